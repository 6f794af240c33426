// Best-matching-unit search for gfx950: fused score contraction + running arg-max, never storing N x K.
//
// For sample x and node k the kernel maximises  score(x, k) = x . w_k - |w_k|^2 / 2, which orders the nodes
// exactly as the squared distance |x - w_k|^2 = |x|^2 - 2 score does (paper Section 3.3.1: b(x) is the
// best-matching unit under the current weights).  The contraction runs as float32 MFMA
// (v_mfma_f32_32x32x2_f32): one instruction multiplies a 32-node x 2-feature slab of W by a 2-feature x 32-sample
// slab of X into a 32 x 32 block of scores, its accumulator pre-loaded with -|w_k|^2 / 2.
//
// Work split.  A wavefront owns MS blocks of 32 samples and keeps their features in registers for the whole
// kernel (lane l holds sample l % 32, features 2 s + l / 32).  The K nodes stream through LDS in stages of 128
// (double-buffered copies of padded weight rows), shared by the four wavefronts of a workgroup.  After each
// 32 x 32 block every lane folds its 16 scores into a running (best, runner-up, position) triple, so one lane
// only ever tracks the nodes of its own half of the rows; the two halves meet once at the end.  On this chip
// float32 MFMA and ordinary vector instructions occupy the same lanes (they do not overlap, not even across
// wavefronts), so the fold is held to four vector instructions per score.
//
// Exactness.  Scores are formed on centred values x - c, w - c (c = column means of W: distances are unchanged,
// magnitudes shrink to the spread of the map).  float32 accumulation leaves an error of at most
// (roundings) * 2^-24 * (|x - c| max|w - c| + max|w - c|^2 / 2) in a score, so a sample whose best two scores are
// closer than that worst-case bound is put on a list and re-decided by direct differences sum_d (x_d - w_kd)^2 on
// the values as given (lowest index wins ties): over every node (bmu_exact_kernel), or, for long lists, over the
// few nodes whose score lies inside the bound, which a second pass of the search collects (bmu_cand_kernel +
// bmu_cand_exact_kernel; the bf16 search for D <= 64 takes the differences at the end of its candidate tile).
// Where the caller asks for distances, the winner's squared distance of all other samples is recomputed by direct
// differences as well, so the reported distances never carry the cancellation error of the score form.
//
// The default search (bmu_split_kernel and bmu_split_wide_kernel further down) is the same scheme with the
// contraction on the bf16 matrix pipe, samples and weights cut into two bf16 parts each.
#include "som_internal.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <math.h>

namespace som {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWavesPerGroup = 4;
constexpr int kThreads = kWavesPerGroup * 64;

constexpr uint32_t kCandMin = 6144;             // shortest list the candidate pass serves (about 25 us; the all-nodes pass takes 4.6 ns a sample)
constexpr uint32_t kCandHalfTiles = 65536;      // up to this length its tiles are halved (one per compute unit and more)
constexpr size_t kCandCapMax = (size_t)1 << 24; // longest one (bounds the candidate buffer at 512 MB + 64 MB)
constexpr int kCandGrid = 2048;

// floats of one 128-node stage (padded rows + half squared norms), rounded up to one float4 per thread
constexpr int stage_floats_for(int stride)
{
    return ((kNodesPerStage * (stride + 1) + 4 * kThreads - 1) / (4 * kThreads)) * (4 * kThreads);
}

// ---------------------------------------------------------------------------------------------------------
// Weight preparation: padded rows + half squared norms per (128-node stage, feature chunk), transposed copy,
// largest squared norm (scal[0], cleared beforehand), and the zeroing of the result words the later kernels count
// into.  A chunk holds stride - 1 features and one zero column (odd row stride); maps with D <= 64 have a single
// chunk.  One thread per element of the padded matrix (coalesced reads of W); the first kpad / 4 wavefronts also
// compute four nodes' norms each, in float64.
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// centre[f] = mean over nodes of W[k][f], f < D; zero up to the next multiple of 64.  Any vector would do (distances do not change when the same vector is
// taken off samples and weights); the mean keeps |w_k - centre| as small as the spread of the map.
__global__ void __launch_bounds__(1024) bmu_centre_kernel(const float* __restrict__ W, int K, int D, float* __restrict__ centre,
                                                          unsigned int* __restrict__ scal)
{
    __shared__ double part[16][64];
    const int fl = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int f = blockIdx.x * 64 + fl;
    // this kernel runs first in every preparation: it also clears the result words (maximum norm, list lengths)
    if (blockIdx.x == 0 && threadIdx.x < 8) scal[threadIdx.x] = 0u;
    double s = 0.0;
    if (f < D) {
        // sixteen loads in flight per thread: the kernel is a chain of memory round trips otherwise
        int k = grp;
        for (; k + 15 * 16 < K; k += 16 * 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = W[(size_t)(k + 16 * u) * D + f];
#pragma unroll
            for (int u = 0; u < 16; ++u) s += (double)v[u];
        }
        for (; k < K; k += 16) s += (double)W[(size_t)k * D + f];
    }
    part[grp][fl] = s;
    __syncthreads();
    if (grp == 0) {                       // the padding up to the next multiple of 64 entries is zeroed
        double t = 0.0;
        for (int q = 0; q < 16; ++q) t += part[q][fl];
        centre[f] = (f < D) ? (float)(t / K) : 0.0f;
    }
}

struct SplitPrep {
    char* stage16;       // null: no split search for this shape
    float* wwin;         // float32 copy of the slots (D <= 64 only), or null
    int kb_count, tail_r, nch16, row_bytes, stage16_bytes;
};
constexpr float kSplitPadNorm = -3.0e38f;     // padding nodes of the split search: finite, so that position bits cannot make a NaN

// One slot of the rows for the bf16 matrix pipe: thread e takes (node, slot), chunks of kb_count 16-feature blocks (one
// chunk for D <= 64, chunks of 64 features above).
// tail_r > 0 (D <= 64 only): the last tail_r <= 4 features do not get a 16-feature block of their own (three MFMAs
// for a block that is mostly padding) but one packed block whose sixteen slots hold the three products side by side,
//     weights  [ hi(r) | hi(r) | lo(r) | norm parts (3) | 0 ... ]   against samples  [ hi(r) | lo(r) | hi(r) | 1 1 1 | 0 ... ],
// one MFMA (the norm parts are written by the wavefront that sums the node's norm).  The float32 copy of the packed
// block (wwin) carries the r centred weights in its first slots.
__device__ __forceinline__ void split_prep_slot(const float* __restrict__ W, int K, int D, int kpad,
                                                const float* __restrict__ centre, const SplitPrep& sp, int e)
{
    const int per_chunk = sp.kb_count * 16 + (sp.tail_r ? 16 : 0), slots = sp.nch16 * per_chunk;
    if (e >= kpad * slots) return;
    const int k = e / slots, sl = e - k * slots;
    const int chunk = sl / per_chunk, within = sl - chunk * per_chunk;
    const int kb = within >> 4, g = (within >> 3) & 1, t = within & 7;
    char* row = sp.stage16 + ((size_t)(k / kNodesPerStage) * sp.nch16 + chunk) * sp.stage16_bytes +
                (size_t)(k % kNodesPerStage) * sp.row_bytes;
    if (kb < sp.kb_count) {
        const int f0 = 64 * chunk + 4 * (4 * kb + 2 * g + (t >> 2));      // the slot group's own first feature
        const int f = (f0 < D - 4 ? f0 : D - 4) + (t & 3);               // its window, always inside the row
        const bool real = k < K && f >= f0;
        const float v = real ? W[(size_t)k * D + f] - centre[f] : 0.0f;
        const __bf16 hi = (__bf16)v;
        const __bf16 lo = (__bf16)(v - (float)hi);
        __bf16* cell = reinterpret_cast<__bf16*>(row + kb * 64 + g * 32) + t;
        cell[0] = hi;
        cell[8] = lo;
        if (sp.wwin) sp.wwin[e] = v;   // the same slots in float32, [node][kb][g][8]: the winner's row for the distances
    } else {
        // packed tail: slot s = 8 g + t holds copy s / r of feature D - r + s % r (copies 0, 1: hi, copy 2: lo); the
        // three slots behind them belong to the norm
        const int sidx = 8 * g + t, copy = sidx / sp.tail_r, f = D - sp.tail_r + sidx % sp.tail_r;
        const float v = (k < K && copy < 3) ? W[(size_t)k * D + f] - centre[f] : 0.0f;
        const __bf16 hi = (__bf16)v;
        const __bf16 lo = (__bf16)(v - (float)hi);
        const int ns = sidx - 3 * sp.tail_r;
        if (ns < 0 || ns >= 3) reinterpret_cast<__bf16*>(row + sp.kb_count * 64 + g * 16)[t] = (copy == 2) ? lo : hi;
        if (sp.wwin) sp.wwin[e] = (copy == 0) ? v : 0.0f;
    }
}

// The rows for the bf16 matrix pipe (stage16 != null; layout at bmu_split_tile) are written by the same launch: one thread per
// (node, slot), and the wavefront that sums a node's norm also writes it where the split search reads it.

__global__ void __launch_bounds__(256) bmu_prep_kernel(const float* __restrict__ W, int K, int D, int kpad, int stride,
                                                       int nch, int stage_floats, const float* __restrict__ centre,
                                                       float* __restrict__ stage, float* __restrict__ wt,
                                                       unsigned int* __restrict__ scal, double* __restrict__ qe,
                                                       int32_t* __restrict__ small, const SplitPrep sp)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    const int cols = nch * stride;
    if (e < 2 && qe) qe[e] = 0.0;
    if (e < 4 && small) small[e] = 0;
    if (sp.stage16) split_prep_slot(W, K, D, kpad, centre, sp, e);
    if (e < kpad * cols) {
        const int k = e / cols, c = e - k * cols;
        const int ch = c / stride, fl = c - ch * stride;
        // stage column fl = 2 s + g feeds MFMA step s, half-wavefront g.  One chunk (D <= 64): feature fl.  Several
        // chunks: the lane's STEPS features are contiguous in a sample row, own range [first, first + STEPS) with
        // first = CH ch + STEPS g.  Where that range would run past D the lane reads the window [D - STEPS, D)
        // instead (always whole, always inside the row) and the columns in front of its own range hold zero
        // weights, so no feature is counted twice.
        const int steps = (stride - 1) / 2;
        const int first = ch * (stride - 1) + (fl & 1) * steps;
        const int window = first < D - steps ? first : D - steps;
        const int f = (nch == 1) ? fl : window + (fl >> 1);
        const bool own = fl < stride - 1 && f < D && (nch == 1 || f >= first);
        const bool real = k < K && own;
        const float v = real ? W[(size_t)k * D + f] : 0.0f;
        const int st = k / kNodesPerStage, r = k % kNodesPerStage;
        stage[((size_t)st * nch + ch) * stage_floats + (size_t)r * stride + fl] = real ? v - centre[f] : 0.0f;
    }
    // transposed copy, one thread per element with the node running fastest: coalesced writes (the reads, one row
    // apart, come from L2; written from the loop above the copy was 50,000 scattered 4-byte stores)
    if (e < D * kpad) {
        const int f = e / kpad, kk = e - f * kpad;
        wt[e] = (kk < K) ? W[(size_t)kk * D + f] : 0.0f;
    }
    // squared norm of the centred row exactly as the stage holds it (float32 differences), summed in float64: the
    // first kpad / 4 wavefronts of the grid take four nodes each (coalesced reads of their rows), and a workgroup
    // hands its largest norm to scal[0] with one atomic (one per node, all on the same word, took 10 us)
    __shared__ float wg_up[4];
    const int wv = e >> 6, lane = e & 63;
    float up_max = 0.0f;
    if (wv * 4 < kpad) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = wv * 4 + q;
            double nrm = 0.0;
            if (k < K)
                for (int f = lane; f < D; f += 64) {
                    const double v = (double)(W[(size_t)k * D + f] - centre[f]);
                    nrm += v * v;
                }
            nrm = wave_sum(nrm);
            if (lane == 0 && k < kpad) {
                const int st = k / kNodesPerStage, r = k % kNodesPerStage;
                const float nh = (k < K) ? (float)(-0.5 * nrm) : -INFINITY;
                for (int ch = 0; ch < nch; ++ch)
                    stage[((size_t)st * nch + ch) * stage_floats + (size_t)kNodesPerStage * stride + r] = nh;
                if (sp.stage16) {
                    const float nf = nh > kSplitPadNorm ? nh : kSplitPadNorm;
                    for (int ch = 0; ch < sp.nch16; ++ch) {
                        char* blob = sp.stage16 + ((size_t)st * sp.nch16 + ch) * sp.stage16_bytes;
                        reinterpret_cast<float*>(blob + (size_t)kNodesPerStage * sp.row_bytes)[r] = nf;
                        if (sp.tail_r) {
                            // -|w|^2 / 2 cut into three bf16 parts (exactly: 3 x 8 bits) in the three slots behind the
                            // packed block's features; they meet ones on the samples' side
                            const __bf16 p0 = (__bf16)nf;
                            const __bf16 p1 = (__bf16)(nf - (float)p0);
                            const __bf16 p2 = (__bf16)((nf - (float)p0) - (float)p1);
                            __bf16* cell = reinterpret_cast<__bf16*>(blob + (size_t)r * sp.row_bytes + sp.kb_count * 64);
                            cell[3 * sp.tail_r] = p0;          // slots 8 g + t are contiguous: [g = 0: 8][g = 1: 8]
                            cell[3 * sp.tail_r + 1] = p1;
                            cell[3 * sp.tail_r + 2] = p2;
                        }
                    }
                }
                if (k < K) {
                    float up = (float)nrm;
                    if ((double)up < nrm) up = nextafterf(up, INFINITY);
                    up_max = fmaxf(up_max, up);
                }
            }
        }
    }
    if (lane == 0) wg_up[threadIdx.x >> 6] = up_max;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float m = fmaxf(fmaxf(wg_up[0], wg_up[1]), fmaxf(wg_up[2], wg_up[3]));
        if (m > 0.0f) atomicMax(&scal[0], __float_as_uint(m));
    }
}

__global__ void fill_zero_kernel(uint32_t* p, size_t words)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// ---------------------------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------------------------

// Sum of distances and squared distances of a workgroup's samples -> one of kQeSlots partial-sum slots.  Every
// wavefront adding to the same two words would serialise tens of thousands of atomics on one address; one pair
// per workgroup spread over 256 slots does not show in the kernel time.  Called by all threads of the workgroup.
__device__ __forceinline__ void group_qe_add(double* __restrict__ part, double qs, double qs2)
{
    __shared__ double wsum[16][2];
    qs = wave_sum(qs);
    qs2 = wave_sum(qs2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        wsum[wave][0] = qs;
        wsum[wave][1] = qs2;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t0 = 0.0, t1 = 0.0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) {
            t0 += wsum[w][0];
            t1 += wsum[w][1];
        }
        if (t0 != 0.0 || t1 != 0.0) {
            const int slot = blockIdx.x & (kQeSlots - 1);
            unsafeAtomicAdd(&part[2 * slot], t0);
            unsafeAtomicAdd(&part[2 * slot + 1], t1);
        }
    }
}

// Append sample i (and its score cut) to the re-decision list for every lane with `push` set: one atomic per wavefront (the list
// length is a single word; one atomic per listed sample serialises on it when a tenth of all samples is listed).
// Called in converged control flow by all lanes of the wavefront.
__device__ __forceinline__ void list_push(unsigned int* __restrict__ counter, uint32_t* __restrict__ list,
                                          float* __restrict__ cutv, bool push, int64_t i, float cut)
{
    const unsigned long long mask = __ballot(push);
    if (mask == 0ull) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((long long)mask) - 1;
    unsigned int base = 0u;
    if (lane == leader) base = atomicAdd(counter, (unsigned int)__popcll(mask));
    base = __shfl(base, leader);
    const unsigned int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
    if (push) {
        list[base + below] = (uint32_t)i;
        if (cutv) cutv[base + below] = cut;     // scores at or above this value may belong to the true winner
    }
}

// The re-decision list of a pass.  The search kernels do not append to it themselves: one atomic per wavefront on the
// list's single length word serialises in the memory system (about 10 ns each; with a few per cent of the samples
// listed nearly every wavefront has one, and the 15,625 wavefronts of 10^6 samples then spent up to 0.1 ms of a
// 0.4 ms kernel queueing for it).  Each sample instead gets one word, its cut (best score minus the rounding bound)
// or kNotListed, and this kernel compacts the listed ones: a workgroup takes 4096 samples at a time, counts with a
// scan, and reserves its entries with one atomic.  The order of the list is immaterial (every entry is decided on its
// own).
constexpr float kNotListed = __builtin_nanf("");
constexpr int kListThreads = 1024, kListPerThread = 4;

__global__ void __launch_bounds__(kListThreads) bmu_list_kernel(const BmuArgs a)
{
    __shared__ unsigned int wave_base[kListThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int64_t per_block = (int64_t)kListThreads * kListPerThread;
    for (int64_t chunk = blockIdx.x; chunk * per_block < a.m; chunk += gridDim.x) {
        const int64_t i0 = chunk * per_block + (int64_t)tid * kListPerThread;
        float c[kListPerThread];
        if (i0 + kListPerThread <= a.m) {
            const float4 t = *reinterpret_cast<const float4*>(a.cut_all + i0);      // i0 is a multiple of four
            c[0] = t.x;
            c[1] = t.y;
            c[2] = t.z;
            c[3] = t.w;
        } else {
#pragma unroll
            for (int q = 0; q < kListPerThread; ++q) c[q] = (i0 + q < a.m) ? a.cut_all[i0 + q] : kNotListed;
        }
        static_assert(kListPerThread == 4, "a thread's cuts travel as one float4");
        unsigned int mine = 0u;
#pragma unroll
        for (int q = 0; q < kListPerThread; ++q) mine += (c[q] == c[q]) ? 1u : 0u;
        unsigned int incl = mine;                         // inclusive scan over the wavefront
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wave_base[wave] = incl;
        __syncthreads();
        if (wave == 0) {
            // exclusive scan of the wavefronts' totals; the last lane reserves the workgroup's entries
            const unsigned int w = lane < kListThreads / 64 ? wave_base[lane] : 0u;
            unsigned int wi = w;
#pragma unroll
            for (int o = 1; o < kListThreads / 64; o <<= 1) {
                const unsigned int t = __shfl_up(wi, o);
                if (lane >= o) wi += t;
            }
            const unsigned int total = __shfl(wi, kListThreads / 64 - 1);
            unsigned int base = 0u;
            if (lane == 0 && total) base = atomicAdd(&a.scal[a.slot], total);
            base = __shfl(base, 0);
            if (lane < kListThreads / 64) wave_base[lane] = base + wi - w;
        }
        __syncthreads();
        unsigned int pos = wave_base[wave] + incl - mine;
#pragma unroll
        for (int q = 0; q < kListPerThread; ++q) {
            if (c[q] == c[q]) {
                a.recheck[pos] = (uint32_t)(i0 + q);
                a.cutv[pos] = c[q];
                ++pos;
            }
        }
        __syncthreads();                                 // wave_base is rewritten by the next chunk
    }
}

// sixteen bytes from a 4-byte aligned address in one load (global memory needs no more than dword alignment)
__device__ __forceinline__ float4 load4(const float* p)
{
    float4 v;
    __builtin_memcpy(&v, p, sizeof(v));
    return v;
}

// Up to seven 16-bit node ids and their count in 128 bits of registers.  A hit shifts the ids up by one place (the
// oldest drops out at the top, the count keeps counting, so an overflow shows): no memory traffic while the scores
// are being formed, one 16-byte store per lane at the end.
struct CandSet {
    unsigned long long lo = 0ull, hi = 0ull;
    int n = 0;
    // id = base + off
    __device__ __forceinline__ void note(int base, int off)
    {
        // (The empty statement keeps the branch that skips these instructions when no lane of the wavefront has a
        // hit, which is four times out of five: without it the compiler runs them under an empty mask, and every
        // vector instruction here is paid for in matrix time.  Passing the base through it keeps the addition
        // inside the skipped region as well.)
        asm volatile("" : "+v"(base));
        const int id = base + off;
        hi = (hi << 16) | (lo >> 48);
        lo = (lo << 16) | (unsigned long long)(unsigned int)id;
        ++n;
    }
    __device__ __forceinline__ ulonglong2 packed() const
    {
        const unsigned long long c = (unsigned long long)(n < 0xffff ? n : 0xffff);
        return make_ulonglong2(lo, (hi & 0xffffffffffffull) | (c << 48));
    }
};
__device__ __forceinline__ int cand_count(const ulonglong2& v) { return (int)(v.y >> 48); }
__device__ __forceinline__ int cand_id(const ulonglong2& v, int t)
{
    return (int)(((t < 4) ? (v.x >> (16 * t)) : (v.y >> (16 * (t - 4)))) & 0xffffull);
}

// plain v_max_f32: the scores are never signalling NaNs worth quieting, and every VALU instruction here is paid
// for in matrix time (float32 MFMA and the vector ALU share the same lanes)
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// plain v_max3_f32, for the same reason
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// ---------------------------------------------------------------------------------------------------------
// main kernel
// ---------------------------------------------------------------------------------------------------------
// One tile = the kWavesPerGroup * MS * 32 samples of a workgroup against all nodes.
// CAND = false: the search proper (samples wave0 ..., running best / runner-up, results and list at the end).
// CAND = true: the candidate pass over the first `count` entries of the re-decision list: the same scores are
// formed again, and instead of the fold every score that reaches the entry's cut is noted (node id into the
// lane's own slots: lane (j, g) sees the nodes of half g only, so no two lanes share a slot and no atomics are
// needed).  One compare per score instead of four fold instructions.
// PAD = true: the last stage ends in whole blocks of padding nodes (K is at least 32 short of a multiple of 128),
// which are skipped; a variant of its own so that the stage body of the other maps stays one basic block.
template <int STEPS, int MS, bool CAND, bool PAD = false>
__device__ __forceinline__ void bmu_tile(const BmuArgs& a, int64_t first, int64_t tile_index, unsigned int count,
                                         float4* lds4)
{
    constexpr int STRIDE = 2 * STEPS + 1;
    constexpr int STAGE_FLOATS = stage_floats_for(STRIDE);   // whole float4s per thread: no tail handling
    constexpr int STAGE_F4 = STAGE_FLOATS / 4;
    constexpr int PRE = STAGE_F4 / kThreads;
    float* lds = reinterpret_cast<float*>(lds4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 31;
    const int g = lane >> 5;
    const int64_t wave0 = first + (tile_index * kWavesPerGroup + wave) * (MS * 32);   // first = position of tile 0

    // centre[2 s + g]: both candidates are read through wave-uniform addresses (scalar loads), the lane picks one
    // (the array is zero-padded to a multiple of 64 entries, so no index needs a bound)
    auto centre_of = [&](int s) {
        const float c0 = a.centre[2 * s], c1 = a.centre[2 * s + 1];
        return g ? c1 : c0;
    };

    // ---- this wavefront's samples, kept in registers
    float x[MS][STEPS];
    bool valid[MS];
    float cut[MS];          // CAND
    CandSet noted[MS];      // CAND
    // (Staging the workgroup's rows through LDS with coalesced 16-byte loads was measured against this direct
    // gather and lost by 3 to 10 %: the gather is served by the vector L1, the staging adds two barriers.)
#pragma unroll
    for (int mb = 0; mb < MS; ++mb) {
        int64_t i = wave0 + mb * 32 + j;
        const int64_t total = CAND ? (int64_t)count : a.m;
        valid[mb] = i < total;
        int64_t ii = valid[mb] ? i : total - 1;
        if constexpr (CAND) {
            cut[mb] = valid[mb] ? a.cutv[ii] : NAN;     // no score compares >= NaN
            ii = (int64_t)a.recheck[ii];
        }
        const int64_t row = a.idx ? (int64_t)a.idx[ii] : ii;
        const float* xr = a.X + row * a.ldx;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int f = 2 * s + g;
            // Unconditional load through a clamped index.  Beyond D the value is a copy of the last feature; it
            // meets zero weights in the stage rows, and the epilogue masks it out of the norms.
            x[mb][s] = xr[f < a.D ? f : a.D - 1];
        }
    }

    // running best / runner-up scores of this lane's half of the rows, and where the best one sits
    float best[MS], second[MS];
    int rsel[MS], tsel[MS];
#pragma unroll
    for (int mb = 0; mb < MS; ++mb) {
        best[mb] = -INFINITY;
        second[mb] = -INFINITY;
        rsel[mb] = 0;
        tsel[mb] = 0;
    }

    // ---- stream the nodes through LDS
    const int nstages = a.kpad / kNodesPerStage;
    const float4* src4 = reinterpret_cast<const float4*>(a.stage);
    {
        float4 first[PRE];
#pragma unroll
        for (int p = 0; p < PRE; ++p) first[p] = src4[tid + p * kThreads];
        // the samples are centred only now, with the first stage's loads already on their way
#pragma unroll
        for (int mb = 0; mb < MS; ++mb)
#pragma unroll
            for (int s = 0; s < STEPS; ++s) x[mb][s] -= centre_of(s);
#pragma unroll
        for (int p = 0; p < PRE; ++p) lds4[tid + p * kThreads] = first[p];
    }
    __syncthreads();

    for (int st = 0; st < nstages; ++st) {
        const int buf = st & 1;
        // the next stage travels global -> registers now and registers -> LDS after this stage's arithmetic
        // (the last iteration reloads its own stage into the idle buffer, which keeps the loop branch-free).
        // Named scalars rather than an array, and a scheduling fence behind the loads: otherwise the compiler
        // sinks every load to its use after the MFMAs and the copy is no longer hidden.
        float4 pre0, pre1, pre2, pre3, pre4, pre5, pre6, pre7, pre8;
        static_assert(PRE <= 9, "stage copy holds at most nine float4 per thread");
        {
            const int nxt = (st + 1 < nstages) ? st + 1 : st;
            const float4* s4 = src4 + (size_t)nxt * STAGE_F4 + tid;
#define SOM_PRE_LOAD(i) if constexpr (PRE > i) pre##i = s4[i * kThreads];
            SOM_PRE_LOAD(0) SOM_PRE_LOAD(1) SOM_PRE_LOAD(2) SOM_PRE_LOAD(3) SOM_PRE_LOAD(4)
            SOM_PRE_LOAD(5) SOM_PRE_LOAD(6) SOM_PRE_LOAD(7) SOM_PRE_LOAD(8)
#undef SOM_PRE_LOAD
        }
        __builtin_amdgcn_sched_barrier(0);
        const float* wbuf = lds + buf * STAGE_FLOATS;
        const float* nbuf = wbuf + kNodesPerStage * STRIDE;

        // Fully unrolled: with the stage body in one basic block the prefetch loads above stay ahead of the MFMAs.
        // The LDS reads of node block nb + 1 (weights and -|w|^2/2) are written into the MFMA sequence of block nb,
        // one read per pair of MFMAs, and pinned there: left alone the scheduler sometimes gathers all reads of a
        // block in front of its first MFMA, and the matrix pipe then idles for an LDS round trip per block.
        float wa[STEPS];
        floatx16 c;
        {
            const float* wrow = wbuf + j * STRIDE + g;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) wa[s] = wrow[2 * s];
            const float4* nh = reinterpret_cast<const float4*>(nbuf + 4 * g);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 t = nh[2 * q];
                c[4 * q + 0] = t.x;
                c[4 * q + 1] = t.y;
                c[4 * q + 2] = t.z;
                c[4 * q + 3] = t.w;
            }
        }
#pragma unroll
        for (int nb = 0; nb < kNodesPerStage / 32; ++nb) {
            constexpr int NB = kNodesPerStage / 32;
            if constexpr (PAD) {
                if (st * kNodesPerStage + nb * 32 >= a.K) break;           // padding from here to the end of the stage
            }
            const int nx = (nb + 1 < NB) ? nb + 1 : nb;                    // the last block re-reads itself (unused)
            const float* wnext = wbuf + (nx * 32 + j) * STRIDE + g;
            const float4* nhnext = reinterpret_cast<const float4*>(nbuf + nx * 32 + 4 * g);
            float wn[STEPS];
            floatx16 cn;
            floatx16 acc[MS];
#pragma unroll
            for (int mb = 0; mb < MS; ++mb) acc[mb] = c;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
#pragma unroll
                for (int mb = 0; mb < MS; ++mb)
                    acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[s], x[mb][s], acc[mb], 0, 0, 0);
                if (nb + 1 < NB) {
                    wn[s] = wnext[2 * s];
                    if (s < 4) {
                        const float4 t = nhnext[2 * s];
                        cn[4 * s + 0] = t.x;
                        cn[4 * s + 1] = t.y;
                        cn[4 * s + 2] = t.z;
                        cn[4 * s + 3] = t.w;
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, MS, 0);    // MS MFMAs
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
                }
            }
            const int tile = st * (kNodesPerStage / 32) + nb;
            if constexpr (CAND) {
#pragma unroll
                for (int mb = 0; mb < MS; ++mb) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (acc[mb][r] >= cut[mb]) noted[mb].note(tile * 32 + 4 * g, 8 * (r >> 2) + (r & 3));
                }
            }
            // fold the 16 scores of each block into the running triple: four VALU instructions per score
#pragma unroll
            for (int mb = 0; mb < (CAND ? 0 : MS); ++mb) {
                const float before = best[mb];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[mb][r];
                    rsel[mb] = (v > best[mb]) ? r : rsel[mb];
                    second[mb] = __builtin_amdgcn_fmed3f(best[mb], second[mb], v);
                    best[mb] = vmax(best[mb], v);
                }
                tsel[mb] = (best[mb] > before) ? tile : tsel[mb];
            }
            if (nb + 1 < NB) {
#pragma unroll
                for (int s = 0; s < STEPS; ++s) wa[s] = wn[s];
                c = cn;
            }
        }

        {
            float4* d4 = lds4 + (buf ^ 1) * STAGE_F4 + tid;
#define SOM_PRE_STORE(i) if constexpr (PRE > i) d4[i * kThreads] = pre##i;
            SOM_PRE_STORE(0) SOM_PRE_STORE(1) SOM_PRE_STORE(2) SOM_PRE_STORE(3) SOM_PRE_STORE(4)
            SOM_PRE_STORE(5) SOM_PRE_STORE(6) SOM_PRE_STORE(7) SOM_PRE_STORE(8)
#undef SOM_PRE_STORE
        }
        __syncthreads();
    }

    if constexpr (CAND) {
#pragma unroll
        for (int mb = 0; mb < MS; ++mb)
            if (valid[mb])
                a.cand[(size_t)(wave0 + mb * 32 + j) * 2 + g] = noted[mb].packed();
        return;
    }
    // ---- join the two half-wavefronts, then lane (j, g) finishes block mp + g
    const float wmax2 = __uint_as_float(a.scal[0]);
    const float wmax = sqrtf(wmax2) * 1.000001f;
    // two scores, each with two roundings per MFMA step (k = 2) and one in -|w|^2/2; the roundings of x - centre
    // and w - centre move a score difference by at most 2 and 4 more units: (4 STEPS + 8) * 2^-24, plus slack
    const float rel = (float)(4 * STEPS + 12) * 5.9604645e-08f;
    double qs = 0.0, qs2 = 0.0;
#pragma unroll
    for (int mp = 0; mp < MS; mp += 2) {
        float r_best = 0.f, r_second = 0.f, r_xn = 0.f, r_part = 0.f;
        int r_node = 0;
        bool r_valid = false;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int mb = mp + q;
            if (mb >= MS) break;
            int node = tsel[mb] * 32 + 8 * (rsel[mb] >> 2) + 4 * g + (rsel[mb] & 3);
            const float ob = __shfl_xor(best[mb], 32);
            const float os = __shfl_xor(second[mb], 32);
            const int on = __shfl_xor(node, 32);
            const float sec = fmaxf(fmaxf(second[mb], os), fminf(best[mb], ob));
            const bool other = (ob > best[mb]) || (ob == best[mb] && on < node);
            const float bst = other ? ob : best[mb];
            node = other ? on : node;
            node = node < a.K ? node : a.K - 1;
            // squared norm of the centred sample and squared distance to the winner (both centred the same way),
            // half the features per lane
            // (the winner's centred weights come from its stage row, which holds them in this lane's order with
            // zeros beyond D: no centring and no bounds here)
            float xn = 0.f, part = 0.f;
            const float* wr = a.stage + (size_t)(node / kNodesPerStage) * STAGE_FLOATS +
                              (size_t)(node % kNodesPerStage) * STRIDE + g;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float xm = (2 * s + g < a.D) ? x[mb][s] : 0.0f;
                const float df = xm - wr[2 * s];
                xn = fmaf(xm, xm, xn);
                part = fmaf(df, df, part);
            }
            xn += __shfl_xor(xn, 32);
            part += __shfl_xor(part, 32);
            if (q == g) {
                r_best = bst;
                r_second = sec;
                r_node = node;
                r_xn = xn;
                r_part = part;
                r_valid = valid[mb];
            }
        }
        const int64_t i = wave0 + (mp + g) * 32 + j;
        // magnitude bound of every partial sum of the score: |w|^2/2 + |sum x_d w_d| <= |w|^2/2 + |x| |w|
        const float xl = sqrtf(r_xn);
        const float bound = (xl * wmax + 0.5f * wmax2) * rel;
        // the two centring roundings leave an error of 2^-23 d (|x| + |w|) in d^2: hand the few samples that
        // sit within 2^-9 (|x| + |w|) of their node to the exact pass, which works on the values as given
        const float tiny = (xl + wmax) * (xl + wmax) * 3.8146973e-06f;
        const bool close = r_valid && a.K > 1 && (!((r_best - r_second) > bound) || r_part < tiny);
        if (r_valid) {
            a.bmu[i] = r_node;
            if (a.d2) a.d2[i] = r_part;
            if (!close) {
                qs += sqrt((double)r_part);
                qs2 += (double)r_part;
            }
        }
        if (r_valid) a.cut_all[i] = close ? r_best - bound : kNotListed;
    }
    if (a.qe) group_qe_add(a.qe_part, qs, qs2);
}

// two workgroups per compute unit (LDS-bound), i.e. two wavefronts per SIMD: the register budget is 256 VGPRs
template <int STEPS, int MS, bool PAD>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    // The first full_tiles workgroups take MS blocks per wavefront; the rest of the grid, the last partial round
    // of the launch, takes tiles of half that size, which spread more evenly over the compute units.
    if ((int64_t)blockIdx.x < a.full_tiles) {
        bmu_tile<STEPS, MS, false, PAD>(a, 0, blockIdx.x, 0u, lds4);
    } else if constexpr (MS > 1) {
        constexpr int64_t per_full = (int64_t)kWavesPerGroup * MS * 32;
        bmu_tile<STEPS, MS / 2, false, PAD>(a, a.full_tiles * per_full, (int64_t)blockIdx.x - a.full_tiles, 0u, lds4);
    }
}

// true when this call's list is long enough for the candidate pass to pay and fits its buffers (device-side: the
// host does not know the list length)
__device__ __forceinline__ bool cand_pass_serves(const BmuArgs& a, unsigned int count)
{
    return count > a.cand_min && count <= a.cand_cap;
}

// candidate pass: a fixed grid walks the tiles of the list
template <int STEPS, int MS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_cand_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    const unsigned int count = a.scal[a.slot];
    if (!cand_pass_serves(a, count)) return;
    constexpr int64_t per_tile = (int64_t)kWavesPerGroup * MS * 32;
    if constexpr (MS > 1) {
        // a list that leaves compute units idle goes through in tiles of half the size: twice as many workgroups,
        // each done in half the time
        if (count <= kCandHalfTiles) {
            for (int64_t t = blockIdx.x; t * (per_tile / 2) < (int64_t)count; t += gridDim.x)
                bmu_tile<STEPS, MS / 2, true>(a, 0, t, count, lds4);
            return;
        }
    }
    for (int64_t t = blockIdx.x; t * per_tile < (int64_t)count; t += gridDim.x) bmu_tile<STEPS, MS, true>(a, 0, t, count, lds4);
}

// ---------------------------------------------------------------------------------------------------------
// The same search with the contraction on the bf16 matrix pipe (this kernel: 4 <= D <= 64, bmu_split_wide_kernel
// below: D > 64; the default for every map of more than one node).
//
// A float32 value v is cut into two bf16 parts, hi = bf16(v) and lo = bf16(v - hi) (both rounded to nearest, the
// difference is exact in float32), so that |v - hi - lo| <= 2^-18 |v|.  A score then takes three bf16 MFMAs per 16
// features (v_mfma_f32_32x32x16_bf16, products exact, float32 accumulation):
//     x . w  ~  xh . wh + xl . wh + xh . wl,
// the dropped parts together below 3 * 2^-18 |x| |w|.  The bf16 pipe runs these three in 96 cycles where the
// float32 MFMAs of the same 16 features take 512, and unlike those it leaves three quarters of the vector issue
// slots to the fold, which runs beside it.  Nothing else changes: the error bound is wider (the split, and the pipe's
// accumulation error per MFMA, charged as any-order float32 summation), samples inside it go on the same list and are decided by the same direct
// differences, so the results are those of the float32 search.
//
// Layout.  Lane (j, g) of a wavefront holds, for k-block kb, the eight features of slot groups q = 4 kb + 2 g and
// q + 1, group q being the window [min(4 q, D - 4), + 4) of the row: always whole and inside the row, so a group is
// one 16-byte load; where the window is shifted back the stage rows hold zero weights in front of the group's own
// features, and no feature is counted twice.  A stage row is [kb][g][hi x 8 | lo x 8] bf16 plus 16 bytes of padding
// (row stride 64 * blocks + 16 bytes: the 16-byte reads of sixteen consecutive rows fall into distinct banks), followed
// by the stage's 128 half squared norms in float32.
// The fold keeps the position inside a block in the low four bits of the score (one and-or instead of a compare
// and a select; 16 units of the last place are part of the bound), so padding nodes carry a large finite negative
// norm here instead of -inf.
// ---------------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// bytes of a stage row: kb whole 16-feature blocks of 64 bytes, 32 bytes for a packed tail block, 16 bytes of padding
constexpr int split_row_bytes(int kb, bool tail = false) { return kb * 64 + (tail ? 32 : 0) + 16; }
constexpr int split_stage_f4(int kb, bool tail = false)
{
    return ((kNodesPerStage * split_row_bytes(kb, tail) + kNodesPerStage * 4) / 16 + kThreads - 1) / kThreads * kThreads;
}
constexpr int kSplitMinNodes = 1;              // SOM_SEARCH_AUTO: every map of more than this many nodes (measured faster than the
                                               // float32 search from 2 x 2 nodes and from D = 4 on)
constexpr size_t kPartsBytes = (size_t)8 << 30;    // workspace of the samples' bf16 parts (D > 64), per pass
constexpr int kSplitMS = 2;

__device__ __forceinline__ void split8(const float (&v)[8], bf16x8& hi, bf16x8& lo)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        hi[i] = (__bf16)v[i];
        lo[i] = (__bf16)(v[i] - (float)hi[i]);
    }
}

// first feature of slot group q (four consecutive features)
__device__ __forceinline__ int split_window(int q, int D) { return 4 * q < D - 4 ? 4 * q : D - 4; }

// CAND = true: the candidate pass over the first `count` entries of the re-decision list (as in bmu_tile): the same
// scores are formed again, bit for bit, and every node whose score reaches the entry's cut is noted.
// KB whole 16-feature blocks (three MFMAs each) and, with TAIL, one packed block for the last a.tail_r <= 4 features
// (one MFMA; layout in bmu_prep_split_kernel).
template <int KB, bool TAIL, int MS, bool CAND>
__device__ __forceinline__ void bmu_split_tile(const BmuArgs& a, int64_t first, int64_t tile_index, unsigned int count,
                                               float4* lds4)
{
    constexpr int RS = split_row_bytes(KB, TAIL);
    constexpr int STAGE_F4 = split_stage_f4(KB, TAIL);
    constexpr int KBA = KB > 0 ? KB : 1;               // array lengths (no zero-length arrays when D <= 4)
    constexpr int WROW = KB * 16 + (TAIL ? 16 : 0);    // floats of a node's row in wwin
    constexpr int PRE = STAGE_F4 / kThreads;
    const char* ldsb = reinterpret_cast<const char*>(lds4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 31;
    const int g = lane >> 5;
    const int64_t wave0 = first + (tile_index * kWavesPerGroup + wave) * (MS * 32);

    // This lane's 8 KB slots of a sample row, centred; slots in front of a shifted window's own features read zero
    // (they meet zero weights in the stage rows, and stay out of the norms and distances).
    auto centred_slots = [&](const float* xr, int D, float (&v)[KBA][8]) {
        float4 raw[KBA][2], cen[KBA][2];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int start = split_window(4 * kb + 2 * g + h, D);
                raw[kb][h] = load4(xr + start);
                cen[kb][h] = load4(a.centre + start);
            }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int q = 4 * kb + 2 * g + h;
                const int shift = 4 * q - split_window(q, D);            // own slots: i >= shift
                v[kb][4 * h + 0] = shift <= 0 ? raw[kb][h].x - cen[kb][h].x : 0.0f;
                v[kb][4 * h + 1] = shift <= 1 ? raw[kb][h].y - cen[kb][h].y : 0.0f;
                v[kb][4 * h + 2] = shift <= 2 ? raw[kb][h].z - cen[kb][h].z : 0.0f;
                v[kb][4 * h + 3] = shift <= 3 ? raw[kb][h].w - cen[kb][h].w : 0.0f;
            }
    };

    // the last tail_r features of a row, centred: vt[t] = feature D - tail_r + t (zero for t >= tail_r); one 16-byte
    // load of the window [D - 4, D), which lies inside the row because D >= 4
    const int tail_r = TAIL ? a.tail_r : 0;
    auto tail_values = [&](const float* xr, int D, float (&vt)[4]) {
        const float4 raw = load4(xr + D - 4), cen = load4(a.centre + D - 4);
        const float c4[4] = {raw.x - cen.x, raw.y - cen.y, raw.z - cen.z, raw.w - cen.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int src = 4 - tail_r + t;              // 0 .. 3 for t < tail_r
            float v = c4[3];
            v = src == 2 ? c4[2] : v;
            v = src == 1 ? c4[1] : v;
            v = src == 0 ? c4[0] : v;
            vt[t] = t < tail_r ? v : 0.0f;
        }
    };
    // this lane's eight slots of the packed block: slot s = 8 g + i holds copy s / tail_r of tail feature s % tail_r,
    // the samples' copies being hi, lo, hi (against the weights' hi, hi, lo)
    auto tail_pack = [&](const float (&vt)[4]) {
        bf16x8 out;
        __bf16 hi[4], lo[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            hi[t] = (__bf16)vt[t];
            lo[t] = (__bf16)(vt[t] - (float)hi[t]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int sidx = 8 * g + i;
            const int copy = (sidx >= tail_r) + (sidx >= 2 * tail_r) + (sidx >= 3 * tail_r);
            const int t = sidx - copy * tail_r;
            __bf16 h = hi[3], l = lo[3];
            h = t == 2 ? hi[2] : h;
            l = t == 2 ? lo[2] : l;
            h = t == 1 ? hi[1] : h;
            l = t == 1 ? lo[1] : l;
            h = t == 0 ? hi[0] : h;
            l = t == 0 ? lo[0] : l;
            const __bf16 zero = (__bf16)0.0f, one = (__bf16)1.0f;
            const int ns = sidx - 3 * tail_r;                 // 0, 1, 2: opposite the three parts of -|w|^2 / 2
            out[i] = copy > 2 ? ((ns >= 0 && ns < 3) ? one : zero) : (copy == 1 ? l : h);
        }
        return out;
    };

    // ---- this wavefront's samples: centred, cut into bf16 parts, kept in registers
    bf16x8 xh[MS][KBA], xl[MS][KBA], xt[MS];
    bool valid[MS];
    const float* xrow[MS];
    float xnorm2[MS];       // search: squared norm of the centred sample (both lane halves hold the whole row's)
    float cut[MS];          // CAND
    CandSet noted[MS];      // CAND
#pragma unroll
    for (int mb = 0; mb < MS; ++mb) {
        const int64_t i = wave0 + mb * 32 + j;
        const int64_t total = CAND ? (int64_t)count : a.m;
        valid[mb] = i < total;
        int64_t ii = valid[mb] ? i : total - 1;
        if constexpr (CAND) {
            cut[mb] = valid[mb] ? a.cutv[ii] : NAN;     // no score compares >= NaN
            ii = (int64_t)a.recheck[ii];
        }
        const int64_t row = a.idx ? (int64_t)a.idx[ii] : ii;
        xrow[mb] = a.X + row * a.ldx;
        float xs = 0.0f;     // this lane's slots, in the order the end of the tile adds them up
        if constexpr (TAIL) {
            float vt[4];
            tail_values(xrow[mb], a.D, vt);
            xt[mb] = tail_pack(vt);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float xv = g == 0 ? vt[t] : 0.0f;      // the packed block's features once each
                xs = fmaf(xv, xv, xs);
            }
        }
        if constexpr (KB > 0) {
            float v[KBA][8];
            centred_slots(xrow[mb], a.D, v);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                split8(v[kb], xh[mb][kb], xl[mb][kb]);
#pragma unroll
                for (int t = 0; t < 8; ++t) xs = fmaf(v[kb][t], v[kb][t], xs);
            }
        }
        xnorm2[mb] = CAND ? 0.0f : xs + __shfl_xor(xs, 32);
    }

    // running best / runner-up scores of this lane's half of the rows (position in the block in the low four bits
    // of the score) and the block the best one came from
    float best[MS], second[MS], before[MS];
    int tsel[MS];
#pragma unroll
    for (int mb = 0; mb < MS; ++mb) {
        best[mb] = -INFINITY;
        second[mb] = -INFINITY;
        before[mb] = -INFINITY;
        tsel[mb] = 0;
    }
    // one fold step: scores r0, r0 + 1 of sample block mb of the node block `tile`.  With v1, v2 the two scores (position
    // in their low bits), the largest of {best, second, v1, v2} is max3(best, v1, v2) and, because second <= best, the
    // second largest is max(second, med3(best, v1, v2)): five vector instructions per two scores, plus two per block
    // for the block number
    auto fold_step = [&](const floatx16 (&acc)[MS], int step, int tile) {
        const int mb = step >> 3, r0 = 2 * (step & 7);
        if constexpr (CAND) {
            // (the set that the very first block "folds" holds the padding value, which reaches no cut)
            if (acc[mb][r0] >= cut[mb]) noted[mb].note(tile * 32 + 4 * g, 8 * (r0 >> 2) + (r0 & 3));
            if (acc[mb][r0 + 1] >= cut[mb]) noted[mb].note(tile * 32 + 4 * g, 8 * ((r0 + 1) >> 2) + ((r0 + 1) & 3));
            return;
        }
        if (r0 == 0) before[mb] = best[mb];
        const float v1 = __uint_as_float((__float_as_uint(acc[mb][r0]) & 0xfffffff0u) | (unsigned)r0);
        const float v2 = __uint_as_float((__float_as_uint(acc[mb][r0 + 1]) & 0xfffffff0u) | (unsigned)(r0 + 1));
        const float mid = __builtin_amdgcn_fmed3f(best[mb], v1, v2);
        best[mb] = vmax3(best[mb], v1, v2);
        second[mb] = vmax(second[mb], mid);
        if (r0 == 14) tsel[mb] = (best[mb] > before[mb]) ? tile : tsel[mb];
    };

    // ---- stream the nodes through LDS
    const int nstages = a.kpad / kNodesPerStage;
    const float4* src4 = reinterpret_cast<const float4*>(a.stage16);
    {
#pragma unroll
        for (int p = 0; p < PRE; ++p) lds4[tid + p * kThreads] = src4[tid + p * kThreads];
    }
    __syncthreads();

    // The scores of a node block are folded while the matrix pipe works on the next block: two sets of accumulators
    // take turns, and the fold's instructions are written between the MFMAs (the pipe is busy 32 cycles per MFMA,
    // of which the issue of the MFMA itself takes 16 on the vector port).  The very first block folds a set that
    // holds the padding value, which any real score replaces.
    floatx16 accA[MS], accB[MS];
#pragma unroll
    for (int mb = 0; mb < MS; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) accB[mb][r] = kSplitPadNorm;

    constexpr int GROUPS = 3 * KB + (TAIL ? 1 : 0);   // groups of MS MFMAs per node block
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    constexpr int STEPS_ALL = 8 * MS;          // fold steps (two scores each) per node block
    auto block = [&](floatx16 (&cur)[MS], const floatx16 (&prev)[MS], bf16x8 (&wh)[KBA], bf16x8 (&wl)[KBA], bf16x8& wtl,
                     floatx16& c, const char* wnext, const float4* nhnext, bool more, int tile) {
        // the norms of the next block replace c once the block's first group has read it
        auto next_norms = [&]() {
            if constexpr (TAIL) return;      // the norms travel inside the packed block
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 t = nhnext[2 * q];
                c[4 * q + 0] = t.x;
                c[4 * q + 1] = t.y;
                c[4 * q + 2] = t.z;
                c[4 * q + 3] = t.w;
            }
        };
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int term = 0; term < 3; ++term) {
                const int grp = 3 * kb + term;
                const bf16x8 wa = (term == 2) ? wl[kb] : wh[kb];
#pragma unroll
                for (int mb = 0; mb < MS; ++mb) {
                    cur[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, (term == 1) ? xl[mb][kb] : xh[mb][kb],
                                                                      grp == 0 ? (TAIL ? zero16 : c) : cur[mb], 0, 0, 0);
                    // this MFMA's share of the previous block's fold, fenced so that it stays behind it
                    const int m = grp * MS + mb;
                    const int s0 = m * STEPS_ALL / (GROUPS * MS), s1 = (m + 1) * STEPS_ALL / (GROUPS * MS);
#pragma unroll
                    for (int sidx = s0; sidx < s1; ++sidx) fold_step(prev, sidx, tile - 1);
                    if (mb + 1 < MS) __builtin_amdgcn_sched_barrier(0);
                }
                // LDS reads of the next block, into the registers this group has just finished with
                if (more) {
                    if (grp == 0) next_norms();
                    if (term == 2) {
                        wh[kb] = *reinterpret_cast<const bf16x8*>(wnext + kb * 64);
                        wl[kb] = *reinterpret_cast<const bf16x8*>(wnext + kb * 64 + 16);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (TAIL) {
            constexpr int grp = 3 * KB;
#pragma unroll
            for (int mb = 0; mb < MS; ++mb) {
                cur[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wtl, xt[mb], grp == 0 ? zero16 : cur[mb], 0, 0, 0);
                const int m = grp * MS + mb;
                const int s0 = m * STEPS_ALL / (GROUPS * MS), s1 = (m + 1) * STEPS_ALL / (GROUPS * MS);
#pragma unroll
                for (int sidx = s0; sidx < s1; ++sidx) fold_step(prev, sidx, tile - 1);
                if (mb + 1 < MS) __builtin_amdgcn_sched_barrier(0);
            }
            if (more) {
                if (grp == 0) next_norms();
                wtl = *reinterpret_cast<const bf16x8*>(wnext + KB * 64 - g * 16);    // (wnext carries g * 32)
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The first node block's operands; every later block's are read while the block before it is on the matrix pipe.
    bf16x8 wh[KBA], wl[KBA], wtl;
    floatx16 c;
    {
        const char* wrow = ldsb + j * RS + g * 32;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            wh[kb] = *reinterpret_cast<const bf16x8*>(wrow + kb * 64);
            wl[kb] = *reinterpret_cast<const bf16x8*>(wrow + kb * 64 + 16);
        }
        if constexpr (TAIL) wtl = *reinterpret_cast<const bf16x8*>(wrow + KB * 64 - g * 16);
        const float4* nh = reinterpret_cast<const float4*>(ldsb + kNodesPerStage * RS) + g;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 t = TAIL ? float4{0.f, 0.f, 0.f, 0.f} : nh[2 * q];
            c[4 * q + 0] = t.x;
            c[4 * q + 1] = t.y;
            c[4 * q + 2] = t.z;
            c[4 * q + 3] = t.w;
        }
    }
    // One stage: the next stage travels global -> registers at the start and registers -> the idle LDS buffer after
    // the second block; the stage's only barrier stands in front of its last block, whose spare LDS slots then read
    // the first block of the next stage.  (With the barrier at the end of the stage a wavefront stood still for an
    // LDS write, the barrier and an LDS read once per stage; alone on its SIMD, while the unit's other workgroup
    // loads or stores its samples, that cost a fifth of its time.)  Why this is safe: a buffer's last reads, the
    // operands of its stage's last block, are issued during the block before that barrier and waited for before
    // it, so once a wavefront is past the barrier of stage s the buffer of stage s is free for stage s + 2, which
    // nobody writes before the middle of stage s + 1; and the barrier of stage s stands between every wavefront's
    // writes of stage s + 1 and the first reads of it.
    constexpr int NB = kNodesPerStage / 32;
    static_assert(NB == 4, "two blocks, the LDS writes, one block, the barrier, one block");
    for (int st = 0; st < nstages; ++st) {
        const int buf = st & 1;
        // (the last iteration reloads its own stage into the idle buffer, which keeps the loop branch-free)
        float4 pre0, pre1, pre2, pre3, pre4, pre5, pre6, pre7, pre8;
        static_assert(PRE <= 9, "stage copy holds at most nine float4 per thread");
        {
            const int nxt = (st + 1 < nstages) ? st + 1 : st;
            const float4* s4 = src4 + (size_t)nxt * STAGE_F4 + tid;
#define SOM_PRE_LOAD(i) if constexpr (PRE > i) pre##i = s4[i * kThreads];
            SOM_PRE_LOAD(0) SOM_PRE_LOAD(1) SOM_PRE_LOAD(2) SOM_PRE_LOAD(3) SOM_PRE_LOAD(4)
            SOM_PRE_LOAD(5) SOM_PRE_LOAD(6) SOM_PRE_LOAD(7) SOM_PRE_LOAD(8)
#undef SOM_PRE_LOAD
        }
        __builtin_amdgcn_sched_barrier(0);
        const char* wbuf = ldsb + (size_t)buf * STAGE_F4 * 16;
        const char* obuf = ldsb + (size_t)(buf ^ 1) * STAGE_F4 * 16;
        auto rows_of = [&](const char* base, int nb) { return base + (nb * 32 + j) * RS + g * 32; };
        auto norms_of = [&](const char* base, int nb) {
            return reinterpret_cast<const float4*>(base + kNodesPerStage * RS + nb * 32 * 4) + g;
        };
        const int tile = st * NB;
        block(accA, accB, wh, wl, wtl, c, rows_of(wbuf, 1), norms_of(wbuf, 1), true, tile);
        block(accB, accA, wh, wl, wtl, c, rows_of(wbuf, 2), norms_of(wbuf, 2), true, tile + 1);
        {
            float4* d4 = lds4 + (buf ^ 1) * STAGE_F4 + tid;
#define SOM_PRE_STORE(i) if constexpr (PRE > i) d4[i * kThreads] = pre##i;
            SOM_PRE_STORE(0) SOM_PRE_STORE(1) SOM_PRE_STORE(2) SOM_PRE_STORE(3) SOM_PRE_STORE(4)
            SOM_PRE_STORE(5) SOM_PRE_STORE(6) SOM_PRE_STORE(7) SOM_PRE_STORE(8)
#undef SOM_PRE_STORE
        }
        __builtin_amdgcn_sched_barrier(0);
        block(accA, accB, wh, wl, wtl, c, rows_of(wbuf, 3), norms_of(wbuf, 3), true, tile + 2);
        __syncthreads();
        block(accB, accA, wh, wl, wtl, c, rows_of(obuf, 0), norms_of(obuf, 0), true, tile + 3);
    }
    // the last block's scores
#pragma unroll
    for (int sidx = 0; sidx < STEPS_ALL; ++sidx) fold_step(accB, sidx, nstages * (kNodesPerStage / 32) - 1);

    if constexpr (CAND) {
        // Direct float32 differences over the nodes this lane noted for its sample (the true winner is among the two
        // lane halves' candidates: its score lies within the rounding bound of the best one found), features in order,
        // lowest distance, then lowest node index; the halves are joined at the end.  An entry whose set overflowed
        // in either half (more than seven candidates) or that noted nothing goes to the second list, which the
        // all-nodes kernel serves.  The row stays in registers across the candidates: D <= 64.
        double qs = 0.0, qs2 = 0.0;
#pragma unroll
        for (int mb = 0; mb < MS; ++mb) {
            const int n = noted[mb].n;
            const bool over = n >= kCandSlots;
            const int mine = (valid[mb] && !over) ? n : 0;
            const float* xr = xrow[mb];
            const int D = a.D, whole = D / 4, rest = D - 4 * whole;
            float4 xv[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) xv[q] = (mine > 0 && q < whole) ? load4(xr + 4 * q) : float4{0.f, 0.f, 0.f, 0.f};
            // the last one to three features: the window [D - 4, D), its leading elements already counted
            const float4 xt4 = (mine > 0 && rest > 0) ? load4(xr + D - 4) : float4{0.f, 0.f, 0.f, 0.f};
            float bd = INFINITY;
            int bk = 0x7fffffff;
            for (int t = 0; t < kCandSlots - 1; ++t) {
                if (__ballot(t < mine) == 0ull) break;
                if (t < mine) {
                    const unsigned long long word = t < 4 ? noted[mb].lo >> (16 * t) : noted[mb].hi >> (16 * (t - 4));
                    const int id = (int)(word & 0xffffull);
                    if (id < a.K) {
                        const float* wr = a.W + (size_t)id * D;
                        float d = 0.0f;
#pragma unroll
                        for (int q = 0; q < 16; ++q) {
                            if (q < whole) {
                                const float4 w4 = load4(wr + 4 * q);
                                const float d0 = xv[q].x - w4.x, d1 = xv[q].y - w4.y, d2 = xv[q].z - w4.z, d3 = xv[q].w - w4.w;
                                d = fmaf(d0, d0, d);
                                d = fmaf(d1, d1, d);
                                d = fmaf(d2, d2, d);
                                d = fmaf(d3, d3, d);
                            }
                        }
                        if (rest > 0) {
                            const float4 w4 = load4(wr + D - 4);
                            const float d1 = xt4.y - w4.y, d2 = xt4.z - w4.z, d3 = xt4.w - w4.w;
                            if (rest > 2) d = fmaf(d1, d1, d);
                            if (rest > 1) d = fmaf(d2, d2, d);
                            d = fmaf(d3, d3, d);
                        }
                        if (d < bd || (d == bd && id < bk)) {
                            bd = d;
                            bk = id;
                        }
                    }
                }
            }
            const float od = __shfl_xor(bd, 32);
            const int ok = __shfl_xor(bk, 32);
            const bool oover = __shfl_xor(over ? 1 : 0, 32) != 0;
            if (od < bd || (od == bd && ok < bk)) {
                bd = od;
                bk = ok;
            }
            const bool served = !over && !oover && bk < a.K;
            const bool writer = valid[mb] && g == 0;
            const int64_t i = writer ? (int64_t)a.recheck[wave0 + mb * 32 + j] : 0;
            if (writer && served) {
                a.bmu[i] = bk;
                if (a.d2) a.d2[i] = bd;
                qs += sqrt((double)bd);
                qs2 += (double)bd;
            }
            list_push(&a.scal[a.slot2], a.recheck2, nullptr, writer && !served, i, 0.0f);
        }
        if (a.qe) group_qe_add(a.qe_part, qs, qs2);
        return;
    }
    // ---- join the two half-wavefronts, then lane (j, g) finishes block mp + g
    const float wmax2 = __uint_as_float(a.scal[0]);
    const float wmax = sqrtf(wmax2) * 1.000001f;
    // Difference of two scores.  Per score: the split leaves 3 * 2^-18 (1 + 2^-7) |x||w|.  Every MFMA adds sixteen
    // exact products to its accumulator C; how the pipe orders and rounds those additions is not documented, so each
    // MFMA is charged what seventeen float32 terms can lose when added in ANY order with one rounding to nearest per
    // addition: 16 * 2^-24 (|C| + sum |products|).  |C| + sum |products| never exceeds |w|^2 / 2 + (|xh| + |xl|)
    // (|wh| + |wl|) <= 1.016 times the magnitude bound, hence 49 units for each of the 3 KB MFMAs.  (The largest error
    // seen on operands built against aligning, truncating and sequential adders stays well inside 16 units:
    // tests/test_gpu_matrix_pipe.py fails on the first result outside them.)  The packed tail block is one MFMA
    // more.  The position bits take 16 units of the last place; -|w|^2/2 and the two centrings as in the float32 kernel.
    const float rel = 2.0f * (3.0f * 3.8146973e-06f * 1.0078125f + (float)(49 * KB + (TAIL ? 17 : 0) + 1) * 5.9604645e-08f + 1.9073486e-06f) +
                      12.0f * 5.9604645e-08f;
    // (the window offsets are worked out again rather than carried through the stage loop in registers)
    int d_again = a.D;
    asm volatile("" : "+s"(d_again));
    // Squared distances (d2, the quantisation-error sums) only where the caller wants them: without them the rows are
    // not read a second time, the sample's norm comes from the start of the tile and the winner's from the stage
    // blob (-|w|^2 / 2 in float32 behind the rows of its stage).
    const bool distances = a.d2 != nullptr || a.qe != nullptr;
    double qs = 0.0, qs2 = 0.0;
#pragma unroll
    for (int mp = 0; mp < MS; mp += 2) {
        float r_best = 0.f, r_second = 0.f, r_xn = 0.f, r_part = 0.f, r_wn = 0.f;
        int r_node = 0;
        bool r_valid = false;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int mb = mp + q;
            if (mb >= MS) break;
            const int rsel = (int)(__float_as_uint(best[mb]) & 15u);
            int node = tsel[mb] * 32 + 8 * (rsel >> 2) + 4 * g + (rsel & 3);
            const float ob = __shfl_xor(best[mb], 32);
            const float os = __shfl_xor(second[mb], 32);
            const int on = __shfl_xor(node, 32);
            const float sec = fmaxf(fmaxf(second[mb], os), fminf(best[mb], ob));
            const bool other = (ob > best[mb]) || (ob == best[mb] && on < node);
            const float bst = other ? ob : best[mb];
            node = other ? on : node;
            node = node < a.K ? node : a.K - 1;
            // squared norm of the centred sample and squared distance to the winner by direct differences on the
            // float32 values, this lane's slots (the row is read again: it is still in the cache; the winner's
            // centred weights come from the float32 copy of the stage rows, in the same slot order)
            float xn = 0.f, part = 0.f, wn = 0.f;
            if (!distances) {
                xn = xnorm2[mb];
                const char* blob = reinterpret_cast<const char*>(a.stage16) + (size_t)(node / kNodesPerStage) * STAGE_F4 * 16;
                wn = -2.0f * reinterpret_cast<const float*>(blob + (size_t)kNodesPerStage * RS)[node % kNodesPerStage];
            }
            if constexpr (TAIL) if (distances) {
                // the packed block's features once each: lane half 0 takes them (its first slots of wwin hold the weights)
                float vt[4];
                tail_values(xrow[mb], d_again, vt);
                const float4 w0 = *reinterpret_cast<const float4*>(a.wwin + (size_t)node * WROW + KB * 16);
                const float w[4] = {w0.x, w0.y, w0.z, w0.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float xv = g == 0 ? vt[t] : 0.0f, wv = g == 0 ? w[t] : 0.0f;
                    const float df = xv - wv;
                    xn = fmaf(xv, xv, xn);
                    part = fmaf(df, df, part);
                    wn = fmaf(wv, wv, wn);
                }
            }
            if constexpr (KB > 0) if (distances) {
                float v[KBA][8];
                centred_slots(xrow[mb], d_again, v);
                const float* wr = a.wwin + (size_t)node * WROW + g * 8;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const float4 w0 = *reinterpret_cast<const float4*>(wr + kb * 16);
                    const float4 w1 = *reinterpret_cast<const float4*>(wr + kb * 16 + 4);
                    const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        const float df = v[kb][t] - w[t];
                        xn = fmaf(v[kb][t], v[kb][t], xn);
                        part = fmaf(df, df, part);
                        wn = fmaf(w[t], w[t], wn);
                    }
                }
            }
            if (distances) {
                xn += __shfl_xor(xn, 32);
                part += __shfl_xor(part, 32);
                wn += __shfl_xor(wn, 32);
            }
            if (q == g) {
                r_best = bst;
                r_second = sec;
                r_node = node;
                r_xn = xn;
                r_part = part;
                r_wn = wn;
                r_valid = valid[mb];
            }
        }
        const int64_t i = wave0 + (mp + g) * 32 + j;
        const float xl2 = sqrtf(r_xn);
        // The winner's score errs by at most rel / 2 of its own magnitude bound, |x||w_b| + |w_b|^2 / 2 with the
        // winner's own norm; any other node's by at most rel / 2 of the bound with the largest norm.
        const float wb = fminf(sqrtf(r_wn) * 1.00001f, wmax);
        const float bound = 0.5f * rel * ((xl2 * wb + 0.5f * wb * wb) + (xl2 * wmax + 0.5f * wmax2));
        // (a sample that close to its node is re-decided for the sake of its distance: the centring roundings)
        const float tiny = (xl2 + wmax) * (xl2 + wmax) * 3.8146973e-06f;
        const bool close = r_valid && a.K > 1 && (!((r_best - r_second) > bound) || (distances && r_part < tiny));
        if (r_valid) {
            a.bmu[i] = r_node;
            if (a.d2) a.d2[i] = r_part;
            if (!close) {
                qs += sqrt((double)r_part);
                qs2 += (double)r_part;
            }
        }
        if (r_valid) a.cut_all[i] = close ? r_best - bound : kNotListed;
    }
    if (a.qe) group_qe_add(a.qe_part, qs, qs2);
}

// full tiles for the workgroups below a.full_tiles, half tiles for the last partial round (as bmu_kernel)
template <int KB, bool TAIL, int MS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_split_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    if ((int64_t)blockIdx.x < a.full_tiles) {
        bmu_split_tile<KB, TAIL, MS, false>(a, 0, blockIdx.x, 0u, lds4);
    } else if constexpr (MS > 1) {
        constexpr int64_t per_full = (int64_t)kWavesPerGroup * MS * 32;
        bmu_split_tile<KB, TAIL, MS / 2, false>(a, a.full_tiles * per_full, (int64_t)blockIdx.x - a.full_tiles, 0u, lds4);
    }
}

// candidate pass of the split search: a fixed grid walks the tiles of the list (as bmu_cand_kernel)
template <int KB, bool TAIL, int MS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_split_cand_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    const unsigned int count = a.scal[a.slot];
    if (!cand_pass_serves(a, count)) return;
    constexpr int64_t per_tile = (int64_t)kWavesPerGroup * MS * 32;
    if constexpr (MS > 1) {
        if (count <= kCandHalfTiles) {
            for (int64_t t = blockIdx.x; t * (per_tile / 2) < (int64_t)count; t += gridDim.x)
                bmu_split_tile<KB, TAIL, MS / 2, true>(a, 0, t, count, lds4);
            return;
        }
    }
    for (int64_t t = blockIdx.x; t * per_tile < (int64_t)count; t += gridDim.x)
        bmu_split_tile<KB, TAIL, MS, true>(a, 0, t, count, lds4);
}

// ---------------------------------------------------------------------------------------------------------
// the same search for D > 64: features go through in chunks of 50, 56 or 64.  A wavefront owns one block of 32
// samples; the accumulators of a stage's four node blocks stay live across the chunks, the samples' features of
// the current chunk are re-read from memory once per stage (one workgroup touches 128 rows).
// ---------------------------------------------------------------------------------------------------------
// CAND as in bmu_tile: the candidate pass over the first `count` entries of the re-decision list.
template <int STEPS, bool CAND>
__device__ __forceinline__ void bmu_wide_tile(const BmuArgs& a, int64_t tile_index, unsigned int count, float4* lds4)
{
    constexpr int CH = 2 * STEPS;                        // features per chunk
    constexpr int STRIDE = 2 * STEPS + 1, NBS = kNodesPerStage / 32;
    constexpr int STAGE_FLOATS = stage_floats_for(STRIDE);
    constexpr int STAGE_F4 = STAGE_FLOATS / 4;
    constexpr int PRE = STAGE_F4 / kThreads;
    static_assert(PRE <= 9, "stage copy holds at most nine float4 per thread");
    float* lds = reinterpret_cast<float*>(lds4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, g = lane >> 5;
    const int64_t i = (tile_index * kWavesPerGroup + wave) * 32 + j;      // sample position, or list entry (CAND)
    const int64_t total = CAND ? (int64_t)count : a.m;
    const bool valid = i < total;
    int64_t ii = valid ? i : total - 1;
    float cut = NAN;                                                        // CAND; no score compares >= NaN
    CandSet noted;
    if constexpr (CAND) {
        if (valid) cut = a.cutv[ii];
        ii = (int64_t)a.recheck[ii];
    }
    const int64_t row = a.idx ? (int64_t)a.idx[ii] : ii;
    const float* xr = a.X + row * a.ldx;

    float best = -INFINITY, second = -INFINITY;
    int rsel = 0, tsel = 0;
    const int nstages = a.kpad / kNodesPerStage;
    const int nch = (a.D + CH - 1) / CH;
    const int nq = nstages * nch;
    const float4* src4 = reinterpret_cast<const float4*>(a.stage);
    {
        float4 first[PRE];
#pragma unroll
        for (int p = 0; p < PRE; ++p) first[p] = src4[tid + p * kThreads];
#pragma unroll
        for (int p = 0; p < PRE; ++p) lds4[tid + p * kThreads] = first[p];
    }
    __syncthreads();

    floatx16 acc[NBS];
    int st = 0, ch = 0;
    // Centred features of the current chunk.  Lane (j, g) holds STEPS contiguous features of the chunk, the window the weight preparation laid the stage
    // columns out for: [CH ch + STEPS g, + STEPS), moved back to [D - STEPS, D) where it would pass the end of the
    // row.  Every chunk therefore comes in as STEPS / 4 16-byte loads per lane (4-byte aligned addresses are
    // enough for them; STEPS = 25 adds one dword), with no bounds to check and nothing read outside the row.
    auto window_of = [&](int chunk) {
        const int first = CH * chunk + STEPS * g;
        return first < a.D - STEPS ? first : a.D - STEPS;
    };
    float x[STEPS];
    {
        const float* xc = xr + window_of(0);
        const float* cc = a.centre + window_of(0);
#pragma unroll
        for (int t = 0; t < STEPS / 4; ++t) {
            const float4 v = load4(xc + 4 * t), c = load4(cc + 4 * t);
            x[4 * t + 0] = v.x - c.x;
            x[4 * t + 1] = v.y - c.y;
            x[4 * t + 2] = v.z - c.z;
            x[4 * t + 3] = v.w - c.w;
        }
#pragma unroll
        for (int s = STEPS / 4 * 4; s < STEPS; ++s) x[s] = xc[s] - cc[s];
    }
    for (int q = 0; q < nq; ++q) {
        const int buf = q & 1;
        float4 pre0, pre1, pre2, pre3, pre4, pre5, pre6, pre7, pre8;
        {
            const int nxt = (q + 1 < nq) ? q + 1 : q;
            const float4* s4 = src4 + (size_t)nxt * STAGE_F4 + tid;
#define SOM_PRE_LOAD(i) if constexpr (PRE > i) pre##i = s4[i * kThreads];
            SOM_PRE_LOAD(0) SOM_PRE_LOAD(1) SOM_PRE_LOAD(2) SOM_PRE_LOAD(3) SOM_PRE_LOAD(4)
            SOM_PRE_LOAD(5) SOM_PRE_LOAD(6) SOM_PRE_LOAD(7) SOM_PRE_LOAD(8)
#undef SOM_PRE_LOAD
        }
        // the samples' next chunk travels to registers during this chunk's arithmetic, like the next stage blob
        // (and with them the matching entries of the centre vector: vector loads cost no matrix-pipe time, a
        // select between two scalar values per entry would)
        float xn[STEPS], cn[STEPS];
        {
            const int chn = (ch + 1 == nch) ? 0 : ch + 1;
            const int w0 = window_of(chn);
            const float* cc = a.centre + w0;
            const float* xc = xr + w0;
#pragma unroll
            for (int t = 0; t < STEPS / 4; ++t) {
                const float4 c = load4(cc + 4 * t);
                cn[4 * t + 0] = c.x;
                cn[4 * t + 1] = c.y;
                cn[4 * t + 2] = c.z;
                cn[4 * t + 3] = c.w;
                const float4 v = load4(xc + 4 * t);
                xn[4 * t + 0] = v.x;
                xn[4 * t + 1] = v.y;
                xn[4 * t + 2] = v.z;
                xn[4 * t + 3] = v.w;
            }
#pragma unroll
            for (int s = STEPS / 4 * 4; s < STEPS; ++s) {
                cn[s] = cc[s];
                xn[s] = xc[s];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        const float* wbuf = lds + buf * STAGE_FLOATS;
        const float* nbuf = wbuf + kNodesPerStage * STRIDE;
        // As in bmu_kernel the LDS reads of node block nb + 1 are written into the MFMA sequence of block nb (one
        // read per MFMA) where the registers allow it (STEPS <= 28); only the first block of a chunk waits for LDS.
        constexpr bool PIPE = STEPS <= 28;
        float wa[PIPE ? STEPS : 1];
        if constexpr (PIPE) {
            const float* wrow = wbuf + j * STRIDE + g;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) wa[s] = wrow[2 * s];
        }
#pragma unroll
        for (int nb = 0; nb < NBS; ++nb) {
            if (ch == 0) {
                const float4* nh = reinterpret_cast<const float4*>(nbuf + nb * 32 + 4 * g);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float4 v = nh[2 * t];
                    acc[nb][4 * t + 0] = v.x;
                    acc[nb][4 * t + 1] = v.y;
                    acc[nb][4 * t + 2] = v.z;
                    acc[nb][4 * t + 3] = v.w;
                }
            }
            // The chunk's 64-feature partial product is summed on its own, from zero, and then added to the
            // running score: every rounding inside the chunk is relative to the chunk's own magnitude
            // |x_chunk| |w_chunk|, and those add up to at most |x| |w| over the chunks (Cauchy-Schwarz), so the
            // error bound grows with 2 STEPS + nch roundings per score instead of 2 STEPS nch.
            const float* wrow = wbuf + (nb * 32 + j) * STRIDE + g;
            floatx16 part;
#pragma unroll
            for (int r = 0; r < 16; ++r) part[r] = 0.0f;
            if constexpr (PIPE) {
                const float* wnext = wrow + 32 * STRIDE;
                float wn[STEPS];
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    part = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[s], x[s], part, 0, 0, 0);
                    if (nb + 1 < NBS) {
                        wn[s] = wnext[2 * s];
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
                    }
                }
                if (nb + 1 < NBS) {
#pragma unroll
                    for (int s = 0; s < STEPS; ++s) wa[s] = wn[s];
                }
            } else {
#pragma unroll
                for (int s = 0; s < STEPS; ++s)
                    part = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[2 * s], x[s], part, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nb][r] += part[r];
            if (CAND && ch == nch - 1) {
                const int tile = st * NBS + nb;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (acc[nb][r] >= cut) noted.note(tile * 32 + 4 * g, 8 * (r >> 2) + (r & 3));
            }
            if (!CAND && ch == nch - 1) {
                const int tile = st * NBS + nb;
                const float before = best;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[nb][r];
                    rsel = (v > best) ? r : rsel;
                    second = __builtin_amdgcn_fmed3f(best, second, v);
                    best = vmax(best, v);
                }
                tsel = (best > before) ? tile : tsel;
            }
        }
        {
            float4* d4 = lds4 + (buf ^ 1) * STAGE_F4 + tid;
#define SOM_PRE_STORE(i) if constexpr (PRE > i) d4[i * kThreads] = pre##i;
            SOM_PRE_STORE(0) SOM_PRE_STORE(1) SOM_PRE_STORE(2) SOM_PRE_STORE(3) SOM_PRE_STORE(4)
            SOM_PRE_STORE(5) SOM_PRE_STORE(6) SOM_PRE_STORE(7) SOM_PRE_STORE(8)
#undef SOM_PRE_STORE
        }
        __syncthreads();
        if (++ch == nch) {
            ch = 0;
            ++st;
        }
#pragma unroll
        for (int s = 0; s < STEPS; ++s) x[s] = xn[s] - cn[s];
    }

    if constexpr (CAND) {
        if (valid) a.cand[(size_t)i * 2 + g] = noted.packed();
        return;
    }
    // ---- join the two half-wavefronts; squared norm and exact winner distance from memory, half the features each
    int node = tsel * 32 + 8 * (rsel >> 2) + 4 * g + (rsel & 3);
    const float ob = __shfl_xor(best, 32), os = __shfl_xor(second, 32);
    const int on = __shfl_xor(node, 32);
    const float sec = fmaxf(fmaxf(second, os), fminf(best, ob));
    const bool other = (ob > best) || (ob == best && on < node);
    const float bst = other ? ob : best;
    node = other ? on : node;
    node = node < a.K ? node : a.K - 1;
    float xn = 0.f, part = 0.f;
    const float* wr = a.W + (size_t)node * a.D;
    for (int f = g; f < a.D; f += 2) {
        const float xv = xr[f];
        const float xc = xv - a.centre[f];
        const float df = xv - wr[f];
        xn = fmaf(xc, xc, xn);
        part = fmaf(df, df, part);
    }
    xn += __shfl_xor(xn, 32);
    part += __shfl_xor(part, 32);
    double qs = 0.0, qs2 = 0.0;
    const float wmax2 = __uint_as_float(a.scal[0]);
    const float wmax = sqrtf(wmax2) * 1.000001f;
    // per score: 2 STEPS roundings inside the chunks (see the stage loop), nch chunk additions, one for
    // -|w|^2/2; two scores, plus the centring roundings and slack as in bmu_kernel
    const float rel = (float)(4 * STEPS + 2 * nch + 12) * 5.9604645e-08f;
    const float bound = (sqrtf(xn) * wmax + 0.5f * wmax2) * rel;
    const bool mine = valid && g == 0;
    const bool close = mine && a.K > 1 && !((bst - sec) > bound);
    if (mine) {
        a.bmu[i] = node;
        if (a.d2) a.d2[i] = part;
        if (!close) {
            qs = sqrt((double)part);
            qs2 = (double)part;
        }
    }
    if (mine) a.cut_all[i] = close ? bst - bound : kNotListed;
    if (a.qe) group_qe_add(a.qe_part, qs, qs2);
}

template <int STEPS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_wide_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    bmu_wide_tile<STEPS, false>(a, blockIdx.x, 0u, lds4);
}

template <int STEPS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_wide_cand_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    const unsigned int count = a.scal[a.slot];
    if (!cand_pass_serves(a, count)) return;
    constexpr int64_t per_tile = (int64_t)kWavesPerGroup * 32;
    for (int64_t t = blockIdx.x; t * per_tile < (int64_t)count; t += gridDim.x) bmu_wide_tile<STEPS, true>(a, t, count, lds4);
}

// ---------------------------------------------------------------------------------------------------------
// The split search for D > 64: chunks of 64 features (four 16-feature blocks) through the same stage rows, one block
// of 32 samples per wavefront, the four node blocks' accumulators of a stage live across the chunks (as
// bmu_wide_tile).  A wavefront meets every chunk of its samples once per stage, so the samples' bf16 parts are not
// made in this kernel (tried: the conversion, 250 vector instructions per chunk and stage beside 48 MFMAs, made it
// slower than the float32 kernel) but once per pass by bmu_split_convert_kernel, into a[parts]: per presented
// sample and slot group of eight features 32 bytes, [hi x 8 | lo x 8], which a lane reads as they are.
// Every chunk's partial product is summed on its own from zero and then added, so that the roundings inside a chunk
// are relative to |x_chunk| |w_chunk| and add up to at most |x| |w| over the chunks (Cauchy-Schwarz).
// Slot group q of chunk ch is the row's window [min(64 ch + 4 q, D - 4), + 4); the weights (bmu_prep_split_kernel)
// and the samples (the conversion) are zero in front of a shifted window's own features.
// ---------------------------------------------------------------------------------------------------------
// one thread per (presented sample, group of eight slots): centred, cut into bf16 parts
__global__ void __launch_bounds__(256) bmu_split_convert_kernel(const BmuArgs a, int nch16)
{
    const int groups = nch16 * 8;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= a.m * groups) return;
    const int64_t i = e / groups;
    const int grp = (int)(e - i * groups);
    const int chunk = grp >> 3, kb = (grp >> 1) & 3, g = grp & 1;
    const int64_t row = a.idx ? (int64_t)a.idx[i] : i;
    const float* xr = a.X + row * a.ldx;
    float v[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int f0 = 64 * chunk + 4 * (4 * kb + 2 * g + h);
        const int start = f0 < a.D - 4 ? f0 : a.D - 4;
        const int shift = f0 - start;                                     // own slots: index >= shift
        const float4 x4 = load4(xr + start), c4 = load4(a.centre + start);
        v[4 * h + 0] = shift <= 0 ? x4.x - c4.x : 0.0f;
        v[4 * h + 1] = shift <= 1 ? x4.y - c4.y : 0.0f;
        v[4 * h + 2] = shift <= 2 ? x4.z - c4.z : 0.0f;
        v[4 * h + 3] = shift <= 3 ? x4.w - c4.w : 0.0f;
    }
    bf16x8 hi, lo;
    split8(v, hi, lo);
    bf16x8* out = reinterpret_cast<bf16x8*>(a.parts) + e * 2;
    out[0] = hi;
    out[1] = lo;
}

template <bool CAND>
__device__ __forceinline__ void bmu_split_wide_tile(const BmuArgs& a, int64_t tile_index, unsigned int count, float4* lds4)
{
    constexpr int KB = 4, NBS = kNodesPerStage / 32;
    constexpr int RS = split_row_bytes(KB);
    constexpr int STAGE_F4 = split_stage_f4(KB);
    constexpr int PRE = STAGE_F4 / kThreads;
    static_assert(PRE <= 9, "stage copy holds at most nine float4 per thread");
    const char* ldsb = reinterpret_cast<const char*>(lds4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, g = lane >> 5;
    const int64_t i = (tile_index * kWavesPerGroup + wave) * 32 + j;      // sample position, or list entry (CAND)
    const int64_t total = CAND ? (int64_t)count : a.m;
    const bool valid = i < total;
    int64_t ii = valid ? i : total - 1;
    float cut = NAN;                                                        // CAND; no score compares >= NaN
    CandSet noted;
    if constexpr (CAND) {
        if (valid) cut = a.cutv[ii];
        ii = (int64_t)a.recheck[ii];
    }
    const int64_t row = a.idx ? (int64_t)a.idx[ii] : ii;
    const float* xr = a.X + row * a.ldx;

    float best = -INFINITY, second = -INFINITY;
    int rsel = 0, tsel = 0;
    const int nstages = a.kpad / kNodesPerStage;
    const int nch = (a.D + 63) / 64;
    const int nq = nstages * nch;
    const float4* src4 = reinterpret_cast<const float4*>(a.stage16);
#pragma unroll
    for (int p = 0; p < PRE; ++p) lds4[tid + p * kThreads] = src4[tid + p * kThreads];
    __syncthreads();

    // this lane's parts of a chunk: four groups of eight slots, 32 bytes each
    const bf16x8* prow = reinterpret_cast<const bf16x8*>(a.parts) + (size_t)ii * (nch * 8) * 2;
    auto read_chunk = [&](int chunk, bf16x8 (&h8)[KB], bf16x8 (&l8)[KB]) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const bf16x8* p = prow + (size_t)((chunk * 4 + kb) * 2 + g) * 2;
            h8[kb] = p[0];
            l8[kb] = p[1];
        }
    };
    bf16x8 xh[KB], xl[KB];
    read_chunk(0, xh, xl);

    floatx16 acc[NBS];
    int st = 0, ch = 0;
    for (int q = 0; q < nq; ++q) {
        const int buf = q & 1;
        float4 pre0, pre1, pre2, pre3, pre4, pre5, pre6, pre7, pre8;
        {
            const int nxt = (q + 1 < nq) ? q + 1 : q;
            const float4* s4 = src4 + (size_t)nxt * STAGE_F4 + tid;
#define SOM_PRE_LOAD(i) if constexpr (PRE > i) pre##i = s4[i * kThreads];
            SOM_PRE_LOAD(0) SOM_PRE_LOAD(1) SOM_PRE_LOAD(2) SOM_PRE_LOAD(3) SOM_PRE_LOAD(4)
            SOM_PRE_LOAD(5) SOM_PRE_LOAD(6) SOM_PRE_LOAD(7) SOM_PRE_LOAD(8)
#undef SOM_PRE_LOAD
        }
        // the samples' next chunk travels to registers during this chunk's arithmetic
        const int chn = (ch + 1 == nch) ? 0 : ch + 1;
        bf16x8 xhn[KB], xln[KB];
        read_chunk(chn, xhn, xln);
        __builtin_amdgcn_sched_barrier(0);
        const char* wbuf = ldsb + (size_t)buf * STAGE_F4 * 16;
        const float* nbuf = reinterpret_cast<const float*>(wbuf + kNodesPerStage * RS);
        bf16x8 wh[KB], wl[KB];
        {
            const char* wrow = wbuf + j * RS + g * 32;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                wh[kb] = *reinterpret_cast<const bf16x8*>(wrow + kb * 64);
                wl[kb] = *reinterpret_cast<const bf16x8*>(wrow + kb * 64 + 16);
            }
        }
#pragma unroll
        for (int nb = 0; nb < NBS; ++nb) {
            if (ch == 0) {
                const float4* nh = reinterpret_cast<const float4*>(nbuf + nb * 32 + 4 * g);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float4 v = nh[2 * t];
                    acc[nb][4 * t + 0] = v.x;
                    acc[nb][4 * t + 1] = v.y;
                    acc[nb][4 * t + 2] = v.z;
                    acc[nb][4 * t + 3] = v.w;
                }
            }
            const char* wnext = wbuf + ((nb + 1) * 32 + j) * RS + g * 32;
            floatx16 part;
#pragma unroll
            for (int r = 0; r < 16; ++r) part[r] = 0.0f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                part = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh[kb], xh[kb], part, 0, 0, 0);
                part = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wh[kb], xl[kb], part, 0, 0, 0);
                part = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wl[kb], xh[kb], part, 0, 0, 0);
                // the next block's rows, into the registers this block has finished with
                if (nb + 1 < NBS) {
                    wh[kb] = *reinterpret_cast<const bf16x8*>(wnext + kb * 64);
                    wl[kb] = *reinterpret_cast<const bf16x8*>(wnext + kb * 64 + 16);
                    __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);     // three MFMAs
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);     // two LDS reads
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nb][r] += part[r];
            if (CAND && ch == nch - 1) {
                const int tile = st * NBS + nb;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (acc[nb][r] >= cut) noted.note(tile * 32 + 4 * g, 8 * (r >> 2) + (r & 3));
            }
            if (!CAND && ch == nch - 1) {
                const int tile = st * NBS + nb;
                const float before = best;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[nb][r];
                    rsel = (v > best) ? r : rsel;
                    second = __builtin_amdgcn_fmed3f(best, second, v);
                    best = vmax(best, v);
                }
                tsel = (best > before) ? tile : tsel;
            }
        }
        {
            float4* d4 = lds4 + (buf ^ 1) * STAGE_F4 + tid;
#define SOM_PRE_STORE(i) if constexpr (PRE > i) d4[i * kThreads] = pre##i;
            SOM_PRE_STORE(0) SOM_PRE_STORE(1) SOM_PRE_STORE(2) SOM_PRE_STORE(3) SOM_PRE_STORE(4)
            SOM_PRE_STORE(5) SOM_PRE_STORE(6) SOM_PRE_STORE(7) SOM_PRE_STORE(8)
#undef SOM_PRE_STORE
        }
        __syncthreads();
        if (++ch == nch) {
            ch = 0;
            ++st;
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            xh[kb] = xhn[kb];
            xl[kb] = xln[kb];
        }
    }

    if constexpr (CAND) {
        if (valid) a.cand[(size_t)i * 2 + g] = noted.packed();
        return;
    }
    // ---- join the two half-wavefronts; squared norm and exact winner distance from memory, half the features each
    int node = tsel * 32 + 8 * (rsel >> 2) + 4 * g + (rsel & 3);
    const float ob = __shfl_xor(best, 32), os = __shfl_xor(second, 32);
    const int on = __shfl_xor(node, 32);
    const float sec = fmaxf(fmaxf(second, os), fminf(best, ob));
    const bool other = (ob > best) || (ob == best && on < node);
    const float bst = other ? ob : best;
    node = other ? on : node;
    node = node < a.K ? node : a.K - 1;
    float xn = 0.f, part = 0.f;
    const float* wr = a.W + (size_t)node * a.D;
    for (int f = g; f < a.D; f += 2) {
        const float xv = xr[f];
        const float xc = xv - a.centre[f];
        const float df = xv - wr[f];
        xn = fmaf(xc, xc, xn);
        part = fmaf(df, df, part);
    }
    xn += __shfl_xor(xn, 32);
    part += __shfl_xor(part, 32);
    double qs = 0.0, qs2 = 0.0;
    const float wmax2 = __uint_as_float(a.scal[0]);
    const float wmax = sqrtf(wmax2) * 1.000001f;
    // per score: the split leaves 3 * 2^-18 (1 + 2^-7); inside a chunk 12 MFMAs charged 16 units of 2^-24 each,
    // times 1.016 for the parts' own magnitudes (any order of round-to-nearest additions, as in bmu_split_tile; relative
    // to the chunk's magnitude, see above), one addition per chunk, one rounding for -|w|^2/2; two scores, plus the
    // centring roundings and slack as in bmu_kernel
    const float rel = 2.0f * (3.0f * 3.8146973e-06f * 1.0078125f + (float)(196 + nch + 1) * 5.9604645e-08f) + 12.0f * 5.9604645e-08f;
    const float bound = (sqrtf(xn) * wmax + 0.5f * wmax2) * rel;
    const bool mine = valid && g == 0;
    const bool close = mine && a.K > 1 && !((bst - sec) > bound);
    if (mine) {
        a.bmu[i] = node;
        if (a.d2) a.d2[i] = part;
        if (!close) {
            qs = sqrt((double)part);
            qs2 = (double)part;
        }
    }
    if (mine) a.cut_all[i] = close ? bst - bound : kNotListed;
    if (a.qe) group_qe_add(a.qe_part, qs, qs2);
}

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_split_wide_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    bmu_split_wide_tile<false>(a, blockIdx.x, 0u, lds4);
}

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) bmu_split_wide_cand_kernel(const BmuArgs a)
{
    extern __shared__ float4 lds4[];
    const unsigned int count = a.scal[a.slot];
    if (!cand_pass_serves(a, count)) return;
    constexpr int64_t per_tile = (int64_t)kWavesPerGroup * 32;
    for (int64_t t = blockIdx.x; t * per_tile < (int64_t)count; t += gridDim.x) bmu_split_wide_tile<true>(a, t, count, lds4);
}

// ---------------------------------------------------------------------------------------------------------
// exact re-decision of the listed samples by direct differences, sum_d (x_d - w_kd)^2 for every node.
// A workgroup takes kExactGroup samples at a time; thread t owns nodes t, t + 256, ... so one coalesced read of
// the transposed weights serves all samples of the group, and the samples' features are broadcast from LDS.
// The inner loop is one v_sub and one v_fmac per (sample, node, feature) with nothing else in the way, i.e. the
// plain vector-ALU rate: 2 K D lane-operations per sample (2.6 ns at K = 1024, D = 50 on 256 compute units; 3.8 ns
// measured with every sample listed).  Larger groups or prefetched weights were measured and change nothing.
// ---------------------------------------------------------------------------------------------------------
constexpr int kExactGroup = 8;
constexpr int kExactNodesPerThread = 4;

// ---------------------------------------------------------------------------------------------------------
// Direct differences over the nodes the candidate pass noted (the true winner is among them: its score lies
// within the rounding bound of the best one found).  Sixteen lanes per list entry, each a sixteenth of the
// features; lowest distance, then lowest node index.  Entries whose slots overflowed (more than seven candidates
// in one half) or that noted nothing (non-finite scores) go to the second list, which the all-nodes kernel serves.
// ---------------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) bmu_cand_exact_kernel(const BmuArgs a)
{
    const unsigned int count = a.scal[a.slot];
    if (!cand_pass_serves(a, count)) return;
    const int sub = threadIdx.x & 15;
    constexpr unsigned int per_group = 256 / 16;
    constexpr int kMost = 2 * (kCandSlots - 1);        // candidates of one sample at most
    double qs = 0.0, qs2 = 0.0;
    for (unsigned int p0 = blockIdx.x * per_group; p0 < count; p0 += gridDim.x * per_group) {
        const unsigned int p = p0 + (threadIdx.x >> 4);
        const bool live = p < count;
        const unsigned int pc = live ? p : count - 1;
        const int64_t i = (int64_t)a.recheck[pc];
        const ulonglong2 h0 = a.cand[(size_t)pc * 2], h1 = a.cand[(size_t)pc * 2 + 1];
        const int64_t row = a.idx ? (int64_t)a.idx[i] : i;
        const float* xr = a.X + row * a.ldx;
        const int c0 = cand_count(h0), c1 = cand_count(h1);
        bool served = c0 < kCandSlots && c1 < kCandSlots && c0 + c1 > 0;
        const int c = served ? c0 + c1 : 0;
        // Both halves' candidates form one dense list of c places, taken four at a time (most samples have no more):
        // the loads of a batch (four rows of W, a quarter of 64 features per lane) are issued together, and batches
        // nobody in the wavefront needs are skipped.
        float bd = INFINITY;
        int bk = 0x7fffffff;
        constexpr int kBatch = 4;
        for (int t0 = 0; t0 < kMost; t0 += kBatch) {
            if (__ballot(c > t0) == 0ull) break;
            int node[kBatch];
            float d[kBatch];
#pragma unroll
            for (int tt = 0; tt < kBatch; ++tt) {
                const int t = t0 + tt, u = t - c0;
                const int k = (t < c0) ? cand_id(h0, t < kCandSlots - 1 ? t : 0)
                                       : cand_id(h1, u < kCandSlots - 1 ? u : 0);
                node[tt] = (t < c && k < a.K) ? k : -1;
                d[tt] = 0.0f;
            }
            for (int f0 = 0; f0 < a.D; f0 += 64) {
                float xv[4], wv[kBatch][4];
                int fo[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int f = f0 + 16 * q + sub;
                    fo[q] = f < a.D ? f : -1;
                    xv[q] = xr[fo[q] >= 0 ? f : a.D - 1];
                }
#pragma unroll
                for (int tt = 0; tt < kBatch; ++tt) {
                    const float* wr = a.W + (size_t)(node[tt] >= 0 ? node[tt] : 0) * a.D;
#pragma unroll
                    for (int q = 0; q < 4; ++q) wv[tt][q] = wr[fo[q] >= 0 ? fo[q] : a.D - 1];
                }
#pragma unroll
                for (int tt = 0; tt < kBatch; ++tt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float df = fo[q] >= 0 ? xv[q] - wv[tt][q] : 0.0f;
                        d[tt] = fmaf(df, df, d[tt]);
                    }
            }
#pragma unroll
            for (int tt = 0; tt < kBatch; ++tt) {
                float v = d[tt];
                v += __shfl_xor(v, 8);
                v += __shfl_xor(v, 4);
                v += __shfl_xor(v, 2);
                v += __shfl_xor(v, 1);
                const int k = node[tt];
                if (k >= 0 && (v < bd || (v == bd && k < bk))) {
                    bd = v;
                    bk = k;
                }
            }
        }
        served = served && bk < a.K;
        const bool mine = live && sub == 0;
        if (mine && served) {
            a.bmu[i] = bk;
            if (a.d2) a.d2[i] = bd;
            qs += sqrt((double)bd);
            qs2 += (double)bd;
        }
        list_push(&a.scal[a.slot2], a.recheck2, nullptr, mine && !served, i, 0.0f);
    }
    if (a.qe) group_qe_add(a.qe_part, qs, qs2);
}

__global__ void __launch_bounds__(256) bmu_exact_kernel(const BmuArgs a)
{
    __shared__ float4 xs4[64][kExactGroup / 4];   // [feature within a 64-wide slab][sample]
    __shared__ float red_d[4][kExactGroup];
    __shared__ int red_k[4][kExactGroup];
    float* xs = reinterpret_cast<float*>(xs4);
    const float* __restrict__ wt = a.wt;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // the whole list, or what the candidate pass left over
    const unsigned int listed = a.scal[a.slot];
    const bool by_cand = cand_pass_serves(a, listed);
    const unsigned int count = by_cand ? a.scal[a.slot2] : listed;
    const uint32_t* __restrict__ list = by_cand ? a.recheck2 : a.recheck;
    if (blockIdx.x == 0 && tid == 0) {
        atomicAdd(&a.scal[3], listed);  // running total over the calls that share one weight preparation
        a.scal[3 - a.slot] = 0u;        // the next call counts into the other slots (1 and 2, 4 and 5)
        a.scal[9 - a.slot2] = 0u;
    }
    double qs = 0.0, qs2 = 0.0;
    for (unsigned int g0 = blockIdx.x * kExactGroup; g0 < count; g0 += gridDim.x * kExactGroup) {
        float bestd[kExactGroup];
        int bestk[kExactGroup];
#pragma unroll
        for (int s = 0; s < kExactGroup; ++s) {
            bestd[s] = INFINITY;
            bestk[s] = 0x7fffffff;
        }
        for (int kb = 0; kb < a.kpad; kb += 256 * kExactNodesPerThread) {
            float dist[kExactGroup][kExactNodesPerThread];
#pragma unroll
            for (int s = 0; s < kExactGroup; ++s)
#pragma unroll
                for (int u = 0; u < kExactNodesPerThread; ++u) dist[s][u] = 0.f;
            for (int d0 = 0; d0 < a.D; d0 += 64) {
                const int dn = (a.D - d0 < 64) ? a.D - d0 : 64;
                __syncthreads();
                for (int e = tid; e < kExactGroup * dn; e += 256) {
                    const int s = e / dn, d = e % dn;
                    const unsigned int ge = (g0 + s < count) ? g0 + s : count - 1;
                    const int64_t i = (int64_t)list[ge];
                    const int64_t r = a.idx ? (int64_t)a.idx[i] : i;
                    xs[d * kExactGroup + s] = a.X[r * a.ldx + d0 + d];
                }
                __syncthreads();
                // four features at a time: their sixteen weight loads are in flight together
                for (int d = 0; d < dn; d += 4) {
                    float w[4][kExactNodesPerThread];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int u = 0; u < kExactNodesPerThread; ++u) {
                            const int k = kb + u * 256 + tid;
                            w[t][u] = (k < a.kpad && d + t < dn) ? wt[(size_t)(d0 + d + t) * a.kpad + k] : 0.f;
                        }
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (d + t < dn) {
                            float xv[kExactGroup];
#pragma unroll
                            for (int q = 0; q < kExactGroup / 4; ++q) {
                                const float4 v4 = xs4[d + t][q];
                                xv[4 * q + 0] = v4.x;
                                xv[4 * q + 1] = v4.y;
                                xv[4 * q + 2] = v4.z;
                                xv[4 * q + 3] = v4.w;
                            }
#pragma unroll
                            for (int s = 0; s < kExactGroup; ++s)
#pragma unroll
                                for (int u = 0; u < kExactNodesPerThread; ++u) {
                                    const float df = xv[s] - w[t][u];
                                    dist[s][u] = fmaf(df, df, dist[s][u]);
                                }
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kExactNodesPerThread; ++u) {
                const int k = kb + u * 256 + tid;
#pragma unroll
                for (int s = 0; s < kExactGroup; ++s)
                    if (k < a.K && dist[s][u] < bestd[s]) {
                        bestd[s] = dist[s][u];
                        bestk[s] = k;
                    }
            }
        }
        // lowest distance, then lowest node index, across the workgroup
#pragma unroll
        for (int s = 0; s < kExactGroup; ++s) {
            float bd = bestd[s];
            int bk = bestk[s];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float od = __shfl_xor(bd, o);
                const int ok = __shfl_xor(bk, o);
                if (od < bd || (od == bd && ok < bk)) {
                    bd = od;
                    bk = ok;
                }
            }
            if (lane == 0) {
                red_d[wave][s] = bd;
                red_k[wave][s] = bk;
            }
        }
        __syncthreads();
        if (tid < kExactGroup && g0 + tid < count) {
            float bd = red_d[0][tid];
            int bk = red_k[0][tid];
            for (int w = 1; w < 4; ++w) {
                const float od = red_d[w][tid];
                const int ok = red_k[w][tid];
                if (od < bd || (od == bd && ok < bk)) {
                    bd = od;
                    bk = ok;
                }
            }
            if (bk >= a.K) bk = 0; // only reachable with non-finite input
            const int64_t i = (int64_t)list[g0 + tid];
            a.bmu[i] = bk;
            if (a.d2) a.d2[i] = bd;
            qs += sqrt((double)bd);
            qs2 += (double)bd;
        }
    }
    if (a.qe) group_qe_add(a.qe_part, tid < kExactGroup ? qs : 0.0, tid < kExactGroup ? qs2 : 0.0);
}

// qe[0..1] += the call's partial sums, which are left zero for the next call
__global__ void __launch_bounds__(kQeSlots) qe_finish_kernel(double* __restrict__ part, double* __restrict__ qe)
{
    __shared__ double w[kQeSlots / 64][2];
    const int tid = threadIdx.x;
    double s0 = part[2 * tid], s1 = part[2 * tid + 1];
    part[2 * tid] = 0.0;
    part[2 * tid + 1] = 0.0;
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    if ((tid & 63) == 0) {
        w[tid >> 6][0] = s0;
        w[tid >> 6][1] = s1;
    }
    __syncthreads();
    if (tid == 0) {
        double t0 = 0.0, t1 = 0.0;
        for (int q = 0; q < kQeSlots / 64; ++q) {
            t0 += w[q][0];
            t1 += w[q][1];
        }
        qe[0] += t0;
        qe[1] += t1;
    }
}

// ---------------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------------
static int steps_for(int D)
{
    const int need = (D + 1) / 2;
    const int avail[] = {4, 8, 12, 16, 20, 25, 28, 32};   // MFMA steps per block; the smallest that holds D
    for (int s : avail)
        if (need <= s) return s;
    return 0;
}

int launch_fill_zero(som_ctx* ctx, void* p, size_t bytes)
{
    if (bytes == 0) return SOM_OK;
    const size_t words = bytes / 4;
    int blocks = (int)((words + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, ctx->stream, (uint32_t*)p, words);
    return check_hip(ctx, hipGetLastError(), "fill_zero launch");
}

int bmu_prepare(som_ctx* ctx, const float* W, int32_t K, int32_t D, BmuPrep* out, double* qe, int32_t* small)
{
    int steps, nch;
    if (D <= 2 * kMaxStepsResident) {
        steps = steps_for(D);
        nch = 1;
    } else {
        // chunk width 50, 56 or 64 features, whichever wastes least (a chunk costs about three MFMA steps of
        // overhead); the wider one on a tie
        steps = 0;
        nch = 0;
        for (int cand : {32, 28, 25}) {
            const int n = (D + 2 * cand - 1) / (2 * cand);
            if (steps == 0 || n * (cand + 3) < nch * (steps + 3)) {
                steps = cand;
                nch = n;
            }
        }
    }
    const int stride = 2 * steps + 1;
    const int kpad = ((K + kNodesPerStage - 1) / kNodesPerStage) * kNodesPerStage;
    const size_t stage_bytes = (size_t)(kpad / kNodesPerStage) * nch * stage_floats_for(stride) * sizeof(float);
    const size_t wt_bytes = (size_t)D * kpad * sizeof(float);
    // the centre vector is zero-padded to whole chunks (and to the 64 entries the resident kernel reads)
    const size_t centre_floats = (size_t)(nch > 1 ? nch * 2 * steps : 64);
    const size_t centre_bytes = ((centre_floats > (size_t)D ? centre_floats : (size_t)D) * sizeof(float) + 255) / 256 * 256;
    // rows for the bf16 matrix pipe where the split search applies
    // (small maps stay with the float32 search: a tile is mostly prologue and epilogue there, and the split search's
    // are the longer ones; measured at 10^7 x 50: 256 nodes 3.5 ms against 4.5, 576 nodes 5.7 against 5.1)
    const bool split = D >= 4 && K > kSplitMinNodes && ctx->search != SOM_SEARCH_FLOAT32;
    // D <= 64: whole 16-feature blocks, and a remainder of one to four features goes into one packed block (one MFMA
    // instead of three for a block that would be mostly padding); larger remainders get a block of their own
    const int tail_r = (split && nch == 1 && D % 16 >= 1 && D % 16 <= 4) ? D % 16 : 0;
    const int kb = !split ? 0 : (nch == 1 ? (tail_r ? D / 16 : (D + 15) / 16) : 4);
    const int nch16 = !split ? 0 : (nch == 1 ? 1 : (D + 63) / 64);
    const size_t stage16_one = split ? (size_t)split_stage_f4(kb, tail_r > 0) * 16 : 0;
    const size_t stage16_bytes = (size_t)(kpad / kNodesPerStage) * nch16 * stage16_one;
    const size_t wwin_bytes = (split && nch == 1) ? (size_t)kpad * (kb * 16 + (tail_r ? 16 : 0)) * sizeof(float) : 0;
    const size_t need = stage_bytes + wt_bytes + centre_bytes + stage16_bytes + wwin_bytes + 256;
    if (need > ctx->prep_bytes) {
        if (ctx->prep_blob) {
            if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
            (void)hipFree(ctx->prep_blob);
            ctx->prep_blob = nullptr;
            ctx->prep_bytes = 0;
        }
        if (hipMalloc(&ctx->prep_blob, need) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for the weight workspace", need);
        }
        ctx->prep_bytes = need;
    }
    char* base = (char*)ctx->prep_blob;
    out->scal = (unsigned int*)base;
    out->stage = (float*)(base + 256);
    out->wt = (float*)(base + 256 + stage_bytes);
    out->centre = (float*)(base + 256 + stage_bytes + wt_bytes);
    out->stage16 = split ? (void*)(base + 256 + stage_bytes + wt_bytes + centre_bytes) : nullptr;
    out->tail_r = tail_r;
    out->wwin = wwin_bytes ? (float*)(base + 256 + stage_bytes + wt_bytes + centre_bytes + stage16_bytes) : nullptr;
    out->nch16 = nch16;
    out->kb = kb;
    out->kpad = kpad;
    out->steps = steps;
    out->stride = stride;
    out->nch = nch;
    out->calls = 0;
    hipLaunchKernelGGL(bmu_centre_kernel, dim3((unsigned)(centre_bytes / 256)), dim3(1024), 0, ctx->stream, W, K, D,
                       out->centre, out->scal);
    // one thread per element of the padded stage matrix and of the transposed copy, one wavefront per four nodes
    long long elems = (long long)kpad * nch * stride;
    if (elems < (long long)kpad * 16) elems = (long long)kpad * 16;
    if (elems < (long long)kpad * D) elems = (long long)kpad * D;
    SplitPrep sp{};
    if (split) {
        sp.stage16 = (char*)out->stage16;
        sp.wwin = out->wwin;
        sp.kb_count = kb;
        sp.tail_r = tail_r;
        sp.nch16 = nch16;
        sp.row_bytes = split_row_bytes(kb, tail_r > 0);
        sp.stage16_bytes = (int)stage16_one;
        const long long slots = (long long)kpad * nch16 * (kb * 16 + (tail_r ? 16 : 0));
        if (elems < slots) elems = slots;
    }
    hipLaunchKernelGGL(bmu_prep_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, ctx->stream, W, K, D, kpad,
                       stride, nch, stage_floats_for(stride), out->centre, out->stage, out->wt, out->scal, qe, small, sp);
    return check_hip(ctx, hipGetLastError(), "bmu_prep launch");
}

template <int STEPS>
static int launch_bmu_wide(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)stage_floats_for(2 * STEPS + 1) * sizeof(float);
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = bmu_wide_kernel<STEPS>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    const int64_t per_group = (int64_t)kWavesPerGroup * 32;
    const int64_t groups = (a.m + per_group - 1) / per_group;
    hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(kThreads), lds_bytes, ctx->stream, a);
    return check_hip(ctx, hipGetLastError(), "bmu (wide) kernel launch");
}

static int launch_bmu_split_wide(som_ctx* ctx, const BmuArgs& a, int nch16)
{
    constexpr size_t lds_bytes = 2 * (size_t)split_stage_f4(4) * 16;
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(bmu_split_wide_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    // the pass's samples as bf16 parts first
    const int64_t groups8 = a.m * nch16 * 8;
    hipLaunchKernelGGL(bmu_split_convert_kernel, dim3((unsigned)((groups8 + 255) / 256)), dim3(256), 0, ctx->stream, a, nch16);
    if (int rc = check_hip(ctx, hipGetLastError(), "bmu (split, wide) conversion launch")) return rc;
    const int64_t per_group = (int64_t)kWavesPerGroup * 32;
    const int64_t groups = (a.m + per_group - 1) / per_group;
    hipLaunchKernelGGL(bmu_split_wide_kernel, dim3((unsigned)groups), dim3(kThreads), lds_bytes, ctx->stream, a);
    return check_hip(ctx, hipGetLastError(), "bmu (split, wide) kernel launch");
}

// grid of the candidate kernels: the tiles of the longest list they may serve, at most kCandGrid workgroups
static unsigned cand_grid(const BmuArgs& a, int64_t per_tile)
{
    const int64_t most = a.m < (int64_t)a.cand_cap ? a.m : (int64_t)a.cand_cap;
    const int64_t tiles = (most + per_tile - 1) / per_tile;
    return (unsigned)(tiles < kCandGrid ? tiles : kCandGrid);
}

template <int STEPS>
static int launch_bmu_wide_cand(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)stage_floats_for(2 * STEPS + 1) * sizeof(float);
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = bmu_wide_cand_kernel<STEPS>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(cand_grid(a, (int64_t)kWavesPerGroup * 32)), dim3(kThreads), lds_bytes, ctx->stream, a);
    return check_hip(ctx, hipGetLastError(), "bmu (wide) candidate kernel launch");
}

static int launch_bmu_split_wide_cand(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)split_stage_f4(4) * 16;
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(bmu_split_wide_cand_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    hipLaunchKernelGGL(bmu_split_wide_cand_kernel, dim3(cand_grid(a, (int64_t)kWavesPerGroup * 32)), dim3(kThreads),
                       lds_bytes, ctx->stream, a);
    return check_hip(ctx, hipGetLastError(), "bmu (split, wide) candidate kernel launch");
}

template <int STEPS, int MS>
static int launch_bmu_cand(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)stage_floats_for(2 * STEPS + 1) * sizeof(float);
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = bmu_cand_kernel<STEPS, MS>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(cand_grid(a, (int64_t)kWavesPerGroup * MS * 32)), dim3(kThreads), lds_bytes, ctx->stream,
                       a);
    return check_hip(ctx, hipGetLastError(), "bmu candidate kernel launch");
}

static int dispatch_bmu_cand(som_ctx* ctx, int steps, const BmuArgs& a)
{
    switch (steps) {
    case 4: return launch_bmu_cand<4, 2>(ctx, a);
    case 8: return launch_bmu_cand<8, 2>(ctx, a);
    case 12: return launch_bmu_cand<12, 2>(ctx, a);
    case 16: return launch_bmu_cand<16, 2>(ctx, a);
    case 20: return launch_bmu_cand<20, 2>(ctx, a);
    case 25: return launch_bmu_cand<25, 2>(ctx, a);
    case 28: return launch_bmu_cand<28, 2>(ctx, a);
    case 32: return launch_bmu_cand<32, 2>(ctx, a);
    }
    return fail(ctx, SOM_EINVAL, "no BMU kernel for %d steps", steps);
}

template <int STEPS, int MS>
static int launch_bmu(som_ctx* ctx, const BmuArgs& a)
{
    constexpr int STRIDE = 2 * STEPS + 1;
    constexpr size_t lds_bytes = 2 * (size_t)stage_floats_for(STRIDE) * sizeof(float);
    // maps that end in whole blocks of padding nodes take the variant that skips them
    const bool pad = a.kpad - a.K >= 32;
    static bool attr_set[2] = {false, false};
    auto kern = pad ? bmu_kernel<STEPS, MS, true> : bmu_kernel<STEPS, MS, false>;
    if (!attr_set[pad]) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set[pad] = true;
    }
    // Two workgroups fit a compute unit, so the grid runs in rounds of 2 * units tiles and a unit's time in the
    // last, partial round goes with the number of sample blocks it gets.  When halving the tiles of that round
    // lowers the largest share (measured at 10^6 samples on 256 units: 7.63 rounds cost as much as 8), they are
    // halved.
    if (ctx->units == 0) {
        int units = 0;
        if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess || units < 1)
            units = 256;
        ctx->units = units;
    }
    const int64_t per_group = (int64_t)kWavesPerGroup * MS * 32;
    const int64_t tiles = (a.m + per_group - 1) / per_group;
    const int64_t units = ctx->units, rem = tiles % (2 * units);
    BmuArgs b = a;
    b.full_tiles = tiles;
    int64_t groups = tiles;
    if (MS > 1 && tiles >= 2 * units && rem > 0 && (2 * rem + units - 1) / units < 2 * ((rem + units - 1) / units)) {
        b.full_tiles = tiles - rem;
        const int64_t left = a.m - b.full_tiles * per_group, per_half = per_group / 2;
        groups = b.full_tiles + (left + per_half - 1) / per_half;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(kThreads), lds_bytes, ctx->stream, b);
    return check_hip(ctx, hipGetLastError(), "bmu kernel launch");
}

template <int KB, bool TAIL, int MS>
static int launch_bmu_split(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)split_stage_f4(KB, TAIL) * 16;
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = bmu_split_kernel<KB, TAIL, MS>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    if (ctx->units == 0) {
        int units = 0;
        if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess || units < 1)
            units = 256;
        ctx->units = units;
    }
    // full tiles, and half tiles for the last partial round where that lowers the largest share (as launch_bmu)
    const int64_t per_group = (int64_t)kWavesPerGroup * MS * 32;
    const int64_t tiles = (a.m + per_group - 1) / per_group;
    const int64_t units = ctx->units, rem = tiles % (2 * units);
    BmuArgs b = a;
    b.full_tiles = tiles;
    int64_t groups = tiles;
    if (MS > 1 && tiles >= 2 * units && rem > 0 && (2 * rem + units - 1) / units < 2 * ((rem + units - 1) / units)) {
        b.full_tiles = tiles - rem;
        const int64_t left = a.m - b.full_tiles * per_group, per_half = per_group / 2;
        groups = b.full_tiles + (left + per_half - 1) / per_half;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(kThreads), lds_bytes, ctx->stream, b);
    return check_hip(ctx, hipGetLastError(), "bmu split kernel launch");
}

template <int KB, bool TAIL, int MS>
static int launch_bmu_split_cand(som_ctx* ctx, const BmuArgs& a)
{
    constexpr size_t lds_bytes = 2 * (size_t)split_stage_f4(KB, TAIL) * 16;
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = bmu_split_cand_kernel<KB, TAIL, MS>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(cand_grid(a, (int64_t)kWavesPerGroup * MS * 32)), dim3(kThreads), lds_bytes, ctx->stream,
                       a);
    return check_hip(ctx, hipGetLastError(), "bmu split candidate kernel launch");
}

static int dispatch_bmu_split_cand(som_ctx* ctx, int kb, bool tail, const BmuArgs& a)
{
    switch (kb * 2 + (tail ? 1 : 0)) {
    case 1: return launch_bmu_split_cand<0, true, kSplitMS>(ctx, a);
    case 2: return launch_bmu_split_cand<1, false, kSplitMS>(ctx, a);
    case 3: return launch_bmu_split_cand<1, true, kSplitMS>(ctx, a);
    case 4: return launch_bmu_split_cand<2, false, kSplitMS>(ctx, a);
    case 5: return launch_bmu_split_cand<2, true, kSplitMS>(ctx, a);
    case 6: return launch_bmu_split_cand<3, false, kSplitMS>(ctx, a);
    case 7: return launch_bmu_split_cand<3, true, kSplitMS>(ctx, a);
    case 8: return launch_bmu_split_cand<4, false, kSplitMS>(ctx, a);
    }
    return fail(ctx, SOM_EINVAL, "no split candidate kernel for %d blocks%s", kb, tail ? " and a tail" : "");
}

static int dispatch_bmu_split(som_ctx* ctx, int kb, bool tail, const BmuArgs& a)
{
    switch (kb * 2 + (tail ? 1 : 0)) {
    case 1: return launch_bmu_split<0, true, kSplitMS>(ctx, a);
    case 2: return launch_bmu_split<1, false, kSplitMS>(ctx, a);
    case 3: return launch_bmu_split<1, true, kSplitMS>(ctx, a);
    case 4: return launch_bmu_split<2, false, kSplitMS>(ctx, a);
    case 5: return launch_bmu_split<2, true, kSplitMS>(ctx, a);
    case 6: return launch_bmu_split<3, false, kSplitMS>(ctx, a);
    case 7: return launch_bmu_split<3, true, kSplitMS>(ctx, a);
    case 8: return launch_bmu_split<4, false, kSplitMS>(ctx, a);
    }
    return fail(ctx, SOM_EINVAL, "no split BMU kernel for %d blocks%s", kb, tail ? " and a tail" : "");
}

static int dispatch_bmu(som_ctx* ctx, int steps, const BmuArgs& a)
{
    switch (steps) {
    case 4: return launch_bmu<4, 2>(ctx, a);
    case 8: return launch_bmu<8, 2>(ctx, a);
    case 12: return launch_bmu<12, 2>(ctx, a);
    case 16: return launch_bmu<16, 2>(ctx, a);
    case 20: return launch_bmu<20, 2>(ctx, a);
    case 25: return launch_bmu<25, 2>(ctx, a);
    case 28: return launch_bmu<28, 2>(ctx, a);
    case 32: return launch_bmu<32, 2>(ctx, a);
    }
    return fail(ctx, SOM_EINVAL, "no BMU kernel for %d steps", steps);
}

static int bmu_run_pass(som_ctx* ctx, BmuPrep& prep, BmuArgs a);

// The rows go through in passes of at most 2^27: the re-decision workspace then stays near 2.2 GB whatever m is,
// and a pass's list stays within what the candidate pass can hold (2^24 entries, an eighth of a pass) — one call over
// 10^9 rows listed more than that and fell back to direct differences over all nodes for every listed sample.
int bmu_run(som_ctx* ctx, BmuPrep& prep, BmuArgs a)
{
    int64_t kRowsPerPass = (int64_t)1 << 27;
    const int64_t m = a.m;
    // the split search for D > 64 reads the pass's samples as bf16 parts from a workspace of its own: 256 bytes per
    // sample and chunk of 64 features, at most kPartsBytes in all (shorter passes for wide rows)
    if (prep.stage16 && prep.nch > 1) {
        const size_t row_bytes = (size_t)prep.nch16 * 256;
        int64_t rows = (int64_t)(kPartsBytes / row_bytes) / 128 * 128;
        if (rows < 128) rows = 128;
        if (rows < kRowsPerPass) kRowsPerPass = rows;
        const size_t need = (size_t)(m < kRowsPerPass ? m : kRowsPerPass) * row_bytes;
        if (need > ctx->parts_bytes) {
            if (ctx->parts_blob) {
                if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
                (void)hipFree(ctx->parts_blob);
                ctx->parts_blob = nullptr;
                ctx->parts_bytes = 0;
            }
            if (hipMalloc(&ctx->parts_blob, need) != hipSuccess) {
                (void)hipGetLastError();
                return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for the samples' bf16 parts", need);
            }
            ctx->parts_bytes = need;
        }
        a.parts = ctx->parts_blob;
    }
    for (int64_t off = 0; off < m; off += kRowsPerPass) {
        BmuArgs b = a;
        b.m = m - off < kRowsPerPass ? m - off : kRowsPerPass;
        if (a.idx)
            b.idx = a.idx + off;
        else
            b.X = a.X + off * a.ldx;
        b.bmu = a.bmu + off;
        if (a.d2) b.d2 = a.d2 + off;
        if (int rc = bmu_run_pass(ctx, prep, b)) return rc;
    }
    return SOM_OK;
}

static int bmu_run_pass(som_ctx* ctx, BmuPrep& prep, BmuArgs a)
{
    if (a.m <= 0) return SOM_OK;
    auto cand_cap_for = [](size_t cap) { return cap < kCandCapMax ? cap : kCandCapMax; };
    if ((size_t)a.m > ctx->recheck_cap) {
        if (ctx->recheck) {
            if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
            (void)hipFree(ctx->recheck);
            ctx->recheck = nullptr;
            ctx->recheck_cap = 0;
        }
        // sample positions [cap], cuts [cap], per-sample cuts [cap], second list [cand_cap], candidate sets [cand_cap][2]; the capacity is a
        // multiple of four entries so that the 16-byte candidate sets stay aligned
        const size_t cap = ((size_t)a.m + 3) / 4 * 4, ccap = cand_cap_for(cap);
        const size_t bytes = cap * 12 + ccap * (4 + 2 * sizeof(ulonglong2));
        if (hipMalloc((void**)&ctx->recheck, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, SOM_ENOMEM, "cannot allocate the %lld-entry recheck list", (long long)a.m);
        }
        ctx->recheck_cap = cap;
    }
    a.kpad = prep.kpad;
    a.stage = prep.stage;
    a.stride = prep.stride;
    a.stage16 = prep.stage16;
    a.wwin = prep.wwin;
    a.tail_r = prep.tail_r;
    a.wt = prep.wt;
    a.centre = prep.centre;
    a.scal = prep.scal;
    a.recheck = ctx->recheck;
    a.cutv = (float*)(ctx->recheck + ctx->recheck_cap);
    a.cut_all = (float*)(ctx->recheck + 2 * ctx->recheck_cap);
    a.recheck2 = ctx->recheck + 3 * ctx->recheck_cap;
    a.cand = (ulonglong2*)(a.recheck2 + cand_cap_for(ctx->recheck_cap));
    a.cand_cap = (uint32_t)cand_cap_for(ctx->recheck_cap);
    // The candidate pass repeats the search for the listed samples at matrix speed (under a nanosecond per sample
    // at K D = 51200, against 3.8 ns for direct differences over all nodes) but has the latency of a whole tile, so
    // it only serves lists above a minimum length; node ids are 16-bit there.
    const bool cand_possible = a.K > 1 && a.K <= 65536 && a.m > (int64_t)kCandMin;
    a.cand_min = cand_possible ? kCandMin : 0xffffffffu;
    a.qe_part = ctx->qe_part;
    // the list length restarts for every call (chunk): calls alternate between two counters, and each call's
    // exact pass clears the counter of the next one
    a.slot = 1 + (prep.calls & 1);
    a.slot2 = 4 + (prep.calls & 1);
    ++prep.calls;
    hipEvent_t stop = nullptr;
    if (ctx->profiling) {
        if (ctx->prof_used == ctx->prof_events.size()) {
            hipEvent_t e0, e1;
            if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
                return fail(ctx, SOM_EHIP, "event creation failed");
            ctx->prof_events.emplace_back(e0, e1);
        }
        (void)hipEventRecord(ctx->prof_events[ctx->prof_used].first, ctx->stream);
        stop = ctx->prof_events[ctx->prof_used].second;
        ++ctx->prof_used;
    }
    int rc = prep.nch > 1 ? (prep.stage16        ? launch_bmu_split_wide(ctx, a, prep.nch16)
                             : prep.steps == 25 ? launch_bmu_wide<25>(ctx, a)
                             : prep.steps == 28 ? launch_bmu_wide<28>(ctx, a)
                                                : launch_bmu_wide<32>(ctx, a))
                          : (prep.stage16 ? dispatch_bmu_split(ctx, prep.kb, prep.tail_r > 0, a) : dispatch_bmu(ctx, prep.steps, a));
    if (rc) return rc;
    if (a.K > 1) {
        const int64_t chunks = (a.m + kListThreads * kListPerThread - 1) / (kListThreads * kListPerThread);
        hipLaunchKernelGGL(bmu_list_kernel, dim3((unsigned)(chunks < 1024 ? chunks : 1024)), dim3(kListThreads), 0, ctx->stream, a);
        if ((rc = check_hip(ctx, hipGetLastError(), "bmu list launch"))) return rc;
    }
    if (stop) (void)hipEventRecord(stop, ctx->stream);
    if (cand_possible) {
        rc = prep.nch > 1 ? (prep.stage16        ? launch_bmu_split_wide_cand(ctx, a)
                             : prep.steps == 25 ? launch_bmu_wide_cand<25>(ctx, a)
                             : prep.steps == 28 ? launch_bmu_wide_cand<28>(ctx, a)
                                                : launch_bmu_wide_cand<32>(ctx, a))
                          : (prep.stage16 ? dispatch_bmu_split_cand(ctx, prep.kb, prep.tail_r > 0, a) : dispatch_bmu_cand(ctx, prep.steps, a));
        if (rc) return rc;
        // (the split search for D <= 64 takes the direct differences over its candidates at the end of the candidate
        // tile itself; the others hand their candidate sets to a kernel of their own)
        if (!(prep.stage16 && prep.nch == 1)) {
            hipLaunchKernelGGL(bmu_cand_exact_kernel, dim3(2048), dim3(256), 0, ctx->stream, a);
            if ((rc = check_hip(ctx, hipGetLastError(), "bmu candidate-distance launch"))) return rc;
        }
    }
    if (a.K > 1) {
        hipLaunchKernelGGL(bmu_exact_kernel, dim3(1024), dim3(256), 0, ctx->stream, a);
        if ((rc = check_hip(ctx, hipGetLastError(), "bmu exact-pass launch"))) return rc;
    }
    if (a.qe) {
        hipLaunchKernelGGL(qe_finish_kernel, dim3(1), dim3(kQeSlots), 0, ctx->stream, a.qe_part, a.qe);
        rc = check_hip(ctx, hipGetLastError(), "quantisation-error reduction launch");
    }
    return rc;
}

} // namespace som
