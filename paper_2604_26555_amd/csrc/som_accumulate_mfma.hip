// Per-BMU sample sums and counts with the partial sums held in MFMA accumulators:
//     S_k += x_i,  n_k += 1   for k = b_i       (the inner sums of Eq. 3 grouped by best-matching unit).
//
// S = A^T X with A the N x K one-hot matrix of the BMUs.  Dense, that contraction would cost as much as the BMU
// search; restricted to the rows that can be non-zero it is tiny.  A workgroup owns a contiguous range of
// samples and ALL of S for that range: the K x (D + 1) partial (the extra column counts samples: its X entry is a
// constant 1) is cut into 32-node x 32-feature blocks of 16 accumulator VGPRs, dealt round-robin over the 8
// wavefronts (node block nb belongs to wavefront nb % 8).  Samples arrive in LDS tiles of 256 full rows.  For
// every tile a wavefront compacts, per node block it owns, the tile positions whose BMU falls into the block
// (ballot + prefix count; ascending, so the order of additions is fixed), then feeds them two at a time to
// v_mfma_f32_32x32x2_f32:  A = 32 nodes x 2 samples, 1.0 where the node is the sample's BMU;  B = 2 samples x 32
// features read straight from the LDS tile (the ones column and the zero padding live in the tile as well, so
// building an operand costs no vector instructions).  No atomics anywhere, X is read exactly once, and a node
// that attracts a quarter of all samples only lengthens one wavefront's MFMA chain.
// The accumulators move into the workgroup's slice of a global workspace every kFlushRows samples (bounding any
// float32 summation chain); a second kernel adds the slices in a fixed order into S and n.  Slices are padded to
// whole 32-node x 32-column blocks so that every accumulator store is unconditional and covers whole, aligned
// 128-byte runs.  Eight wavefronts of up to 256 VGPRs per workgroup: with sixteen the 128 accumulator registers of
// a 1024-node, 64-column partial do not fit and spill.
#include "som_internal.hpp"

namespace som {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Elements between consecutive workgroups' slices: the padded K x columns block, rounded up to an odd number of
// 4 KiB pages.  All workgroups store the same slice offsets at the same time; with a power-of-two distance those
// stores land on a few memory channels only.
__host__ __device__ inline size_t slice_stride(int K, int cols, size_t elem_bytes)
{
    size_t pages = ((size_t)((K + 31) / 32) * 32 * cols * elem_bytes + 4095) / 4096;
    pages |= 1;
    return pages * 4096 / elem_bytes;
}

constexpr int kMThreads = 512;
constexpr int kMWaves = kMThreads / 64;
constexpr int kMTile = 256;        // rows per LDS tile; tile positions fit a byte
constexpr int kMFlushRows = 16384;
constexpr int kMWindow = 63;       // features per pass: 63 + the count column fill two 32-column blocks

// NBW = node blocks per wavefront, FB = feature blocks (of 32 columns, the count column included)
template <typename SliceT, int NBW, int FB>
__global__ void __launch_bounds__(kMThreads) accumulate_mfma_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                    const uint32_t* __restrict__ idx, int64_t m,
                                                                    const int32_t* __restrict__ bmu, int K,
                                                                    int64_t rows_per_range, SliceT* __restrict__ part)
{
    constexpr int COLS = FB * 32;
    constexpr int STRIDE = COLS + 1;                      // odd row stride: the two rows of an operand never alias banks
    constexpr int PASSES = kMTile / (kMThreads / 64);     // tile rows per thread when 64 lanes span a row
    extern __shared__ float4 macc_lds4[];
    float* T = reinterpret_cast<float*>(macc_lds4);                         // [kMTile][STRIDE]
    int* Bt = reinterpret_cast<int*>(T + kMTile * STRIDE);                  // [kMTile]
    unsigned short* Lst = reinterpret_cast<unsigned short*>(Bt + kMTile);   // [kMWaves * NBW][kMTile]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: row addresses of the tile loads stay in SGPRs
    const int64_t lo = (int64_t)blockIdx.x * rows_per_range;
    int64_t hi = lo + rows_per_range;
    if (hi > m) hi = m;
    constexpr int LS = FB * 32;                                             // padded slice row: whole cache lines per store
    const int KP = ((K + 31) / 32) * 32;                                    // slice rows: whole node blocks
    SliceT* mine = part + (size_t)blockIdx.x * slice_stride(K, LS, sizeof(SliceT));

    // constant columns of the tile: 1.0 in column D, 0.0 behind it
    for (int e = tid; e < kMTile * (COLS - D); e += kMThreads) {
        const int r = e / (COLS - D), c = D + e % (COLS - D);
        T[r * STRIDE + c] = (c == D) ? 1.0f : 0.0f;
    }

    floatx16 acc[NBW][FB];
#pragma unroll
    for (int q = 0; q < NBW; ++q)
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][fb][r] = 0.0f;

    // tile loading: wavefront w brings rows w, w + 8, ...; lane = feature (D <= 63 on this path)
    float pre[PASSES];
    int preb = -1;
    const int lanecol = lane < D ? lane : D - 1;              // clamped, so every load is unconditional
    // Row numbers are wave-uniform: the row base stays in scalar registers and the lane adds its column.  The
    // fetch only issues loads; anything computed from a loaded value waits for the stash, after the tile before
    // has been consumed.
    auto fetch = [&](int64_t t0, int64_t top) {
        if (!idx && t0 + kMTile <= top) {
            // whole tile of consecutive rows: one base, a constant stride (two scalar adds per row)
            const float* rowp = X + (t0 + wave) * ldx;
            const int64_t step = (int64_t)kMWaves * ldx;
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                pre[p] = rowp[lanecol];
                rowp += step;
            }
        } else {
            // ragged tail or an index list: clamp, translate, then address every row on its own
            int64_t row[PASSES];
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int64_t i = t0 + wave + p * kMWaves;
                row[p] = i < top ? i : top - 1;
            }
            if (idx) {
#pragma unroll
                for (int p = 0; p < PASSES; ++p) row[p] = (int64_t)idx[row[p]];
            }
#pragma unroll
            for (int p = 0; p < PASSES; ++p) pre[p] = X[row[p] * ldx + lanecol];
        }
        const int64_t i = t0 + (tid & (kMTile - 1));
        preb = bmu[i < top ? i : top - 1];
    };
    auto stash = [&](int64_t t0, int64_t top) {
        if (lane < D) {
#pragma unroll
            for (int p = 0; p < PASSES; ++p) T[(wave + p * kMWaves) * STRIDE + lane] = pre[p];
        }
        if (tid < kMTile) Bt[tid] = (t0 + tid < top && preb >= 0 && preb < K) ? preb : -1;
    };
    auto consume = [&]() {
        // 1. per owned node block: ascending list of (tile position | node-in-block << 8)
        int cnt[NBW];
#pragma unroll
        for (int q = 0; q < NBW; ++q) cnt[q] = 0;
        for (int c = 0; c < kMTile; c += 64) {
            const int b = Bt[c + lane];
#pragma unroll
            for (int q = 0; q < NBW; ++q) {
                const int nb = wave + q * kMWaves;
                const bool own = b >= 0 && (b >> 5) == nb;
                const unsigned long long bal = __ballot(own);
                const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0));
                if (own) Lst[(wave * NBW + q) * kMTile + cnt[q] + below] = (unsigned short)((c + lane) | ((b & 31) << 8));
                cnt[q] += __popcll(bal);
            }
        }
        // 2. two samples per MFMA step: lanes 0..31 carry one sample, lanes 32..63 the next
        const int half = lane >> 5, j = lane & 31;
#pragma unroll
        for (int q = 0; q < NBW; ++q) {
            const unsigned short* lst = Lst + (wave * NBW + q) * kMTile;
            const int n = cnt[q];
            // four steps at a time: their list entries, then their operands, are in flight together
            for (int s0 = 0; s0 < n; s0 += 8) {
                int e[4];
                bool v[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int s = s0 + 2 * t + half;
                    v[t] = s < n;
                    e[t] = (int)lst[v[t] ? s : s0];
                }
                float a[4], bv[4][FB];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    a[t] = (v[t] && (e[t] >> 8) == j) ? 1.0f : 0.0f;
                    const float* row = T + (e[t] & 0xff) * STRIDE + j;
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) bv[t][fb] = row[32 * fb];
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (s0 + 2 * t < n) {
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
                            acc[q][fb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], bv[t][fb], acc[q][fb], 0, 0, 0);
                    }
                }
            }
        }
    };

    bool first = true;
    for (int64_t base = lo; base < hi || first; base += kMFlushRows) {
        const int64_t top = (base + kMFlushRows < hi) ? base + kMFlushRows : hi;
        if (base < top) {
            fetch(base, top);
            for (int64_t t0 = base; t0 < top; t0 += kMTile) {
                __syncthreads();                                  // tile free (and the constant columns written)
                stash(t0, top);
                __syncthreads();
                if (t0 + kMTile < top) fetch(t0 + kMTile, top);   // in flight while this tile is consumed
                consume();
            }
        }
        // accumulators -> slice (first flush stores, later ones add), then clear.  Register r of lane l holds
        // node 8 (r / 4) + 4 (l / 32) + r % 4 of the block, column l % 32.  Slices are padded to whole node
        // blocks and whole column blocks, so every store is unconditional and covers aligned 128-byte runs.
#pragma unroll
        for (int q = 0; q < NBW; ++q) {
            const int nb = wave + q * kMWaves;
            if (nb * 32 < KP) {
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    // the offset is made opaque so that the store addresses are formed here, not kept in
                    // registers for the whole kernel
                    int off = (nb * 32 + 4 * (lane >> 5)) * LS + fb * 32 + (lane & 31);
                    asm volatile("" : "+v"(off));
                    SliceT* cell = mine + off;
                    if (first) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) cell[(8 * (r >> 2) + (r & 3)) * LS] = (SliceT)acc[q][fb][r];
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) cell[(8 * (r >> 2) + (r & 3)) * LS] += (SliceT)acc[q][fb][r];
                    }
                }
            }
#pragma unroll
            for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[q][fb][r] = 0.0f;
        }
        first = false;
    }
}

// S[k][f] (+)= sum over the workgroups' slices, n[k] (+)= sum of their count columns, always in the same order:
// a workgroup takes 64 cells, its four wavefronts a quarter of the slices each, then the quarters are added 0..3.
template <typename SliceT>
__global__ void __launch_bounds__(256) accumulate_mfma_reduce_kernel(const SliceT* __restrict__ part, int K, int D,
                                                                     int ranges, int zero_first, double* __restrict__ S,
                                                                     int ldS, unsigned long long* __restrict__ n)
{
    // D = columns of this launch's feature window, S points at the window's first column, ldS = row length of S;
    // n may be null (the counts are taken from the first window only)
    __shared__ double qsum[4][64];
    const int q = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int DS = ((D + 1 + 31) / 32) * 32;              // padded slice row (only columns 0..D carry data)
    const int c = blockIdx.x * 64 + l;                    // cell of the K x DS slice layout
    const int per = (ranges + 3) / 4;
    const int r_lo = q * per, r_hi = (r_lo + per < ranges) ? r_lo + per : ranges;
    double s = 0.0;
    if (c < K * DS && c % DS <= D) {
        const size_t stride = slice_stride(K, DS, sizeof(SliceT));
#pragma unroll 8
        for (int r = r_lo; r < r_hi; ++r) s += (double)part[(size_t)r * stride + c];
    }
    qsum[q][l] = s;
    __syncthreads();
    if (q == 0 && c < K * DS) {
        const double tot = ((qsum[0][l] + qsum[1][l]) + qsum[2][l]) + qsum[3][l];
        const int k = c / DS, f = c % DS;
        if (f < D)
            S[(size_t)k * ldS + f] = (zero_first ? 0.0 : S[(size_t)k * ldS + f]) + tot;
        else if (f == D && n)
            n[k] = (zero_first ? 0ull : n[k]) + (unsigned long long)(tot + 0.5);
    }
}

template <typename SliceT, int NBW, int FB>
static int launch_mfma(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                       const int32_t* bmu, int32_t K, int64_t ranges, int64_t rows_per_range, SliceT* part)
{
    constexpr size_t lds = (size_t)kMTile * (FB * 32 + 1) * 4 + kMTile * 4 + (size_t)kMWaves * NBW * kMTile * 2;
    static bool attr_set_dev[kMaxDevices] = {};       // the attribute belongs to the device, not to the process
    bool& attr_set = attr_set_dev[ctx->device];
    auto kern = accumulate_mfma_kernel<SliceT, NBW, FB>;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)ranges), dim3(kMThreads), lds, ctx->stream, X, D, ldx, idx, m, bmu, K,
                       rows_per_range, part);
    return check_hip(ctx, hipGetLastError(), "accumulate (MFMA) launch");
}

template <typename SliceT>
static int dispatch_mfma(som_ctx* ctx, int nbw, int fb, const float* X, int32_t D, int64_t ldx, const uint32_t* idx,
                         int64_t m, const int32_t* bmu, int32_t K, int64_t ranges, int64_t rpr, SliceT* part)
{
#define SOM_MFMA_CASE(N, F) \
    if (nbw == N && fb == F) return launch_mfma<SliceT, N, F>(ctx, X, D, ldx, idx, m, bmu, K, ranges, rpr, part);
    SOM_MFMA_CASE(1, 1) SOM_MFMA_CASE(2, 1) SOM_MFMA_CASE(4, 1) SOM_MFMA_CASE(8, 1)
    SOM_MFMA_CASE(1, 2) SOM_MFMA_CASE(2, 2) SOM_MFMA_CASE(4, 2)
#undef SOM_MFMA_CASE
    return fail(ctx, SOM_EINVAL, "no MFMA accumulation kernel for %d node blocks x %d feature blocks", nbw, fb);
}

// Returns 1 when the shape is not served by this path (the caller then uses the LDS-atomic kernel), SOM_OK on
// success, a negative code on failure.  Served: up to 8 accumulator blocks per wavefront (K <= 1024 when a feature
// window needs two column blocks, K <= 2048 when D <= 31); D above 63 goes through in windows of 63 features.
int accumulate_mfma_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                        const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first)
{
    // feature windows of at most 63 columns (+ the count column = two blocks of 32); one window after the other
    // through the same slices
    const int window = (D <= kMWindow) ? D : kMWindow;
    const int fb = (window + 1 + 31) / 32;
    const int nblocks = (K + 31) / 32;
    int nbw = 1;
    while (nbw * kMWaves < nblocks) nbw *= 2;
    if (nbw * fb > 8 || m <= 0) return 1;
    // one workgroup per compute unit, at least one tile each
    int64_t ranges = 256;
    const int64_t by_rows = (m + kMTile - 1) / kMTile;
    if (ranges > by_rows) ranges = by_rows;
    const int64_t rows_per_range = (((m + ranges - 1) / ranges + kMTile - 1) / kMTile) * kMTile;
    ranges = (m + rows_per_range - 1) / rows_per_range;
    const bool single_flush = rows_per_range <= kMFlushRows;
    const size_t esz = single_flush ? sizeof(float) : sizeof(double);
    const size_t need = (size_t)ranges * slice_stride(K, fb * 32, esz) * esz;
    if (need > ctx->acc_bytes) {
        if (ctx->acc_blob) {
            if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
            (void)hipFree(ctx->acc_blob);
            ctx->acc_blob = nullptr;
            ctx->acc_bytes = 0;
        }
        if (hipMalloc(&ctx->acc_blob, need) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for the accumulation workspace", need);
        }
        ctx->acc_bytes = need;
    }
    for (int f0 = 0; f0 < D; f0 += window) {
        const int dw = (D - f0 < window) ? D - f0 : window;
        const int fbw = (dw + 1 + 31) / 32;
        const dim3 rgrid((K * fbw * 32 + 63) / 64);
        unsigned long long* nw = (f0 == 0) ? n : nullptr;
        if (single_flush) {
            float* part = (float*)ctx->acc_blob;
            if (int rc = dispatch_mfma<float>(ctx, nbw, fbw, X + f0, dw, ldx, idx, m, bmu, K, ranges, rows_per_range, part))
                return rc;
            hipLaunchKernelGGL(accumulate_mfma_reduce_kernel<float>, rgrid, dim3(256), 0, ctx->stream, part, K, dw,
                               (int)ranges, zero_first ? 1 : 0, S + f0, D, nw);
        } else {
            double* part = (double*)ctx->acc_blob;
            if (int rc = dispatch_mfma<double>(ctx, nbw, fbw, X + f0, dw, ldx, idx, m, bmu, K, ranges, rows_per_range, part))
                return rc;
            hipLaunchKernelGGL(accumulate_mfma_reduce_kernel<double>, rgrid, dim3(256), 0, ctx->stream, part, K, dw,
                               (int)ranges, zero_first ? 1 : 0, S + f0, D, nw);
        }
        if (int rc = check_hip(ctx, hipGetLastError(), "accumulate (MFMA) reduce launch")) return rc;
    }
    return SOM_OK;
}

} // namespace som
