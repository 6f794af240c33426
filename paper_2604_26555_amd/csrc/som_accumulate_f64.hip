// Per-BMU sample sums and counts in LDS with float64 atomics:
//     S_k += x_i,  n_k += 1   for k = b_i       (the inner sums of Eq. 3 grouped by best-matching unit).
//
// Measured on gfx950: ds_add_f64 and the integer LDS atomics complete a 64-lane instruction in about 15 cycles,
// ds_add_f32 needs about 190.  With 8-byte cells the K x (D + 1) partial (the extra column counts samples) does
// not fit one compute unit's LDS, so the NODES are cut into slabs: a workgroup owns a contiguous range of samples
// and one slab of nodes, reads the BMU of every sample of its range (4 bytes), and loads and adds only the rows
// whose BMU falls into its slab.  Every row of X is therefore read exactly once, by exactly one workgroup, as one
// coalesced 64-lane load (lane 0 adds the count, lane l > 0 feature l - 1), followed by one LDS atomic instruction.
// Wavefronts work independently: each reads the BMUs of 256 consecutive samples with one 16-byte load per lane (a
// round ahead), and in four passes of 64 samples takes the rows that belong to the slab off a ballot mask with
// scalar instructions, up to sixteen rows at a time (that many row loads in flight); there is no barrier and no LDS traffic
// other than the atomics inside the range loop.  Where the time goes (10^7 rows of 50 features on 1024 nodes, 431 us
// against 331 us for a kernel that only reads X): a 64-lane LDS atomic takes 15.6 cycles per instruction and COMPUTE
// UNIT whatever its width, 16 cycles a row where the plain read needs 8, and the kernel spends 21; the scan alone
// (every row skipped) costs 64 us for three slabs; more row loads in flight change nothing.  At 10^6 rows, 26 of the
// 57 us do not depend on the rows at all (clearing LDS, the slices, the reduce kernel, two launches).
// At the end the slab moves to the range's slice of a global workspace and a second kernel adds the slices in a
// fixed order.  Counts are exact; the sums are float64 throughout (the order of the atomic additions varies from
// run to run, which moves a sum by a few units in the 16th digit).
// The slabs of one sample range get workgroup numbers 8 apart so that they run on the same XCD: rows are not
// aligned to cache lines, and the lines two neighbouring rows share are then fetched into that XCD's L2 once.
#include "som_internal.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <type_traits>

namespace som {

constexpr int kFThreads = 1024;
constexpr size_t kFLdsBytes = 150 * 1024;     // slab
constexpr int kFMaxSlabs = 16;

// GATHER: rows are taken through the index list (a scalar load per row; kept out of the plain variant because its
// wait would also wait for the LDS atomics in flight)
template <bool GATHER>
__global__ void __launch_bounds__(kFThreads) accumulate_f64_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                   const uint32_t* __restrict__ idx, int64_t m,
                                                                   const int32_t* __restrict__ bmu, int K, int ks,
                                                                   int nslabs, int64_t rows_per_range,
                                                                   double* __restrict__ part)
{
    extern __shared__ double f64_lds[];
    const int DS = D + 1;
    double* P = f64_lds;                                                   // [ks][DS]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroup number -> (range, slab): slabs of a range sit 8 apart inside a block of 8 * nslabs workgroups
    const int blk = blockIdx.x / (8 * nslabs), within = blockIdx.x % (8 * nslabs);
    const int slab = within / 8;
    const int64_t range = (int64_t)blk * 8 + (within % 8);
    const int k0 = slab * ks;
    const int kn = (k0 + ks <= K) ? ks : K - k0;                           // nodes of this slab (may be <= 0)
    const int64_t lo = range * rows_per_range;
    if (lo >= m) return;                                   // padding of the last block of 8 ranges (whole workgroup)
    int64_t hi = lo + rows_per_range;
    if (hi > m) hi = m;

    for (int c = tid; c < ks * DS; c += kFThreads) P[c] = 0.0;
    __syncthreads();

    constexpr int G = 16;                                                 // rows in flight per wavefront
    constexpr int U = 4;                                                  // 64-row passes per load of BMU indices
    // A wavefront takes 64 U consecutive samples at a time: lane l holds the BMUs of samples base + U l .. + U - 1
    // (one 16-byte load, requested a whole round of U passes ahead: with one pass per load the wait for the indices
    // was the longest part of a pass), and pass q works on the samples base + U l + q.
    auto load_bmus = [&](int64_t base, int (&bq)[U]) {
        const int64_t i0 = base + U * lane;
        if (i0 + U <= hi) {
            int4 t;
            __builtin_memcpy(&t, bmu + i0, sizeof(t));
            bq[0] = t.x;
            bq[1] = t.y;
            bq[2] = t.z;
            bq[3] = t.w;
        } else {
#pragma unroll
            for (int q = 0; q < U; ++q) bq[q] = (i0 + q < hi) ? bmu[i0 + q] : -1;
        }
    };
    static_assert(U == 4, "the BMU indices of a round travel as one int4");
    int bq_next[U];
    load_bmus(lo + (int64_t)wave * 64 * U, bq_next);
    const int ldxu = (int)ldx * U;                                         // distance between a pass's rows
    for (int64_t base = lo + (int64_t)wave * 64 * U; base < hi; base += (int64_t)kFThreads * U) {
        int bq[U];
#pragma unroll
        for (int q = 0; q < U; ++q) bq[q] = bq_next[q];
        load_bmus(base + (int64_t)kFThreads * U, bq_next);                 // beyond the range: all -1, nothing is read
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int b = bq[q];
            const bool in = b >= k0 && b < k0 + kn;
            unsigned long long todo = __ballot(in);                        // wave-uniform: lanes whose row is ours
            const float* xpass = X + (base + q) * ldx;
            const int ncell = (b - k0) * DS;                                // this lane's row of P, if its sample is ours
            // Rows are taken off the mask with scalar instructions only (find-first-set, read-lane): no list in
            // LDS, no wait between a row's decoding and its load, so up to G row loads are in flight per wavefront.
            // The scalar unit is shared by the compute unit's wavefronts and this bookkeeping is what it is busy
            // with, so whole batches (sixteen rows, then eight, then four) run without per-row conditions, three
            // scalar instructions a row; what is left of the pass goes through one batch of four places whose empty
            // ones repeat the last row's load and skip the addition.
            int left = __popcll(todo);
            const int f = lane - 1;                                         // lane 0 carries the count
            const int fcl = f < 0 ? 0 : (f < D ? f : D - 1);
            auto whole_batch = [&](auto width) {
                constexpr int GB = decltype(width)::value;
                float v[GB];
                int cell[GB];
#pragma unroll
                for (int t = 0; t < GB; ++t) {
                    const int p = __builtin_ctzll(todo);                    // todo has at least GB bits set here
                    asm("s_bitset0_b64 %0, %1" : "+s"(todo) : "s"(p));
                    // plain variant: 32-bit offset from the pass's first row (63 U rows of ldx floats stay far
                    // below 2^31)
                    const float* xrow = GATHER ? X + (int64_t)idx[base + U * p + q] * ldx : xpass + (unsigned)(p * ldxu);
                    cell[t] = __builtin_amdgcn_readlane(ncell, p);
                    const float xv = xrow[fcl];
                    v[t] = (lane == 0) ? 1.0f : xv;
                }
                if (lane < DS) {
#pragma unroll
                    for (int t = 0; t < GB; ++t) unsafeAtomicAdd(&P[cell[t] + lane], (double)v[t]);
                }
                left -= GB;
            };
            while (left >= G) whole_batch(std::integral_constant<int, G>{});
            if (left >= G / 2) whole_batch(std::integral_constant<int, G / 2>{});
            if (left >= G / 4) whole_batch(std::integral_constant<int, G / 4>{});
            if (left > 0) {
                constexpr int GB = G / 4;
                float v[GB];
                int cell[GB];
                bool live[GB];
                int p_last = 0;
#pragma unroll
                for (int t = 0; t < GB; ++t) {
                    live[t] = todo != 0ull;
                    const int p = live[t] ? (int)__ffsll((long long)todo) - 1 : p_last;
                    if (live[t]) {
                        todo &= todo - 1ull;
                        p_last = p;
                    }
                    const float* xrow = GATHER ? X + (int64_t)idx[base + U * p + q] * ldx : xpass + (unsigned)(p * ldxu);
                    cell[t] = __builtin_amdgcn_readlane(ncell, p);
                    const float xv = xrow[fcl];
                    v[t] = (lane == 0) ? 1.0f : xv;
                }
#pragma unroll
                for (int t = 0; t < GB; ++t) {
                    if (live[t]) {
                        if (lane < DS) unsafeAtomicAdd(&P[cell[t] + lane], (double)v[t]);
                    }
                }
            }
        }
    }
    __syncthreads();
    // slab -> the range's slice [K][DS]
    if (kn > 0) {
        double* out = part + ((size_t)range * K + k0) * DS;
        for (int c = tid; c < kn * DS; c += kFThreads) out[c] = P[c];
    }
}

// S[k][f] (+)= sum over the ranges' slices, n[k] (+)= sum of their count columns, always in the same order:
// a workgroup takes 64 cells, its four wavefronts a quarter of the slices each, then the quarters are added 0..3.
// D = columns of this launch's feature window, S points at the window's first column, ldS = row length of S; n may
// be null (the counts are taken from the first window only).
__global__ void __launch_bounds__(256) accumulate_f64_reduce_kernel(const double* __restrict__ part, int K, int D,
                                                                    int ranges, int zero_first, double* __restrict__ S,
                                                                    int ldS, unsigned long long* __restrict__ n)
{
    __shared__ double qsum[4][64];
    const int q = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int DS = D + 1;
    const int c = blockIdx.x * 64 + l;
    const int per = (ranges + 3) / 4;
    const int r_lo = q * per, r_hi = (r_lo + per < ranges) ? r_lo + per : ranges;
    double s = 0.0;
    if (c < K * DS) {
        const size_t stride = (size_t)K * DS;
#pragma unroll 8
        for (int r = r_lo; r < r_hi; ++r) s += part[(size_t)r * stride + c];
    }
    qsum[q][l] = s;
    __syncthreads();
    if (q == 0 && c < K * DS) {
        const double tot = ((qsum[0][l] + qsum[1][l]) + qsum[2][l]) + qsum[3][l];
        const int k = c / DS, f = c % DS;
        if (f == 0) {
            if (n) n[k] = (zero_first ? 0ull : n[k]) + (unsigned long long)(tot + 0.5);
        } else {
            S[(size_t)k * ldS + f - 1] = (zero_first ? 0.0 : S[(size_t)k * ldS + f - 1]) + tot;
        }
    }
}

// Returns 1 when the shape is not served by this path (the caller then tries the others), SOM_OK on success, a
// negative code on failure.  Rows wider than 63 features go through in windows of 63 (one kernel + reduce per
// window through the same slices).  Served: a K x 64 float64 partial that fits kFMaxSlabs slabs of LDS.
int accumulate_f64_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                       const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first)
{
    if (m <= 0 || ldx >= (1 << 22)) return 1;               // row offsets inside a round of passes are 32-bit
    const int window = D < 63 ? D : 63;                      // features per pass; lane 0 carries the count
    const size_t row_bytes = (size_t)(window + 1) * sizeof(double);
    const int ks_max = (int)(kFLdsBytes / row_bytes);
    const int nslabs = (K + ks_max - 1) / ks_max;
    if (nslabs > kFMaxSlabs) return 1;
    const int ks = (K + nslabs - 1) / nslabs;                  // balanced slabs
    // One workgroup per compute unit and never more workgroups than compute units (with one resident workgroup
    // per unit a grid of 264 ran 60 % slower than one of 240): 256 / nslabs ranges, in whole blocks of 8 so that
    // the slabs of a range share an XCD.
    int64_t ranges = (256 / nslabs) / 8 * 8;
    if (ranges < 8) ranges = 256 / nslabs;
    if (ranges < 1) ranges = 1;
    const int64_t by_rows = (m + kFThreads - 1) / kFThreads;
    if (ranges > by_rows) ranges = by_rows;
    // an odd number of 64-row units per range keeps the range starts off a common power-of-two stride
    int64_t units = ((m + ranges - 1) / ranges + 63) / 64;
    units |= 1;
    const int64_t rows_per_range = units * 64;
    ranges = (m + rows_per_range - 1) / rows_per_range;      // every remaining range holds at least one row
    const int64_t ranges_padded = (ranges + 7) / 8 * 8;
    const size_t need = (size_t)ranges * K * (window + 1) * sizeof(double);
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
    double* part = (double*)ctx->acc_blob;
    const dim3 grid((unsigned)(ranges_padded * nslabs));
    auto kern = idx ? accumulate_f64_kernel<true> : accumulate_f64_kernel<false>;
    if (int rc = check_hip(ctx,
                           hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFLdsBytes),
                           "raising the dynamic LDS limit"))
        return rc;
    for (int f0 = 0; f0 < D; f0 += window) {
        const int dw = (D - f0 < window) ? D - f0 : window;
        const size_t lds = (size_t)ks * (dw + 1) * sizeof(double);
        hipLaunchKernelGGL(kern, grid, dim3(kFThreads), lds, ctx->stream, X + f0, dw, ldx, idx, m, bmu, K, ks, nslabs,
                           rows_per_range, part);
        if (int rc = check_hip(ctx, hipGetLastError(), "accumulate (float64 LDS) launch")) return rc;
        const int cells = K * (dw + 1);
        hipLaunchKernelGGL(accumulate_f64_reduce_kernel, dim3((cells + 63) / 64), dim3(256), 0, ctx->stream, part, K, dw,
                           (int)ranges, zero_first ? 1 : 0, S + f0, D, (f0 == 0) ? n : (unsigned long long*)nullptr);
        if (int rc = check_hip(ctx, hipGetLastError(), "accumulate (float64 LDS) reduce launch")) return rc;
    }
    return SOM_OK;
}

} // namespace som
