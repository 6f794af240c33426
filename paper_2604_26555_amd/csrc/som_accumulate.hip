// Per-BMU sample sums and counts (the inner sums of Eq. 3 grouped by best-matching unit):
//     S_k += x_i,  n_k += 1   for k = b_i.
// The pass is bound by reading X once.  Global floating-point atomics serialise in the memory system, so every
// workgroup owns a contiguous range of samples and a slab of `ws` features, adds its samples into a float32
// partial P[K][ws] held in LDS (LDS atomics; consecutive lanes take consecutive features of a sample, so a
// sample's lanes never collide), and moves the partial into its own slice of a global workspace every kFlushRows
// samples, which bounds the length of any float32 summation chain.  A second kernel then adds the slices in a
// fixed order into S.  The feature slabs of one sample range are given workgroup numbers 8 apart so that they
// run on the same XCD and share the range's cache lines in that XCD's L2.
#include "som_internal.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace som {

constexpr int kAccThreads = 1024;
constexpr int kAccUnroll = 16;
constexpr int kFlushRows = 16384;
constexpr size_t kAccLdsBytes = 144 * 1024;

// LDS bytes for a K-node map with ws features per slab: partial + counters
static inline size_t acc_lds_bytes(int K, int ws) { return ((size_t)K * ws + K) * 4; }

// SliceT = float when a range is flushed once (its float32 chain is at most kFlushRows long), double otherwise.
template <typename SliceT>
__global__ void __launch_bounds__(kAccThreads) accumulate_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                 const uint32_t* __restrict__ idx, int64_t m,
                                                                 const int32_t* __restrict__ bmu, int K, int ws,
                                                                 int nslabs, int64_t rows_per_range,
                                                                 SliceT* __restrict__ part_S,
                                                                 unsigned int* __restrict__ part_n)
{
    extern __shared__ float4 acc_lds4[];
    float* P = reinterpret_cast<float*>(acc_lds4);                          // [K][ws]
    unsigned int* C = reinterpret_cast<unsigned int*>(P + (size_t)K * ws);  // [K], used by slab 0 only
    const int tid = threadIdx.x;
    // workgroup number -> (range, slab): slabs of a range sit 8 apart inside a block of 8 * nslabs workgroups
    const int blk = blockIdx.x / (8 * nslabs), within = blockIdx.x % (8 * nslabs);
    const int slab = within / 8;
    const int64_t range = (int64_t)blk * 8 + (within % 8);
    const int f0 = slab * ws;
    const int wcur = (D - f0 < ws) ? (D - f0) : ws;                          // features in this slab
    const int64_t lo = range * rows_per_range;
    int64_t hi = lo + rows_per_range;
    if (hi > m) hi = m;
    const int cells = K * ws;
    SliceT* myS = part_S + (size_t)blockIdx.x * cells;                       // this workgroup's slice
    unsigned int* myN = part_n + (size_t)range * K;
    for (int c = tid; c < cells + K; c += kAccThreads) P[c] = 0.0f;          // zero bits also clear the counters
    __syncthreads();

    // the (sample, feature) pairs of a flush block are numbered e = s * wcur + f and dealt to the threads in order,
    // so every LDS atomic instruction carries 64 useful lanes; e / wcur is a multiply-high by ceil(2^32 / wcur),
    // exact while e * wcur < 2^32 (e < kFlushRows * wcur, wcur <= 256)
    const unsigned int magic = (unsigned int)((0x100000000ull + (unsigned)wcur - 1) / (unsigned)wcur);

    bool first = true;
    for (int64_t base = lo; base < hi || first; base += kFlushRows) {
        const int64_t top = (base + kFlushRows < hi) ? base + kFlushRows : hi;
        const int elems = (top > base) ? (int)(top - base) * wcur : 0;       // at most kFlushRows * 256 = 2^22
        for (int e0 = 0; e0 < elems; e0 += kAccThreads * kAccUnroll) {
            // all loads of a step are issued back to back: positions are clamped into range, not predicated
            int64_t rows[kAccUnroll];
            int f[kAccUnroll], b[kAccUnroll];
            float v[kAccUnroll];
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                const int e = e0 + u * kAccThreads + tid;
                const unsigned int ec = (unsigned int)(e < elems ? e : elems - 1);
                const unsigned int sidx = __umulhi(ec, magic);
                f[u] = (int)(ec - sidx * (unsigned)wcur);
                rows[u] = base + sidx;
            }
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) b[u] = bmu[rows[u]];
            if (idx) {
#pragma unroll
                for (int u = 0; u < kAccUnroll; ++u) rows[u] = (int64_t)idx[rows[u]];
            }
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) v[u] = X[rows[u] * ldx + f0 + f[u]];
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                const int e = e0 + u * kAccThreads + tid;
                if (e < elems && b[u] >= 0 && b[u] < K) {
                    unsafeAtomicAdd(&P[b[u] * ws + f[u]], v[u]);
                    if (slab == 0 && f[u] == 0) atomicAdd(&C[b[u]], 1u);
                }
            }
        }
        __syncthreads();
        // LDS partial -> this workgroup's slice (first flush stores, later ones add), then clear
        for (int c = tid; c < cells; c += kAccThreads) {
            const float p = P[c];
            if (first)
                myS[c] = (SliceT)p;
            else if (p != 0.0f)
                myS[c] += (SliceT)p;
            P[c] = 0.0f;
        }
        if (slab == 0) {
            for (int k = tid; k < K; k += kAccThreads) {
                const unsigned int c = C[k];
                if (first)
                    myN[k] = c;
                else if (c)
                    myN[k] += c;
                C[k] = 0u;
            }
        }
        first = false;
        __syncthreads();
    }
}

// S[k][f] (+)= sum over ranges of the slices, n[k] (+)= sum over ranges of the counts, always in the same order:
// a workgroup takes 64 cells, its four wavefronts a quarter of the ranges each, then the quarters are added 0..3.
template <typename SliceT>
__global__ void __launch_bounds__(256) accumulate_reduce_kernel(const SliceT* __restrict__ part_S,
                                                                const unsigned int* __restrict__ part_n, int K, int D,
                                                                int ws, int nslabs, int ranges, int zero_first,
                                                                double* __restrict__ S,
                                                                unsigned long long* __restrict__ n)
{
    __shared__ double qsum[4][64];
    __shared__ unsigned long long qcnt[4][64];
    const int q = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);   // cell of S, then the K counters
    const int cells = K * ws;
    const int per = (ranges + 3) / 4;
    const int r_lo = q * per, r_hi = (r_lo + per < ranges) ? r_lo + per : ranges;
    double s = 0.0;
    unsigned long long t = 0ull;
    if (c < K * D) {
        const int k = c / D, f = c % D;
        const int slab = f / ws, fl = f - slab * ws;
        const size_t off = (size_t)k * ws + fl;
#pragma unroll 8
        for (int r = r_lo; r < r_hi; ++r) {
            const int wg = (r / 8) * (8 * nslabs) + slab * 8 + (r % 8);
            s += (double)part_S[(size_t)wg * cells + off];
        }
    } else if (c < K * D + K) {
        const int k = c - K * D;
#pragma unroll 8
        for (int r = r_lo; r < r_hi; ++r) t += part_n[(size_t)r * K + k];
    }
    qsum[q][threadIdx.x & 63] = s;
    qcnt[q][threadIdx.x & 63] = t;
    __syncthreads();
    if (q == 0) {
        const int l = threadIdx.x;
        if (c < K * D) {
            const double tot = ((qsum[0][l] + qsum[1][l]) + qsum[2][l]) + qsum[3][l];
            S[c] = (zero_first ? 0.0 : S[c]) + tot;
        } else if (c < K * D + K) {
            const int k = c - K * D;
            n[k] = (zero_first ? 0ull : n[k]) + qcnt[0][l] + qcnt[1][l] + qcnt[2][l] + qcnt[3][l];
        }
    }
}

// Fallback for maps whose partial does not fit LDS: one wavefront per sample, straight to the global sums.
__global__ void __launch_bounds__(256) accumulate_direct_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                const uint32_t* __restrict__ idx, int64_t m,
                                                                const int32_t* __restrict__ bmu, int K,
                                                                double* __restrict__ S,
                                                                unsigned long long* __restrict__ n)
{
    const int lane = threadIdx.x & 63;
    const int64_t nw = (int64_t)gridDim.x * 4;
    for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < m; i += nw) {
        const int b = bmu[i];
        if (b < 0 || b >= K) continue;
        const int64_t r = idx ? (int64_t)idx[i] : i;
        for (int f = lane; f < D; f += 64) unsafeAtomicAdd(&S[(size_t)b * D + f], (double)X[r * ldx + f]);
        if (lane == 0) atomicAdd(&n[b], 1ull);
    }
}

int accumulate_run(som_ctx* ctx, const float* X, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                   const int32_t* bmu, int32_t K, double* S, unsigned long long* n, bool zero_first)
{
    // fixed-order sums in MFMA accumulators when asked for (and the shape fits one workgroup's registers)
    if (ctx->reproducible) {
        const int rc = accumulate_mfma_run(ctx, X, D, ldx, idx, m, bmu, K, S, n, zero_first);
        if (rc != 1) return rc;
    }
    // float64 LDS atomics over node slabs when the K x 64 partial fits a few slabs
    {
        const int rc = accumulate_f64_run(ctx, X, D, ldx, idx, m, bmu, K, S, n, zero_first);
        if (rc != 1) return rc;
    }
    if (!ctx->reproducible) {
        const int rc = accumulate_mfma_run(ctx, X, D, ldx, idx, m, bmu, K, S, n, zero_first);
        if (rc != 1) return rc;
    }
    // widest feature slab whose LDS footprint fits
    int ws = D < 256 ? D : 256;   // the kernel's multiply-high division is exact for slabs up to 512 wide
    while (ws >= 1 && acc_lds_bytes(K, ws) > kAccLdsBytes) --ws;
    if (ws < 1) {
        if (zero_first) {
            if (int rc = launch_fill_zero(ctx, S, (size_t)K * D * sizeof(double))) return rc;
            if (int rc = launch_fill_zero(ctx, n, (size_t)K * sizeof(unsigned long long))) return rc;
        }
        if (m <= 0) return SOM_OK;
        int blocks = (int)((m + 3) / 4 < 4096 ? (m + 3) / 4 : 4096);
        hipLaunchKernelGGL(accumulate_direct_kernel, dim3(blocks), dim3(256), 0, ctx->stream, X, D, ldx, idx, m, bmu, K,
                           S, n);
        return check_hip(ctx, hipGetLastError(), "accumulate (direct) launch");
    }
    if (m <= 0) {
        if (!zero_first) return SOM_OK;
        if (int rc = launch_fill_zero(ctx, S, (size_t)K * D * sizeof(double))) return rc;
        return launch_fill_zero(ctx, n, (size_t)K * sizeof(unsigned long long));
    }
    const int nslabs = (D + ws - 1) / ws;
    ws = (D + nslabs - 1) / nslabs; // balance the slabs
    const size_t lds_bytes = acc_lds_bytes(K, ws);
    // one workgroup per compute unit: ranges = 256 / nslabs, at least 2048 rows each, in multiples of 8 ranges
    int64_t ranges = 256 / nslabs;
    const int64_t by_rows = (m + 2047) / 2048;
    if (ranges > by_rows) ranges = by_rows;
    if (ranges < 1) ranges = 1;
    ranges = ((ranges + 7) / 8) * 8;
    const int64_t rows_per_range = (m + ranges - 1) / ranges;
    const bool single_flush = rows_per_range <= kFlushRows;
    const size_t slice_elem = single_flush ? sizeof(float) : sizeof(double);
    const size_t groups = (size_t)ranges * nslabs;
    const size_t slices_bytes = ((groups * (size_t)K * ws * slice_elem) + 255) & ~(size_t)255;
    const size_t need = slices_bytes + (size_t)ranges * K * sizeof(unsigned int);
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
    unsigned int* part_n = (unsigned int*)((char*)ctx->acc_blob + slices_bytes);
    const int total = K * D + K;
    const dim3 rgrid((total + 63) / 64), grid((unsigned)groups);
    static bool attr_set_dev[kMaxDevices][2] = {};    // the attribute belongs to the device, not to the process
    bool* attr_set = attr_set_dev[ctx->device];
    auto launch = [&](auto kern, auto* part_S, int slot) -> int {
        if (!attr_set[slot]) {
            if (int rc = check_hip(ctx,
                                   hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLdsBytes),
                                   "raising the dynamic LDS limit"))
                return rc;
            attr_set[slot] = true;
        }
        hipLaunchKernelGGL(kern, grid, dim3(kAccThreads), lds_bytes, ctx->stream, X, D, ldx, idx, m, bmu, K, ws, nslabs,
                           rows_per_range, part_S, part_n);
        return check_hip(ctx, hipGetLastError(), "accumulate launch");
    };
    if (single_flush) {
        float* part_S = (float*)ctx->acc_blob;
        if (int rc = launch(accumulate_kernel<float>, part_S, 0)) return rc;
        hipLaunchKernelGGL(accumulate_reduce_kernel<float>, rgrid, dim3(256), 0, ctx->stream, part_S, part_n, K, D, ws,
                           nslabs, (int)ranges, zero_first ? 1 : 0, S, n);
    } else {
        double* part_S = (double*)ctx->acc_blob;
        if (int rc = launch(accumulate_kernel<double>, part_S, 1)) return rc;
        hipLaunchKernelGGL(accumulate_reduce_kernel<double>, rgrid, dim3(256), 0, ctx->stream, part_S, part_n, K, D, ws,
                           nslabs, (int)ranges, zero_first ? 1 : 0, S, n);
    }
    return check_hip(ctx, hipGetLastError(), "accumulate reduce launch");
}

} // namespace som
