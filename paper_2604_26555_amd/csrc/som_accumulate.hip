// Per-BMU sample sums and counts (the inner sums of Eq. 3 grouped by best-matching unit):
//     S_k += x_i,  n_k += 1   for k = b_i.
// The pass is bound by reading X once, so all arithmetic is kept off the memory path: every workgroup owns a
// contiguous range of samples and a slab of `ws` features, adds its samples into a float32 partial
// P[K][ws] held in LDS (LDS atomics, conflict-free within a sample because consecutive lanes take consecutive
// features), and flushes the partial into the float64 global sums with hardware atomics every kFlushRows
// samples, which bounds the length of any float32 summation chain.  Counts are LDS integers flushed likewise.
// The feature slabs of one sample range are given workgroup numbers 8 apart so that they run on the same XCD
// and share the range's cache lines in that XCD's L2.
#include "som_internal.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace som {

constexpr int kAccThreads = 1024;
constexpr int kFlushRows = 16384;
constexpr size_t kAccLdsBudget = 144 * 1024;

__global__ void __launch_bounds__(kAccThreads) accumulate_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                 const uint32_t* __restrict__ idx, int64_t m,
                                                                 const int32_t* __restrict__ bmu, int K, int ws,
                                                                 int nslabs, int64_t rows_per_range,
                                                                 double* __restrict__ S,
                                                                 unsigned long long* __restrict__ n)
{
    extern __shared__ float4 acc_lds4[];
    float* P = reinterpret_cast<float*>(acc_lds4);              // [K][ws]
    unsigned int* C = reinterpret_cast<unsigned int*>(P + (size_t)K * ws); // [K], used by slab 0 only
    const int tid = threadIdx.x;
    // workgroup number -> (range, slab): slabs of a range sit 8 apart inside a block of 8 * nslabs workgroups
    const int blk = blockIdx.x / (8 * nslabs), within = blockIdx.x % (8 * nslabs);
    const int slab = within / 8;
    const int64_t range = (int64_t)blk * 8 + (within % 8);
    const int f0 = slab * ws;
    const int wcur = (D - f0 < ws) ? (D - f0) : ws;              // features in this slab
    const int64_t lo = range * rows_per_range;
    int64_t hi = lo + rows_per_range;
    if (hi > m) hi = m;
    const int cells = K * ws;
    for (int c = tid; c < cells + K; c += kAccThreads) P[c] = 0.0f; // zero bits also clear the counters
    __syncthreads();
    if (lo >= hi || wcur <= 0) return;

    for (int64_t base = lo; base < hi; base += kFlushRows) {
        const int64_t top = (base + kFlushRows < hi) ? base + kFlushRows : hi;
        const int elems = (int)(top - base) * wcur;   // at most kFlushRows * ws, far below 2^31
        for (int e0 = 0; e0 < elems; e0 += kAccThreads * 8) {
            float v[8];
            int cell[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * kAccThreads + tid;
                cell[u] = -1;
                v[u] = 0.f;
                if (e < elems) {
                    const int64_t i = base + e / wcur;
                    const int f = e % wcur;
                    const int b = bmu[i];
                    if (b >= 0 && b < K) {
                        const int64_t r = idx ? (int64_t)idx[i] : i;
                        v[u] = X[r * ldx + f0 + f];
                        cell[u] = b * ws + f;
                        if (slab == 0 && f == 0) atomicAdd(&C[b], 1u);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (cell[u] >= 0) unsafeAtomicAdd(&P[cell[u]], v[u]);
        }
        __syncthreads();
        for (int c = tid; c < K * wcur; c += kAccThreads) {
            const int k = c / wcur, f = c % wcur;
            const float p = P[k * ws + f];
            if (p != 0.0f) {
                unsafeAtomicAdd(&S[(size_t)k * D + f0 + f], (double)p);
                P[k * ws + f] = 0.0f;
            }
        }
        if (slab == 0) {
            for (int k = tid; k < K; k += kAccThreads) {
                const unsigned int c = C[k];
                if (c) {
                    atomicAdd(&n[k], (unsigned long long)c);
                    C[k] = 0u;
                }
            }
        }
        __syncthreads();
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
                   const int32_t* bmu, int32_t K, double* S, unsigned long long* n)
{
    if (m <= 0) return SOM_OK;
    // widest feature slab whose float32 partial (plus the counters) fits the LDS budget
    const size_t per_feature = (size_t)K * sizeof(float);
    const size_t room = kAccLdsBudget > (size_t)K * 4 ? kAccLdsBudget - (size_t)K * 4 : 0;
    int ws = (int)(room / per_feature);
    if (ws < 1) {
        int blocks = (int)((m + 3) / 4 < 4096 ? (m + 3) / 4 : 4096);
        hipLaunchKernelGGL(accumulate_direct_kernel, dim3(blocks), dim3(256), 0, ctx->stream, X, D, ldx, idx, m, bmu, K,
                           S, n);
        return check_hip(ctx, hipGetLastError(), "accumulate (direct) launch");
    }
    if (ws > D) ws = D;
    const int nslabs = (D + ws - 1) / ws;
    ws = (D + nslabs - 1) / nslabs; // balance the slabs
    const size_t lds_bytes = ((size_t)K * ws + K) * sizeof(float);
    static size_t attr_bytes = 0;
    if (lds_bytes > attr_bytes) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(accumulate_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLdsBudget),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_bytes = kAccLdsBudget;
    }
    // one workgroup per compute unit: ranges = 256 / nslabs, at least 2048 rows each, in multiples of 8 ranges
    int64_t ranges = 256 / nslabs;
    const int64_t by_rows = (m + 2047) / 2048;
    if (ranges > by_rows) ranges = by_rows;
    if (ranges < 1) ranges = 1;
    ranges = ((ranges + 7) / 8) * 8;
    const int64_t rows_per_range = (m + ranges - 1) / ranges;
    hipLaunchKernelGGL(accumulate_kernel, dim3((unsigned)(ranges * nslabs)), dim3(kAccThreads), lds_bytes, ctx->stream,
                       X, D, ldx, idx, m, bmu, K, ws, nslabs, rows_per_range, S, n);
    return check_hip(ctx, hipGetLastError(), "accumulate launch");
}

} // namespace som
