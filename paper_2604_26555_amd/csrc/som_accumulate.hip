// Per-BMU sample sums and counts (the inner sums of Eq. 3 grouped by best-matching unit):
//     S_k += x_i,  n_k += 1   for k = b_i.
// The pass is bound by reading X once, so the arithmetic is kept off the memory path and no global atomics are
// used (they serialise in the memory system).  Every workgroup owns a contiguous range of samples and a slab of
// `ws` features.  It adds its samples into a float32 partial P[K][ws] held in LDS (LDS atomics; consecutive lanes
// take consecutive features of a sample, so a sample's lanes never collide) and moves the partial into its own
// float64 slice of a global workspace every kFlushRows samples, which bounds the length of any float32
// summation chain.  A second kernel then adds the slices in a fixed order into S: the result does not depend on
// scheduling.  The feature slabs of one sample range are given workgroup numbers 8 apart so that they run on the
// same XCD and share the range's cache lines in that XCD's L2.
#include "som_internal.hpp"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace som {

constexpr int kAccThreads = 1024;
constexpr int kAccUnroll = 8;
constexpr int kFlushRows = 16384;
constexpr size_t kAccLdsBudget = 144 * 1024;

__global__ void __launch_bounds__(kAccThreads) accumulate_kernel(const float* __restrict__ X, int D, int64_t ldx,
                                                                 const uint32_t* __restrict__ idx, int64_t m,
                                                                 const int32_t* __restrict__ bmu, int K, int ws,
                                                                 int nslabs, int64_t rows_per_range,
                                                                 double* __restrict__ part_S,
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
    double* myS = part_S + (size_t)blockIdx.x * cells;                       // this workgroup's float64 slice
    unsigned int* myN = part_n + (size_t)range * K;
    for (int c = tid; c < cells + K; c += kAccThreads) P[c] = 0.0f;          // zero bits also clear the counters
    __syncthreads();

    bool first = true;
    for (int64_t base = lo; base < hi || first; base += kFlushRows) {
        const int64_t top = (base + kFlushRows < hi) ? base + kFlushRows : hi;
        const int elems = (top > base) ? (int)(top - base) * wcur : 0;       // at most kFlushRows * ws
        for (int e0 = 0; e0 < elems; e0 += kAccThreads * kAccUnroll) {
            float v[kAccUnroll];
            int b[kAccUnroll], f[kAccUnroll];
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                const int e = e0 + u * kAccThreads + tid;
                const int ec = e < elems ? e : elems - 1;                    // clamped: loads stay unconditional
                const int s = ec / wcur;
                f[u] = ec - s * wcur;
                const int64_t i = base + s;
                const int64_t r = idx ? (int64_t)idx[i] : i;
                b[u] = bmu[i];
                v[u] = X[r * ldx + f0 + f[u]];
                if (e >= elems) b[u] = -1;
            }
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                if (b[u] >= 0 && b[u] < K) {
                    unsafeAtomicAdd(&P[b[u] * ws + f[u]], v[u]);
                    if (slab == 0 && f[u] == 0) atomicAdd(&C[b[u]], 1u);
                }
            }
        }
        __syncthreads();
        // LDS partial -> this workgroup's float64 slice (first flush stores, later ones add), then clear
        for (int c = tid; c < cells; c += kAccThreads) {
            const float p = P[c];
            if (first)
                myS[c] = (double)p;
            else if (p != 0.0f)
                myS[c] += (double)p;
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

// S[k][f] (+)= sum over ranges of the slices, n[k] (+)= sum over ranges of the counts; fixed order
__global__ void __launch_bounds__(256) accumulate_reduce_kernel(const double* __restrict__ part_S,
                                                                const unsigned int* __restrict__ part_n, int K, int D,
                                                                int ws, int nslabs, int ranges, int zero_first,
                                                                double* __restrict__ S,
                                                                unsigned long long* __restrict__ n)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;   // cell of S, then the K counters
    const int cells = K * ws;
    if (c < K * D) {
        const int k = c / D, f = c % D;
        const int slab = f / ws, fl = f - slab * ws;
        double s = zero_first ? 0.0 : S[c];
        for (int r = 0; r < ranges; ++r) {
            const int wg = (r / 8) * (8 * nslabs) + slab * 8 + (r % 8);
            s += part_S[(size_t)wg * cells + (size_t)k * ws + fl];
        }
        S[c] = s;
    } else if (c < K * D + K) {
        const int k = c - K * D;
        unsigned long long t = zero_first ? 0ull : n[k];
        for (int r = 0; r < ranges; ++r) t += part_n[(size_t)r * K + k];
        n[k] = t;
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
    // widest feature slab whose float32 partial (plus the counters) fits the LDS budget
    const size_t per_feature = (size_t)K * sizeof(float);
    const size_t room = kAccLdsBudget > (size_t)K * 4 ? kAccLdsBudget - (size_t)K * 4 : 0;
    int ws = (int)(room / per_feature);
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
    if (ws > D) ws = D;
    const int nslabs = (D + ws - 1) / ws;
    ws = (D + nslabs - 1) / nslabs; // balance the slabs
    const size_t lds_bytes = ((size_t)K * ws + K) * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        if (int rc = check_hip(ctx,
                               hipFuncSetAttribute(reinterpret_cast<const void*>(accumulate_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLdsBudget),
                               "raising the dynamic LDS limit"))
            return rc;
        attr_set = true;
    }
    // one workgroup per compute unit: ranges = 256 / nslabs, at least 2048 rows each, in multiples of 8 ranges
    int64_t ranges = 256 / nslabs;
    const int64_t by_rows = (m + 2047) / 2048;
    if (ranges > by_rows) ranges = by_rows;
    if (ranges < 1) ranges = 1;
    ranges = ((ranges + 7) / 8) * 8;
    const int64_t rows_per_range = (m + ranges - 1) / ranges;
    const size_t groups = (size_t)ranges * nslabs;
    const size_t need = groups * (size_t)K * ws * sizeof(double) + (size_t)ranges * K * sizeof(unsigned int);
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
    double* part_S = (double*)ctx->acc_blob;
    unsigned int* part_n = (unsigned int*)((char*)ctx->acc_blob + groups * (size_t)K * ws * sizeof(double));
    hipLaunchKernelGGL(accumulate_kernel, dim3((unsigned)groups), dim3(kAccThreads), lds_bytes, ctx->stream, X, D, ldx,
                       idx, m, bmu, K, ws, nslabs, rows_per_range, part_S, part_n);
    if (int rc = check_hip(ctx, hipGetLastError(), "accumulate launch")) return rc;
    const int total = K * D + K;
    hipLaunchKernelGGL(accumulate_reduce_kernel, dim3((total + 255) / 256), dim3(256), 0, ctx->stream, part_S, part_n, K,
                       D, ws, nslabs, (int)ranges, zero_first ? 1 : 0, S, n);
    return check_hip(ctx, hipGetLastError(), "accumulate reduce launch");
}

} // namespace som
