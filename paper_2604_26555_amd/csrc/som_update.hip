// Neighbourhood-weighted batch update in float64 (the normalised update U_j / H_j after Eq. 4, with the
// per-sample sums of Eq. 3 grouped by best-matching unit):
//     Num_j = sum_k h(G[k][j]) S_k,   Den_j = sum_k h(G[k][j]) n_k,   h(g) = exp(-g^2 / (2 sigma^2)),
//     w_j <- Num_j / Den_j  where Den_j >= eps_h, otherwise w_j stays.
// One workgroup owns kTJ updated nodes and 64 features; it walks the K contributing nodes in chunks of 64,
// evaluating the influences of the chunk once (one exp per thread) and staging the chunk's rows of S in LDS.
#include "som_internal.hpp"

#include <math.h>

namespace som {

constexpr int kTJ = 4;   // updated nodes per workgroup (one wavefront each)
constexpr int kKC = 64;  // contributing nodes per chunk

__global__ void __launch_bounds__(kTJ * 64) update_kernel(const double* __restrict__ S,
                                                          const unsigned long long* __restrict__ n,
                                                          const float* __restrict__ G, int K, int D, double inv2s2,
                                                          double eps_h, float* __restrict__ W,
                                                          int32_t* __restrict__ small)
{
    __shared__ double hs[kKC][kTJ];
    __shared__ double ns[kKC];
    __shared__ double Ss[kKC][64];
    const int tid = threadIdx.x;
    const int jj = tid >> 6;          // which of the workgroup's nodes
    const int dl = tid & 63;          // feature within the 64-wide slab
    const int j0 = blockIdx.x * kTJ;
    const int d0 = blockIdx.y * 64;
    const int j = j0 + jj;
    const int d = d0 + dl;
    double num = 0.0, den = 0.0;
    for (int kc = 0; kc < K; kc += kKC) {
        // influences of this chunk on the workgroup's nodes: thread -> (k = tid / kTJ, node tid % kTJ)
        {
            const int kk = tid / kTJ, q = tid % kTJ;
            const int k = kc + kk;
            double h = 0.0;
            if (k < K && j0 + q < K) {
                const double gd = (double)G[(size_t)k * K + j0 + q];
                h = isinf(gd) ? 0.0 : exp(-(gd * gd) * inv2s2);
            }
            hs[kk][q] = h;
            if (q == 0) ns[kk] = (k < K) ? (double)n[k] : 0.0;
        }
        for (int e = tid; e < kKC * 64; e += kTJ * 64) {
            const int kk = e >> 6, f = e & 63;
            const int k = kc + kk;
            Ss[kk][f] = (k < K && d0 + f < D) ? S[(size_t)k * D + d0 + f] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < kKC; ++kk) {
            const double h = hs[kk][jj];
            num = fma(h, Ss[kk][dl], num);
            den = fma(h, ns[kk], den);
        }
        __syncthreads();
    }
    if (j < K) {
        const bool ok = den >= eps_h;
        if (ok && d < D) W[(size_t)j * D + d] = (float)(num / den);
        if (dl == 0 && blockIdx.y == 0 && small) {
            if (!ok) atomicAdd(&small[0], 1);
            if (n[j] == 0ull) atomicAdd(&small[1], 1);
        }
    }
}

int update_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K, int32_t D,
               double sigma, double eps_h, float* W, int32_t* small)
{
    const double s = sigma;
    const double inv2s2 = 1.0 / (2.0 * s * s);
    dim3 grid((K + kTJ - 1) / kTJ, (D + 63) / 64);
    hipLaunchKernelGGL(update_kernel, grid, dim3(kTJ * 64), 0, ctx->stream, S, n, G, K, D, inv2s2, eps_h, W, small);
    return check_hip(ctx, hipGetLastError(), "update kernel launch");
}

} // namespace som
