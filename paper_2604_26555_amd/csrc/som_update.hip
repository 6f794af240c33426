// Neighbourhood-weighted batch update in float64 (the normalised update U_j / H_j after Eq. 4, with the
// per-sample sums of Eq. 3 grouped by best-matching unit):
//     Num_j = sum_k h(G[k][j]) S_k,   Den_j = sum_k h(G[k][j]) n_k,   h(g) = exp(-g^2 / (2 sigma^2)),
//     w_j <- Num_j / Den_j  where Den_j >= eps_h, otherwise w_j stays.
// Three small launches, all latency-bound at K ~ 1000, so each is shaped for many independent workgroups:
//   1. influence_kernel    h[k][j] for all K x K pairs, one exp per thread (K^2 threads);
//   2. contract_kernel     partial Num / Den over an eighth of the k range per workgroup (split-k keeps several
//                          workgroups per compute unit in flight; partials are stored, not atomically added);
//   3. finish_kernel       adds the partials in a fixed order, applies the threshold, writes W, counts.
// The contraction is 2 K^2 (D + 1) float64 flops (0.1 GFLOP at K = 1024, D = 50): microseconds on the vector
// ALUs, so it stays a plain FMA loop.
#include "som_internal.hpp"

#include <math.h>

namespace som {

constexpr int kTJ = 4;       // updated nodes per workgroup (one wavefront each)
constexpr int kKC = 32;      // contributing nodes staged per step (two LDS buffers of kKC x 64 doubles)
constexpr int kSplitK = 8;   // workgroups sharing one block of updated nodes

__global__ void __launch_bounds__(256) influence_kernel(const float* __restrict__ G, int K, double inv2s2,
                                                        double* __restrict__ H)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)K * K) return;
    const double gd = (double)G[e];
    H[e] = isinf(gd) ? 0.0 : exp(-(gd * gd) * inv2s2);
}

// grid (K / kTJ, ceil(D / 64), kSplitK); thread = (node jj = tid / 64, feature dl = tid % 64)
__global__ void __launch_bounds__(kTJ * 64) contract_kernel(const double* __restrict__ H, const double* __restrict__ S,
                                                            const unsigned long long* __restrict__ n, int K, int D,
                                                            double* __restrict__ part)
{
    __shared__ double hs[2][kKC][kTJ];
    __shared__ double ns[2][kKC];
    __shared__ double Ss[2][kKC][64];
    const int tid = threadIdx.x;
    const int jj = tid >> 6, dl = tid & 63;
    const int j0 = blockIdx.x * kTJ;
    const int d0 = blockIdx.y * 64;
    const int kper = ((K + kSplitK * kKC - 1) / (kSplitK * kKC)) * kKC;
    const int k_lo = blockIdx.z * kper;
    const int k_hi = (k_lo + kper < K) ? k_lo + kper : K;
    constexpr int SLOADS = kKC * 64 / (kTJ * 64);
    double num = 0.0, den = 0.0;
    double pre_s[SLOADS], pre_h = 0.0, pre_n = 0.0;

    auto fetch = [&](int kc) {
#pragma unroll
        for (int p = 0; p < SLOADS; ++p) {
            const int e = tid + p * kTJ * 64;
            const int kk = e >> 6, f = e & 63;
            const int k = kc + kk;
            pre_s[p] = (k < k_hi && d0 + f < D) ? S[(size_t)k * D + d0 + f] : 0.0;
        }
        const int kk = tid / kTJ, q = tid % kTJ;      // the first kKC * kTJ threads bring the influences
        const int k = kc + kk;
        const bool mine = kk < kKC && k < k_hi;
        pre_h = (mine && j0 + q < K) ? H[(size_t)k * K + j0 + q] : 0.0;
        pre_n = (mine && q == 0) ? (double)n[k] : 0.0;
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int p = 0; p < SLOADS; ++p) {
            const int e = tid + p * kTJ * 64;
            Ss[buf][e >> 6][e & 63] = pre_s[p];
        }
        if (tid < kKC * kTJ) {
            hs[buf][tid / kTJ][tid % kTJ] = pre_h;
            if (tid % kTJ == 0) ns[buf][tid / kTJ] = pre_n;
        }
    };

    if (k_lo < k_hi) {
        fetch(k_lo);
        stash(0);
    }
    __syncthreads();
    int buf = 0;
    for (int kc = k_lo; kc < k_hi; kc += kKC, buf ^= 1) {
        const bool more = kc + kKC < k_hi;
        if (more) fetch(kc + kKC);
#pragma unroll 8
        for (int kk = 0; kk < kKC; ++kk) {
            const double h = hs[buf][kk][jj];
            num = fma(h, Ss[buf][kk][dl], num);
            den = fma(h, ns[buf][kk], den);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    }
    const int j = j0 + jj, d = d0 + dl;
    if (j < K) {
        double* row = part + ((size_t)blockIdx.z * K + j) * (D + 1);
        if (d < D) row[d] = num;
        if (dl == 0 && blockIdx.y == 0) row[D] = den;
    }
}

// plain = true: w <- Num / Den (eta = 1, no momentum);  otherwise delta = eta (Num / Den - w) + mu v, w += delta
__global__ void __launch_bounds__(256) finish_kernel(const double* __restrict__ part,
                                                     const unsigned long long* __restrict__ n, int K, int D,
                                                     double eps_h, bool plain, double eta, double mu,
                                                     float* __restrict__ V, float* __restrict__ W,
                                                     int32_t* __restrict__ small)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= K * D) return;
    const int j = e / D, d = e % D;
    const size_t stride = (size_t)K * (D + 1);
    const double* row = part + (size_t)j * (D + 1);
    double num = 0.0, den = 0.0;
#pragma unroll
    for (int z = 0; z < kSplitK; ++z) {
        num += row[z * stride + d];
        den += row[z * stride + D];
    }
    const bool ok = den >= eps_h;
    if (plain) {
        if (ok) W[e] = (float)(num / den);
    } else {
        const double w = (double)W[e];
        const double delta = (ok ? eta * (num / den - w) : 0.0) + (V ? mu * (double)V[e] : 0.0);
        W[e] = (float)(w + delta);
        if (V) V[e] = (float)delta;
    }
    if (d == 0 && small) {
        if (!ok) atomicAdd(&small[0], 1);
        if (n[j] == 0ull) atomicAdd(&small[1], 1);
    }
}

int update_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K, int32_t D,
               double sigma, double eps_h, float* W, int32_t* small)
{
    const size_t h_elems = (size_t)K * K;
    const size_t need = (h_elems + (size_t)kSplitK * K * (D + 1)) * sizeof(double);
    if (need > ctx->upd_bytes) {
        if (ctx->upd_blob) {
            if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
            (void)hipFree(ctx->upd_blob);
            ctx->upd_blob = nullptr;
            ctx->upd_bytes = 0;
        }
        if (hipMalloc(&ctx->upd_blob, need) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for the update workspace", need);
        }
        ctx->upd_bytes = need;
    }
    double* H = (double*)ctx->upd_blob;
    double* part = H + h_elems;
    const double inv2s2 = 1.0 / (2.0 * sigma * sigma);
    hipLaunchKernelGGL(influence_kernel, dim3((unsigned)((h_elems + 255) / 256)), dim3(256), 0, ctx->stream, G, K, inv2s2, H);
    if (int rc = check_hip(ctx, hipGetLastError(), "influence kernel launch")) return rc;
    dim3 grid((K + kTJ - 1) / kTJ, (D + 63) / 64, kSplitK);
    hipLaunchKernelGGL(contract_kernel, grid, dim3(kTJ * 64), 0, ctx->stream, H, S, n, K, D, part);
    if (int rc = check_hip(ctx, hipGetLastError(), "contraction kernel launch")) return rc;
    const bool plain = ctx->eta == 1.0 && ctx->mu == 0.0;
    hipLaunchKernelGGL(finish_kernel, dim3((K * D + 255) / 256), dim3(256), 0, ctx->stream, part, n, K, D, eps_h, plain,
                       ctx->eta, ctx->mu, ctx->velocity, W, small);
    return check_hip(ctx, hipGetLastError(), "update finish launch");
}

} // namespace som
