// Neighbourhood-weighted batch update in float64 (the normalised update U_j / H_j after Eq. 4, with the
// per-sample sums of Eq. 3 grouped by best-matching unit):
//     Num_j = sum_k h(G[k][j]) S_k,   Den_j = sum_k h(G[k][j]) n_k,   h(g) = exp(-g^2 / (2 sigma^2)),
//     w_j <- Num_j / Den_j  where Den_j >= eps_h, otherwise w_j stays.
// The contraction Num = H^T S (with n as one more column of S) is a dense K x K . K x (D + 1) product in float64:
// it runs on v_mfma_f64_16x16x4_f64.
//   1. contract_kernel     one wavefront = 16 updated nodes x up to 64 columns x one sixteenth of the k range; for
//                          D + 1 <= 64 the influences h = exp(-G^2 / 2 sigma^2) are computed in the wavefront right
//                          where the MFMA needs them (each one is needed exactly once), otherwise influence_kernel
//                          writes them out first and the wavefronts of the column slabs read them;
//   2. finish_kernel       adds the sixteen partials in a fixed order, applies the threshold, writes W, counts.
#include "som_internal.hpp"

#include <math.h>

#include <mutex>

namespace som {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int kSplitK = 16;  // wavefronts sharing one block of updated nodes (partials are stored, then summed in order)

// shift[j] = min over occupied nodes k of G[k][j]^2 (+inf when there is none): one thread per updated node j
__global__ void __launch_bounds__(256) shift_kernel(const float* __restrict__ G, const unsigned long long* __restrict__ n,
                                                    int K, double* __restrict__ shift)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= K) return;
    double m = INFINITY;
    for (int k = 0; k < K; ++k) {
        const double gd = (double)G[(size_t)k * K + j];
        if (n[k] != 0ull && gd * gd < m) m = gd * gd;
    }
    shift[j] = m;
}

// h = exp(-(g^2 - shift_j) / 2 sigma^2); with a shift only occupied nodes k contribute (their exponent is <= 0)
__device__ __forceinline__ double influence_of(double gd, double inv2s2, double shift_j, bool occupied)
{
    const double e = -(gd * gd - shift_j) * inv2s2;
    return (isinf(gd) || isinf(shift_j) || !occupied) ? 0.0 : exp(e);
}

__global__ void __launch_bounds__(256) influence_kernel(const float* __restrict__ G, int K, double inv2s2,
                                                        const double* __restrict__ shift,
                                                        const unsigned long long* __restrict__ n, double* __restrict__ H)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)K * K) return;
    const int k = (int)(e / K), j = (int)(e % K);
    H[e] = influence_of((double)G[e], inv2s2, shift ? shift[j] : 0.0, !shift || n[k] != 0ull);
}

// grid (ceil(K / 16), ceil((D + 1) / 64), kSplitK / 4), 4 wavefronts per workgroup, one k-split each.
// MFMA operands (16 x 16 x 4, float64): lane l supplies A[i = l % 16][k = l / 16] = h[k][j0 + i] and
// B[k = l / 16][c = l % 16] = S[k][c0 + c] (column D is n); its register r receives row l / 16 + 4 r, column l % 16.
template <bool FUSED>
__global__ void __launch_bounds__(256) contract_kernel(const float* __restrict__ G, const double* __restrict__ H,
                                                       double inv2s2, const double* __restrict__ shift,
                                                       const double* __restrict__ S,
                                                       const unsigned long long* __restrict__ n, int K, int D,
                                                       double* __restrict__ part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int z = blockIdx.z * 4 + wave;
    const int j0 = blockIdx.x * 16, c0 = blockIdx.y * 64;
    const int kper = ((K + kSplitK * 4 - 1) / (kSplitK * 4)) * 4;
    const int k_lo = z * kper;
    const int k_hi = (k_lo + kper < K) ? k_lo + kper : K;
    const int li = lane & 15, lk = lane >> 4;
    const int j = j0 + li;
    doublex4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = doublex4{0.0, 0.0, 0.0, 0.0};
    // Sixteen k-steps at a time: first every load of the batch (one wavefront per SIMD has nothing else to cover a
    // round trip to L2 with), then the sixteen exponentials, then the MFMAs.
    constexpr int kBatch = 16;
    const int jc = j < K ? j : K - 1;
    const double shift_j = (FUSED && shift) ? shift[jc] : 0.0;
    for (int kb = k_lo; kb < k_hi; kb += 4 * kBatch) {
        float gv[kBatch];
        double nv[kBatch], sv[kBatch][4];
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
            const int k = kb + 4 * s + lk;
            const int kc = k < K ? k : K - 1;                 // clamped row: the loads are unconditional
            if (FUSED) gv[s] = G[(size_t)kc * K + jc];
            else nv[s] = H[(size_t)kc * K + jc];              // holds h until it is replaced by n below
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = c0 + 16 * t + li;
                sv[s][t] = (c == D) ? (double)n[kc] : S[(size_t)kc * D + (c < D ? c : D - 1)];
            }
        }
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
            const int k = kb + 4 * s + lk;
            const bool in = k < k_hi && j < K;
            double h;
            if (FUSED) {
                const bool occupied = !shift || n[k < K ? k : K - 1] != 0ull;
                h = in ? influence_of((double)gv[s], inv2s2, shift_j, occupied) : 0.0;
            } else {
                h = in ? nv[s] : 0.0;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = c0 + 16 * t + li;
                const double b = (k < k_hi && c <= D) ? sv[s][t] : 0.0;
                acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(h, b, acc[t], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int c = c0 + 16 * t + li;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int jr = j0 + lk + 4 * r;
            if (jr < K && c <= D) part[((size_t)z * K + jr) * (D + 1) + c] = acc[t][r];
        }
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

// the three launches of one update on the given workspaces: H [K*K] (only when D + 1 > 64), part [kSplitK*K*(D+1)],
// shift [K] (only with the shifted-exponent safeguard)
static int update_launch(som_ctx* ctx, double* H, double* part, double* shift_ws, const double* S,
                         const unsigned long long* n, const float* G, int32_t K, int32_t D, double sigma, double eps_h,
                         float* W, int32_t* small)
{
    const size_t h_elems = (size_t)K * K;
    const double inv2s2 = 1.0 / (2.0 * sigma * sigma);
    const dim3 grid((K + 15) / 16, (D + 1 + 63) / 64, kSplitK / 4);
    double* shift = nullptr;
    if (ctx->safeguard == SOM_SAFEGUARD_SHIFT) {
        shift = shift_ws;
        hipLaunchKernelGGL(shift_kernel, dim3((K + 255) / 256), dim3(256), 0, ctx->stream, G, n, K, shift);
        if (int rc = check_hip(ctx, hipGetLastError(), "exponent shift launch")) return rc;
    }
    if (grid.y == 1) {
        hipLaunchKernelGGL(contract_kernel<true>, grid, dim3(256), 0, ctx->stream, G, (const double*)nullptr, inv2s2,
                           (const double*)shift, S, n, K, D, part);
    } else {
        hipLaunchKernelGGL(influence_kernel, dim3((unsigned)((h_elems + 255) / 256)), dim3(256), 0, ctx->stream, G, K, inv2s2,
                           (const double*)shift, n, H);
        if (int rc = check_hip(ctx, hipGetLastError(), "influence kernel launch")) return rc;
        hipLaunchKernelGGL(contract_kernel<false>, grid, dim3(256), 0, ctx->stream, G, (const double*)H, inv2s2,
                           (const double*)nullptr, S, n, K, D, part);
    }
    if (int rc = check_hip(ctx, hipGetLastError(), "contraction kernel launch")) return rc;
    const bool plain = ctx->eta == 1.0 && ctx->mu == 0.0;
    hipLaunchKernelGGL(finish_kernel, dim3((K * D + 255) / 256), dim3(256), 0, ctx->stream, part, n, K, D, eps_h, plain,
                       ctx->eta, ctx->mu, ctx->velocity, W, small);
    return check_hip(ctx, hipGetLastError(), "update finish launch");
}

int update_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K, int32_t D,
               double sigma, double eps_h, float* W, int32_t* small)
{
    const size_t h_elems = (size_t)K * K;
    const size_t need = (h_elems + (size_t)kSplitK * K * (D + 1) + K) * sizeof(double);
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
    return update_launch(ctx, H, part, part + (size_t)kSplitK * K * (D + 1), S, n, G, K, D, sigma, eps_h, W, small);
}

// ---------------------------------------------------------------------------------------------------------
// The same update for callers that cannot allocate (som_neighborhood_update_static): the split-k partials and the
// exponent shifts live in a fixed device array instead of a grown workspace.  One array per GPU, shared by every
// call on that GPU and holding the last call's contents; every cell a call reads it has written first (the
// contraction writes all kSplitK partials of every node and column, the shift kernel every node), so nothing needs
// clearing.  Host code never uses the array's name as an address: the device address is looked up once per device.
// ---------------------------------------------------------------------------------------------------------
static __device__ __align__(256) double scratch[(size_t)kSplitK * kUpdateStaticCells + kUpdateStaticNodes];

static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices] = {};     // per device: its own copy of the array, at its own address

// called by som_create with the context's device current
int update_static_init(som_ctx* ctx)
{
    if (ctx->device < 0 || ctx->device >= kMaxDevices) return SOM_OK;   // the static entry point reports it when used
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[ctx->device]) {
        void* p = nullptr;
        if (int rc = check_hip(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "looking up the static update workspace")) return rc;
        g_scratch_ptr[ctx->device] = (double*)p;
    }
    ctx->upd_static = g_scratch_ptr[ctx->device];
    return SOM_OK;
}

int update_static_run(som_ctx* ctx, const double* S, const unsigned long long* n, const float* G, int32_t K, int32_t D,
                      double sigma, double eps_h, float* W, int32_t* small)
{
    if (D + 1 > 64 || K > kUpdateStaticNodes || (int64_t)K * (D + 1) > kUpdateStaticCells)
        return fail(ctx, SOM_EINVAL,
                    "som_neighborhood_update_static serves D <= 63, K <= %d and K * (D + 1) <= %d (got K = %d, D = %d)",
                    kUpdateStaticNodes, kUpdateStaticCells, K, D);
    if (!ctx->upd_static) return fail(ctx, SOM_ESTATE, "the static update workspace was not set up on this device");
    double* part = ctx->upd_static;
    return update_launch(ctx, nullptr, part, part + (size_t)kSplitK * kUpdateStaticCells, S, n, G, K, D, sigma, eps_h, W, small);
}

} // namespace som
