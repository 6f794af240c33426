// Measurement support: one v_mfma_f32_32x32x16_bf16 per problem, exactly the instruction whose accumulation error
// the rounding bound of the default BMU search counts (som_bmu.hip, bmu_split_tile).  Operands go in and come out
// as plain row-major matrices so that a caller can compare the pipe's result with the exact sum.
#include "som_internal.hpp"

namespace som {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// A: [n][32][16] (row i, k) and Bt: [n][32][16] (column j, k) as bf16 bit patterns; C, Dout: [n][32][32] float32.
// One wavefront per problem.  Lane (j, g) feeds k = 8 g .. 8 g + 7 of row j of A and of column j of B, as the
// search does; accumulator register r of lane (j, g) is row 8 (r / 4) + 4 g + r % 4, column j.
__global__ void __launch_bounds__(256) mfma_probe_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Bt,
                                                        const float* __restrict__ C, float* __restrict__ Dout, int64_t n)
{
    const int lane = threadIdx.x & 63, j = lane & 31, g = lane >> 5;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n) return;
    const uint4 ar = *reinterpret_cast<const uint4*>(A + (size_t)t * 512 + j * 16 + 8 * g);
    const uint4 br = *reinterpret_cast<const uint4*>(Bt + (size_t)t * 512 + j * 16 + 8 * g);
    bf16x8 av, bv;
    __builtin_memcpy(&av, &ar, 16);
    __builtin_memcpy(&bv, &br, 16);
    const float* c = C + (size_t)t * 1024;
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r >> 2) + 4 * g + (r & 3)) * 32 + j];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
    float* d = Dout + (size_t)t * 1024;
#pragma unroll
    for (int r = 0; r < 16; ++r) d[(8 * (r >> 2) + 4 * g + (r & 3)) * 32 + j] = acc[r];
}

// Plain streaming read of a buffer (16-byte loads, one contiguous range per workgroup): what the memory system delivers
// to a kernel that does nothing else, the yardstick for the HBM-bound accumulation pass.
__global__ void __launch_bounds__(256) read_probe_kernel(const float4* __restrict__ p, size_t n4, float* __restrict__ out)
{
    float acc = 0.f;
    const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * blockIdx.x, hi = lo + per < n4 ? lo + per : n4;
    size_t i = lo + threadIdx.x;
    for (; i + 7 * 256 < hi; i += 8 * 256) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[i + u * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    for (; i < hi; i += 256) {
        const float4 v = p[i];
        acc += (v.x + v.y) + (v.z + v.w);
    }
    // (the sum is only there to keep the loads; one lane in a million ever stores it)
    if (acc == 12345.6789f) out[0] = acc;
}

// Sustained rate of v_mfma_f32_32x32x16_bf16 on pseudo-random operands, with FOLD fold steps (three vector instructions
// each: and-or, med3, max, on registers no MFMA in flight writes) beside every MFMA: eight MFMAs on two accumulators
// per loop trip.  Run for a second or more it shows the rate the chip holds under its power limit, which is what
// bounds the BMU search (random data draws far more power in the matrix pipe than zeros do).
#define SOM_FOLD1 "v_and_or_b32 %2, %7, %8, 5\nv_med3_f32 %3, %4, %3, %2\nv_max_f32 %4, %4, %2\n"
#define SOM_PAIR(VS) "v_mfma_f32_32x32x16_bf16 %0, %5, %6, %0\n" VS "v_mfma_f32_32x32x16_bf16 %1, %5, %6, %1\n" VS
template <int FOLD>
__global__ void __launch_bounds__(256) mfma_rate_kernel(int iters, unsigned seed, float* __restrict__ sink)
{
    // operands: uniform in [-1, 1) from a per-lane linear congruential sequence
    unsigned st = seed * 747796405u + (blockIdx.x * 256u + threadIdx.x) * 2891336453u + 1u;
    auto next = [&]() {
        st = st * 1664525u + 1013904223u;
        return (float)(int)st * 4.6566129e-10f;
    };
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)next();
        b[i] = (__bf16)next();
    }
    floatx16 c0 = {}, c1 = {};
    float t = 0.f, second = next(), best = next(), src = next();
    const unsigned mask = 0xfffffff0u;
    for (int it = 0; it < iters; ++it) {
        if (FOLD == 0)
            asm volatile(SOM_PAIR("") SOM_PAIR("") SOM_PAIR("") SOM_PAIR("")
                         : "+v"(c0), "+v"(c1), "+v"(t), "+v"(second), "+v"(best)
                         : "v"(a), "v"(b), "v"(src), "s"(mask));
        if (FOLD == 1)
            asm volatile(SOM_PAIR(SOM_FOLD1) SOM_PAIR(SOM_FOLD1) SOM_PAIR(SOM_FOLD1) SOM_PAIR(SOM_FOLD1)
                         : "+v"(c0), "+v"(c1), "+v"(t), "+v"(second), "+v"(best)
                         : "v"(a), "v"(b), "v"(src), "s"(mask));
        if (FOLD == 2)
            asm volatile(SOM_PAIR(SOM_FOLD1 SOM_FOLD1) SOM_PAIR(SOM_FOLD1 SOM_FOLD1) SOM_PAIR(SOM_FOLD1 SOM_FOLD1)
                             SOM_PAIR(SOM_FOLD1 SOM_FOLD1)
                         : "+v"(c0), "+v"(c1), "+v"(t), "+v"(second), "+v"(best)
                         : "v"(a), "v"(b), "v"(src), "s"(mask));
    }
    const float r = c0[0] + c1[3] + t + second + best;
    if (r == 12345.6789f) sink[0] = r;           // keeps the loop; practically never stores
}
#undef SOM_PAIR
#undef SOM_FOLD1

} // namespace som

using namespace som;

extern "C" int som_mfma_rate_probe(som_ctx* ctx, int fold_steps, int waves_per_simd, int iters)
{
    if (!ctx) return SOM_EINVAL;
    if (fold_steps < 0 || fold_steps > 2 || waves_per_simd < 1 || waves_per_simd > 2 || iters < 1 || iters > (1 << 24))
        return fail(ctx, SOM_EINVAL, "fold_steps in 0..2, waves_per_simd in 1..2, iters in 1..2^24");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    if (ctx->units == 0) {
        int units = 0;
        if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess || units < 1) units = 256;
        ctx->units = units;
    }
    const dim3 grid((unsigned)(ctx->units * waves_per_simd));
    auto kern = fold_steps == 0 ? mfma_rate_kernel<0> : fold_steps == 1 ? mfma_rate_kernel<1> : mfma_rate_kernel<2>;
    hipLaunchKernelGGL(kern, grid, dim3(256), 0, ctx->stream, iters, 12345u, (float*)ctx->small);
    return check_hip(ctx, hipGetLastError(), "launching the MFMA rate probe");
}

extern "C" int som_read_probe(som_ctx* ctx, const void* p, int64_t bytes)
{
    if (!ctx) return SOM_EINVAL;
    if (bytes < 0 || (bytes > 0 && !p)) return fail(ctx, SOM_EINVAL, "bad buffer");
    if (((uintptr_t)p & 15) || (bytes & 15)) return fail(ctx, SOM_EINVAL, "buffer and size must be multiples of 16 bytes");
    if (bytes == 0) return SOM_OK;
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    hipLaunchKernelGGL(read_probe_kernel, dim3(4096), dim3(256), 0, ctx->stream, (const float4*)p, (size_t)bytes / 16,
                       (float*)ctx->small);
    return check_hip(ctx, hipGetLastError(), "launching the read probe");
}

extern "C" int som_matrix_pipe_probe(som_ctx* ctx, const uint16_t* A, const uint16_t* Bt, const float* C, float* Dout, int64_t n)
{
    if (!ctx) return SOM_EINVAL;
    if (n < 0 || n > ((int64_t)1 << 24)) return fail(ctx, SOM_EINVAL, "n must be in [0, 2^24]");
    if (n == 0) return SOM_OK;
    if (!A || !Bt || !C || !Dout) return fail(ctx, SOM_EINVAL, "null operand");
    if (((uintptr_t)A | (uintptr_t)Bt) & 15) return fail(ctx, SOM_EINVAL, "A and Bt must be 16-byte aligned");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, ctx->stream, A, Bt, C, Dout, n);
    return check_hip(ctx, hipGetLastError(), "launching the matrix-pipe probe");
}
