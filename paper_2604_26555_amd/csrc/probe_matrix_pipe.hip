// Stand-alone probe of the two properties of gfx950's bf16 matrix pipe that bmu_split_kernel is built on; not part
// of libsom.so.  Build: python -m paper_2604_26555_amd.build; run: paper_2604_26555_amd/probe_matrix_pipe
//
// 1. Accumulation error of v_mfma_f32_32x32x16_bf16 (and _f16).  The products of 16-bit operands are exact in
//    float32, but how the pipe adds 16 of them to the accumulator is not specified.  The probe compares
//    D = C + sum_k A[i][k] B[k][j] with the exact value (float64 is exact for these operand ranges) over random
//    operands with several exponent spreads and reports the largest error in units of
//    2^-24 * max(|C|, sum_k |A B|), and how often the result equals the correctly rounded exact sum.  The error
//    bound of the split BMU search counts 8 such units per MFMA.
// 2. Vector instructions beside an MFMA.  Eight bf16 MFMAs on two accumulators, each followed by n fold steps
//    (v_and_or_b32, v_med3_f32, v_max_f32 on registers no MFMA in flight writes), timed with one and with two
//    wavefronts per SIMD: cycles per MFMA slot.  The pipe is busy 32 cycles per MFMA; whatever stays at about 32-35
//    is issued for free.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                       \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

// A: [32][16] (i, k), Bt: [32][16] (j, k), C, D: [32][32], one problem per loop trip
template <bool F16>
__global__ void __launch_bounds__(64) mfma_once(const float* A, const float* Bt, const float* C, float* D, int n)
{
    const int lane = threadIdx.x, j = lane & 31, g = lane >> 5;
    for (int t = blockIdx.x; t < n; t += gridDim.x) {
        const float* a = A + (size_t)t * 512;
        const float* b = Bt + (size_t)t * 512;
        const float* c = C + (size_t)t * 1024;
        floatx16 acc;
        for (int r = 0; r < 16; ++r) acc[r] = c[(8 * (r >> 2) + 4 * g + (r & 3)) * 32 + j];
        if (F16) {
            f16x8 av, bv;
            for (int i = 0; i < 8; ++i) {
                av[i] = (_Float16)a[j * 16 + 8 * g + i];
                bv[i] = (_Float16)b[j * 16 + 8 * g + i];
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);
        } else {
            bf16x8 av, bv;
            for (int i = 0; i < 8; ++i) {
                av[i] = (__bf16)a[j * 16 + 8 * g + i];
                bv[i] = (__bf16)b[j * 16 + 8 * g + i];
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
        }
        float* d = D + (size_t)t * 1024;
        for (int r = 0; r < 16; ++r) d[(8 * (r >> 2) + 4 * g + (r & 3)) * 32 + j] = acc[r];
    }
}

static float to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    u = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
    memcpy(&v, &u, 4);
    return v;
}
static float to_f16(float v) { return (float)(_Float16)v; }

#define FOLD1 "v_and_or_b32 %2, %7, %8, 5\nv_med3_f32 %3, %4, %3, %2\nv_max_f32 %4, %4, %2\n"
#define PAIR(VS) "v_mfma_f32_32x32x16_bf16 %0, %5, %6, %0\n" VS "v_mfma_f32_32x32x16_bf16 %1, %5, %6, %1\n" VS
template <int N>
__global__ void __launch_bounds__(256) beside(const float* x, float* out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)x[(threadIdx.x + i) & 1023];
        b[i] = (__bf16)x[(threadIdx.x * 3 + i) & 1023];
    }
    floatx16 c0 = {}, c1 = {};
    float t = 0.f, second = x[threadIdx.x & 1023], best = x[(threadIdx.x + 7) & 1023], src = x[(threadIdx.x + 9) & 1023];
    unsigned mask = 0xfffffff0u;
    for (int it = 0; it < iters; ++it) {
#define RUN(VS)                                                                                                        \
    asm volatile(PAIR(VS) PAIR(VS) PAIR(VS) PAIR(VS)                                                                   \
                 : "+v"(c0), "+v"(c1), "+v"(t), "+v"(second), "+v"(best)                                               \
                 : "v"(a), "v"(b), "v"(src), "s"(mask));
        if (N == 0) RUN("")
        if (N == 1) RUN(FOLD1)
        if (N == 2) RUN(FOLD1 FOLD1)
        if (N == 3) RUN(FOLD1 FOLD1 FOLD1)
    }
    out[blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[3] + t + second + best;
}

template <int N>
static int time_beside(const float* x, float* out, int grid)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int iters = 20000;
    float best = 1e9f;
    for (int rep = 0; rep < 3; ++rep) {
        CHECK(hipEventRecord(e0));
        beside<N><<<grid, 256>>>(x, out, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    printf("%d wavefront(s) per SIMD, %d fold steps (%d vector instructions) per MFMA: %.2f ns per MFMA slot = %.1f cycles at 2.4 GHz\n",
           grid / 256, N, 3 * N, best * 1e6 / (8.0 * iters * (grid / 256)), best * 1e-3 * 2.4e9 / (8.0 * iters * (grid / 256)));
    fflush(stdout);
    return 0;
}

int main()
{
    const int n = 2048;
    std::mt19937_64 rng(12345);
    std::uniform_real_distribution<double> U(-1.0, 1.0);
    float *dA, *dB, *dC, *dD;
    CHECK(hipMalloc(&dA, n * 512 * 4));
    CHECK(hipMalloc(&dB, n * 512 * 4));
    CHECK(hipMalloc(&dC, n * 1024 * 4));
    CHECK(hipMalloc(&dD, n * 1024 * 4));
    std::vector<float> A(n * 512), B(n * 512), C(n * 1024), D(n * 1024);
    double worst_all[2] = {0, 0};
    for (int f16 = 0; f16 < 2; ++f16)
        for (int spread = 0; spread <= 12; spread += 4)
            for (int cexp = -8; cexp <= 8; cexp += 8) {
                std::uniform_int_distribution<int> E(-spread, spread);
                for (auto& v : A) {
                    const float x = (float)std::ldexp(U(rng), E(rng));
                    v = f16 ? to_f16(x) : to_bf16(x);
                }
                for (auto& v : B) {
                    const float x = (float)std::ldexp(U(rng), E(rng));
                    v = f16 ? to_f16(x) : to_bf16(x);
                }
                for (auto& v : C) v = (float)std::ldexp(U(rng), cexp);
                CHECK(hipMemcpy(dA, A.data(), n * 512 * 4, hipMemcpyHostToDevice));
                CHECK(hipMemcpy(dB, B.data(), n * 512 * 4, hipMemcpyHostToDevice));
                CHECK(hipMemcpy(dC, C.data(), n * 1024 * 4, hipMemcpyHostToDevice));
                if (f16)
                    mfma_once<true><<<256, 64>>>(dA, dB, dC, dD, n);
                else
                    mfma_once<false><<<256, 64>>>(dA, dB, dC, dD, n);
                CHECK(hipMemcpy(D.data(), dD, n * 1024 * 4, hipMemcpyDeviceToHost));
                double worst = 0;
                long total = 0, correctly_rounded = 0;
                for (int t = 0; t < n; ++t)
                    for (int i = 0; i < 32; ++i)
                        for (int j = 0; j < 32; ++j) {
                            double exact = C[(size_t)t * 1024 + i * 32 + j], mag = std::fabs(exact), sabs = 0;
                            for (int k = 0; k < 16; ++k) {
                                const double p = (double)A[(size_t)t * 512 + i * 16 + k] * (double)B[(size_t)t * 512 + j * 16 + k];
                                exact += p;
                                sabs += std::fabs(p);
                            }
                            if (sabs > mag) mag = sabs;
                            const float got = D[(size_t)t * 1024 + i * 32 + j];
                            const double units = std::fabs((double)got - exact) / (mag * 5.9604644775390625e-08);
                            if (units > worst) worst = units;
                            if ((float)exact == got) ++correctly_rounded;
                            ++total;
                        }
                if (worst > worst_all[f16]) worst_all[f16] = worst;
                printf("%s operands 2^+-%-2d, C ~ 2^%-2d: largest error %.3f x 2^-24 x max(|C|, sum|products|); correctly rounded in %.4f of %ld outputs\n",
                       f16 ? "f16 " : "bf16", spread, cexp, worst, (double)correctly_rounded / total, total);
                fflush(stdout);
            }
    printf("largest error overall: bf16 %.3f units, f16 %.3f units (the search's bound counts 8)\n", worst_all[0], worst_all[1]);

    float *x, *out;
    CHECK(hipMalloc(&x, 4096));
    CHECK(hipMalloc(&out, 2048 * 256 * 4));
    CHECK(hipMemset(x, 0, 4096));
    for (int grid = 256; grid <= 512; grid += 256) {       // one and two workgroups of four wavefronts per compute unit
        if (time_beside<0>(x, out, grid) || time_beside<1>(x, out, grid) || time_beside<2>(x, out, grid) ||
            time_beside<3>(x, out, grid))
            return 1;
    }
    return worst_all[0] <= 8.0 ? 0 : 2;
}
