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

} // namespace som

using namespace som;

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
