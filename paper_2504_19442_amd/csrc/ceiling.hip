// Measured ceiling for the roofline: what the matrix pipes of this chip sustain on the GEMM's own instruction and
// register pattern when nothing else happens -- no global loads, no LDS traffic, no barriers.  Every wave keeps 14
// blocks of 32x32 fp32 accumulators (224 registers, as one wave of the 256x224 tile does) and feeds them with
// v_mfma_f32_32x32x16_bf16 from nine operand fragments held in registers, filled with pseudo-random bf16 values in
// the ranges of the benchmark's inputs (A uniform in [-1, 1), B scaled by 0.02): the power the pipes draw, and with it
// the clock the chip holds, depends on how much the operand bits toggle.
#include "agg_internal.h"

namespace agg {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8c;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16c;

__device__ inline unsigned mix(unsigned x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(256) void mfma_ceiling_kernel(float* sink, int iters, int constant_operands)
{
    bf16x8c fr[9];
    for (int s = 0; s < 9; ++s)
        for (int i = 0; i < 8; ++i) {
            const unsigned h = mix(threadIdx.x * 131u + blockIdx.x * 7919u + s * 17u + i);
            const float u = constant_operands ? 1.0f : (h & 0xffff) / 32768.0f - 1.0f;
            fr[s][i] = (__bf16)(u * (s >= 2 ? 0.02f : 1.0f));
        }
    f32x16c acc[14];
    for (int j = 0; j < 14; ++j)
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 14; ++q)
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[q % 2], fr[2 + q / 2], acc[q], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < 14; ++j)
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 123.456f) sink[threadIdx.x] = s;      // keeps the loop alive; practically never taken
}

hipError_t launch_mfma_ceiling(float* sink, int grid, int iters, int constant_operands, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(grid), dim3(256), 0, stream, sink, iters, constant_operands);
    return hipGetLastError();
}

}  // namespace agg
