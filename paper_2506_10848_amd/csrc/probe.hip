// Measurement hook: the rate at which the matrix cores run when nothing else does.  Every wave multiplies
// operands it keeps in registers (v_mfma_f32_32x32x16_bf16, eight independent accumulator tiles, no memory
// access inside the loop), one wave per SIMD on every CU.  With random operands the chip's power limit, not
// the instruction rate, sets the result, which is the ceiling any bf16 GEMM of this library can approach.
#include "internal.h"

namespace dllm {
namespace {

union Frag { uint4 u; bf16x8 b; };

__global__ __launch_bounds__(256) void mfma_rate_kernel(const uint4 *__restrict__ operands, int n_operands,
                                                        float *__restrict__ sink, int iters)
{
    const int tid = blockIdx.x * 256 + threadIdx.x;
    Frag a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = operands[(unsigned)(tid * 8 + i) % (unsigned)n_operands];
        b[i].u = operands[(unsigned)(tid * 8 + 4 + i) % (unsigned)n_operands];
    }
    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3].b, b[(i >> 1) & 3].b, acc[i], 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += acc[i][e];
    sink[tid] = sum;
}

}  // namespace

hipError_t launch_mfma_rate(hipStream_t stream, const void *operands, int n_operands, float *sink, int workgroups,
                            int iters)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(256), 0, stream,
                       reinterpret_cast<const uint4 *>(operands), n_operands, sink, iters);
    return hipGetLastError();
}

}  // namespace dllm
