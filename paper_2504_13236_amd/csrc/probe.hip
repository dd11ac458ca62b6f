// Measurement aids of the library: kernels that do no useful work and exist to find the rates the
// chip sustains, against which the product kernels are judged.
//
// nnt_probe_mfma_rate: every wavefront issues matrix instructions back to back on operands that
// live in registers (no memory traffic, no dependence between consecutive instructions), for fp32
// (v_mfma_f32_32x32x2_f32) or bf16 (v_mfma_f32_32x32x16_bf16).  With `random_operands` the operand
// registers hold pseudo-random values that differ from instruction to instruction, as the operands
// of a real product do; with constants the inputs of the matrix cores never toggle.  The matrix
// cores of this chip run measurably slower on toggling operands (the clock is lowered under the
// higher power draw), so the two figures bracket what a product kernel can reach.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nntile_mi.h"

namespace nnt {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// a value in (-2, 2) from a counter
__device__ __forceinline__ float unit_value(uint32_t c) { return (float)(int32_t)(mix(c) >> 8) * (1.f / 4194304.f) - 2.f; }

constexpr int kOperands = 8;      // operand registers in rotation

__global__ void __launch_bounds__(256) mfma_rate_f32(int random_operands, int iters, float* sink) {
    float a[kOperands], b[kOperands];
    const uint32_t id = (blockIdx.x * 256u + threadIdx.x) * 2u * kOperands;
#pragma unroll
    for (int i = 0; i < kOperands; i++) {
        a[i] = random_operands ? unit_value(id + 2 * i) : 1.f;
        b[i] = random_operands ? unit_value(id + 2 * i + 1) : 1.f;
    }
    f32x16 acc[4] = {};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < kOperands; i++) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[i], acc[i & 3], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 4; q++)
#pragma unroll
        for (int i = 0; i < 16; i++) t += acc[q][i];
    if (t == 12345.678f) sink[0] = t;      // keeps the instructions alive; practically never true
}

__global__ void __launch_bounds__(256) mfma_rate_bf16(int random_operands, int iters, float* sink) {
    bf16x8 a[kOperands], b[kOperands];
    const uint32_t id = (blockIdx.x * 256u + threadIdx.x) * 16u * kOperands;
#pragma unroll
    for (int i = 0; i < kOperands; i++)
#pragma unroll
        for (int e = 0; e < 8; e++) {
            a[i][e] = (__bf16)(random_operands ? unit_value(id + 16 * i + e) : 1.f);
            b[i][e] = (__bf16)(random_operands ? unit_value(id + 16 * i + 8 + e) : 1.f);
        }
    f32x16 acc[4] = {};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < kOperands; i++) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i & 3], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 4; q++)
#pragma unroll
        for (int i = 0; i < 16; i++) t += acc[q][i];
    if (t == 12345.678f) sink[0] = t;
}

}  // namespace
}  // namespace nnt

using namespace nnt;

extern "C" int32_t nnt_probe_mfma_rate(void* stream, int32_t dtype, int32_t random_operands, int32_t iters, int32_t workgroups,
                                       float* sink, double* flops_out) {
    if (dtype != NNT_F32 && dtype != NNT_BF16) return NNT_EDTYPE;
    if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20) || !sink) return NNT_EINVAL;
    const dim3 grid((unsigned)workgroups), block(256);
    if (dtype == NNT_F32) hipLaunchKernelGGL(mfma_rate_f32, grid, block, 0, (hipStream_t)stream, random_operands, iters, sink);
    else hipLaunchKernelGGL(mfma_rate_bf16, grid, block, 0, (hipStream_t)stream, random_operands, iters, sink);
    if (hipGetLastError() != hipSuccess) return NNT_EHIP;
    // flops issued: wavefronts x iterations x instructions per iteration x flops per instruction
    if (flops_out) *flops_out = (double)workgroups * 4.0 * iters * kOperands * (dtype == NNT_F32 ? 4096.0 : 32768.0);
    return NNT_OK;
}
