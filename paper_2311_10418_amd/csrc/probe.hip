// Measurement aid: the rate the matrix cores sustain on their own, as the yardstick beside the published peak.
//
// One work-group per compute unit slot (512 threads = 2 wavefronts per SIMD, the occupancy of the GEMM kernel; a
// 100 KB LDS allocation keeps a second work-group off the CU), every wavefront holding the GEMM kernel's register
// tile: 8 x 4 accumulator blocks of v_mfma_f32_16x16x32_bf16 and the 8 + 4 operand fragments of two k steps, read
// once from memory.  The loop issues the 64 MFMAs of a K tile in the GEMM kernel's order and nothing else: no LDS,
// no transfers, no barrier.  What it reaches depends on the operands (the chip runs at its power limit): about
// 2.47 PFLOP/s on zeros, 2.0 - 2.1 on random values.
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace {

__global__ __launch_bounds__(512, 1) void mfma_loop_kernel(const bf16x8_t* __restrict__ operands, float* __restrict__ sink, int iters) {
    const int t = threadIdx.x;
    bf16x8_t fa[2][8], fb[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 8; ++i) fa[s][i] = operands[(s * 12 + i) * 512 + t];
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[s][j] = operands[(s * 12 + 8 + j) * 512 + t];
    }
    f32x4_t acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int j = (i & 1) ? 3 - jj : jj;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[s][j], fa[s][i], acc[i][j], 0, 0, 0);
                }
    }
    // one value per thread leaves the kernel so that the loop cannot be dropped
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) r += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    sink[(size_t)blockIdx.x * 512 + t] = r;
}

}  // namespace

extern "C" ds_status ds_mfma_probe(const void* operands, float* sink, int32_t n_groups, int32_t iters, void* hip_stream) {
    if (!operands || !sink || n_groups <= 0 || iters <= 0 || ((uintptr_t)operands & 15)) return DS_EINVAL;
    static bool attr_set = false;
    constexpr int kLds = 100 * 1024;
    if (!attr_set) {
        DS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_loop_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        attr_set = true;
    }
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(n_groups), dim3(512), kLds, (hipStream_t)hip_stream,
                       static_cast<const bf16x8_t*>(operands), sink, iters);
    DS_LAUNCH_CHECK();
    return DS_OK;
}
