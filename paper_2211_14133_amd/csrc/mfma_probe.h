// Register-only MFMA loops: what the matrix cores sustain on this chip when
// nothing else (memory, LDS, barriers) is in the way.  The benchmark reports the
// curvature kernel against this measured ceiling next to the published peak.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tn_gemm.h"

namespace kfac {

constexpr int PROBE_MFMA_PER_ITER = 8;   // independent accumulators per wave and loop iteration (acc[2][4] below)

// 4 waves per workgroup; each wave runs `iters` iterations of 8 independent MFMA 32x32x2 (fp32).
__global__ __launch_bounds__(256, 2) void mfma_probe_f32_kernel(float a0, float b0, int iters, float *sink)
{
    static_assert(PROBE_MFMA_PER_ITER == 2 * 4, "the loops below issue acc[2][4] = 8 MFMAs per iteration");
    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float a[2], b[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = a0 + (float)(threadIdx.x + i);
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = b0 - (float)(threadIdx.x * 2 + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    if (s == 12345.678f) sink[threadIdx.x & 63] = s;  // keeps the loop alive; practically never taken
}

// Same with MFMA 32x32x16 on bfloat16 operands.
__global__ __launch_bounds__(256, 2) void mfma_probe_bf16_kernel(unsigned a0, unsigned b0, int iters, float *sink)
{
    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    uint4 a[2], b[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = make_uint4(a0 + threadIdx.x, a0 + i, a0, a0 ^ threadIdx.x);
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = make_uint4(b0 + threadIdx.x, b0 + j, b0, b0 ^ threadIdx.x);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                                    __builtin_bit_cast(bf16x8, b[j]), acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    if (s == 12345.678f) sink[threadIdx.x & 63] = s;
}

}  // namespace kfac
