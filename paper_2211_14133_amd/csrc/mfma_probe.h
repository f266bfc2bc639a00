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

// The same loops on operands with random sign and mantissa bits (exponent of 1.0), four operand sets in
// rotation: what the matrix cores sustain when their inputs toggle as real data does.  (With constant operands
// the bf16 loop reaches the published peak; with random bits the chip lowers its clock: the power drawn by the
// matrix cores depends on the data.)
constexpr int PROBE_SETS = 4;

__device__ inline unsigned probe_hash(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(256, 2) void mfma_probe_f32_random_kernel(int iters, float *sink)
{
    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float a[PROBE_SETS][2], b[PROBE_SETS][4];
    const unsigned t = threadIdx.x + 256 * blockIdx.x;
#pragma unroll
    for (int s = 0; s < PROBE_SETS; ++s) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            a[s][i] = __builtin_bit_cast(float, (probe_hash(t * 131 + s * 17 + i) & 0x807fffffu) | 0x3f800000u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            b[s][j] = __builtin_bit_cast(float, (probe_hash(t * 257 + s * 29 + j + 99) & 0x807fffffu) | 0x3f800000u);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < PROBE_SETS; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
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

__global__ __launch_bounds__(256, 2) void mfma_probe_bf16_random_kernel(int iters, float *sink)
{
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    u32x4 a[PROBE_SETS][2], b[PROBE_SETS][4];
    const unsigned t = threadIdx.x + 256 * blockIdx.x;
#pragma unroll
    for (int s = 0; s < PROBE_SETS; ++s) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) a[s][i][c] = (probe_hash(t * 131 + s * 17 + i * 5 + c) & 0x807f807fu) | 0x3f803f80u;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c) b[s][j][c] = (probe_hash(t * 257 + s * 29 + j * 7 + c + 99) & 0x807f807fu) | 0x3f803f80u;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < PROBE_SETS; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[s][i]),
                                                                        __builtin_bit_cast(bf16x8, b[s][j]), acc[i][j], 0, 0, 0);
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
