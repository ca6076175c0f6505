// Measurement aids: what this GPU sustains on the two resources the convolution kernels
// are priced against.  A register-only MFMA loop (no LDS, no memory, no barrier) gives the
// matrix-core rate at the clock the chip really holds; a plain 16-byte copy gives the rate
// of one read stream plus one write stream through HBM.  Neither is part of the block.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "kern_igemm_bf16.h"

namespace mcn {

#define PROBE_BLOCKS 2048   // 8 blocks of 4 waves per compute unit
#define PROBE_THREADS 256
#define PROBE_ACC 4         // independent accumulators per wave: hides the MFMA latency

// precision 0: v_mfma_f32_32x32x2_f32 (4096 flop each); 1: v_mfma_f32_32x32x16_bf16 (32768 flop each).
template <int BF>
__global__ __launch_bounds__(PROBE_THREADS) void probe_mfma_kernel(float *sink, int iters, float seed) {
    floatx16 acc[PROBE_ACC];
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float a = seed + (float)(threadIdx.x & 7), b = seed * 0.5f;
    bf16x8 a8, b8;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        a8[v] = (__bf16)(a + v);
        b8[v] = (__bf16)b;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i) {
            if (BF)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8, b8, acc[i], 0, 0, 0);
            else
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// dst[0..n) = src[0..n); n4 = n / 4 whole 16-byte words, the tail goes float by float.
__global__ __launch_bounds__(PROBE_THREADS) void probe_copy_kernel(const float *__restrict__ src,
                                                                   float *__restrict__ dst, size_t n) {
    const size_t n4 = n >> 2;
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    const float4 *s4 = reinterpret_cast<const float4 *>(src);
    float4 *d4 = reinterpret_cast<float4 *>(dst);
    for (size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x; i < n4; i += stride) d4[i] = s4[i];
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) dst[(n4 << 2) + threadIdx.x] = src[(n4 << 2) + threadIdx.x];
}

}  // namespace mcn
