// Measurement hook: the rate of the bf16 matrix instructions in a loop that touches nothing but registers.
// It frames every MFMA-bound figure of the library: the published peak assumes 2.4 GHz, and what the part
// sustains depends on the operand values (switching activity) through its power limit.
//
// Every wave keeps four independent accumulator sets and four operand pairs in registers and issues
// iters x 4 matrix instructions; operands are all zero, or pseudo-random bf16 values with magnitudes 1/8 .. 16.
// The sums go to `sink` so that the loop cannot be dropped.
#pragma once
#include "acc_common.h"

namespace acc {

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// bf16 with random sign and mantissa and an exponent of 124 .. 131
__device__ __forceinline__ bf16 probe_value(uint32_t h) {
  const uint16_t bits = (uint16_t)((h & 0x807Fu) | ((124u + ((h >> 8) & 7u)) << 7));
  return __builtin_bit_cast(bf16, bits);
}

// fp8 (e4m3) byte with random sign and mantissa and an exponent field of 4 .. 11 (magnitudes 1/8 .. 30)
__device__ __forceinline__ uint32_t probe_fp8(uint32_t h) { return (h & 0x87u) | ((4u + ((h >> 8) & 7u)) << 3); }

// SHAPE 0: v_mfma_f32_32x32x16_bf16 (32768 flops), SHAPE 1: v_mfma_f32_16x16x32_bf16 (16384 flops),
// SHAPE 2: v_mfma_f32_16x16x128_f8f6f4 on fp8 (e4m3) operands (65536 flops)
template <int SHAPE>
__global__ __launch_bounds__(512) void mfma_probe_kernel(int random_data, int64_t iters, float* __restrict__ sink) {
  const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[j][e] = random_data ? probe_value(probe_hash(gid * 64u + j * 16u + e)) : (bf16)0.f;
      b[j][e] = random_data ? probe_value(probe_hash(gid * 64u + j * 16u + 8u + e)) : (bf16)0.f;
    }
  float total = 0.f;
  if constexpr (SHAPE == 2) {
    i32x8 a8[4], b8[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint32_t wa = 0, wb = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          wa |= probe_fp8(probe_hash(gid * 256u + j * 64u + e * 4u + t)) << (8 * t);
          wb |= probe_fp8(probe_hash(gid * 256u + j * 64u + 32u + e * 4u + t)) << (8 * t);
        }
        a8[j][e] = random_data ? (int)wa : 0;
        b8[j][e] = random_data ? (int)wb : 0;
      }
    f32x4 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8[j], b8[j], acc[j], 0, 0, 0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) total += acc[j][e];
  } else if constexpr (SHAPE == 0) {
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) total += acc[j][e];
  } else {
    f32x4 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j], b[j], acc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) total += acc[j][e];
  }
  sink[gid] = total;
}

}  // namespace acc
