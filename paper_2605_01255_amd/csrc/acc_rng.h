// Device-side regeneration of the sketch matrix S (step F0).
//
// Integer stream: Philox4x32-10 (Salmon et al., SC'11), key = (seed lo, seed hi),
// counter = ((g >> 2) lo, column j, stream 0, g >> 34) for global token g; output word w
// is token 4*(g >> 2) + w.  Uniform u = ((x >> 9) + 0.5) 2^-23 (exact in fp32).
// Box-Muller on (x0, x1) and (x2, x3): z_even = R cos(theta), z_odd = R sin(theta).
#pragma once
#include "acc_common.h"

namespace acc {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float uniform_from_word(uint32_t x) {
  // ((x >> 9) + 0.5) 2^-23 in two instructions, both exact: v_alignbit_b32 puts the 23 bits under the exponent of
  // 1.0 (a = 1 + (x >> 9) 2^-23), and a - (1 - 2^-24) = (2 (x >> 9) + 1) 2^-24 is representable, so the
  // subtraction does not round.  (Shift, convert, add, multiply take four.)
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_alignbit(0x7Fu, x, 9u));
  return a - 0x1.fffffep-1f;
}

// a ^ b ^ k in one instruction (v_bitop3_b32 with truth table 0x96 = three-input xor; k wave-uniform).
// The compiler emits two v_xor_b32 here.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t k) {
  uint32_t r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "s"(k));
  return r;
}

// One Philox4x32 round on a counter held in c[0..3]; round_index selects the bumped key (wave-uniform).
__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t key0, uint32_t key1, int round_index) {
  const uint32_t k0 = key0 + (uint32_t)round_index * 0x9E3779B9u;
  const uint32_t k1 = key1 + (uint32_t)round_index * 0xBB67AE85u;
  const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
  const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
  const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
  const uint32_t n0 = xor3(hi1, c[1], k0), n2 = xor3(hi0, c[3], k1);
  c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
}

// One Box-Muller pair from two words (fast hardware generator, already scaled by 1/sqrt(r)).
__device__ __forceinline__ void box_muller_fast(uint32_t wa, uint32_t wb, float neg2_ln2_over_r, float& z_even,
                                                float& z_odd) {
  const float u1 = uniform_from_word(wa), u2 = uniform_from_word(wb);
  const float radius = __builtin_amdgcn_sqrtf(neg2_ln2_over_r * __builtin_amdgcn_logf(u1));
  z_even = radius * __builtin_amdgcn_cosf(u2);
  z_odd = radius * __builtin_amdgcn_sinf(u2);
}

// The four Philox words of token group g4 = (global token >> 2) and column j.
__device__ __forceinline__ void sketch_words(uint32_t key0, uint32_t key1, uint64_t g4, uint32_t j,
                                             uint32_t (&w)[4]) {
  philox4x32_10((uint32_t)g4, j, 0u, (uint32_t)(g4 >> 32), key0, key1, w);
}

// Four entries of S (tokens 4*g4 .. 4*g4+3 of one column), already scaled by 1/sqrt(r).
//   ACCURATE: libm-grade log / sincospi (fp32 layers, tolerance 1e-5).
//   fast:     v_log_f32, v_sqrt_f32, v_sin_f32, v_cos_f32 (the last two take revolutions,
//             so theta = 2 pi u needs no multiply); error ~1e-6 absolute, far below bf16 rounding.
// neg2_ln2_over_r = -2 ln(2) / r folds the 1/sqrt(r) scale under the square root.
template <bool ACCURATE>
__device__ __forceinline__ void normals_from_words(const uint32_t (&w)[4], float inv_sqrt_r,
                                                   float neg2_ln2_over_r, float (&z)[4]) {
#pragma unroll
  for (int a = 0; a < 4; a += 2) {
    const float u1 = uniform_from_word(w[a]);
    const float u2 = uniform_from_word(w[a + 1]);
    if (ACCURATE) {
      const float radius = sqrtf(-2.0f * logf(u1)) * inv_sqrt_r;
      float s, c;
      sincospif(2.0f * u2, &s, &c);
      z[a] = radius * c;
      z[a + 1] = radius * s;
    } else {
      const float radius = __builtin_amdgcn_sqrtf(neg2_ln2_over_r * __builtin_amdgcn_logf(u1));
      z[a] = radius * __builtin_amdgcn_cosf(u2);
      z[a + 1] = radius * __builtin_amdgcn_sinf(u2);
    }
  }
}

struct SketchParams {
  uint32_t key0, key1;     // Philox key = seed words
  uint64_t row_offset;     // global index of local token 0 (multiple of 4)
  float inv_sqrt_r;        // 1 / sqrt(r)
  float neg2_ln2_over_r;   // -2 ln 2 / r
};

}  // namespace acc
