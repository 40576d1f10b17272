// Shape-generic MFMA kernels: any sizes and strides, fp32 or bf16.  They serve the fp32 layers
// and every shape the tuned bf16 kernels do not take; correctness first, 64x64x32 tiles.
#pragma once
#include "acc_common.h"
#include "acc_rng.h"

namespace acc {

struct GemmParams {
  const void* A;   // element (m, k) at A[m * a_sm + k * a_sk]
  const void* B;   // element (k, n) at B[k * b_sk + n * b_sn]   (ignored when B is the sketch)
  void* C;         // element (m, n) at C[m * c_sm + n * c_sn] (+ split * c_split_stride)
  int64_t M, N, K;
  int64_t a_sm, a_sk, b_sk, b_sn, c_sm, c_sn;
  int64_t k_per_split;     // K range handled by one blockIdx.z (multiple of 32)
  int64_t c_split_stride;  // elements between the partial results of consecutive splits
  int accumulate;          // 0: C = A . B;  1: C = beta C + alpha (A . B) (read-modify-write, one rounding)
  float alpha, beta;       // used when accumulate; 1, 1 is the plain sum
  SketchParams sk;         // B = S[k = token, n = column] when B_SKETCH
};

// C = A . B with fp32 accumulation.  CT is the MFMA operand type (float -> v_mfma_f32_32x32x2_f32,
// bf16 -> v_mfma_f32_32x32x16_bf16); inputs are converted to CT when staged in LDS.
// Grid: x = M tiles, y = N tiles, z = K splits.  256 threads = 4 waves in a 2x2 arrangement.
template <typename TA, typename TB, typename TC, typename CT, bool B_SKETCH, bool ACCURATE>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmParams p) {
  constexpr int BM = 64, BN = 64, BK = 32;
  constexpr int LDT = BK + (sizeof(CT) == 2 ? 8 : 1);
  __shared__ __attribute__((aligned(16))) CT As[BM * LDT];
  __shared__ __attribute__((aligned(16))) CT Bs[BN * LDT];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.x * BM, n0 = (int64_t)blockIdx.y * BN;
  const int64_t kbeg = (int64_t)blockIdx.z * p.k_per_split;
  const int64_t kend = (kbeg + p.k_per_split < p.K) ? kbeg + p.k_per_split : p.K;
  const TA* __restrict__ A = (const TA*)p.A;
  const TB* __restrict__ B = (const TB*)p.B;

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
    // ---- stage A[64 x 32] ----
    if (p.a_sk == 1) {
      const int kk = tid & 31;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int mm = (tid >> 5) + 8 * i;
        const int64_t gm = m0 + mm, gk = k0 + kk;
        const float v = (gm < p.M && gk < kend) ? to_f32(A[gm * p.a_sm + gk]) : 0.f;
        As[mm * LDT + kk] = from_f32<CT>(v);
      }
    } else {
      const int mm = tid & 63;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kk = (tid >> 6) + 4 * i;
        const int64_t gm = m0 + mm, gk = k0 + kk;
        const float v = (gm < p.M && gk < kend) ? to_f32(A[gm * p.a_sm + gk * p.a_sk]) : 0.f;
        As[mm * LDT + kk] = from_f32<CT>(v);
      }
    }
    // ---- stage B[32 x 64], kept as [n][k] ----
    if (B_SKETCH) {
      const int nn = tid & 63;
      const int64_t gn = n0 + nn;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int quad = (tid >> 6) + 4 * i;
        const int64_t gk = k0 + 4 * quad;  // local token of word 0
        float z[4] = {0.f, 0.f, 0.f, 0.f};
        if (gn < p.N && gk < kend) {
          uint32_t w[4];
          sketch_words(p.sk.key0, p.sk.key1, (p.sk.row_offset + (uint64_t)gk) >> 2, (uint32_t)gn, w);
          normals_from_words<ACCURATE>(w, p.sk.inv_sqrt_r, p.sk.neg2_ln2_over_r, z);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
          Bs[nn * LDT + 4 * quad + t] = from_f32<CT>((gk + t < kend) ? z[t] : 0.f);
      }
    } else if (p.b_sn == 1) {
      const int nn = tid & 63;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kk = (tid >> 6) + 4 * i;
        const int64_t gn = n0 + nn, gk = k0 + kk;
        const float v = (gn < p.N && gk < kend) ? to_f32(B[gk * p.b_sk + gn]) : 0.f;
        Bs[nn * LDT + kk] = from_f32<CT>(v);
      }
    } else {
      const int kk = tid & 31;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int nn = (tid >> 5) + 8 * i;
        const int64_t gn = n0 + nn, gk = k0 + kk;
        const float v = (gn < p.N && gk < kend) ? to_f32(B[gk * p.b_sk + gn * p.b_sn]) : 0.f;
        Bs[nn * LDT + kk] = from_f32<CT>(v);
      }
    }
    __syncthreads();
    // ---- one 32x32 MFMA tile per wave ----
    const CT* arow = &As[(wm * 32 + (lane & 31)) * LDT];
    const CT* brow = &Bs[(wn * 32 + (lane & 31)) * LDT];
    if constexpr (sizeof(CT) == 2) {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        const bf16x8 a = *(const bf16x8*)(arow + kk + (lane >> 5) * 8);
        const bf16x8 b = *(const bf16x8*)(brow + kk + (lane >> 5) * 8);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        const float a = arow[kk + (lane >> 5)];
        const float b = brow[kk + (lane >> 5)];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
      }
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds column (lane & 31), rows 8*(i/4) + 4*(lane>>5) + i%4 ----
  TC* __restrict__ C = (TC*)p.C + (int64_t)blockIdx.z * p.c_split_stride;
  const int64_t gn = n0 + wn * 32 + (lane & 31);
  if (gn < p.N) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t gm = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      if (gm < p.M) {
        float v = acc[i];
        if (p.accumulate) v = p.alpha * v + p.beta * to_f32(C[gm * p.c_sm + gn * p.c_sn]);
        C[gm * p.c_sm + gn * p.c_sn] = from_f32<TC>(v);
      }
    }
  }
}

// K4: out[e] = sum_g part[g * stride + e], converted to the factor type.  count % 4 == 0.
template <typename TO>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int G,
                                                              int64_t stride, int64_t count,
                                                              TO* __restrict__ out, int64_t row, int64_t ld) {
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e >= count) return;
  f32x4 s = *(const f32x4*)(part + e);
  for (int g = 1; g < G; ++g) {
    const f32x4 v = *(const f32x4*)(part + (int64_t)g * stride + e);
    s += v;
  }
  const int64_t eo = ld == row ? e : (e / row) * ld + e % row;  // rows of `row` elements stored `ld` apart
#pragma unroll
  for (int t = 0; t < 4; ++t) out[eo + t] = from_f32<TO>(s[t]);
}

// Column sums over a slab of rows (bias gradient, proof of Thm 3.2.2, bias term):
// part[g * C + c] = sum over rows i of slab g of A[i, c], fp32.  Grid (ceil(C / (64 * VEC)), G).
// A work-group has 16 waves; a lane owns VEC consecutive columns (one 16-byte load per row); wave w takes
// rows w, w + 16, ... of the slab in order, and the per-wave sums are added in a fixed order, so the
// result does not depend on scheduling.  C % VEC == 0; rows are 16-byte aligned.
constexpr int kColsumWaves = 16;
template <typename T>
__global__ __launch_bounds__(64 * kColsumWaves) void colsum_partial_kernel(const T* __restrict__ A, int64_t n,
                                                                            int64_t C, int64_t lda,
                                                                            int64_t rows_per_split,
                                                                            float* __restrict__ part) {
  constexpr int VEC = 16 / sizeof(T);
  typedef T vecT __attribute__((ext_vector_type(VEC)));
  __shared__ float red[kColsumWaves][64 * VEC];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = ((int64_t)blockIdx.x * 64 + lane) * VEC;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_split;
  const int64_t r1 = r0 + rows_per_split < n ? r0 + rows_per_split : n;
  float s[VEC];
#pragma unroll
  for (int t = 0; t < VEC; ++t) s[t] = 0.f;
  if (c < C) {
#pragma unroll 8
    for (int64_t i = r0 + wave; i < r1; i += kColsumWaves) {
      const vecT v = *(const vecT*)(A + i * lda + c);
#pragma unroll
      for (int t = 0; t < VEC; ++t) s[t] += to_f32(v[t]);
    }
  }
#pragma unroll
  for (int t = 0; t < VEC; ++t) red[wave][lane * VEC + t] = s[t];
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * VEC; e += 64 * kColsumWaves) {
    const int64_t col = (int64_t)blockIdx.x * 64 * VEC + e;
    float sum = red[0][e];
#pragma unroll
    for (int w = 1; w < kColsumWaves; ++w) sum += red[w][e];
    if (col < C) part[(int64_t)blockIdx.y * C + col] = sum;
  }
}

// out[c] = sum_g part[g * C + c] for a short vector (C columns, G partials): a work-group owns 64
// columns, its wave w adds partials w, w + 4, ... in order, then the four wave sums are added in order.
template <typename TO>
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, int G, int64_t C,
                                                           TO* __restrict__ out) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c = (int64_t)blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < C) {
#pragma unroll 8
    for (int g = wave; g < G; g += 4) s += part[(int64_t)g * C + c];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && c < C) out[c] = from_f32<TO>(((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane]);
}

// Test hook kernels -----------------------------------------------------------------------
__global__ __launch_bounds__(256) void philox_dump_kernel(uint32_t key0, uint32_t key1,
                                                          uint64_t row_offset, int64_t nq, int64_t r,
                                                          uint32_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // = q * r + j
  if (idx >= nq * r) return;
  const int64_t q = idx / r;
  const uint32_t j = (uint32_t)(idx - q * r);
  uint32_t w[4];
  sketch_words(key0, key1, (row_offset >> 2) + (uint64_t)q, j, w);
  *(u32x4*)(out + idx * 4) = u32x4{w[0], w[1], w[2], w[3]};
}

template <bool ACCURATE>
__global__ __launch_bounds__(256) void sketch_dump_kernel(SketchParams sk, int64_t n, int64_t r,
                                                          float* __restrict__ S) {
  const int64_t nq = (n + 3) / 4;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // = q * r + j
  if (idx >= nq * r) return;
  const int64_t q = idx / r;
  const uint32_t j = (uint32_t)(idx - q * r);
  uint32_t w[4];
  float z[4];
  sketch_words(sk.key0, sk.key1, (sk.row_offset >> 2) + (uint64_t)q, j, w);
  normals_from_words<ACCURATE>(w, sk.inv_sqrt_r, sk.neg2_ln2_over_r, z);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int64_t i = 4 * q + t;
    if (i < n) S[i * r + j] = ACCURATE ? z[t] : (float)(bf16)z[t];
  }
}

}  // namespace acc
