// Small dense kernels of the RSVD compressor (Experimental Setup: randomized SVD of Halko et al.): the
// triangular factor of a k x k Gram matrix and its inverse, the middle step of a Cholesky QR.  The large
// products around it (X.Omega, Yr^T.Yr, Yr.R^-1, X^T.U, U^T.dY) run on the generic MFMA kernels.
#pragma once
#include "acc_common.h"
#include "acc_rng.h"

namespace acc {

constexpr int kRsvdMaxRank = 64;   // the k x k factorisation runs on one wave, one matrix row per lane

// G [k, k] (symmetric positive semi-definite, fp32) -> Rinv [k, k] fp32 with G = R^T R, R upper triangular
// with positive diagonal, Rinv = R^-1 (upper triangular), for k <= K (K = 32 or 64), by ONE wave entirely in
// registers: lane i holds row i of the symmetric matrix (padded to K with the identity), values move
// between lanes by v_readlane broadcasts; no LDS, no barriers (the k sequential steps are pure latency, and
// an LDS version with a barrier per step measured 2-4x slower).
// A pivot that is not positive beyond rounding (column j of the factored matrix depends on the earlier
// ones) is dropped: row and column j of Rinv are zero, so the corresponding basis vector comes out as zero
// and the span of the others is unchanged.
__device__ __forceinline__ float lane_bcast(float v, int src_lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
}
__device__ __forceinline__ double lane_bcast(double v, int src_lane) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)u, src_lane);
  const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), src_lane);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

template <int K, typename R>
__global__ __launch_bounds__(64) void chol_inverse_small_kernel(const float* __restrict__ G, float* __restrict__ Rinv,
                                                                int k) {
  const int lane = threadIdx.x;
  R a[K], x[K];
#pragma unroll
  for (int c = 0; c < K; ++c) {
    a[c] = (lane < k && c < k) ? (R)G[lane * k + c] : (lane == c ? (R)1 : (R)0);
    x[c] = (R)0;
  }
  R diag = (R)0;
#pragma unroll
  for (int c = 0; c < K; ++c) diag = (c == lane && lane < k) ? a[c] : diag;
  R maxdiag = (R)0;
#pragma unroll
  for (int l = 0; l < K; ++l) {
    const R d = lane_bcast(diag, l);
    maxdiag = d > maxdiag ? d : maxdiag;
  }
  const R tol = maxdiag * (R)1e-6;
  uint64_t dead_mask = 0;
#pragma unroll
  for (int j = 0; j < K; ++j) {
    const R piv = lane_bcast(a[j], j);
    const bool dead = !(piv > tol);
    if (dead) dead_mask |= 1ull << j;
    const R inv_d = dead ? (R)0 : (R)1 / (R)sqrt((double)piv);
    const R rji = lane > j ? a[j] * inv_d : (R)0;   // R[j][lane] (the matrix is kept symmetric)
#pragma unroll
    for (int c = j + 1; c < K; ++c) {
      const R rjc = lane_bcast(a[c], j) * inv_d;   // R[j][c]
      a[c] = lane == j ? rjc : a[c] - rji * rjc;        // lane j keeps row j of R; lanes > j update
    }
    a[j] = lane == j ? (dead ? (R)0 : piv * inv_d) : a[j];
  }
  // lane i now holds row i of R in a[i..K-1].  Lane c builds column c of the inverse, top row last.
  const bool dead_c = (dead_mask >> lane) & 1;
#pragma unroll
  for (int i = K - 1; i >= 0; --i) {
    R sum = lane == i ? (R)1 : (R)0;
#pragma unroll
    for (int t = i + 1; t < K; ++t) sum -= lane_bcast(a[t], i) * x[t];
    const R rii = lane_bcast(a[i], i);
    const bool dead_i = (dead_mask >> i) & 1;
    x[i] = (i <= lane && !dead_i && !dead_c) ? sum / rii : (R)0;
  }
  if (lane < k) {
#pragma unroll
    for (int i = 0; i < K; ++i)
      if (i < k) Rinv[i * k + lane] = (float)x[i];
  }
}

// out[e] = sum over p of part[p * E + e], p in order within fixed groups: a work-group owns 64 elements, its
// wave w adds parts w, w + 16, ..., then the 16 wave sums are added in order.  Grid ceil(E / 64) x 1024 threads.
__global__ __launch_bounds__(1024) void sum_parts_kernel(const float* __restrict__ part, int P, int64_t E,
                                                         float* __restrict__ out) {
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t e = (int64_t)blockIdx.x * 64 + lane;
  float s = 0.f;
  if (e < E) {
#pragma unroll 8
    for (int p = wave; p < P; p += 16) s += part[(int64_t)p * E + e];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && e < E) {
    float sum = red[0][lane];
#pragma unroll
    for (int w = 1; w < 16; ++w) sum += red[w][lane];
    out[e] = sum;
  }
}

// Partial Gram matrices of a tall matrix: part[g] [k, k] = Y[rows of slab g]^T . Y[rows of slab g], fp32
// matrix instructions (v_mfma_f32_32x32x2_f32).  Y [n, k] fp32 row-major; grid = slabs of `rows_per_wg`
// rows; 4 waves share the (k/32)^2 output blocks (k is padded to a multiple of 32 with zero columns).
__global__ __launch_bounds__(256) void gram_partial_kernel(const float* __restrict__ Y, int64_t n, int k,
                                                           int rows_per_wg, float* __restrict__ part) {
  constexpr int CH = 64;                       // rows staged at a time
  __shared__ float Ys[CH * (kRsvdMaxRank + 32)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kp = (k + 31) / 32 * 32, nb = kp / 32, blocks = nb * nb;
  const int ld = (kp % 64 == 0) ? kp + 32 : kp;  // rows r and r + 1 on different halves of the 64 banks
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg;
  const int64_t r1 = r0 + rows_per_wg < n ? r0 + rows_per_wg : n;
  f32x16 acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
  for (int64_t c0 = r0; c0 < r1; c0 += CH) {
    for (int e = tid; e < CH * kp; e += 256) {
      const int r = e / kp, c = e % kp;
      Ys[r * ld + c] = (c0 + r < r1 && c < k) ? Y[(c0 + r) * k + c] : 0.f;
    }
    __syncthreads();
    if (blocks == 1) {  // k <= 32: the four waves split the rows of the chunk, their sums are added below
      for (int rr = wave * (CH / 4); rr < (wave + 1) * (CH / 4); rr += 2) {
        const float a = Ys[(rr + (lane >> 5)) * ld + (lane & 31)];
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, acc[0], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int blk = wave + 4 * q;
        if (blk < blocks) {
          const int i0 = (blk / nb) * 32, j0 = (blk % nb) * 32;
          for (int rr = 0; rr < CH; rr += 2) {
            const float a = Ys[(rr + (lane >> 5)) * ld + i0 + (lane & 31)];
            const float b = Ys[(rr + (lane >> 5)) * ld + j0 + (lane & 31)];
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }
  if (blocks == 1) {  // fold the four waves' sums in a fixed order (Ys is free: the loop ended on a barrier)
#pragma unroll
    for (int e = 0; e < 16; ++e) Ys[(wave * 16 + e) * 64 + lane] = acc[0][e];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        acc[0][e] = ((Ys[e * 64 + lane] + Ys[(16 + e) * 64 + lane]) + Ys[(32 + e) * 64 + lane]) + Ys[(48 + e) * 64 + lane];
    } else {
      return;  // wave 0 stores
    }
  }
  float* out = part + (int64_t)blockIdx.x * k * k;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int blk = wave + 4 * q;
    if (blk < blocks) {
      const int i0 = (blk / nb) * 32, j0 = (blk % nb) * 32;
      const int col = j0 + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = i0 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (row < k && col < k) out[row * k + col] = acc[q][e];
      }
    }
  }
}

// Q = Y . Rinv for a tall Y [n, k] fp32 and a k x k fp32 Rinv, fp32 matrix instructions.  One work-group
// per 64 rows, rows up to n_rows_out (>= n; rows past n count as zero).  Outputs, each optional:
//   Qf  [n, k] fp32;  Qt [n, k] in TU (the stored factor);  Ut [k, ldt] bf16, the transpose with its
//   columns n .. n_rows_out - 1 written as zero (K padding of the later products over tokens); with
//   `hilo` Ut is [2k, ldt]: rows 0 .. k-1 the bf16 rounding of Q^T, rows k .. 2k-1 the bf16 rounding of
//   the remainder, so that hi + lo carries Q to about 2^-17 relative through a bf16 matrix product.
template <typename TU>
__global__ __launch_bounds__(256) void tall_times_small_kernel(const float* __restrict__ Y, int64_t n, int k,
                                                               const float* __restrict__ Rinv,
                                                               float* __restrict__ Qf, TU* __restrict__ Qt,
                                                               bf16* __restrict__ Ut, int64_t ldt,
                                                               int64_t n_rows_out, int hilo) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kp = (k + 31) / 32 * 32, nb = kp / 32;
  const int ldy = kp + 1, ldr = (kp % 64 == 0) ? kp + 32 : kp;
  float* Ys = (float*)smem_raw;           // [64][ldy]
  float* Rs = Ys + 64 * ldy;              // [kp][ldr]
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  for (int e = tid; e < 64 * kp; e += 256) {
    const int r = e / kp, c = e % kp;
    Ys[r * ldy + c] = (r0 + r < n && c < k) ? Y[(r0 + r) * k + c] : 0.f;
  }
  for (int e = tid; e < kp * kp; e += 256) {
    const int r = e / kp, c = e % kp;
    Rs[r * ldr + c] = (r < k && c < k) ? Rinv[r * k + c] : 0.f;
  }
  __syncthreads();
  // 2 x nb output blocks of 32 x 32 over 4 waves
  for (int blk = wave; blk < 2 * nb; blk += 4) {
    const int m0 = (blk / nb) * 32, c0 = (blk % nb) * 32;
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    for (int kk = 0; kk < kp; kk += 2) {
      const float a = Ys[(m0 + (lane & 31)) * ldy + kk + (lane >> 5)];
      const float b = Rs[(kk + (lane >> 5)) * ldr + c0 + (lane & 31)];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
    const int col = c0 + (lane & 31);
    if (col < k) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = r0 + m0 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (row < n) {
          if (Qf) Qf[row * k + col] = acc[e];
          if (Qt) Qt[row * k + col] = from_f32<TU>(acc[e]);
        }
        if (Ut && row < n_rows_out) {
          const bf16 hi = row < n ? (bf16)acc[e] : (bf16)0.f;
          Ut[(int64_t)col * ldt + row] = hi;
          if (hilo) Ut[(int64_t)(k + col) * ldt + row] = row < n ? (bf16)(acc[e] - (float)hi) : (bf16)0.f;
        }
      }
    }
  }
}

// Omega [d_in, k] of the range finder as two bfloat16 matrices, Omega = hi + lo to about 2^-17 relative
// (one bfloat16 MFMA pass per part gives fp32-grade products with exact bf16 inputs).  Output layout
// [2k, ld] K-contiguous rows: row j = hi of column j, row k + j = lo of column j; entry (c, j) is the
// Philox normal of (token index := c, column j), scaled by 1 / sqrt(k) like S.  One thread per (4
// channels, column).  d_in % 4 == 0.
__global__ __launch_bounds__(256) void omega_hilo_kernel(SketchParams sk, int64_t d_in, int k, int64_t ld,
                                                         bf16* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // = q * k + j
  const int64_t nq = d_in / 4;
  if (idx >= nq * k) return;
  const int64_t q = idx / k;
  const int j = (int)(idx - q * k);
  uint32_t w[4];
  sketch_words(sk.key0, sk.key1, (uint64_t)q, (uint32_t)j, w);
  float z[4];
  normals_from_words<true>(w, sk.inv_sqrt_r, sk.neg2_ln2_over_r, z);
  bf16x4 hi, lo;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    hi[t] = (bf16)z[t];
    lo[t] = (bf16)(z[t] - (float)hi[t]);
  }
  *(bf16x4*)(out + (int64_t)j * ld + 4 * q) = hi;
  *(bf16x4*)(out + (int64_t)(k + j) * ld + 4 * q) = lo;
}

// Yr[i, j] = sum over splits of (part[s][i][j] + part[s][i][k + j]): folds the K splits and the hi / lo
// halves of X . [Omega_hi Omega_lo] in a fixed order.  One thread per element.
__global__ __launch_bounds__(256) void combine_hilo_kernel(const float* __restrict__ part, int splits, int64_t n,
                                                           int k, float* __restrict__ Yr) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n * k) return;
  const int64_t i = idx / k;
  const int j = (int)(idx - i * k);
  float sum = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float* row = part + ((int64_t)s * n + i) * (2 * k);
    sum += row[j] + row[k + j];
  }
  Yr[idx] = sum;
}

// Z [cols, k] = transpose of the sum over splits of (part[s][j][c] + part[s][k + j][c]), part[s] being
// [2k, cols] fp32: folds the K splits and the hi / lo halves of [Q_hi; Q_lo]^T-type products in a fixed
// order.  One thread per input column pair (c, j), coalesced reads.
__global__ __launch_bounds__(256) void combine_hilo_t_kernel(const float* __restrict__ part, int splits, int64_t cols,
                                                             int k, float* __restrict__ Z) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // = j * cols + c
  if (idx >= (int64_t)k * cols) return;
  const int64_t j = idx / cols, c = idx - j * cols;
  float sum = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float* p = part + (int64_t)s * 2 * k * cols;
    sum += p[j * cols + c] + p[(k + j) * cols + c];
  }
  Z[c * k + j] = sum;
}

// Ut [k, ld] = U^T with the columns n .. ld - 1 zeroed (ld = n rounded up to 64: the K padding of the
// products over tokens).  One thread per output element.
template <typename TU>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const TU* __restrict__ U, int64_t n, int k, int64_t ld,
                                                            bf16* __restrict__ Ut) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;  // = i * k + j: coalesced read
  if (idx >= ld * k) return;
  const int64_t i = idx / k;
  const int j = (int)(idx - i * k);
  Ut[(int64_t)j * ld + i] = i < n ? (bf16)to_f32(U[idx]) : (bf16)0.f;
}

// out = sum over splits of part[s] ([rows, cols] fp32 each), stored transposed ([cols, rows]) when
// TRANSPOSE, converted to TO.  One thread per input element (coalesced reads).
template <typename TO, bool TRANSPOSE>
__global__ __launch_bounds__(256) void reduce_store_kernel(const float* __restrict__ part, int splits, int64_t rows,
                                                           int64_t cols, TO* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cols) return;
  float sum = part[idx];
  for (int s = 1; s < splits; ++s) sum += part[(int64_t)s * rows * cols + idx];
  if (TRANSPOSE) {
    const int64_t r = idx / cols, c = idx - r * cols;
    out[c * rows + r] = from_f32<TO>(sum);
  } else {
    out[idx] = from_f32<TO>(sum);
  }
}

}  // namespace acc
