// Small dense kernels of the RSVD compressor (Experimental Setup: randomized SVD of Halko et al.): the
// triangular factor R of a k x k Gram matrix and Yr.R^-1 by substitution, the middle steps of a Cholesky QR,
// with the Gram products and the helpers around them.  The large products (X.Omega, X^T.U, U^T.dY) run on the
// GEMM kernels.
#pragma once
#include "acc_common.h"
#include "acc_rng.h"

namespace acc {

constexpr int kRsvdMaxRank = 64;   // a k x k factorisation of this size runs on one wave, one matrix row per lane
constexpr int kRsvdMaxRankBlocked = 512;  // larger ranks: the same kernels on 64 x 64 diagonal blocks (blocked Cholesky)

__device__ __forceinline__ float lane_bcast(float v, int src_lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
}

// G [k, k] (symmetric positive semi-definite, fp32) -> the upper triangular factor R of G = R^T R with positive
// diagonal, for k <= K (K = 32 or 64), by ONE wave: lane i holds row i of the symmetric matrix (padded to K
// with the identity) in registers; at each step the pivot row goes through LDS to all lanes (same-address reads
// broadcast; v_readlane broadcasts of the same values measured 20 % slower).  The elimination is done in the
// square-root-free form (A = L D L^T: one reciprocal per step on the critical path, no square root), eight
// steps per trip of a rolled loop: after each trip the eight finished rows go to LDS and every lane's registers
// move down by eight columns, so register indices stay compile-time constants while the loop body stays small.
// Work done on columns that are already eliminated is harmless: those registers are never read again.  The k
// steps are a serial chain (LDS round trip, reciprocal, K multiply-adds): 11.9 us at K = 32, 38 us at K = 64.
// Output, in the form tall_solve_kernel copies to its LDS: Rimg [K * K + 2 K] floats, Rimg[t * K + c] = R[t][c]
// for t < c < k and zero elsewhere up to index K * K + K, then 1 / R[c][c] for c < k (zero for c >= k).  A pivot
// that is not positive beyond rounding (column j of the factored matrix depends on the earlier ones) is dropped:
// its reciprocal is stored as 0 and row j of R is zero, so the corresponding basis vector comes out as zero and
// the span of the others is unchanged.
template <int K>
__global__ __launch_bounds__(64) void chol_factor_kernel(const float* __restrict__ G, float* __restrict__ Rimg,
                                                         int k, int64_t ldg, const float* __restrict__ scale_ref,
                                                         float rel_tol) {
  // ldg: row stride of G.  scale_ref: when not null, the largest diagonal entry of the WHOLE matrix this block
  // belongs to (blocked factorisation: a trailing block that is nothing but rounding noise must be measured against
  // the matrix it came from, not against itself); null: the largest diagonal entry of G itself.  rel_tol: a pivot
  // at or below rel_tol times that scale counts as zero (1e-6 for one block; the blocked form passes its rank
  // times 2^-23, the size of the rounding noise that `rank` elimination steps leave on an exactly dependent column).
  __shared__ float rows[K][K + 1];
  __shared__ float scale[K];
  const int lane = threadIdx.x;
  float a[K];
  {  // every lane loads from a valid address (clamped), then selects: no branches around the loads
    const int lr = lane < k ? lane : k - 1;
#pragma unroll
    for (int c = 0; c < K; ++c) {
      const float g = G[lr * ldg + (c < k ? c : k - 1)];
      a[c] = (lane < k && c < k) ? g : (lane == c ? 1.f : 0.f);
    }
  }
  float diag = 0.f;
#pragma unroll
  for (int c = 0; c < K; ++c) diag = (c == lane && lane < k) ? a[c] : diag;
  float maxdiag = 0.f;
#pragma unroll
  for (int l = 0; l < K; ++l) {
    const float d = lane_bcast(diag, l);
    maxdiag = d > maxdiag ? d : maxdiag;
  }
  const float tol = (scale_ref ? *scale_ref : maxdiag) * rel_tol;
  float my_piv = 0.f;   // pivot of my row, 0 for a dropped one
  __shared__ __attribute__((aligned(16))) float bc[2][K];   // the pivot row of a step, for all lanes to read
#pragma unroll 1
  for (int jb = 0; jb < K; jb += 8) {
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int j = jb + jj;
      // lane j publishes its row (columns j .. of the current register window) through LDS: one wave, so LDS
      // operations complete in order and no hardware barrier is needed; two buffers alternate so that a step's
      // writes cannot overtake the previous step's reads
      float* row = bc[jj & 1];
      if (lane == j) {
#pragma unroll
        for (int c = jj & ~3; c < K; c += 4) *(f32x4*)(&row[c]) = f32x4{a[c], a[c + 1], a[c + 2], a[c + 3]};
      }
      // other lanes' writes become visible to this lane's reads only across a fence the compiler honours (without
      // it the reads are hoisted out of the loop as if no one else wrote); at wavefront scope it costs nothing
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      f32x4 rj[K / 4];
#pragma unroll
      for (int c = jj & ~3; c < K; c += 4) rj[c / 4] = *(const f32x4*)(&row[c]);
      const float piv = rj[jj / 4][jj % 4];
      const bool dead = !(piv > tol);
      // reciprocal: hardware estimate + one Newton step (about 1 ulp); the elimination needs no more, the
      // factor's own scaling below uses exact square roots
      float inv_p = __builtin_amdgcn_rcpf(piv);
      inv_p = fmaf(fmaf(-piv, inv_p, 1.f), inv_p, inv_p);
      inv_p = dead ? 0.f : inv_p;
      my_piv = lane == j ? (dead ? 0.f : piv) : my_piv;
      const float t = lane > j ? a[jj] * inv_p : 0.f;
#pragma unroll
      for (int c = jj + 1; c < K; ++c) a[c] = fmaf(-t, rj[c / 4][c % 4], a[c]);
    }
    if (lane >= jb && lane < jb + 8) {
#pragma unroll
      for (int c = 0; c < K; ++c)
        if (jb + c < K) rows[lane][jb + c] = a[c];
    }
#pragma unroll
    for (int c = 0; c < K - 8; ++c) a[c] = a[c + 8];
#pragma unroll
    for (int c = K - 8; c < K; ++c) a[c] = 0.f;
  }
  if (lane < K) scale[lane] = (lane < k && my_piv > 0.f) ? 1.f / sqrtf(my_piv) : 0.f;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < (K * K + 2 * K) / 64; ++i) {
    const int e = lane + 64 * i, t = e / K, c = e % K;
    float v = 0.f;
    if (t < K) v = (t < c && c < k) ? rows[t][c] * scale[t] : 0.f;
    else if (t == K + 1) v = scale[c];
    Rimg[e] = v;
  }
}

// out[0] = the largest diagonal entry of the symmetric matrix G [k, k] (row stride ldg).  One wave.
__global__ __launch_bounds__(64) void diag_max_kernel(const float* __restrict__ G, int k, int64_t ldg,
                                                      float* __restrict__ out) {
  float m = 0.f;
  for (int i = threadIdx.x; i < k; i += 64) {
    const float d = G[i * ldg + i];
    m = d > m ? d : m;
  }
#pragma unroll
  for (int l = 0; l < 64; ++l) {
    const float d = lane_bcast(m, l);
    if (threadIdx.x == 0 && l > 0) m = d > m ? d : m;
  }
  if (threadIdx.x == 0) out[0] = m;
}

// Q = Y . R^-1 for a tall Y [n, k] fp32 by forward substitution along each row, q_c = (y_c - sum_{t<c} q_t
// R[t][c]) / R[c][c]: one row per lane, the row in registers, R read from LDS (all lanes read the same address).
// No explicit inverse is formed.  Columns are taken eight at a time in a rolled loop: substitution inside the
// block, then the block's contribution is removed from all later columns and the registers move down by eight,
// so register indices are compile-time constants and the loop body stays small.  Updates that fall on columns
// past the end touch registers that are never read.
// Rimg as written by chol_factor_kernel<K>.  Outputs, each optional, rows up to n_rows_out (>= n; rows past n
// count as zero):
//   Qf  [n, k] fp32;  Qt [n, k] in TU (the stored factor);  Ut [k, ldt] bf16, the transpose with its
//   columns n .. n_rows_out - 1 written as zero (K padding of the later products over tokens); with
//   `hilo` Ut is [2k, ldt]: rows 0 .. k-1 the bf16 rounding of Q^T, rows k .. 2k-1 the bf16 rounding of
//   the remainder, so that hi + lo carries Q to about 2^-17 relative through a bf16 matrix product.
// Grid: ceil(n_rows_out / 64) x 64 threads.  k % 8 == 0, k <= K.
template <int K, typename TU>
__global__ __launch_bounds__(64) void tall_solve_kernel(const float* __restrict__ Y, int64_t n, int k,
                                                        const float* __restrict__ Rimg, float* __restrict__ Qf,
                                                        TU* __restrict__ Qt, bf16* __restrict__ Ut, int64_t ldt,
                                                        int64_t n_rows_out, int hilo, int64_t ldy, int64_t ldq,
                                                        int lo_rows) {
  // ldy: row stride of Y; ldq: row stride of Qf and Qt (a column block of a wider matrix passes the wide stride);
  // lo_rows: row of Ut where the lo parts start (the full rank when this call handles one column block)
  // Rs[t * K + c] = R[t][c] for t < c < k, zero elsewhere; one spare row: the update of the last columns reads
  // up to K - 9 elements past a row's end
  __shared__ __attribute__((aligned(16))) float Rs[K * K + 2 * K];
  const float* Ds = Rs + K * K + K;
  const int tid = threadIdx.x;
  {
    constexpr int V4 = (K * K + 2 * K) / 4, PER = (V4 + 63) / 64;
    f32x4 tmp[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + 64 * i;
      tmp[i] = *(const f32x4*)(Rimg + 4 * (e < V4 ? e : V4 - 1));
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + 64 * i;
      if (e < V4) *(f32x4*)(&Rs[4 * e]) = tmp[i];
    }
  }
  const int64_t row = (int64_t)blockIdx.x * 64 + tid;
  float y[K];
#pragma unroll
  for (int c = 0; c < K; c += 4) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (row < n && c < k) v = *(const f32x4*)(Y + row * ldy + c);
#pragma unroll
    for (int t = 0; t < 4; ++t) y[c + t] = v[t];
  }
  __syncthreads();
#pragma unroll 1
  for (int cb = 0; cb < k; cb += 8) {
    float q[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      float s = y[jj];
#pragma unroll
      for (int t = 0; t < jj; ++t) s = fmaf(-q[t], Rs[(cb + t) * K + cb + jj], s);
      q[jj] = s * Ds[cb + jj];
    }
    // four later columns at a time: their eight R entries each are read one group ahead of the multiplies; the
    // fences keep the compiler from hoisting every read of the trip to its top (450 registers, spills)
    f32x4 r[8], rn[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) r[jj] = *(const f32x4*)(&Rs[(cb + jj) * K + cb + 8]);
#pragma unroll
    for (int c4 = 8; c4 < K; c4 += 4) {
      if (c4 + 4 < K) {
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) rn[jj] = *(const f32x4*)(&Rs[(cb + jj) * K + cb + c4 + 4]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
#pragma unroll
        for (int u = 0; u < 4; ++u) y[c4 + u] = fmaf(-q[jj], r[jj][u], y[c4 + u]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) r[jj] = rn[jj];
    }
    if (row < n) {
      if (Qf) {
        *(f32x4*)(Qf + row * ldq + cb) = f32x4{q[0], q[1], q[2], q[3]};
        *(f32x4*)(Qf + row * ldq + cb + 4) = f32x4{q[4], q[5], q[6], q[7]};
      }
      if (Qt) {
        if constexpr (sizeof(TU) == 2) {
          bf16x8 o;
#pragma unroll
          for (int t = 0; t < 8; ++t) o[t] = (bf16)q[t];
          *(bf16x8*)(Qt + row * ldq + cb) = o;
        } else {
          *(f32x4*)(Qt + row * ldq + cb) = f32x4{q[0], q[1], q[2], q[3]};
          *(f32x4*)(Qt + row * ldq + cb + 4) = f32x4{q[4], q[5], q[6], q[7]};
        }
      }
    }
    if (Ut && row < n_rows_out) {
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const bf16 hi = row < n ? (bf16)q[jj] : (bf16)0.f;
        Ut[(int64_t)(cb + jj) * ldt + row] = hi;
        if (hilo) Ut[(int64_t)(lo_rows + cb + jj) * ldt + row] = row < n ? (bf16)(q[jj] - (float)hi) : (bf16)0.f;
      }
    }
#pragma unroll
    for (int c = 0; c < K - 8; ++c) y[c] = y[c + 8];
#pragma unroll
    for (int c = K - 8; c < K; ++c) y[c] = 0.f;
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
