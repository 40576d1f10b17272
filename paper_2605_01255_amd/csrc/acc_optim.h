// Optimizer step on the factored gradient (Sec. 4, update strategy (ii)): Adam moments at the size of the small
// factor.  This kernel is the element-wise part; the step back to weight space is a product of the two factors
// accumulated into W by the GEMM kernels' epilogue.
#pragma once
#include "acc_common.h"

namespace acc {

struct AdamParams {
  float beta1, beta2;
  float inv_c1, inv_c2;  // 1 / (1 - beta1^step), 1 / (1 - beta2^step), computed on the host in double
  float eps;
};

// M <- beta1 M + (1 - beta1) g;  V <- beta2 V + (1 - beta2) g^2;  N = (M inv_c1) / (sqrt(V inv_c2) + eps).
// g: the projected gradient (the small factor itself, or the fp32 product with the projector).  Four consecutive
// elements per lane; count % 4 == 0.  M, V fp32 in place; N in the factor type.
template <typename TG, typename TN>
__global__ __launch_bounds__(256) void adam_factor_kernel(const TG* __restrict__ Gr, float* __restrict__ M,
                                                          float* __restrict__ V, TN* __restrict__ N,
                                                          int64_t count, AdamParams h) {
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e >= count) return;
  float g[4];
  if constexpr (sizeof(TG) == 2) {
    const bf16x4 v = *(const bf16x4*)(Gr + e);
#pragma unroll
    for (int t = 0; t < 4; ++t) g[t] = (float)v[t];
  } else {
    const f32x4 v = *(const f32x4*)(Gr + e);
#pragma unroll
    for (int t = 0; t < 4; ++t) g[t] = v[t];
  }
  f32x4 m = *(const f32x4*)(M + e), v2 = *(const f32x4*)(V + e);
  float nrm[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    m[t] = h.beta1 * m[t] + (1.f - h.beta1) * g[t];
    v2[t] = h.beta2 * v2[t] + (1.f - h.beta2) * g[t] * g[t];
    nrm[t] = (m[t] * h.inv_c1) / (sqrtf(v2[t] * h.inv_c2) + h.eps);
  }
  *(f32x4*)(M + e) = m;
  *(f32x4*)(V + e) = v2;
  if constexpr (sizeof(TN) == 2) {
    bf16x4 o;
#pragma unroll
    for (int t = 0; t < 4; ++t) o[t] = (bf16)nrm[t];
    *(bf16x4*)(N + e) = o;
  } else {
    f32x4 o;
#pragma unroll
    for (int t = 0; t < 4; ++t) o[t] = nrm[t];
    *(f32x4*)(N + e) = o;
  }
}

// Projected gradient and moments in one pass (bf16 small factor): R = T1 . Gr with T1 [k, r] fp32 taken as the sum
// of two bfloat16 parts (hi = rounding of T1, lo = rounding of the remainder; two matrix instructions per step
// carry T1 to about 2^-17 relative, Gr is bfloat16 already), then the Adam update of adam_factor_kernel on the
// accumulators.  Element (a, o) of R, M, V and N sits at a * c_sm + o * c_sn (either orientation of the small
// factor); Gr element (j, o) at j * b_sk + o * b_sn.  Grid: x = ceil(k / 64), y = ceil(d_out / 64); 4 waves, one
// 32 x 32 block each.
struct ProjectAdamParams {
  const float* T1;      // [k, r] dense
  const bf16* Gr;
  float* M;
  float* V;
  bf16* N;
  int64_t k, r, d_out;
  int64_t b_sk, b_sn, c_sm, c_sn;
  AdamParams h;
};

__global__ __launch_bounds__(256) void project_adam_kernel(ProjectAdamParams p) {
  // With k / 64 x d_out / 64 work-groups the kernel runs at the latency of its dependent global loads, not at any
  // throughput limit: few, long stages (128 elements of the contraction), the next stage's operands and the
  // moments requested before the current stage is multiplied.
  constexpr int BK = 128, LDT = BK + 8;
  __shared__ __attribute__((aligned(16))) bf16 Ahi[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Alo[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Bs[64 * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.x * 64, n0 = (int64_t)blockIdx.y * 64;
  const float* __restrict__ T1 = p.T1;
  const bf16* __restrict__ Gr = p.Gr;
  float* __restrict__ Mp = p.M;
  float* __restrict__ Vp = p.V;
  bf16* __restrict__ Np = p.N;
  const bool n_major = p.b_sn == 1;   // Gr [r, d_out]

  f32x4 ta[8];
  bf16x8 tb[4];
  auto fetch = [&](int64_t k0) {
    // T1 rows are dense and r % 8 == 0: four floats per load
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int idx = tid + 256 * i, mm = idx >> 5, kq = (idx & 31) * 4;
      const int64_t gm = m0 + mm, gk = k0 + kq;
      ta[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (gm < p.k && gk < p.r) ta[i] = *(const f32x4*)(T1 + gm * p.r + gk);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + 256 * i;
#pragma unroll
      for (int t = 0; t < 8; ++t) tb[i][t] = (bf16)0.f;
      if (n_major) {  // eight output channels of one j per load (d_out % 8 == 0)
        const int kk = idx >> 3, nq = (idx & 7) * 8;
        const int64_t gn = n0 + nq, gk = k0 + kk;
        if (gn < p.d_out && gk < p.r) tb[i] = *(const bf16x8*)(Gr + gk * p.b_sk + gn);
      } else {        // Gr [d_out, r]: eight j of one output channel per load (r % 8 == 0)
        const int nn = idx >> 4, kq = (idx & 15) * 8;
        const int64_t gn = n0 + nn, gk = k0 + kq;
        if (gn < p.d_out && gk < p.r) tb[i] = *(const bf16x8*)(Gr + gn * p.b_sn + gk);
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int idx = tid + 256 * i, mm = idx >> 5, kq = (idx & 31) * 4;
      bf16x4 hi, lo;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        hi[t] = (bf16)ta[i][t];
        lo[t] = (bf16)(ta[i][t] - (float)hi[t]);
      }
      *(bf16x4*)(&Ahi[mm * LDT + kq]) = hi;
      *(bf16x4*)(&Alo[mm * LDT + kq]) = lo;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + 256 * i;
      if (n_major) {  // scattered into the [channel][j] tile
        const int kk = idx >> 3, nq = (idx & 7) * 8;
#pragma unroll
        for (int t = 0; t < 8; ++t) Bs[(nq + t) * LDT + kk] = tb[i][t];
      } else {
        const int nn = idx >> 4, kq = (idx & 15) * 8;
        *(bf16x8*)(&Bs[nn * LDT + kq]) = tb[i];
      }
    }
  };

  fetch(0);
  // lane holds column (lane & 31), rows 8 * (i / 4) + 4 * (lane >> 5) + i % 4 of its wave's 32 x 32 block
  const int64_t gn = n0 + wn * 32 + (lane & 31);
  float m[16], v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t gm = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    const int64_t e = gm * p.c_sm + gn * p.c_sn;
    const bool in = gm < p.k && gn < p.d_out;
    m[i] = in ? Mp[e] : 0.f;
    v[i] = in ? Vp[e] : 0.f;
  }
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  for (int64_t k0 = 0; k0 < p.r; k0 += BK) {
    stage();
    __syncthreads();
    if (k0 + BK < p.r) fetch(k0 + BK);
    const int arow = (wm * 32 + (lane & 31)) * LDT, brow = (wn * 32 + (lane & 31)) * LDT;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      const bf16x8 b = *(const bf16x8*)(&Bs[brow + kk + (lane >> 5) * 8]);
      const bf16x8 ah = *(const bf16x8*)(&Ahi[arow + kk + (lane >> 5) * 8]);
      const bf16x8 al = *(const bf16x8*)(&Alo[arow + kk + (lane >> 5) * 8]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b, acc, 0, 0, 0);
    }
    __syncthreads();
  }
  if (gn >= p.d_out) return;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int64_t gm = m0 + wm * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    if (gm < p.k) {
      const int64_t e = gm * p.c_sm + gn * p.c_sn;
      const float g = acc[i];
      const float mi = p.h.beta1 * m[i] + (1.f - p.h.beta1) * g;
      const float vi = p.h.beta2 * v[i] + (1.f - p.h.beta2) * g * g;
      Mp[e] = mi;
      Vp[e] = vi;
      Np[e] = (bf16)((mi * p.h.inv_c1) / (sqrtf(vi * p.h.inv_c2) + p.h.eps));
    }
  }
}

}  // namespace acc
