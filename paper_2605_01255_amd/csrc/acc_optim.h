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

}  // namespace acc
