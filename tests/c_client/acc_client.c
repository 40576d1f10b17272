/* A client of libacc.so written against include/acc.h alone (C, HIP runtime for memory; no Python, no
 * torch): one forward + backward of a small float32 layer, checked on the host against plain loops for
 * the exact products (Def. 3.1) and against the factorisation identity dW = Xs.Gr (Sec. 4).
 * Exit status 0 = all checks passed. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/acc.h"

#define CHECK_HIP(x)                                                     \
  do {                                                                   \
    hipError_t e_ = (x);                                                 \
    if (e_ != hipSuccess) {                                              \
      fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); \
      return 2;                                                          \
    }                                                                    \
  } while (0)

static float pattern(int i, int j, int salt) { return (float)(((i * 131 + j * 71 + salt * 17) % 23) - 11) / 16.0f; }

int main(void) {
  const int n = 200, d_in = 72, d_out = 40, r = 16;
  acc_linear_desc d;
  d.n = n; d.d_in = d_in; d.d_out = d_out; d.r = r;
  d.ldx = 0; d.ldw = 0; d.ldy = 0;
  d.seed = 1234; d.row_offset = 0;
  d.io_dtype = ACC_F32; d.factor_dtype = ACC_F32; d.dw_dtype = ACC_F32;
  d.flags = 0; d.ldf = 0;
  if (acc_version() < 100) { fprintf(stderr, "bad version\n"); return 1; }

  float *hX = malloc(sizeof(float) * n * d_in), *hW = malloc(sizeof(float) * d_in * d_out);
  float *hdY = malloc(sizeof(float) * n * d_out);
  float *hY = malloc(sizeof(float) * n * d_out), *hdX = malloc(sizeof(float) * n * d_in);
  float *hXs = malloc(sizeof(float) * d_in * r), *hGr = malloc(sizeof(float) * r * d_out);
  float *hdW = malloc(sizeof(float) * d_in * d_out);
  for (int i = 0; i < n; ++i) for (int c = 0; c < d_in; ++c) hX[i * d_in + c] = pattern(i, c, 1);
  for (int c = 0; c < d_in; ++c) for (int o = 0; o < d_out; ++o) hW[c * d_out + o] = pattern(c, o, 2) / 8.0f;
  for (int i = 0; i < n; ++i) for (int o = 0; o < d_out; ++o) hdY[i * d_out + o] = pattern(i, o, 3) / 64.0f;

  const size_t ws_f = acc_linear_workspace_bytes(&d, 0), ws_b = acc_linear_workspace_bytes(&d, 1);
  if (ws_f == 0 || ws_b == 0) { fprintf(stderr, "descriptor refused\n"); return 1; }
  float *X, *W, *dY, *Y, *dX, *Xs, *Gr, *dW;
  void* ws;
  CHECK_HIP(hipMalloc((void**)&X, sizeof(float) * n * d_in));
  CHECK_HIP(hipMalloc((void**)&W, sizeof(float) * d_in * d_out));
  CHECK_HIP(hipMalloc((void**)&dY, sizeof(float) * n * d_out));
  CHECK_HIP(hipMalloc((void**)&Y, sizeof(float) * n * d_out));
  CHECK_HIP(hipMalloc((void**)&dX, sizeof(float) * n * d_in));
  CHECK_HIP(hipMalloc((void**)&Xs, sizeof(float) * d_in * r));
  CHECK_HIP(hipMalloc((void**)&Gr, sizeof(float) * r * d_out));
  CHECK_HIP(hipMalloc((void**)&dW, sizeof(float) * d_in * d_out));
  CHECK_HIP(hipMalloc(&ws, ws_f > ws_b ? ws_f : ws_b));
  CHECK_HIP(hipMemcpy(X, hX, sizeof(float) * n * d_in, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(W, hW, sizeof(float) * d_in * d_out, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dY, hdY, sizeof(float) * n * d_out, hipMemcpyHostToDevice));

  int rc = acc_linear_fwd(&d, X, W, Y, Xs, ws, ws_f, NULL);
  if (rc != ACC_OK) { fprintf(stderr, "acc_linear_fwd: %s\n", acc_status_string(rc)); return 1; }
  rc = acc_linear_bwd(&d, dY, W, Xs, dX, Gr, dW, ws, ws_b, NULL);
  if (rc != ACC_OK) { fprintf(stderr, "acc_linear_bwd: %s\n", acc_status_string(rc)); return 1; }
  CHECK_HIP(hipDeviceSynchronize());
  CHECK_HIP(hipMemcpy(hY, Y, sizeof(float) * n * d_out, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hdX, dX, sizeof(float) * n * d_in, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hXs, Xs, sizeof(float) * d_in * r, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hGr, Gr, sizeof(float) * r * d_out, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hdW, dW, sizeof(float) * d_in * d_out, hipMemcpyDeviceToHost));

  double worst = 0.0;
  for (int i = 0; i < n; ++i)
    for (int o = 0; o < d_out; ++o) {
      double s = 0.0;
      for (int c = 0; c < d_in; ++c) s += (double)hX[i * d_in + c] * hW[c * d_out + o];
      const double e = fabs(s - hY[i * d_out + o]);
      if (e > worst) worst = e;
    }
  for (int i = 0; i < n; ++i)
    for (int c = 0; c < d_in; ++c) {
      double s = 0.0;
      for (int o = 0; o < d_out; ++o) s += (double)hdY[i * d_out + o] * hW[c * d_out + o];
      const double e = fabs(s - hdX[i * d_in + c]);
      if (e > worst) worst = e;
    }
  for (int c = 0; c < d_in; ++c)
    for (int o = 0; o < d_out; ++o) {
      double s = 0.0;
      for (int j = 0; j < r; ++j) s += (double)hXs[c * r + j] * hGr[j * d_out + o];
      const double e = fabs(s - hdW[c * d_out + o]);
      if (e > worst) worst = e;
    }
  /* optimizer update from the factors, left factor as projector, first step from zero moments with eps = 0:
     the normalised step is sign(Gr), so W moves by -lr * Xs . sign(Gr) (checked here with plain loops) */
  {
    float *M, *V;
    void* wso;
    const size_t ws_o = acc_lowrank_workspace_bytes(&d, 0);
    if (ws_o == 0) { fprintf(stderr, "optimizer descriptor refused\n"); return 1; }
    CHECK_HIP(hipMalloc((void**)&M, sizeof(float) * r * d_out));
    CHECK_HIP(hipMalloc((void**)&V, sizeof(float) * r * d_out));
    CHECK_HIP(hipMalloc(&wso, ws_o));
    CHECK_HIP(hipMemset(M, 0, sizeof(float) * r * d_out));
    CHECK_HIP(hipMemset(V, 0, sizeof(float) * r * d_out));
    acc_adamw_hyper h;
    h.lr = 0.01f; h.beta1 = 0.9f; h.beta2 = 0.999f; h.eps = 0.0f; h.weight_decay = 0.0f; h.scale = 1.0f;
    h.step = 1; h.reserved = 0;
    rc = acc_lowrank_adamw_step(&d, &h, NULL, 0, Xs, Gr, M, V, W, wso, ws_o, NULL);
    if (rc != ACC_OK) { fprintf(stderr, "acc_lowrank_adamw_step: %s\n", acc_status_string(rc)); return 1; }
    CHECK_HIP(hipDeviceSynchronize());
    float* hW1 = malloc(sizeof(float) * d_in * d_out);
    CHECK_HIP(hipMemcpy(hW1, W, sizeof(float) * d_in * d_out, hipMemcpyDeviceToHost));
    for (int c = 0; c < d_in; ++c)
      for (int o = 0; o < d_out; ++o) {
        double s = 0.0;
        for (int j = 0; j < r; ++j) {
          const float g = hGr[j * d_out + o];
          s += (double)hXs[c * r + j] * (g > 0.f ? 1.0 : (g < 0.f ? -1.0 : 0.0));
        }
        const double e = fabs((double)hW[c * d_out + o] - 0.01 * s - hW1[c * d_out + o]);
        if (e > worst) worst = e;
      }
    h.step = 0;
    if (acc_lowrank_adamw_step(&d, &h, NULL, 0, Xs, Gr, M, V, W, wso, ws_o, NULL) != ACC_ERR_INVALID_ARG) return 1;
  }
  /* a refused call must come back as an error code, not a crash */
  d.r = 20;
  const int refused = acc_linear_fwd(&d, X, W, Y, Xs, ws, ws_f, NULL);
  printf("worst absolute error %.3g, refused call -> %s\n", worst, acc_status_string(refused));
  if (!(worst < 1e-4) || refused != ACC_ERR_SHAPE) return 1;
  printf("C client OK\n");
  return 0;
}
