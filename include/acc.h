/*
 * acc.h -- C ABI of libacc.so: the compressed linear layer of activation-gradient
 * co-compression (paper Sec. 4; operator workflow of Def. 3.1) for AMD MI355X (gfx950).
 *
 * Notation (row-major everywhere):
 *   X  [n, d_in]      input activation          W  [d_in, d_out]  weight
 *   Y  [n, d_out]     exact output  Y = X.W     dY [n, d_out]     incoming gradient
 *   S  [n, r]         random-projection compressor, i.i.d. N(0, 1/r); NEVER stored:
 *                     S[i, j] is a pure function of (seed, row_offset + i, j)
 *   Xs [d_in, r]      Xs = X^T.S   the only activation kept for backward
 *   dX [n, d_in]      dX = dY.W^T  exact input gradient
 *   Gr [r, d_out]     Gr = S^T.dY  small factor of the weight gradient
 *   dW [d_in, d_out]  dW = Xs.Gr   factored weight gradient, materialised on request
 *   dB [d_out]        dB = 1^T.dY  gradient of a bias broadcast over tokens (exact)
 *
 * With ACC_FLAG_W_OUT_IN the weight side is in the paper's own orientation (Def. 3.1: Z = X.W^T;
 * Sec. 4): W [d_out, d_in], Gr [d_out, r] = dY^T.S, dW [d_out, d_in] = Gr.Xs^T.  X, Y, dY, dX and
 * Xs are unchanged, and every result equals the transpose of its default-orientation counterpart.
 *
 * Random stream: Philox4x32-10 with key (seed low word, seed high word) and counter
 * ((g >> 2) low word, j, 0, g >> 34), g = row_offset + i; output word w of the call is
 * token 4*(g >> 2) + w of column j.  u = ((x >> 9) + 0.5) * 2^-23; Box-Muller on the word
 * pairs (x0, x1), (x2, x3): z_even = R cos(theta), z_odd = R sin(theta),
 * R = sqrt(-2 ln u_first), theta = 2 pi u_second; S = z / sqrt(r).
 *
 * Ownership and behaviour common to every call:
 *   - every data pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or keeps one and never synchronises: a call only enqueues kernels
 *     on `stream` (a hipStream_t passed as void*; NULL = the default stream);
 *   - X, W, Y, dY, dX, Xs, Gr, dW and the workspace must be 16-byte aligned;
 *   - a workspace is scratch for the duration of a call's kernels: calls that share one must be ordered on
 *     one stream (or by events); the library is re-entrant otherwise and keeps no state between calls
 *     except per-kernel launch attributes it sets once;
 *   - return value 0 = success, negative = one of ACC_ERR_*; on error nothing is launched;
 *   - no C++ exception crosses this boundary; the library runs on gfx950 only.
 */
#ifndef ACC_H_
#define ACC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ACC_F32 = 0, ACC_BF16 = 1 } acc_dtype;

enum {
  ACC_OK = 0,
  ACC_ERR_INVALID_ARG = -1, /* NULL descriptor or required pointer, unknown flag            */
  ACC_ERR_SHAPE = -2,       /* a size is <= 0 or above its limit (n <= 2^30, d_in, d_out <= 2^21,
                               r <= 2^16), r % 8 != 0, d_in % 8 or d_out % 8 != 0,
                               a row stride (ldx, ldw, ldy, ldf) smaller than the row or not a multiple of 8,
                               row_offset % 4 != 0                                           */
  ACC_ERR_ALIGN = -3,       /* a pointer is not 16-byte aligned                              */
  ACC_ERR_DTYPE = -4,       /* a dtype field is not ACC_F32 / ACC_BF16                       */
  ACC_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than acc_linear_workspace_bytes()   */
  ACC_ERR_HIP = -6          /* HIP runtime error, or the current device is not gfx950        */
};

enum {
  ACC_FLAG_SKIP_SKETCH = 1u, /* forward only: leave Xs untouched (several linears that share
                                one input, e.g. q/k/v, keep a single Xs; Sec. 5.1)           */
  ACC_FLAG_ONE_LAUNCH = 2u,  /* run the exact GEMM and the sketch of a pass as ONE kernel
                                launch (their work-groups interleaved in one grid) when the
                                shape allows it (bf16, r % 128 == 0, >= 192 output tiles of
                                256 x 256); otherwise ignored.  Results are identical; on
                                MI355X the default (two launches) is measured ~5 % faster. */
  ACC_FLAG_W_OUT_IN = 4u,    /* W is [d_out, ldw >= d_in] (the layout of torch.nn.Linear.weight
                                and of the paper's Def. 3.1); Gr is then [d_out, r] and dW
                                [d_out, d_in].  ACC_FLAG_ONE_LAUNCH is ignored with it.          */
  ACC_FLAG_RSVD_POWER_1 = 1u << 8, /* acc_linear_fwd_rsvd only: one round of subspace iteration after the  */
  ACC_FLAG_RSVD_POWER_2 = 2u << 8, /* range finder (two, three): Z = orth(X^T.U), U = orth(X.Z); refused   */
  ACC_FLAG_RSVD_POWER_3 = 3u << 8, /* by the random-projection calls, ignored by acc_linear_bwd_rsvd.  Each
                                      round costs two more passes over X.                                  */
  ACC_FLAG_DW_ACCUMULATE = 8u /* backward only, with dW != NULL: dW += Xs.Gr, not dW = Xs.Gr
                                (gradient accumulation over micro-batches on the dense gradient,
                                Sec. 4 update strategy (i)).  A float dW is rounded once per call;
                                a bfloat16 dW rounds the product and then the sum.               */
};

#define ACC_FLAG_RSVD_POWER_SHIFT 8 /* flags bits 8..9: rounds of subspace iteration, 0..3 */

typedef struct acc_linear_desc {
  int64_t n;            /* tokens (batch x sequence)                                         */
  int64_t d_in;         /* input features,  multiple of 8                                    */
  int64_t d_out;        /* output features, multiple of 8                                    */
  int64_t r;            /* sketch rank, multiple of 8                                        */
  int64_t ldx;          /* row stride of X and dX in elements; 0 = d_in                      */
  int64_t ldw;          /* row stride of W in elements;        0 = d_out (d_in with W_OUT_IN) */
  int64_t ldy;          /* row stride of Y and dY in elements; 0 = d_out                     */
  uint64_t seed;        /* Philox key                                                        */
  uint64_t row_offset;  /* global index of local token 0 (multiple of 4); 0 on one GPU      */
  int32_t io_dtype;     /* acc_dtype of X, W, Y, dY, dX                                      */
  int32_t factor_dtype; /* acc_dtype of Xs and Gr                                            */
  int32_t dw_dtype;     /* acc_dtype of the dense dW (ignored when dW == NULL)               */
  uint32_t flags;       /* ACC_FLAG_*                                                        */
  int64_t ldf;          /* row stride, in elements, of the factors whose rows hold r elements: Xs
                           [d_in, r] and, under ACC_FLAG_W_OUT_IN, Gr [d_out, r]; 0 = r (dense);
                           otherwise >= r and a multiple of 8.  Lets a call write its factor into a
                           column block of a wider matrix (stacked factors, see acc_linear_dw).      */
} acc_linear_desc;

/* Bytes of device workspace the forward (is_backward == 0) or backward call needs for the
 * split-token fp32 partials of the sketch.  Returns 0 for an invalid descriptor. */
size_t acc_linear_workspace_bytes(const acc_linear_desc* desc, int is_backward);

/* Forward of the compressed linear operator (Def. 3.1: the output is exact, the input is
 * compressed and stored; Sec. 4: the stored factor).  Computes Y = X.W and, unless
 * ACC_FLAG_SKIP_SKETCH is set, Xs = X^T.S with S regenerated from (seed, row_offset).
 * X [n, ldx], W [d_in, ldw] are read; Y [n, ldy] and Xs [d_in, ldf] (columns 0 .. r-1 of each row) are overwritten.
 * workspace: ws_bytes >= acc_linear_workspace_bytes(desc, 0); contents are scratch. */
int acc_linear_fwd(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* Xs,
                   void* workspace, size_t ws_bytes, void* stream);

/* acc_linear_fwd for callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, kernels and results, but the split-token
 * partial tiles of the sketch go to a static device array inside the library, ACC_STATIC_SCRATCH_BYTES
 * (32 MiB) per GPU, held until the process ends.  The call allocates nothing.  A descriptor whose
 * acc_linear_workspace_bytes(desc, 0) exceeds that size returns ACC_ERR_WORKSPACE and launches nothing (the
 * 3B-shaped projection at r = 256 needs 31.5 MB and fits; with ACC_FLAG_SKIP_SKETCH nothing is needed).
 * All calls on one GPU share the array: calls that may overlap there (different streams without an event
 * between them, several host threads) race on it; order them, or use acc_linear_fwd with workspaces of
 * their own.  Nothing in the array has to be cleared between calls: every partial a call reads it has
 * written before. */
#define ACC_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int acc_linear_fwd_static(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* Xs,
                          void* stream);

/* Backward (Def. 3.1 and Thm 3.2.2(a): dX = dY.W^T is exact; Sec. 4: the weight gradient is
 * kept as two rank-r factors).  Computes dX [n, ldx], Gr = S^T.dY [r, d_out] (dense) and, when
 * dW != NULL, the dense dW = Xs.Gr [d_in, d_out] (Sec. 4, update strategy (i)).
 * dY [n, ldy], W and Xs (as written by acc_linear_fwd with the same seed / row_offset / r)
 * are read.  Xs may be NULL when dW is NULL. */
int acc_linear_bwd(const acc_linear_desc* desc, const void* dY, const void* W, const void* Xs,
                   void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes, void* stream);

/* The dense weight gradient from the two factors alone (Sec. 4, update strategy (i): full-gradient
 * reconstruction), as a call of its own: dW [d_in, d_out] = Xs.Gr, or += with ACC_FLAG_DW_ACCUMULATE (under
 * ACC_FLAG_W_OUT_IN dW [d_out, d_in] = Gr.Xs^T).  Xs [d_in, ldf] and Gr ([r, d_out] dense, or [d_out, ldf]) of
 * factor_dtype are read; only d_in, d_out, r, ldf, factor_dtype, dw_dtype and those two flags of desc matter (n
 * must be valid).  No workspace.
 * Accumulation over micro-batches WITHOUT a dense gradient (the paper stops at one batch; the factored form
 * adds up by stacking): micro-batch m of M runs acc_linear_fwd / acc_linear_bwd with rank r, ldf = M r, Xs
 * pointing at column m r of a stacked left factor [d_in, M r], Gr at row m r of a stacked small factor
 * [M r, d_out] (column m r of [d_out, M r] under ACC_FLAG_W_OUT_IN), dW = NULL, and a row_offset (or seed) of
 * its own so that the batches draw independent rows of S.  Then sum_m Xs_m.Gr_m = Xs_stack.Gr_stack exactly: the
 * stacked pair is a rank-M r factored gradient that acc_linear_dw (r := M r, ldf = 0), acc_lowrank_projector and
 * acc_lowrank_adamw_step take like any other; 2 M r (d_in + d_out) bytes are held instead of d_in d_out. */
int acc_linear_dw(const acc_linear_desc* desc, const void* Xs, const void* Gr, void* dW, void* stream);

/* The exact products on 8-bit floating-point operands (a widening of Def. 3.1's exact path; the paper itself
 * computes in bf16): for callers that hold 8-bit copies of X, W and dY next to the bf16 tensors (the usual fp8
 * training recipe: a cast with a per-tensor scale), F1 and B1 run on the fp8 matrix instructions, twice the bf16
 * rate at half the operand bytes; everything else of the path (the sketches of the bf16 X and dY, the factors,
 * the dense dW) is unchanged.
 *   X8 [n, ldx], dY8 [n, ldy], W8 (shape and stride of W): one byte per element, OCP fp8 e4m3 (dY8 may be e5m2:
 *   dy8_format); same strides, counted in elements, as their bf16 counterparts, but here ldx, ldw and ldy must be
 *   multiples of 16.
 *   Y  = scale * (X8 . W8)    (bf16, fp32 accumulation; scale = product of the two dequantisation scales)
 *   dX = scale * (dY8 . W8^T)
 * X / dY (bf16) are read by the sketch only (X and Xs may be NULL with ACC_FLAG_SKIP_SKETCH).  io_dtype must be
 * ACC_BF16.  The contraction length (d_in forward, d_out backward) must be a multiple of 128 and at least 384,
 * otherwise ACC_ERR_SHAPE: this path has no slower fall-back.  ACC_FLAG_ONE_LAUNCH is ignored.  Workspace as for
 * acc_linear_fwd / acc_linear_bwd. */
typedef enum { ACC_FP8_E4M3 = 0, ACC_FP8_E5M2 = 1 } acc_fp8_format;
int acc_linear_fwd_fp8(const acc_linear_desc* desc, const void* X, const void* X8, const void* W8, float scale,
                       void* Y, void* Xs, void* workspace, size_t ws_bytes, void* stream);
int acc_linear_bwd_fp8(const acc_linear_desc* desc, const void* dY, const void* dY8, int dy8_format, const void* W8,
                       float scale, const void* Xs, void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes,
                       void* stream);

/* Gradient of a bias b [d_out] that is broadcast over tokens (proof of Thm 3.2.2, bias term: the
 * gradient of the added term is grad_Z L itself, independent of X, hence exact under compression):
 * dB[o] = sum_i dY[i, o], accumulated in fp32 in a fixed order (bitwise reproducible), stored as
 * desc->dw_dtype.  dY [n, ldy] (io_dtype) is read; dB [d_out] is overwritten.  Needs the backward
 * workspace: ws_bytes >= acc_linear_workspace_bytes(desc, 1); contents are scratch, so on one stream it
 * may be the buffer acc_linear_bwd uses.  Only n, d_out, r, ldy, io_dtype, factor_dtype, dw_dtype of
 * desc matter (r and factor_dtype through the workspace size only). */
int acc_linear_bias_grad(const acc_linear_desc* desc, const void* dY, void* dB, void* workspace,
                         size_t ws_bytes, void* stream);

/* ---- Optimizer step on the factored gradient (Sec. 4, update strategy (ii)) ------------------------
 * The paper names the scheme (optimizer states kept in a compressed low-rank form, in the manner of the
 * gradient low-rank projection of Zhao et al., ICML 2024) and gives no formulas.  Reading: that scheme applied
 * to the two factors a backward call returns, G^_W = left . Gr (left = Xs of acc_linear_bwd or V of
 * acc_linear_bwd_rsvd), whose product is never formed; weight decay is decoupled (AdamW):
 *   R  = P^T G^_W = (P^T . left) . Gr          projected gradient [k, d_out]; the projector P [d_in, k] has
 *                                              orthonormal columns and is held fixed between refreshes
 *   M <- beta1 M + (1 - beta1) R;   V <- beta2 V + (1 - beta2) R o R               (fp32, in place)
 *   N  = (M / (1 - beta1^step)) / (sqrt(V / (1 - beta2^step)) + eps)               (factor_dtype, workspace)
 *   W <- (1 - lr weight_decay) W - lr scale (P . N)                                 (io_dtype, in place)
 * With P == NULL the left factor itself is the projector: k = r, R = Gr, W moves along left . N; the moments
 * then live in the basis of the current batch's compressor.
 * Refreshing the projector (acc_lowrank_projector): an orthonormal basis of a k-dimensional subspace of
 * range(G^_W) by a randomized range finder on the factors,
 *   Omega [d_out, k] Gaussian, Omega[o, j] = the Philox normal of (seed, token index := o, column j);
 *   Yp = left . (Gr . Omega);   Yp = P . T, P^T.P = I, diag(T) > 0 (Cholesky QR, applied twice).
 * For k = r, and whenever rank(G^_W) <= k, range(P) = range(G^_W), which is also what the leading singular
 * vectors span.  No dense gradient and no dense optimizer state exists at any point. */
typedef struct acc_adamw_hyper {
  float lr, beta1, beta2, eps, weight_decay;
  float scale;     /* multiplies the step taken back to weight space (1 = none)          */
  int32_t step;    /* number of this update, counted from 1 (bias correction)            */
  int32_t reserved;/* 0                                                                  */
} acc_adamw_hyper;

/* Bytes of device workspace of acc_lowrank_adamw_step and acc_lowrank_projector for projector rank k (k == 0:
 * the step without a projector); 0 = invalid descriptor or k.  Of desc only d_in, d_out, r, ldw, io_dtype,
 * factor_dtype, seed and ACC_FLAG_W_OUT_IN matter to the three calls (n must be valid; it is not used; the
 * factors are dense: ldf must be 0 or r). */
size_t acc_lowrank_workspace_bytes(const acc_linear_desc* desc, int64_t k);

/* P [d_in, k] (dense, factor_dtype) is overwritten with the projector of the factored gradient left . Gr.
 * left [d_in, r] and Gr ([r, d_out], or [d_out, r] under ACC_FLAG_W_OUT_IN), both factor_dtype, are read.
 * k: multiple of 8, 8 <= k <= 512, k <= r, k <= d_in (else ACC_ERR_SHAPE; above 64 the k x k factorisation runs
 * blocked on 64 x 64 diagonal blocks).  If Yp has dependent columns
 * (rank(G^_W) < k) the corresponding columns of P are zero. */
int acc_lowrank_projector(const acc_linear_desc* desc, int64_t k, const void* left, const void* Gr, void* P,
                          void* workspace, size_t ws_bytes, void* stream);

/* One update of W from the factors of one backward call.  P [d_in, k] (factor_dtype; k a multiple of 8,
 * k <= d_in; any orthonormal projector, not only acc_lowrank_projector's) or NULL (k ignored), left and Gr as
 * above are read; M and V (fp32, dense, [k, d_out], or [d_out, k] under ACC_FLAG_W_OUT_IN, with k = r when P is
 * NULL; zero before step 1) and W ([d_in, ldw], or [d_out, ldw] under ACC_FLAG_W_OUT_IN, io_dtype) are
 * updated in place.  ACC_ERR_INVALID_ARG also for step < 1, beta outside [0, 1), eps < 0 or a non-finite
 * lr / weight_decay / scale, and for ACC_FLAG_SKIP_SKETCH, ACC_FLAG_ONE_LAUNCH or ACC_FLAG_DW_ACCUMULATE.
 * A bf16 W rounds the product P . N to bf16, then the updated weight. */
int acc_lowrank_adamw_step(const acc_linear_desc* desc, const acc_adamw_hyper* hyper, const void* P, int64_t k,
                           const void* left, const void* Gr, float* M, float* V, void* W, void* workspace,
                           size_t ws_bytes, void* stream);

/* ---- RSVD compressor (Experimental Setup: randomized SVD of Halko, Martinsson and Tropp; Sec. 4: the
 * compressed activation is kept as two factors, X^ = U.V^T, U [n, r], V [d_in, r]) -------------------
 * Reading (the paper fixes only the rank): randomized range finder and projection, no oversampling, no
 * final rotation to singular vectors, subspace iterations only on request (ACC_FLAG_RSVD_POWER_*):
 *   Omega [d_in, r] Gaussian, Omega[c, j] = the Philox normal of (seed, token index := c, column j);
 *   Yr = X.Omega;  Yr = U.R, U^T.U = I, diag(R) > 0 (Cholesky QR, applied twice);  V = X^T.U.
 * Here desc->r is the rank: multiple of 8, 8 <= r <= 512, r <= n, r <= d_in, ldf 0 or r (else ACC_ERR_SHAPE; the
 * paper uses 8 and 32; above 64 the r x r factorisation runs blocked on 64 x 64 diagonal blocks);
 * row_offset is ignored; ACC_FLAG_SKIP_SKETCH and ACC_FLAG_ONE_LAUNCH are refused.  If Yr has
 * dependent columns (rank(X) < r) the corresponding columns of U and V are zero; U.V^T is still the
 * projection of X onto the range of Yr.  U and V are stored as factor_dtype.                        */

/* Bytes of device workspace of the RSVD forward (is_backward == 0) or backward call; 0 = invalid. */
size_t acc_rsvd_workspace_bytes(const acc_linear_desc* desc, int is_backward);

/* Forward with the RSVD compressor: Y = X.W exact (Def. 3.1), U [n, r] and V [d_in, r] (dense) are
 * overwritten with the stored factors.  X [n, ldx], W are read. */
int acc_linear_fwd_rsvd(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* U, void* V,
                        void* workspace, size_t ws_bytes, void* stream);

/* Backward with stored RSVD factors (Sec. 4: the weight gradient is ((grad_Z L)^T.U).V^T): dX = dY.W^T
 * exact, Gr = U^T.dY [r, d_out] ([d_out, r] with ACC_FLAG_W_OUT_IN) and, when dW != NULL,
 * dW = V.Gr [d_in, d_out] (Gr.V^T [d_out, d_in] with ACC_FLAG_W_OUT_IN; += with ACC_FLAG_DW_ACCUMULATE).
 * V may be NULL when dW is NULL. */
int acc_linear_bwd_rsvd(const acc_linear_desc* desc, const void* dY, const void* W, const void* U, const void* V,
                        void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes, void* stream);

/* Test hook: the Philox integer stream behind S.  out is a device array of
 * ceil(n/4) * r * 4 uint32 laid out [token group q][column j][word w]. */
int acc_philox_dump_u32(uint64_t seed, uint64_t row_offset, int64_t n, int64_t r, uint32_t* out,
                        void* stream);

/* Test hook: S itself as float32 [n, r] (device).  io_dtype ACC_F32 gives the fp32 generator of the generic
 * kernels (libm-grade log / sincos); ACC_BF16 the hardware-transcendental Box-Muller of the bf16 kernels,
 * rounded to bfloat16 and widened.  The hook runs the straightforward form of that arithmetic (one call per
 * lane, acc_rng.h); the tuned sketch kernels carry their own interleaved copy with its own counter
 * arithmetic, which is pinned separately by running the layer calls on identity inputs (X = I gives Xs = S).
 * Only n, r, seed, row_offset and io_dtype of desc are read. */
int acc_sketch_dump(const acc_linear_desc* desc, float* S, void* stream);

/* Measurement hook: one launch of a loop of matrix instructions that touches only registers, 256
 * work-groups (one per compute unit) of 4 * waves_per_simd waves, each wave iters x 4 instructions on four
 * independent accumulator sets.  shape 0: 32x32x16 bf16, 1: 16x16x32 bf16, 2: 16x16x128 fp8 (e4m3); waves_per_simd 1 or 2;
 * random_data 0: all operands zero, 1: pseudo-random operands.  sink: device scratch of at least 256 * 256 * waves_per_simd
 * floats (overwritten); *flops (host) receives the flops of the launch.  Timing it (events, profiler) gives the
 * rate the matrix pipe sustains under the part's power limit, the practical ceiling of the MFMA-bound steps
 * (Def. 3.1's exact products).  1 <= iters <= 2^24. */
int acc_probe_mfma(int shape, int waves_per_simd, int random_data, int64_t iters, float* sink, size_t sink_bytes,
                   double* flops, void* stream);

/* Human-readable name of a status code (static string, never NULL). */
const char* acc_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int acc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ACC_H_ */
