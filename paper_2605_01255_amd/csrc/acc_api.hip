// Host side of libacc.so: argument validation, launch planning, kernel launches.
// No allocation, no synchronisation: every entry point only enqueues on the caller's stream.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <tuple>
#include <utility>

#include "acc_common.h"
#include "acc_fused.h"
#include "acc_gemm.h"
#include "acc_generic.h"
#include "acc_optim.h"
#include "acc_probe.h"
#include "acc_rsvd.h"
#include "acc_sketch.h"
#include "acc_gemm16.h"
#include "acc_gemm8.h"
#include "acc_gemm_smallk.h"

// Scratch of acc_linear_fwd_static (the entry point for callers that cannot allocate): the split-token partial
// tiles of the sketch live here instead of in a caller's workspace.  Every GPU the library runs on holds its own
// copy of the array until the process ends.  In host code the name is only a handle for hipGetSymbolAddress;
// kernels get the device address looked up once per device (static_scratch()).
constexpr size_t kStaticScratchBytes = ACC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace acc {
namespace {

constexpr int kVersion = 101;  // 0.1.1

bool valid_dtype(int32_t d) { return d == ACC_F32 || d == ACC_BF16; }
size_t dtype_size(int32_t d) { return d == ACC_BF16 ? 2 : 4; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Shape {
  int64_t n, d_in, d_out, r, ldx, ldw, ldy;
  int64_t ldf;  // row stride of the factors whose rows hold r elements
};

int validate_desc(const acc_linear_desc* d, Shape* s, uint32_t extra_flags = 0) {
  if (!d) return ACC_ERR_INVALID_ARG;
  if (d->flags & ~(uint32_t)(ACC_FLAG_SKIP_SKETCH | ACC_FLAG_ONE_LAUNCH | ACC_FLAG_W_OUT_IN | ACC_FLAG_DW_ACCUMULATE |
                             extra_flags))
    return ACC_ERR_INVALID_ARG;
  if (!valid_dtype(d->io_dtype) || !valid_dtype(d->factor_dtype) || !valid_dtype(d->dw_dtype))
    return ACC_ERR_DTYPE;
  if (d->n <= 0 || d->d_in <= 0 || d->d_out <= 0 || d->r <= 0) return ACC_ERR_SHAPE;
  if (d->r % 8 || d->d_in % 8 || d->d_out % 8) return ACC_ERR_SHAPE;  // 16-byte rows of every operand and factor
  // limits that keep every grid dimension and 32-bit tile count in range
  if (d->n > (int64_t)1 << 30 || d->d_in > (1 << 21) || d->d_out > (1 << 21) || d->r > (1 << 16))
    return ACC_ERR_SHAPE;
  if (d->row_offset % 4) return ACC_ERR_SHAPE;
  s->n = d->n; s->d_in = d->d_in; s->d_out = d->d_out; s->r = d->r;
  s->ldx = d->ldx ? d->ldx : d->d_in;
  const int64_t w_row = (d->flags & ACC_FLAG_W_OUT_IN) ? d->d_in : d->d_out;  // elements per row of W
  s->ldw = d->ldw ? d->ldw : w_row;
  s->ldy = d->ldy ? d->ldy : d->d_out;
  if (s->ldx < s->d_in || s->ldw < w_row || s->ldy < s->d_out) return ACC_ERR_SHAPE;
  if (s->ldx % 8 || s->ldw % 8 || s->ldy % 8) return ACC_ERR_SHAPE;
  s->ldf = d->ldf ? d->ldf : d->r;
  if (s->ldf < s->r || s->ldf % 8 || s->ldf > ((int64_t)1 << 24)) return ACC_ERR_SHAPE;
  return ACC_OK;
}

// ACC_VERBOSE=1 in the environment prints the HIP error behind an ACC_ERR_HIP to stderr.
int hip_fail(hipError_t e, const char* what) {
  static const bool verbose = getenv("ACC_VERBOSE") != nullptr;
  if (verbose) fprintf(stderr, "libacc: %s: %s\n", what, hipGetErrorString(e));
  return ACC_ERR_HIP;
}

// The library only runs on gfx950; the answer is cached per device ordinal.
int check_device() {
  static std::atomic<int> cached[64];  // 0 unknown, 1 ok, -1 not gfx950
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= 64) return ACC_ERR_HIP;
  if (cached[dev] == 0) {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDeviceProperties");
    cached[dev] = (strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : -1;
    if (cached[dev] != 1) hip_fail(hipErrorInvalidDevice, prop.gcnArchName);
  }
  return cached[dev] == 1 ? ACC_OK : ACC_ERR_HIP;
}

// Kernels whose dynamic-LDS limit has been raised on a device (the attribute sticks to the function, so
// it is set once per kernel and device, not per launch).  The table is shared by all host threads.
struct RaisedEntry { const void* kernel; int device; };
RaisedEntry g_raised[64];
int g_raised_count = 0;
std::mutex g_raised_mutex;
bool lds_limit_raised(const void* kernel) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  std::lock_guard<std::mutex> lock(g_raised_mutex);
  for (int i = 0; i < g_raised_count; ++i)
    if (g_raised[i].kernel == kernel && g_raised[i].device == dev) return true;
  return false;
}
void lds_limit_note(const void* kernel) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return;
  std::lock_guard<std::mutex> lock(g_raised_mutex);
  if (g_raised_count < 64) g_raised[g_raised_count++] = RaisedEntry{kernel, dev};
}

// Enqueues kernels on one stream and remembers the first launch error.
struct Launcher {
  hipStream_t st;
  hipError_t err = hipSuccess;
  template <typename... KArgs, typename... Args>
  void operator()(void (*kernel)(KArgs...), dim3 grid, dim3 block, Args... args) {
    launch_lds(kernel, grid, block, 0, args...);
  }
  // lds_bytes of dynamic LDS; above 64 KB the kernel's limit is raised first (no allocation involved).
  template <typename... KArgs, typename... Args>
  void launch_lds(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, Args... args) {
    if (err != hipSuccess) return;
    if (lds_bytes > 64 * 1024) {
      if (!lds_limit_raised((const void*)kernel)) {
        err = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (err != hipSuccess) return;
        lds_limit_note((const void*)kernel);
      }
    }
    std::tuple<KArgs...> vals{args...};
    void* ptrs[sizeof...(KArgs)];
    fill(ptrs, vals, std::index_sequence_for<KArgs...>{});
    err = hipLaunchKernel((const void*)kernel, grid, block, ptrs, lds_bytes, st);
  }
  template <typename T, size_t... I>
  static void fill(void** ptrs, T& vals, std::index_sequence<I...>) {
    ((ptrs[I] = (void*)&std::get<I>(vals)), ...);
  }
  int status() const { return err == hipSuccess ? ACC_OK : hip_fail(err, "kernel launch"); }
};

SketchParams make_sketch_params(const acc_linear_desc* d) {
  SketchParams sk;
  sk.key0 = (uint32_t)(d->seed & 0xFFFFFFFFu);
  sk.key1 = (uint32_t)(d->seed >> 32);
  sk.row_offset = d->row_offset;
  sk.inv_sqrt_r = (float)(1.0 / sqrt((double)d->r));
  sk.neg2_ln2_over_r = (float)(-2.0 * 0.6931471805599453 / (double)d->r);
  return sk;
}

// ---- generic path --------------------------------------------------------------------------
// Token splits of the sketch contraction: enough work-groups to fill 256 CUs, at most 32 partials.
int generic_sketch_splits(int64_t n, int64_t c, int64_t r) {
  const int64_t tiles = ceil_div(c, 64) * ceil_div(r, 64);
  int64_t g = ceil_div(1024, tiles);
  const int64_t max_by_k = ceil_div(n, 256);
  if (g > max_by_k) g = max_by_k;
  if (g > 32) g = 32;
  if (g < 1) g = 1;
  return (int)g;
}

template <typename TA, typename TB, typename TC, typename CT, bool SK, bool ACCURATE>
void launch_generic(const GemmParams& p, int splits, Launcher& L) {
  dim3 grid((unsigned)ceil_div(p.M, 64), (unsigned)ceil_div(p.N, 64), (unsigned)splits);
  L(gemm_generic_kernel<TA, TB, TC, CT, SK, ACCURATE>, grid, dim3(256), p);
}

// C[M, N] = A . B, all three of one storage type.
void generic_gemm_io(int32_t dt, const GemmParams& p, Launcher& L) {
  if (dt == ACC_BF16) launch_generic<bf16, bf16, bf16, bf16, false, false>(p, 1, L);
  else launch_generic<float, float, float, float, false, true>(p, 1, L);
}

// partial[g][...] = A^T-slab . S-slab, fp32, then K4 reduce into `out` (factor dtype).
void generic_sketch(const acc_linear_desc* d, const void* A, int64_t lda, int64_t channels, int64_t n,
                    int64_t c_sm, int64_t c_sn, void* out, int64_t out_row, int64_t out_ld, float* ws, Launcher& L) {
  GemmParams p{};
  p.A = A; p.B = nullptr; p.C = ws;
  p.M = channels; p.N = d->r; p.K = n;
  p.a_sm = 1; p.a_sk = lda;
  p.c_sm = c_sm; p.c_sn = c_sn;
  const int G = generic_sketch_splits(n, channels, d->r);
  p.k_per_split = round_up(ceil_div(n, G), 32);
  p.c_split_stride = channels * d->r;
  p.sk = make_sketch_params(d);
  if (d->io_dtype == ACC_BF16) launch_generic<bf16, bf16, float, bf16, true, false>(p, G, L);
  else launch_generic<float, float, float, float, true, true>(p, G, L);
  const int64_t count = channels * d->r;
  const unsigned blocks = (unsigned)ceil_div(count, 1024);
  if (d->factor_dtype == ACC_BF16)
    L(reduce_partials_kernel<bf16>, dim3(blocks), dim3(256), (const float*)ws, G, count, count, (bf16*)out, out_row,
      out_ld);
  else
    L(reduce_partials_kernel<float>, dim3(blocks), dim3(256), (const float*)ws, G, count, count, (float*)out, out_row,
      out_ld);
}

// Where a product of the two factors goes: the dense gradient, or the weight itself (optimizer step).
struct FactorProductOut {
  void* C;
  int32_t dtype;
  int64_t ld;          // row stride in elements
  bool accumulate;     // C = beta C + alpha (product) instead of C = product
  float alpha, beta;
};

void generic_dw(const acc_linear_desc* d, const Shape& s, const void* Xs, const void* Gr, const FactorProductOut& o,
                Launcher& L) {
  GemmParams p{};
  if (d->flags & ACC_FLAG_W_OUT_IN) {  // [d_out, d_in] = Gr [d_out, r] . Xs^T
    p.A = Gr; p.B = Xs; p.C = o.C;
    p.M = s.d_out; p.N = s.d_in; p.K = s.r;
    p.a_sm = s.ldf; p.a_sk = 1; p.b_sk = 1; p.b_sn = s.ldf; p.c_sm = o.ld; p.c_sn = 1;
  } else {
    p.A = Xs; p.B = Gr; p.C = o.C;
    p.M = s.d_in; p.N = s.d_out; p.K = s.r;
    p.a_sm = s.ldf; p.a_sk = 1; p.b_sk = s.d_out; p.b_sn = 1; p.c_sm = o.ld; p.c_sn = 1;
  }
  p.k_per_split = round_up(s.r, 32);
  p.accumulate = o.accumulate ? 1 : 0;
  p.alpha = o.alpha; p.beta = o.beta;
  const bool fb = d->factor_dtype == ACC_BF16, ob = o.dtype == ACC_BF16;
  if (fb && ob) launch_generic<bf16, bf16, bf16, bf16, false, false>(p, 1, L);
  else if (fb) launch_generic<bf16, bf16, float, bf16, false, false>(p, 1, L);
  else if (ob) launch_generic<float, float, bf16, float, false, true>(p, 1, L);
  else launch_generic<float, float, float, float, false, true>(p, 1, L);
}

// ---- tuned bf16 path ------------------------------------------------------------------------
constexpr int64_t kMaxOperandBytes = 0xFFFFFFFFll;  // buffer resources address 4 GiB

// C[M, N] = A[M, K] . B with the tuned kernel; B is [N, K] (KMAJ) or [K, N].
bool fast_gemm_ok(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  return K % 64 == 0 && N % 8 == 0 && M * lda * 2 <= kMaxOperandBytes &&
         (N > K ? N : K) * ldb * 2 <= kMaxOperandBytes && 256 * lda * 2 <= kMaxOperandBytes;
}

// The K4 reduction of a sketch, handed to the GEMM launched right after it (FastGemmParams::red_*)
// instead of taking a launch of its own.  count == 0: nothing pending.
struct ReduceJob {
  const float* part;
  void* out;
  int64_t count;
  int G;
  int out_bf16;
  int64_t row, ld;  // the result's rows hold `row` elements and are stored `ld` apart
};

template <bool KMAJ, typename TC>
void fast_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t lda,
               int64_t ldb, int64_t ldc, Launcher& L, const ReduceJob* job = nullptr, bool accumulate = false,
               float alpha = 1.f, float beta = 1.f) {
  FastGemmParams p{};
  p.accumulate = accumulate ? 1 : 0;
  p.alpha = alpha; p.beta = beta;
  p.A = (const bf16*)A; p.B = (const bf16*)B; p.C = C;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  if (job && job->count) {
    p.red_part = job->part; p.red_out = job->out; p.red_count = job->count; p.red_G = job->G;
    p.red_out_bf16 = job->out_bf16;
    p.red_row = job->row; p.red_ld = job->ld;
  }
  const int64_t big_tiles = ceil_div(M, 256) * ceil_div(N, 256);
  if (big_tiles >= 192) {  // 256 x 256 tiles: enough tiles to fill 256 CUs
    const unsigned grid = gemm_bf16_plan(p, 256, 256);  // a multiple of 256 slots
    p.red_stride = (int64_t)grid * 256 * 4;
    if constexpr (sizeof(TC) == 2) {
      if (!accumulate && K >= 192) {
        // 256 persistent work-groups on the 16x16x32 instruction; one round of tiles takes it too (a 3072 -> 1024
        // projection: GEMM 84.3 against 86.4 us on the 32x32x16 kernel below)
        p.red_stride = (int64_t)256 * 256 * 4;
        L.launch_lds(gemm16_persist_kernel<KMAJ>, dim3(256), dim3(256), (size_t)160 * 1024, p, (int)grid);
        return;
      }
    }
    L.launch_lds(gemm_bf16_kernel<2, 2, 4, 4, KMAJ, TC>, dim3(grid), dim3(256),
                 (size_t)gemm_bf16_lds_bytes<2, 2, 4, 4>(), p);
  } else {                 // 128 x 128 tiles, 4 waves
    const unsigned grid = gemm_bf16_plan(p, 128, 128);
    p.red_stride = (int64_t)grid * 256 * 4;
    L.launch_lds(gemm_bf16_kernel<2, 2, 2, 2, KMAJ, TC>, dim3(grid), dim3(256),
                 (size_t)gemm_bf16_lds_bytes<2, 2, 2, 2>(), p);
  }
}

// C (op)= A[M, K] . B for a short K on the three-stage kernel of acc_gemm_smallk.h (the product of two gradient
// factors: the dense dW, the optimizer's update of W).
template <bool KMAJ, typename TC>
void smallk_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                 int64_t ldc, Launcher& L, bool accumulate, float alpha, float beta) {
  FastGemmParams p{};
  p.accumulate = accumulate ? 1 : 0;
  p.alpha = alpha; p.beta = beta;
  p.A = (const bf16*)A; p.B = (const bf16*)B; p.C = C;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.tiles_m = (int)ceil_div(M, 192);
  p.tiles_n = (int)ceil_div(N, 192);
  L.launch_lds(gemm16_smallk_kernel<KMAJ, TC>, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(256), (size_t)144 * 1024, p);
}

// ---- exact products on 8-bit floating-point operands (acc_gemm8.h) ---------------------------------
// C[M, N] (bf16) = alpha * (A8[M, K] . B8); B8 is [N, K] (KMAJ) or [K, N]; one byte per element, strides in bytes.
bool gemm8_ok(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, bool kmaj) {
  return K % 128 == 0 && K >= 384 && N % 8 == 0 && lda % 16 == 0 && ldb % 16 == 0 && M * lda <= kMaxOperandBytes &&
         (kmaj ? N : K) * ldb <= kMaxOperandBytes && 256 * lda <= kMaxOperandBytes && 256 * ldb <= kMaxOperandBytes;
}

template <bool KMAJ>
void gemm8(const void* A, int a_format, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t lda,
           int64_t ldb, int64_t ldc, float alpha, Launcher& L, const ReduceJob* job) {
  FastGemmParams p{};
  p.alpha = alpha; p.beta = 0.f;
  p.A = (const bf16*)A; p.B = (const bf16*)B; p.C = C;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  if (job && job->count) {
    p.red_part = job->part; p.red_out = job->out; p.red_count = job->count; p.red_G = job->G;
    p.red_out_bf16 = job->out_bf16;
    p.red_row = job->row; p.red_ld = job->ld;
  }
  const unsigned slots = gemm_bf16_plan(p, 256, 256);
  p.red_stride = (int64_t)256 * 256 * 4;
  if (a_format == ACC_FP8_E5M2) L.launch_lds(gemm8_persist_kernel<KMAJ, 1>, dim3(256), dim3(256), (size_t)160 * 1024, p, (int)slots);
  else L.launch_lds(gemm8_persist_kernel<KMAJ, 0>, dim3(256), dim3(256), (size_t)160 * 1024, p, (int)slots);
}

// K splits of a skinny product: as many as fill the chip's resident work-group slots exactly once (a
// second, partly filled round would cost a whole extra pass of load latencies), each with at least
// four K tiles.  lds_bytes: dynamic LDS of the kernel variant (4 waves per work-group).
int64_t splitk_count(int64_t tiles, int64_t K, int lds_bytes) {
  int64_t per_cu = (160 * 1024) / lds_bytes;
  if (per_cu > 4) per_cu = 4;  // measured: five resident 64 x 64 work-groups per CU run slower than four
  int64_t splits = (256 * per_cu) / tiles;
  if (splits > K / 256) splits = K / 256;
  return splits < 1 ? 1 : splits;
}

// Skinny product through the tuned kernel, the K range split over groups of work-groups (splitk_count):
// part[s][M][ldc] = A[:, K range s] . B[K range s, :], fp32.  Returns the number of splits.  kb_rows: rows of an N-contiguous B that exist (K may be A's zero-padded length).
template <int WM, int WN, int TM, int TN, bool KMAJ>
int fast_gemm_splitk(const void* A, const void* B, float* part, int64_t M, int64_t N, int64_t K, int64_t lda,
                     int64_t ldb, int64_t ldc, int64_t kb_rows, Launcher& L) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  FastGemmParams p{};
  p.A = (const bf16*)A; p.B = (const bf16*)B; p.C = part;
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.kb_rows = kb_rows;
  gemm_bf16_plan(p, BM, BN);  // tiles_m, tiles_n; the XCD super-tile order is not used with splits
  const int64_t tiles = ceil_div(M, BM) * ceil_div(N, BN);
  const unsigned tile_blocks = (unsigned)tiles;
  int64_t splits = splitk_count(tiles, K, gemm_bf16_lds_bytes<WM, WN, TM, TN>());
  p.k_per_split = round_up(ceil_div(K, splits), 64);
  splits = ceil_div(K, p.k_per_split);
  p.tile_blocks = (int)tile_blocks;
  p.c_split_stride = M * ldc;
  L.launch_lds(gemm_bf16_kernel<WM, WN, TM, TN, KMAJ, float>, dim3(tile_blocks * (unsigned)splits), dim3(WM * WN * 64),
               (size_t)gemm_bf16_lds_bytes<WM, WN, TM, TN>(), p);
  return (int)splits;
}

// Plan of the tuned sketch kernel for `channels` columns of a [n, ld] matrix.
struct SketchPlan {
  bool fast;
  int ch, rc;            // tile: channels x sketch columns
  int n_cslab, n_js, G;  // channel slabs, column slices, token splits
  int tokens_per_split;
};

SketchPlan plan_sketch(const acc_linear_desc* d, int64_t n, int64_t channels, int64_t ld) {
  SketchPlan sp{};
  sp.fast = d->io_dtype == ACC_BF16 && n * ld * 2 <= kMaxOperandBytes &&
            channels * d->r * 4 <= kMaxOperandBytes / 2;
  if (!sp.fast) {
    sp.G = generic_sketch_splits(n, channels, d->r);
    return sp;
  }
  // 8-wave tiles of 512 channels, one work-group per compute unit.  64 sketch columns (64 accumulators per
  // lane) by default: half the partial bytes of the 128-column tile for the same generator and matrix work.
  // The 128-column tile stays where eight or more column slices would re-read a long token range from L2
  // (measured: r = 512 at 65536 tokens), and in the one-launch kernel, which interleaves it with GEMM tiles;
  // the choice must be the same in every call that sees this descriptor (workspace size, forward, backward).
  sp.ch = 512;
  const bool wide = d->r % 128 == 0 && ((d->flags & ACC_FLAG_ONE_LAUNCH) || (d->r > 256 && n > 32768));
  sp.rc = wide ? 128 : 64;
  sp.n_cslab = (int)ceil_div(channels, sp.ch);
  sp.n_js = (int)ceil_div(d->r, sp.rc);  // the last column slice may be partly empty (rank % 64 != 0)
  int64_t G = 256 / (sp.n_cslab * sp.n_js);  // never more work-groups than compute units
  const int64_t max_by_tokens = ceil_div(n, 256);
  if (G > max_by_tokens) G = max_by_tokens;
  if (G > 64) G = 64;
  if (G < 1) G = 1;
  sp.tokens_per_split = (int)round_up(ceil_div(n, G), 32);
  sp.G = (int)ceil_div(n, sp.tokens_per_split);
  if ((int64_t)sp.tokens_per_split * ld * 2 + 64 * ld * 2 > kMaxOperandBytes) sp.fast = false;
  if (!sp.fast) sp.G = generic_sketch_splits(n, channels, d->r);
  return sp;
}

void reduce_partials(const acc_linear_desc* d, const float* ws, int G, int64_t count, void* out, int64_t row,
                     int64_t ld, Launcher& L) {
  const unsigned blocks = (unsigned)ceil_div(count, 1024);
  if (d->factor_dtype == ACC_BF16)
    L(reduce_partials_kernel<bf16>, dim3(blocks), dim3(256), ws, G, count, count, (bf16*)out, row, ld);
  else
    L(reduce_partials_kernel<float>, dim3(blocks), dim3(256), ws, G, count, count, (float*)out, row, ld);
}

// partial[g] (final orientation) with the tuned kernel, then K4 into `out`.
void fast_sketch(const acc_linear_desc* d, const SketchPlan& sp, const void* A, int64_t lda, int64_t channels,
                 int64_t n, bool transposed, void* out, int64_t out_row, int64_t out_ld, float* ws, Launcher& L,
                 ReduceJob* defer) {
  SketchFastParams p{};
  p.A = (const bf16*)A; p.part = ws; p.n = n; p.C = channels; p.lda = lda; p.r = (int)d->r;
  p.tokens_per_split = sp.tokens_per_split; p.n_cslab = sp.n_cslab; p.n_js = sp.n_js; p.G = sp.G;
  p.sk = make_sketch_params(d);
  const int pairs = sp.n_cslab * sp.G;
  const dim3 grid((unsigned)(8 * sp.n_js * ceil_div(pairs, 8)));
  if (sp.rc == 128) {
    if (transposed) L.launch_lds(sketch8_kernel<true, 4>, grid, dim3(512), (size_t)sketch8_lds_bytes<4>(), p);
    else L.launch_lds(sketch8_kernel<false, 4>, grid, dim3(512), (size_t)sketch8_lds_bytes<4>(), p);
  } else {
    if (transposed) L.launch_lds(sketch8_kernel<true, 2>, grid, dim3(512), (size_t)sketch8_lds_bytes<2>(), p);
    else L.launch_lds(sketch8_kernel<false, 2>, grid, dim3(512), (size_t)sketch8_lds_bytes<2>(), p);
  }
  if (defer) *defer = ReduceJob{ws, out, channels * d->r, sp.G, d->factor_dtype == ACC_BF16 ? 1 : 0, out_row, out_ld};
  else reduce_partials(d, ws, sp.G, channels * d->r, out, out_row, out_ld, L);
}

// One launch for the exact GEMM and the sketch of the same input (see acc_fused.h), then K4.
// A [n, lda] is both the GEMM's left operand and the sketched matrix (X forward, dY backward).
bool fused_ok(const acc_linear_desc* d, const SketchPlan& sp, int64_t n, int64_t N, int64_t K, int64_t lda,
              int64_t ldb) {
  return (d->flags & ACC_FLAG_ONE_LAUNCH) && !(d->flags & ACC_FLAG_W_OUT_IN) && d->io_dtype == ACC_BF16 && fast_gemm_ok(n, N, K, lda, ldb) &&
         ceil_div(n, 256) * ceil_div(N, 256) >= 192 &&
         sp.fast && sp.rc == 128;
}

template <bool KMAJ, bool TRANSPOSED>
void fused_pass(const acc_linear_desc* d, const SketchPlan& sp, const void* A, const void* B, void* C, int64_t n,
                int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc, void* factor_out, int64_t out_row,
                int64_t out_ld, float* ws, Launcher& L) {
  FastGemmParams gp{};
  gp.A = (const bf16*)A; gp.B = (const bf16*)B; gp.C = C;
  gp.M = n; gp.N = N; gp.K = K; gp.lda = lda; gp.ldb = ldb; gp.ldc = ldc;
  const unsigned gemm_grid = gemm_bf16_plan(gp, 256, 256);
  SketchFastParams sk{};
  sk.A = (const bf16*)A; sk.part = ws; sk.n = n; sk.C = K; sk.lda = lda; sk.r = (int)d->r;
  sk.tokens_per_split = sp.tokens_per_split; sk.n_cslab = sp.n_cslab; sk.n_js = sp.n_js; sk.G = sp.G;
  sk.sk = make_sketch_params(d);
  FuseMap fm{};
  const int n_gg = (int)(gemm_grid / 8);
  fm.unit = sp.n_js;
  fm.n_units = (int)ceil_div((int64_t)sp.n_cslab * sp.G, 8);
  fm.period = n_gg / fm.n_units;
  const unsigned grid = (unsigned)(n_gg + fm.n_units * fm.unit) * 8u;
  L.launch_lds(fused_linear_kernel<KMAJ, TRANSPOSED>, dim3(grid), dim3(512), (size_t)128 * 1024, gp, sk, fm);
  reduce_partials(d, ws, sp.G, K * d->r, factor_out, out_row, out_ld, L);
}

// defer != nullptr: the caller launches a tuned GEMM next and wants it to fold the partials; the job is
// filled in when the tuned sketch ran (its partials are pending), left empty otherwise.
// The factor comes out [channels, r] with rows `ldf` apart, or transposed [r, channels] (dense).
void run_sketch(const acc_linear_desc* d, const void* A, int64_t lda, int64_t channels, int64_t n,
                bool transposed, void* out, int64_t ldf, float* ws, Launcher& L, ReduceJob* defer = nullptr) {
  const SketchPlan sp = plan_sketch(d, n, channels, lda);
  const int64_t row = transposed ? channels : d->r, ld = transposed ? channels : ldf;
  if (sp.fast) fast_sketch(d, sp, A, lda, channels, n, transposed, out, row, ld, ws, L, defer);
  else if (transposed) generic_sketch(d, A, lda, channels, n, 1, channels, out, row, ld, ws, L);
  else generic_sketch(d, A, lda, channels, n, d->r, 1, out, row, ld, ws, L);
}

// ---- RSVD compressor ------------------------------------------------------------------------
// Forward chain: Yr = X.Omega -> Cholesky QR twice -> U -> V = X^T.U; every product on the generic MFMA
// kernel (fp32 matrix instructions wherever an fp32 operand is involved), K-splits reduced by K4.
constexpr size_t kCholImageBytes = (size_t)(kRsvdMaxRank * kRsvdMaxRank + 2 * kRsvdMaxRank) * 4;  // chol_factor_kernel's output
struct RsvdPlan {
  bool tuned;   // bf16 inputs and factors, sizes the tuned GEMM kernel takes: skinny products via split K
  int g_gram;   // token splits of the k x k Gram products
  int g_fact;   // token splits of V = X^T.U (forward) or Gr = U^T.dY (backward), generic path
  int64_t n_pad;  // tokens rounded up to 64 (K padding of the products over tokens)
  size_t off_y0, off_q1, off_gram_part, off_gram, off_rinv, off_fact_part;  // byte offsets
  size_t off_omega, off_ut, off_yr_part, off_z0, off_z1, off_zt_part, total;
  size_t off_rt;  // ranks above 64: the transposed triangular factor [k, k] of the blocked Cholesky
};

// Scratch of one Cholesky-QR pass at rank k.  Up to 64 the k x k factorisation is one launch on one wave; above it
// runs blocked on 64 x 64 diagonal blocks and needs the full Gram matrix, the transposed factor and one triangular
// image per block.
constexpr int kGramSplitsBlocked = 16;
struct QrScratch { size_t gram_part, gram, rinv, rt; };
template <typename Take>
QrScratch take_qr_scratch(int64_t k, int g_gram, Take& take) {
  QrScratch q{};
  if (k <= kRsvdMaxRank) {
    q.gram_part = take((size_t)g_gram * k * k * 4);
    q.gram = take((size_t)k * k * 4);
    q.rinv = take(kCholImageBytes);
  } else {
    q.gram_part = take((size_t)kGramSplitsBlocked * k * k * 4);
    q.gram = take((size_t)k * k * 4);
    q.rinv = take(kCholImageBytes * (size_t)ceil_div(k, kRsvdMaxRank) + 256);  // + the matrix's largest diagonal entry
    q.rt = take((size_t)k * k * 4);
  }
  return q;
}

// Rounds of subspace iteration asked for in the descriptor (RSVD entry points only).
int rsvd_power_iters(const acc_linear_desc* d) { return (int)((d->flags >> ACC_FLAG_RSVD_POWER_SHIFT) & 3u); }



RsvdPlan plan_rsvd(const acc_linear_desc* d, const Shape& s, bool backward) {
  RsvdPlan pl{};
  const int64_t k = s.r;
  const int64_t channels = backward ? s.d_out : s.d_in;
  const int64_t ld_in = backward ? s.ldy : s.ldx;
  pl.n_pad = round_up(s.n, 64);
  pl.tuned = d->io_dtype == ACC_BF16 && d->factor_dtype == ACC_BF16 && s.d_in % 64 == 0 && s.n >= 256 &&
             s.n * ld_in * 2 <= kMaxOperandBytes && pl.n_pad * 2 * k * 4 <= kMaxOperandBytes;
  pl.g_gram = 256;  // at most this many slabs per Gram product (one 64-row chunk per work-group where possible)
  pl.g_fact = generic_sketch_splits(s.n, channels, k);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
  if (!backward) {
    pl.off_y0 = take((size_t)s.n * k * 4);
    pl.off_q1 = take((size_t)s.n * k * 4);
    const QrScratch q = take_qr_scratch(k, pl.g_gram, take);
    pl.off_gram_part = q.gram_part; pl.off_gram = q.gram; pl.off_rinv = q.rinv; pl.off_rt = q.rt;
    if (rsvd_power_iters(d)) {  // Z = X^T.U and its orthonormalised form, [d_in, k] fp32
      pl.off_z0 = take((size_t)s.d_in * k * 4);
      pl.off_z1 = take((size_t)s.d_in * k * 4);
    }
  }
  if (pl.tuned) {
    const int64_t fact_splits = splitk_count(ceil_div(k, 64) * ceil_div(channels, 128), pl.n_pad, gemm_bf16_lds_bytes<2, 2, 1, 2>());
    pl.off_fact_part = take((size_t)fact_splits * k * channels * 4);
    pl.off_ut = take((size_t)2 * k * pl.n_pad * 2);  // U^T, or [U_hi; U_lo]^T during subspace iterations
    if (!backward && rsvd_power_iters(d)) {
      const int64_t zt_splits = splitk_count(ceil_div(2 * k, 64) * ceil_div(s.d_in, 128), pl.n_pad, gemm_bf16_lds_bytes<2, 2, 1, 2>());
      pl.off_zt_part = take((size_t)zt_splits * 2 * k * s.d_in * 4);
    }
    if (!backward) {
      const int64_t yr_splits = splitk_count(ceil_div(s.n, 64) * ceil_div(2 * k, 64), s.d_in, gemm_bf16_lds_bytes<2, 2, 1, 1>());
      pl.off_omega = take((size_t)2 * k * s.d_in * 2);
      pl.off_yr_part = take((size_t)yr_splits * s.n * 2 * k * 4);
    }
  } else {
    pl.off_fact_part = take((size_t)pl.g_fact * channels * k * 4);
  }
  pl.total = off;
  return pl;
}

// C[M, N] (+ splits) = A . B with element strides, operand types by dtype code; CT is bf16 only when
// both operands are bf16.
void rsvd_gemm(int a_dt, int b_dt, int c_dt, const GemmParams& p, int splits, Launcher& L) {
  const bool ab = a_dt == ACC_BF16, bb = b_dt == ACC_BF16, cb = c_dt == ACC_BF16;
  if (ab && bb && !cb) launch_generic<bf16, bf16, float, bf16, false, false>(p, splits, L);
  else if (ab && !bb && !cb) launch_generic<bf16, float, float, float, false, true>(p, splits, L);
  else if (!ab && bb && !cb) launch_generic<float, bf16, float, float, false, true>(p, splits, L);
  else if (!ab && !bb && !cb) launch_generic<float, float, float, float, false, true>(p, splits, L);
  else if (!ab && !bb && cb) launch_generic<float, float, bf16, float, false, true>(p, splits, L);
  else L.err = hipErrorInvalidValue;  // not used by the chain
}

void reduce_to(int out_dt, const float* part, int G, int64_t count, void* out, Launcher& L) {
  const unsigned blocks = (unsigned)ceil_div(count, 1024);
  if (out_dt == ACC_BF16)
    L(reduce_partials_kernel<bf16>, dim3(blocks), dim3(256), part, G, count, count, (bf16*)out, count, count);
  else
    L(reduce_partials_kernel<float>, dim3(blocks), dim3(256), part, G, count, count, (float*)out, count, count);
}

// The same pass for ranks above 64 (up to 512), built from the rank-64 kernels: blocked right-looking Cholesky of
// the Gram matrix (diagonal block -> chol_factor_kernel<64>; the block column below it -> tall_solve_kernel<64>,
// which gives the transposed row panel of R; trailing update on the generic GEMM), then Q = Yin . R^-1 block column
// by block column (Y_j -= Q_{<j} . R_{<j, j} on the generic GEMM, Q_j = Y_j . R_jj^-1 by tall_solve_kernel<64>).
// Yin is used as scratch: its columns are overwritten.  Q goes to Qf (fp32; Yin itself when Qf is null), Qt, Ut as
// in cholesky_qr_pass.
void cholesky_qr_pass_blocked(const Shape& s, const RsvdPlan& pl, char* ws, int64_t m, int64_t m_pad, float* Yin,
                              float* Qf, void* Qt, int qt_dt, bf16* Ut, int64_t ldt, bool hilo, Launcher& L) {
  const int64_t k = s.r;
  float* gram_part = (float*)(ws + pl.off_gram_part);
  float* gram = (float*)(ws + pl.off_gram);
  float* rt = (float*)(ws + pl.off_rt);
  float* W = Qf ? Qf : Yin;
  const int nb = (int)ceil_div(k, kRsvdMaxRank);
  auto rimg = [&](int j) { return (float*)(ws + pl.off_rinv + (size_t)j * kCholImageBytes); };
  float* scale_ref = rimg(nb);  // behind the last image
  {  // Gram = Yin^T . Yin, the row range split, partials folded in a fixed order
    GemmParams g{};
    g.A = Yin; g.B = Yin; g.C = gram_part;
    g.M = k; g.N = k; g.K = m;
    g.a_sm = 1; g.a_sk = k; g.b_sk = k; g.b_sn = 1; g.c_sm = k; g.c_sn = 1;
    g.k_per_split = round_up(ceil_div(m, kGramSplitsBlocked), 32);
    g.c_split_stride = k * k;
    const int splits = (int)ceil_div(m, g.k_per_split);
    launch_generic<float, float, float, float, false, true>(g, splits, L);
    L(sum_parts_kernel, dim3((unsigned)ceil_div(k * k, 64)), dim3(1024), (const float*)gram_part, splits, k * k, gram);
    L(diag_max_kernel, dim3(1), dim3(64), (const float*)gram, (int)k, k, scale_ref);
  }
  for (int j = 0; j < nb; ++j) {
    const int64_t jb = (int64_t)j * kRsvdMaxRank;
    const int64_t w = k - jb < kRsvdMaxRank ? k - jb : kRsvdMaxRank, rest = k - jb - w;
    L(chol_factor_kernel<64>, dim3(1), dim3(64), (const float*)(gram + jb * k + jb), rimg(j), (int)w, k,
      (const float*)scale_ref, (float)k * 1.1920929e-7f);
    if (rest == 0) break;
    // Rt[rows below, block column j] = G[rows below, block column j] . R_jj^-1  (= the row panel of R, transposed)
    L(tall_solve_kernel<64, float>, dim3((unsigned)ceil_div(rest, 64)), dim3(64), (const float*)(gram + (jb + w) * k + jb),
      rest, (int)w, (const float*)rimg(j), rt + (jb + w) * k + jb, (float*)nullptr, (bf16*)nullptr, (int64_t)0, rest, 0, k,
      k, 0);
    GemmParams u{};  // trailing block -= panel^T . panel, both triangles (the panels below read the lower one)
    u.A = rt + (jb + w) * k + jb; u.B = u.A; u.C = gram + (jb + w) * k + (jb + w);
    u.M = rest; u.N = rest; u.K = w;
    u.a_sm = k; u.a_sk = 1; u.b_sk = 1; u.b_sn = k; u.c_sm = k; u.c_sn = 1;
    u.k_per_split = round_up(w, 32);
    u.accumulate = 1; u.alpha = -1.f; u.beta = 1.f;
    launch_generic<float, float, float, float, false, true>(u, 1, L);
  }
  const int64_t rows_out = Ut ? m_pad : m;
  const int hl = hilo ? 1 : 0;
  for (int j = 0; j < nb; ++j) {
    const int64_t jb = (int64_t)j * kRsvdMaxRank;
    const int64_t w = k - jb < kRsvdMaxRank ? k - jb : kRsvdMaxRank;
    if (j > 0) {  // Y_j -= Q_{<j} . R_{<j, j};  R[t][jb + c] = Rt[(jb + c) * k + t]
      GemmParams u{};
      u.A = W; u.B = rt + jb * k; u.C = Yin + jb;
      u.M = m; u.N = w; u.K = jb;
      u.a_sm = k; u.a_sk = 1; u.b_sk = 1; u.b_sn = k; u.c_sm = k; u.c_sn = 1;
      u.k_per_split = round_up(jb, 32);
      u.accumulate = 1; u.alpha = -1.f; u.beta = 1.f;
      launch_generic<float, float, float, float, false, true>(u, 1, L);
    }
    const dim3 grid((unsigned)ceil_div(rows_out, 64));
    bf16* ut_j = Ut ? Ut + jb * ldt : nullptr;
    if (qt_dt == ACC_BF16)
      L(tall_solve_kernel<64, bf16>, grid, dim3(64), (const float*)(Yin + jb), m, (int)w, (const float*)rimg(j), W + jb,
        Qt ? (bf16*)Qt + jb : (bf16*)nullptr, ut_j, ldt, rows_out, hl, k, k, (int)k);
    else
      L(tall_solve_kernel<64, float>, grid, dim3(64), (const float*)(Yin + jb), m, (int)w, (const float*)rimg(j), W + jb,
        Qt ? (float*)Qt + jb : (float*)nullptr, ut_j, ldt, rows_out, hl, k, k, (int)k);
  }
}

// One Cholesky-QR pass on a tall matrix Yin [m, k] fp32: Q = Yin . R^-1 with Yin^T.Yin = R^T.R.  Q goes to any
// of: Qf (fp32 [m, k]), Qt (factor dtype [m, k]), Ut (bf16 [k, ldt] zero-padded transpose up to column
// m_pad; [2k, ldt] hi / lo parts with `hilo`).  Ranks above 64 take the blocked form, which overwrites Yin.
void cholesky_qr_pass(const Shape& s, const RsvdPlan& pl, char* ws, int64_t m, int64_t m_pad, float* Yin,
                      float* Qf, void* Qt, int qt_dt, bf16* Ut, int64_t ldt, bool hilo, Launcher& L) {
  const int64_t k = s.r;
  if (k > kRsvdMaxRank) {
    cholesky_qr_pass_blocked(s, pl, ws, m, m_pad, Yin, Qf, Qt, qt_dt, Ut, ldt, hilo, L);
    return;
  }
  float* gram_part = (float*)(ws + pl.off_gram_part);
  float* rinv = (float*)(ws + pl.off_rinv);
  float* gram = (float*)(ws + pl.off_gram);
  const int rows = (int)round_up(ceil_div(m, pl.g_gram), 64);
  const int parts = (int)ceil_div(m, rows);
  L(gram_partial_kernel, dim3((unsigned)parts), dim3(256), (const float*)Yin, m, (int)k, rows, gram_part);
  L(sum_parts_kernel, dim3((unsigned)ceil_div(k * k, 64)), dim3(1024), (const float*)gram_part, parts, k * k, gram);
  if (k <= 32) L(chol_factor_kernel<32>, dim3(1), dim3(64), (const float*)gram, rinv, (int)k, k, (const float*)nullptr, 1e-6f);
  else L(chol_factor_kernel<64>, dim3(1), dim3(64), (const float*)gram, rinv, (int)k, k, (const float*)nullptr, 1e-6f);
  const int64_t rows_out = Ut ? m_pad : m;
  const dim3 grid((unsigned)ceil_div(rows_out, 64));
  const int hl = hilo ? 1 : 0;
  if (k <= 32) {
    if (qt_dt == ACC_BF16)
      L(tall_solve_kernel<32, bf16>, grid, dim3(64), (const float*)Yin, m, (int)k, (const float*)rinv, Qf,
        (bf16*)Qt, Ut, ldt, rows_out, hl, k, k, (int)k);
    else
      L(tall_solve_kernel<32, float>, grid, dim3(64), (const float*)Yin, m, (int)k, (const float*)rinv, Qf,
        (float*)Qt, Ut, ldt, rows_out, hl, k, k, (int)k);
  } else {
    if (qt_dt == ACC_BF16)
      L(tall_solve_kernel<64, bf16>, grid, dim3(64), (const float*)Yin, m, (int)k, (const float*)rinv, Qf,
        (bf16*)Qt, Ut, ldt, rows_out, hl, k, k, (int)k);
    else
      L(tall_solve_kernel<64, float>, grid, dim3(64), (const float*)Yin, m, (int)k, (const float*)rinv, Qf,
        (float*)Qt, Ut, ldt, rows_out, hl, k, k, (int)k);
  }
}

// out[channels, k] (or its transpose) = A^T . U over the token axis, A [n, lda]; splits reduced by K4.
void rsvd_factor(const acc_linear_desc* d, const Shape& s, const RsvdPlan& pl, char* ws, const void* A,
                 int64_t lda, int64_t channels, const void* U, bool transposed, void* out, Launcher& L) {
  const int64_t k = s.r;
  float* part = (float*)(ws + pl.off_fact_part);
  GemmParams p{};
  p.A = A; p.B = U; p.C = part;
  p.M = channels; p.N = k; p.K = s.n;
  p.a_sm = 1; p.a_sk = lda; p.b_sk = k; p.b_sn = 1;
  p.c_sm = transposed ? 1 : k; p.c_sn = transposed ? channels : 1;
  p.k_per_split = round_up(ceil_div(s.n, pl.g_fact), 32);
  p.c_split_stride = channels * k;
  const int splits = (int)ceil_div(s.n, p.k_per_split);
  rsvd_gemm(d->io_dtype, d->factor_dtype, ACC_F32, p, splits, L);
  reduce_to(d->factor_dtype, part, splits, channels * k, out, L);
}

// Tuned form of rsvd_factor: Ut [k, n_pad] = U^T (zero-padded) in the workspace, then
// [k, channels] = Ut . A over the token axis with the K range split, folded (and transposed back to
// [channels, k] unless `transposed`) by one small kernel.
void rsvd_factor_tuned(const acc_linear_desc* d, const Shape& s, const RsvdPlan& pl, char* ws, const void* A,
                       int64_t lda, int64_t channels, const void* U, bool transposed, void* out, Launcher& L) {
  const int64_t k = s.r;
  bf16* ut = (bf16*)(ws + pl.off_ut);
  float* part = (float*)(ws + pl.off_fact_part);
  if (U)  // backward: rebuild the transpose from the stored factor; forward wrote it with the last QR pass
    L(transpose_pad_kernel<bf16>, dim3((unsigned)ceil_div(pl.n_pad * k, 256)), dim3(256), (const bf16*)U, s.n, (int)k,
      pl.n_pad, ut);
  const int splits = fast_gemm_splitk<2, 2, 1, 2, false>(ut, A, part, k, channels, pl.n_pad, pl.n_pad, lda, channels,
                                                       s.n, L);
  const unsigned blocks = (unsigned)ceil_div(k * channels, 256);
  if (transposed) L(reduce_store_kernel<bf16, false>, dim3(blocks), dim3(256), (const float*)part, splits, k, channels, (bf16*)out);
  else L(reduce_store_kernel<bf16, true>, dim3(blocks), dim3(256), (const float*)part, splits, k, channels, (bf16*)out);
}

// The exact products shared with the random-projection entry points.
// Whether the exact product of a pass runs on the tuned kernel (and can fold a pending K4 reduction).
bool forward_gemm_is_tuned(const acc_linear_desc* desc, const Shape& s) {
  return desc->io_dtype == ACC_BF16 && fast_gemm_ok(s.n, s.d_out, s.d_in, s.ldx, s.ldw);
}
bool backward_gemm_is_tuned(const acc_linear_desc* desc, const Shape& s) {
  return desc->io_dtype == ACC_BF16 && fast_gemm_ok(s.n, s.d_in, s.d_out, s.ldy, s.ldw);
}

void exact_forward_gemm(const acc_linear_desc* desc, const Shape& s, const void* X, const void* W, void* Y,
                        Launcher& L, const ReduceJob* job = nullptr) {
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;  // W is [N = d_out, K = d_in]
  if (forward_gemm_is_tuned(desc, s)) {
    if (w_oi) fast_gemm<true, bf16>(X, W, Y, s.n, s.d_out, s.d_in, s.ldx, s.ldw, s.ldy, L, job);
    else fast_gemm<false, bf16>(X, W, Y, s.n, s.d_out, s.d_in, s.ldx, s.ldw, s.ldy, L, job);
  } else {
    GemmParams p{};
    p.A = X; p.B = W; p.C = Y;
    p.M = s.n; p.N = s.d_out; p.K = s.d_in;
    p.a_sm = s.ldx; p.a_sk = 1; p.c_sm = s.ldy; p.c_sn = 1;
    p.b_sk = w_oi ? 1 : s.ldw; p.b_sn = w_oi ? s.ldw : 1;
    p.k_per_split = round_up(s.d_in, 32);
    generic_gemm_io(desc->io_dtype, p, L);
  }
}
void exact_backward_gemm(const acc_linear_desc* desc, const Shape& s, const void* dY, const void* W, void* dX,
                         Launcher& L, const ReduceJob* job = nullptr) {
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  if (backward_gemm_is_tuned(desc, s)) {
    if (w_oi) fast_gemm<false, bf16>(dY, W, dX, s.n, s.d_in, s.d_out, s.ldy, s.ldw, s.ldx, L, job);  // W is [K = d_out, N = d_in]
    else fast_gemm<true, bf16>(dY, W, dX, s.n, s.d_in, s.d_out, s.ldy, s.ldw, s.ldx, L, job);        // W is [N = d_in, K = d_out]
  } else {
    GemmParams p{};
    p.A = dY; p.B = W; p.C = dX;
    p.M = s.n; p.N = s.d_in; p.K = s.d_out;
    p.a_sm = s.ldy; p.a_sk = 1; p.c_sm = s.ldx; p.c_sn = 1;
    p.b_sk = w_oi ? s.ldw : 1; p.b_sn = w_oi ? 1 : s.ldw;
    p.k_per_split = round_up(s.d_out, 32);
    generic_gemm_io(desc->io_dtype, p, L);
  }
}

// Product of the stored left factor (Xs, or V of the RSVD path) and the small factor, left . Gr (or Gr . left^T in
// the paper's orientation), written or accumulated into `o`.
void factor_product(const acc_linear_desc* desc, const Shape& s, const void* Xs, const void* Gr,
                    const FactorProductOut& o, Launcher& L) {
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  // A few K tiles and at most one round of 192 x 192 tiles: the three-stage kernel (one exposed latency per
  // work-group).  More tiles than compute units: the pipelined kernel, two work-groups per compute unit covering
  // each other's waits (measured at 3072 x 8192, r = 256: 23.5 against 27.6 us).  One round, 3072 x 3072: 12.4 against
  // 14.2 us at r = 256, 8.4 against 9.8 at r = 64; read-modify-write of a bf16 W at r = 64: 11.4 against 14.5 us
  // (a plain in-place pass over the same 18.9 MB takes 7.4 us, a fill 4.7).
  const bool short_k = s.r <= 1024 && ceil_div(s.d_in, 192) * ceil_div(s.d_out, 192) <= 256;
  if (w_oi && desc->factor_dtype == ACC_BF16 && fast_gemm_ok(s.d_out, s.d_in, s.r, s.ldf, s.ldf)) {
    if (short_k && o.dtype == ACC_BF16)
      smallk_gemm<true, bf16>(Gr, Xs, o.C, s.d_out, s.d_in, s.r, s.ldf, s.ldf, o.ld, L, o.accumulate, o.alpha, o.beta);
    else if (short_k)
      smallk_gemm<true, float>(Gr, Xs, o.C, s.d_out, s.d_in, s.r, s.ldf, s.ldf, o.ld, L, o.accumulate, o.alpha, o.beta);
    else if (o.dtype == ACC_BF16)
      fast_gemm<true, bf16>(Gr, Xs, o.C, s.d_out, s.d_in, s.r, s.ldf, s.ldf, o.ld, L, nullptr, o.accumulate, o.alpha, o.beta);
    else
      fast_gemm<true, float>(Gr, Xs, o.C, s.d_out, s.d_in, s.r, s.ldf, s.ldf, o.ld, L, nullptr, o.accumulate, o.alpha, o.beta);
  } else if (!w_oi && desc->factor_dtype == ACC_BF16 && fast_gemm_ok(s.d_in, s.d_out, s.r, s.ldf, s.d_out)) {
    if (short_k && o.dtype == ACC_BF16)
      smallk_gemm<false, bf16>(Xs, Gr, o.C, s.d_in, s.d_out, s.r, s.ldf, s.d_out, o.ld, L, o.accumulate, o.alpha, o.beta);
    else if (short_k)
      smallk_gemm<false, float>(Xs, Gr, o.C, s.d_in, s.d_out, s.r, s.ldf, s.d_out, o.ld, L, o.accumulate, o.alpha, o.beta);
    else if (o.dtype == ACC_BF16)
      fast_gemm<false, bf16>(Xs, Gr, o.C, s.d_in, s.d_out, s.r, s.ldf, s.d_out, o.ld, L, nullptr, o.accumulate, o.alpha, o.beta);
    else
      fast_gemm<false, float>(Xs, Gr, o.C, s.d_in, s.d_out, s.r, s.ldf, s.d_out, o.ld, L, nullptr, o.accumulate, o.alpha, o.beta);
  } else {
    generic_dw(desc, s, Xs, Gr, o, L);
  }
}

// dW = left . Gr: dense, of desc->dw_dtype, summed into the caller's dW under ACC_FLAG_DW_ACCUMULATE.
void dense_dw(const acc_linear_desc* desc, const Shape& s, const void* Xs, const void* Gr, void* dW, Launcher& L) {
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  const FactorProductOut o{dW, desc->dw_dtype, w_oi ? s.d_in : s.d_out, (desc->flags & ACC_FLAG_DW_ACCUMULATE) != 0,
                           1.f, 1.f};
  factor_product(desc, s, Xs, Gr, o, L);
}

int validate_rsvd(const acc_linear_desc* d, Shape* s) {
  const int rc = validate_desc(d, s, 3u << ACC_FLAG_RSVD_POWER_SHIFT);
  if (rc != ACC_OK) return rc;
  if (d->flags & (ACC_FLAG_SKIP_SKETCH | ACC_FLAG_ONE_LAUNCH)) return ACC_ERR_INVALID_ARG;
  if (s->ldf != s->r) return ACC_ERR_SHAPE;  // the RSVD factors are dense
  if (s->r > kRsvdMaxRankBlocked || s->n < s->r || s->d_in < s->r) return ACC_ERR_SHAPE;
  return ACC_OK;
}

// ---- optimizer step on the factored gradient ---------------------------------------------------------
// k == 0: no separate projector (the left factor is the projector).  for_projector: the orthonormalisation
// runs on the small-rank Cholesky kernels, which sets the upper limit of k.
int validate_lowrank(const acc_linear_desc* d, Shape* s, int64_t k, bool for_projector) {
  const int rc = validate_desc(d, s);
  if (rc != ACC_OK) return rc;
  if (d->flags & (ACC_FLAG_SKIP_SKETCH | ACC_FLAG_ONE_LAUNCH | ACC_FLAG_DW_ACCUMULATE)) return ACC_ERR_INVALID_ARG;
  if (s->ldf != s->r) return ACC_ERR_SHAPE;  // the optimizer calls read dense factors
  if (k < 0 || k % 8 || k > s->d_in || k > (1 << 16)) return ACC_ERR_SHAPE;
  if (for_projector && (k < 8 || k > kRsvdMaxRankBlocked || k > s->r)) return ACC_ERR_SHAPE;
  return ACC_OK;
}

struct LowrankPlan {
  int t1_splits, z_splits, g_gram;
  int64_t t1_k_per_split, z_k_per_split;
  size_t off_n, off_part, off_t1, off_r;                                  // the step
  size_t off_z, off_yp, off_q1, off_gram_part, off_gram, off_rinv, off_rt;  // the projector (shares off_part)
  size_t step_total, total;
};

// Splits of a reduction of length K whose output has `tiles` 64 x 64 tiles: about 512 work-groups, at least 64
// elements of K each.
int64_t lowrank_splits(int64_t tiles, int64_t K) {
  int64_t g = 512 / tiles;
  if (g > K / 64) g = K / 64;
  return g < 1 ? 1 : g;
}

LowrankPlan plan_lowrank(const acc_linear_desc* d, const Shape& s, int64_t k) {
  LowrankPlan pl{};
  const size_t fsz = dtype_size(d->factor_dtype);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + 255) / 256 * 256; return at; };
  const int64_t kk = k ? k : s.r;
  pl.off_n = take((size_t)kk * s.d_out * fsz);
  if (!k) {
    pl.step_total = pl.total = off;
    return pl;
  }
  int64_t g = lowrank_splits(ceil_div(k, 64) * ceil_div(s.r, 64), s.d_in);
  pl.t1_k_per_split = round_up(ceil_div(s.d_in, g), 32);
  pl.t1_splits = (int)ceil_div(s.d_in, pl.t1_k_per_split);
  g = lowrank_splits(ceil_div(s.r, 64) * ceil_div(k, 64), s.d_out);
  pl.z_k_per_split = round_up(ceil_div(s.d_out, g), 32);
  pl.z_splits = (int)ceil_div(s.d_out, pl.z_k_per_split);
  const int max_splits = pl.t1_splits > pl.z_splits ? pl.t1_splits : pl.z_splits;
  pl.off_part = take((size_t)max_splits * k * s.r * 4);
  pl.off_t1 = take((size_t)k * s.r * 4);
  pl.off_r = take((size_t)k * s.d_out * 4);
  pl.step_total = off;
  if (k <= kRsvdMaxRankBlocked && k <= s.r) {
    pl.g_gram = 256;
    pl.off_z = take((size_t)s.r * k * 4);
    pl.off_yp = take((size_t)s.d_in * k * 4);
    pl.off_q1 = take((size_t)s.d_in * k * 4);
    const QrScratch q = take_qr_scratch(k, pl.g_gram, take);
    pl.off_gram_part = q.gram_part; pl.off_gram = q.gram; pl.off_rinv = q.rinv; pl.off_rt = q.rt;
  }
  pl.total = off;
  return pl;
}

size_t workspace_bytes(const acc_linear_desc* d, const Shape& s, bool backward) {
  const int64_t channels = backward ? s.d_out : s.d_in;
  const SketchPlan sp = plan_sketch(d, s.n, channels, backward ? s.ldy : s.ldx);
  return (size_t)sp.G * (size_t)channels * (size_t)s.r * sizeof(float);
}

// Device address of this device's copy of `scratch`, looked up on the first call with that device current.
int static_scratch(float** out) {
  static void* ptr[64];
  static std::mutex mu;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= 64) return ACC_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    ptr[dev] = p;
  }
  *out = (float*)ptr[dev];
  return ACC_OK;
}

// Enqueues the forward pass; every argument has been validated.
int enqueue_forward(const acc_linear_desc* desc, const Shape& s, const void* X, const void* W, void* Y, void* Xs,
                    float* workspace, hipStream_t stream) {
  const bool sketch = !(desc->flags & ACC_FLAG_SKIP_SKETCH);
  Launcher L{stream};
  const SketchPlan sp_f = plan_sketch(desc, s.n, s.d_in, s.ldx);
  if (sketch && fused_ok(desc, sp_f, s.n, s.d_out, s.d_in, s.ldx, s.ldw)) {
    fused_pass<false, false>(desc, sp_f, X, W, Y, s.n, s.d_out, s.d_in, s.ldx, s.ldw, s.ldy, Xs, s.r, s.ldf, workspace, L);
    return L.status();
  }
  // Sketch first: it pulls X through the memory-side cache, so the GEMM that follows starts from
  // there rather than from HBM (measured 4 % on the whole pass against the opposite order).
  ReduceJob job{};  // with a tuned GEMM next, the sketch leaves its K4 reduction to that launch
  if (sketch)
    run_sketch(desc, X, s.ldx, s.d_in, s.n, false, Xs, s.ldf, workspace, L,
               forward_gemm_is_tuned(desc, s) ? &job : nullptr);
  exact_forward_gemm(desc, s, X, W, Y, L, &job);
  return L.status();
}

}  // namespace
}  // namespace acc

using namespace acc;

extern "C" {

size_t acc_linear_workspace_bytes(const acc_linear_desc* desc, int is_backward) {
  Shape s;
  if (validate_desc(desc, &s) != ACC_OK) return 0;
  return workspace_bytes(desc, s, is_backward != 0);
}

int acc_linear_fwd(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* Xs,
                   void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  const bool sketch = !(desc->flags & ACC_FLAG_SKIP_SKETCH);
  if (!X || !W || !Y || (sketch && !Xs)) return ACC_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(Xs) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  if (sketch && (!workspace || ws_bytes < workspace_bytes(desc, s, false))) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  return enqueue_forward(desc, s, X, W, Y, Xs, (float*)workspace, (hipStream_t)stream);
}

int acc_linear_fwd_static(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* Xs,
                          void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  const bool sketch = !(desc->flags & ACC_FLAG_SKIP_SKETCH);
  if (!X || !W || !Y || (sketch && !Xs)) return ACC_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(Xs)) return ACC_ERR_ALIGN;
  if (sketch && workspace_bytes(desc, s, false) > kStaticScratchBytes) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  float* ws = nullptr;
  if ((rc = static_scratch(&ws)) != ACC_OK) return rc;
  return enqueue_forward(desc, s, X, W, Y, Xs, ws, (hipStream_t)stream);
}

int acc_linear_bwd(const acc_linear_desc* desc, const void* dY, const void* W, const void* Xs,
                   void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  if (desc->flags & ACC_FLAG_SKIP_SKETCH) return ACC_ERR_INVALID_ARG;
  if (!dY || !W || !dX || !Gr || (dW && !Xs)) return ACC_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(W) || !aligned16(Xs) || !aligned16(dX) || !aligned16(Gr) ||
      !aligned16(dW) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  if (!workspace || ws_bytes < workspace_bytes(desc, s, true)) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};

  const SketchPlan sp_b = plan_sketch(desc, s.n, s.d_out, s.ldy);
  const bool fused_b = fused_ok(desc, sp_b, s.n, s.d_in, s.d_out, s.ldy, s.ldw);
  // Gr[j, c] = sum_i S[i, j] dY[i, c]: the contraction of dY^T with S, stored transposed ([r, d_out]), or
  // as it comes ([d_out, r]) in the paper's orientation.  As in the forward pass the sketch goes first
  // and leaves dY in the memory-side cache for the GEMM.
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  if (fused_b) {
    // W is [N = d_in, K = d_out]; the sketched matrix dY is the GEMM's left operand
    fused_pass<true, true>(desc, sp_b, dY, W, dX, s.n, s.d_in, s.d_out, s.ldy, s.ldw, s.ldx, Gr, s.d_out, s.d_out,
                           (float*)workspace, L);
  } else {
    ReduceJob job{};
    run_sketch(desc, dY, s.ldy, s.d_out, s.n, !w_oi, Gr, s.ldf, (float*)workspace, L,
               backward_gemm_is_tuned(desc, s) ? &job : nullptr);
    exact_backward_gemm(desc, s, dY, W, dX, L, &job);
  }
  if (dW) dense_dw(desc, s, Xs, Gr, dW, L);
  return L.status();
}

int acc_linear_fwd_fp8(const acc_linear_desc* desc, const void* X, const void* X8, const void* W8, float scale,
                       void* Y, void* Xs, void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  if (desc->io_dtype != ACC_BF16) return ACC_ERR_DTYPE;
  const bool sketch = !(desc->flags & ACC_FLAG_SKIP_SKETCH);
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;  // W8 is [N = d_out, K = d_in]
  if (!X8 || !W8 || !Y || (sketch && (!X || !Xs)) || !(scale == scale)) return ACC_ERR_INVALID_ARG;
  if (!gemm8_ok(s.n, s.d_out, s.d_in, s.ldx, s.ldw, w_oi)) return ACC_ERR_SHAPE;
  if (!aligned16(X) || !aligned16(X8) || !aligned16(W8) || !aligned16(Y) || !aligned16(Xs) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  if (sketch && (!workspace || ws_bytes < workspace_bytes(desc, s, false))) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  ReduceJob job{};  // the sketch (of the bf16 X) leaves its K4 reduction to the GEMM's prologue
  if (sketch) run_sketch(desc, X, s.ldx, s.d_in, s.n, false, Xs, s.ldf, (float*)workspace, L, &job);
  if (w_oi) gemm8<true>(X8, ACC_FP8_E4M3, W8, Y, s.n, s.d_out, s.d_in, s.ldx, s.ldw, s.ldy, scale, L, &job);
  else gemm8<false>(X8, ACC_FP8_E4M3, W8, Y, s.n, s.d_out, s.d_in, s.ldx, s.ldw, s.ldy, scale, L, &job);
  return L.status();
}

int acc_linear_bwd_fp8(const acc_linear_desc* desc, const void* dY, const void* dY8, int dy8_format, const void* W8,
                       float scale, const void* Xs, void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes,
                       void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  if (desc->io_dtype != ACC_BF16) return ACC_ERR_DTYPE;
  if (dy8_format != ACC_FP8_E4M3 && dy8_format != ACC_FP8_E5M2) return ACC_ERR_DTYPE;
  if (desc->flags & ACC_FLAG_SKIP_SKETCH) return ACC_ERR_INVALID_ARG;
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;  // W8 is [K = d_out, N = d_in]; otherwise [N = d_in, K = d_out]
  if (!dY || !dY8 || !W8 || !dX || !Gr || (dW && !Xs) || !(scale == scale)) return ACC_ERR_INVALID_ARG;
  if (!gemm8_ok(s.n, s.d_in, s.d_out, s.ldy, s.ldw, !w_oi)) return ACC_ERR_SHAPE;
  if (!aligned16(dY) || !aligned16(dY8) || !aligned16(W8) || !aligned16(Xs) || !aligned16(dX) || !aligned16(Gr) ||
      !aligned16(dW) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  if (!workspace || ws_bytes < workspace_bytes(desc, s, true)) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  ReduceJob job{};
  run_sketch(desc, dY, s.ldy, s.d_out, s.n, !w_oi, Gr, s.ldf, (float*)workspace, L, &job);
  if (w_oi) gemm8<false>(dY8, dy8_format, W8, dX, s.n, s.d_in, s.d_out, s.ldy, s.ldw, s.ldx, scale, L, &job);
  else gemm8<true>(dY8, dy8_format, W8, dX, s.n, s.d_in, s.d_out, s.ldy, s.ldw, s.ldx, scale, L, &job);
  if (dW) dense_dw(desc, s, Xs, Gr, dW, L);
  return L.status();
}

size_t acc_rsvd_workspace_bytes(const acc_linear_desc* desc, int is_backward) {
  Shape s;
  if (validate_rsvd(desc, &s) != ACC_OK) return 0;
  return plan_rsvd(desc, s, is_backward != 0).total;
}

int acc_linear_fwd_rsvd(const acc_linear_desc* desc, const void* X, const void* W, void* Y, void* U, void* V,
                        void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_rsvd(desc, &s);
  if (rc != ACC_OK) return rc;
  if (!X || !W || !Y || !U || !V) return ACC_ERR_INVALID_ARG;
  if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(U) || !aligned16(V) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  const RsvdPlan pl = plan_rsvd(desc, s, false);
  if (!workspace || ws_bytes < pl.total) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  char* ws = (char*)workspace;
  float* y0 = (float*)(ws + pl.off_y0);
  float* q1 = (float*)(ws + pl.off_q1);
  const int64_t k = s.r;

  const int power_iters = rsvd_power_iters(desc);
  bf16* omega = (bf16*)(ws + pl.off_omega);  // tuned path: [2k, d_in] hi / lo parts of the right factor of Yr
  bf16* ut = (bf16*)(ws + pl.off_ut);        // tuned path: U^T ([U_hi; U_lo]^T while iterating), zero-padded
  // y0 = X . B, B given as hi + lo bfloat16 parts [2k, d_in]: one split-K pass of the tuned kernel over X,
  // halves and splits folded
  auto times_hilo = [&]() {
    float* yr_part = (float*)(ws + pl.off_yr_part);
    const int splits = fast_gemm_splitk<2, 2, 1, 1, true>(X, omega, yr_part, s.n, 2 * k, s.d_in, s.ldx, s.d_in, 2 * k,
                                                        0, L);
    L(combine_hilo_kernel, dim3((unsigned)ceil_div(s.n * k, 256)), dim3(256), (const float*)yr_part, splits, s.n, (int)k,
      y0);
  };

  // Yr = X . Omega, Omega[c, j] from the Philox map with the channel index in the token's place
  acc_linear_desc od = *desc;
  od.row_offset = 0;
  if (pl.tuned) {
    L(omega_hilo_kernel, dim3((unsigned)ceil_div(s.d_in / 4 * k, 256)), dim3(256), make_sketch_params(&od), s.d_in,
      (int)k, s.d_in, omega);
    times_hilo();
  } else {
    GemmParams p{};
    p.A = X; p.B = nullptr; p.C = y0;
    p.M = s.n; p.N = k; p.K = s.d_in;
    p.a_sm = s.ldx; p.a_sk = 1; p.c_sm = k; p.c_sn = 1;
    p.k_per_split = round_up(s.d_in, 32);
    p.sk = make_sketch_params(&od);
    if (desc->io_dtype == ACC_BF16) launch_generic<bf16, bf16, float, float, true, true>(p, 1, L);
    else launch_generic<float, float, float, float, true, true>(p, 1, L);
  }
  // The final basis gets two Cholesky-QR passes (the second removes the loss of orthogonality of the
  // first).  Before it, `power_iters` rounds of subspace iteration: Z = orth(X^T.U), U = orth(X.Z).  The
  // intermediate bases get ONE pass each: it leaves them orthonormal only to about cond^2 * 2^-24, but any
  // basis of the form Q.T with T upper triangular gives exactly the same final U (the thin QR of X.Z.T has
  // the same Q), and one pass is enough to keep the iterates well conditioned.
  for (int it = 0; it <= power_iters; ++it) {
    if (it == power_iters) {
      cholesky_qr_pass(s, pl, ws, s.n, pl.n_pad, y0, q1, nullptr, ACC_F32, nullptr, 0, false, L);
      cholesky_qr_pass(s, pl, ws, s.n, pl.n_pad, q1, nullptr, U, desc->factor_dtype, pl.tuned ? ut : nullptr, pl.n_pad,
                       false, L);
      break;
    }
    float* z0 = (float*)(ws + pl.off_z0);
    if (pl.tuned) {
      // U as hi + lo parts, transposed; Z^T = [U_hi; U_lo] . X over the tokens with the K range split
      cholesky_qr_pass(s, pl, ws, s.n, pl.n_pad, y0, nullptr, nullptr, ACC_F32, ut, pl.n_pad, true, L);
      float* zt_part = (float*)(ws + pl.off_zt_part);
      const int splits = fast_gemm_splitk<2, 2, 1, 2, false>(ut, X, zt_part, 2 * k, s.d_in, pl.n_pad, pl.n_pad, s.ldx,
                                                           s.d_in, s.n, L);
      L(combine_hilo_t_kernel, dim3((unsigned)ceil_div(k * s.d_in, 256)), dim3(256), (const float*)zt_part, splits,
        s.d_in, (int)k, z0);
      // orth(Z) written as hi + lo parts [2k, d_in]: the right factor of the next X . Z
      cholesky_qr_pass(s, pl, ws, s.d_in, s.d_in, z0, nullptr, nullptr, ACC_F32, omega, s.d_in, true, L);
      times_hilo();
    } else {
      float* z1 = (float*)(ws + pl.off_z1);
      cholesky_qr_pass(s, pl, ws, s.n, pl.n_pad, y0, q1, nullptr, ACC_F32, nullptr, 0, false, L);  // U fp32 -> q1
      float* part = (float*)(ws + pl.off_fact_part);
      GemmParams g{};  // Z [d_in, k] = X^T . U, token range split
      g.A = X; g.B = q1; g.C = part;
      g.M = s.d_in; g.N = k; g.K = s.n;
      g.a_sm = 1; g.a_sk = s.ldx; g.b_sk = k; g.b_sn = 1; g.c_sm = k; g.c_sn = 1;
      g.k_per_split = round_up(ceil_div(s.n, pl.g_fact), 32);
      g.c_split_stride = s.d_in * k;
      const int splits = (int)ceil_div(s.n, g.k_per_split);
      rsvd_gemm(desc->io_dtype, ACC_F32, ACC_F32, g, splits, L);
      reduce_to(ACC_F32, part, splits, s.d_in * k, z0, L);
      cholesky_qr_pass(s, pl, ws, s.d_in, s.d_in, z0, z1, nullptr, ACC_F32, nullptr, 0, false, L);  // orth(Z) -> z1
      GemmParams y{};  // y0 [n, k] = X . Z
      y.A = X; y.B = z1; y.C = y0;
      y.M = s.n; y.N = k; y.K = s.d_in;
      y.a_sm = s.ldx; y.a_sk = 1; y.b_sk = k; y.b_sn = 1; y.c_sm = k; y.c_sn = 1;
      y.k_per_split = round_up(s.d_in, 32);
      rsvd_gemm(desc->io_dtype, ACC_F32, ACC_F32, y, 1, L);
    }
  }
  // V = X^T . U with U as stored (rounded to the factor type), so that U V^T is the projection the
  // backward pass will use
  if (pl.tuned) rsvd_factor_tuned(desc, s, pl, ws, X, s.ldx, s.d_in, nullptr, false, V, L);
  else rsvd_factor(desc, s, pl, ws, X, s.ldx, s.d_in, U, false, V, L);
  exact_forward_gemm(desc, s, X, W, Y, L);
  return L.status();
}

int acc_linear_bwd_rsvd(const acc_linear_desc* desc, const void* dY, const void* W, const void* U, const void* V,
                        void* dX, void* Gr, void* dW, void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_rsvd(desc, &s);
  if (rc != ACC_OK) return rc;
  if (!dY || !W || !U || !dX || !Gr || (dW && !V)) return ACC_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(W) || !aligned16(U) || !aligned16(V) || !aligned16(dX) || !aligned16(Gr) ||
      !aligned16(dW) || !aligned16(workspace))
    return ACC_ERR_ALIGN;
  const RsvdPlan pl = plan_rsvd(desc, s, true);
  if (!workspace || ws_bytes < pl.total) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  // Gr = U^T . dY [k, d_out], or dY^T . U [d_out, k] in the paper's orientation
  if (pl.tuned) rsvd_factor_tuned(desc, s, pl, (char*)workspace, dY, s.ldy, s.d_out, U, !w_oi, Gr, L);
  else rsvd_factor(desc, s, pl, (char*)workspace, dY, s.ldy, s.d_out, U, !w_oi, Gr, L);
  exact_backward_gemm(desc, s, dY, W, dX, L);
  if (dW) dense_dw(desc, s, V, Gr, dW, L);
  return L.status();
}

int acc_linear_dw(const acc_linear_desc* desc, const void* Xs, const void* Gr, void* dW, void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  if (desc->flags & (ACC_FLAG_SKIP_SKETCH | ACC_FLAG_ONE_LAUNCH)) return ACC_ERR_INVALID_ARG;
  if (!Xs || !Gr || !dW) return ACC_ERR_INVALID_ARG;
  if (!aligned16(Xs) || !aligned16(Gr) || !aligned16(dW)) return ACC_ERR_ALIGN;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  dense_dw(desc, s, Xs, Gr, dW, L);
  return L.status();
}

int acc_linear_bias_grad(const acc_linear_desc* desc, const void* dY, void* dB, void* workspace,
                         size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_desc(desc, &s);
  if (rc != ACC_OK) return rc;
  if (!dY || !dB) return ACC_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(dB) || !aligned16(workspace)) return ACC_ERR_ALIGN;
  if (!workspace || ws_bytes < workspace_bytes(desc, s, true)) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  // Row slabs: enough waves in flight to pull dY at memory speed (16 per work-group, about 16 rows each),
  // few enough partials for one short final pass; the backward workspace holds at least 16 rows of
  // d_out floats (r >= 16).
  int64_t G = ceil_div(s.n, 256);
  if (G > 64) G = 64;
  const int64_t fit = (int64_t)(ws_bytes / ((size_t)s.d_out * sizeof(float)));
  if (G > fit) G = fit;
  const int64_t rows = ceil_div(s.n, G);
  G = ceil_div(s.n, rows);
  float* part = (float*)workspace;
  const dim3 block(64 * kColsumWaves);
  if (desc->io_dtype == ACC_BF16)
    L(colsum_partial_kernel<bf16>, dim3((unsigned)ceil_div(s.d_out, 512), (unsigned)G), block, (const bf16*)dY,
      s.n, s.d_out, s.ldy, rows, part);
  else
    L(colsum_partial_kernel<float>, dim3((unsigned)ceil_div(s.d_out, 256), (unsigned)G), block, (const float*)dY,
      s.n, s.d_out, s.ldy, rows, part);
  const unsigned blocks = (unsigned)ceil_div(s.d_out, 64);
  if (desc->dw_dtype == ACC_BF16)
    L(colsum_final_kernel<bf16>, dim3(blocks), dim3(256), (const float*)part, (int)G, s.d_out, (bf16*)dB);
  else
    L(colsum_final_kernel<float>, dim3(blocks), dim3(256), (const float*)part, (int)G, s.d_out, (float*)dB);
  return L.status();
}

size_t acc_lowrank_workspace_bytes(const acc_linear_desc* desc, int64_t k) {
  Shape s;
  if (validate_lowrank(desc, &s, k, false) != ACC_OK) return 0;
  return plan_lowrank(desc, s, k).total;
}

int acc_lowrank_projector(const acc_linear_desc* desc, int64_t k, const void* left, const void* Gr, void* P,
                          void* workspace, size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_lowrank(desc, &s, k, true);
  if (rc != ACC_OK) return rc;
  if (!left || !Gr || !P) return ACC_ERR_INVALID_ARG;
  if (!aligned16(left) || !aligned16(Gr) || !aligned16(P) || !aligned16(workspace)) return ACC_ERR_ALIGN;
  const LowrankPlan pl = plan_lowrank(desc, s, k);
  if (!workspace || ws_bytes < pl.total) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  char* ws = (char*)workspace;
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  float* z = (float*)(ws + pl.off_z);
  float* yp = (float*)(ws + pl.off_yp);
  float* q1 = (float*)(ws + pl.off_q1);
  // Z [r, k] = Gr . Omega over the output channels, Omega[o, j] from the Philox map with the channel index in
  // the token's place, generated in fp32 while it is staged; the channel range split, partials folded by K4
  {
    acc_linear_desc od = *desc;
    od.row_offset = 0;
    od.r = k;
    GemmParams p{};
    p.A = Gr; p.B = nullptr; p.C = ws + pl.off_part;
    p.M = s.r; p.N = k; p.K = s.d_out;
    p.a_sm = w_oi ? 1 : s.d_out; p.a_sk = w_oi ? s.r : 1;
    p.c_sm = k; p.c_sn = 1;
    p.k_per_split = pl.z_k_per_split;
    p.c_split_stride = s.r * k;
    p.sk = make_sketch_params(&od);
    if (desc->factor_dtype == ACC_BF16) launch_generic<bf16, bf16, float, float, true, true>(p, pl.z_splits, L);
    else launch_generic<float, float, float, float, true, true>(p, pl.z_splits, L);
    reduce_to(ACC_F32, (const float*)(ws + pl.off_part), pl.z_splits, s.r * k, z, L);
  }
  // Yp [d_in, k] = left . Z
  {
    GemmParams p{};
    p.A = left; p.B = z; p.C = yp;
    p.M = s.d_in; p.N = k; p.K = s.r;
    p.a_sm = s.r; p.a_sk = 1; p.b_sk = k; p.b_sn = 1; p.c_sm = k; p.c_sn = 1;
    p.k_per_split = round_up(s.r, 32);
    rsvd_gemm(desc->factor_dtype, ACC_F32, ACC_F32, p, 1, L);
  }
  // P = orthonormal factor of Yp: Cholesky QR, twice
  Shape sk = s;
  sk.r = k;
  RsvdPlan rp{};
  rp.g_gram = pl.g_gram; rp.off_gram_part = pl.off_gram_part; rp.off_gram = pl.off_gram; rp.off_rinv = pl.off_rinv;
  rp.off_rt = pl.off_rt;
  cholesky_qr_pass(sk, rp, ws, s.d_in, s.d_in, yp, q1, nullptr, ACC_F32, nullptr, 0, false, L);
  cholesky_qr_pass(sk, rp, ws, s.d_in, s.d_in, q1, nullptr, P, desc->factor_dtype, nullptr, 0, false, L);
  return L.status();
}

int acc_lowrank_adamw_step(const acc_linear_desc* desc, const acc_adamw_hyper* hyper, const void* P, int64_t k,
                           const void* left, const void* Gr, float* M, float* V, void* W, void* workspace,
                           size_t ws_bytes, void* stream) {
  Shape s;
  int rc = validate_lowrank(desc, &s, P ? k : 0, false);
  if (rc != ACC_OK) return rc;
  if (!hyper || !left || !Gr || !M || !V || !W) return ACC_ERR_INVALID_ARG;
  if (hyper->step < 1 || !(hyper->beta1 >= 0.f && hyper->beta1 < 1.f) || !(hyper->beta2 >= 0.f && hyper->beta2 < 1.f) ||
      !(hyper->eps >= 0.f) || !isfinite(hyper->lr) || !isfinite(hyper->weight_decay) || !isfinite(hyper->scale))
    return ACC_ERR_INVALID_ARG;
  if (!aligned16(P) || !aligned16(left) || !aligned16(Gr) || !aligned16(M) || !aligned16(V) || !aligned16(W) ||
      !aligned16(workspace))
    return ACC_ERR_ALIGN;
  const LowrankPlan pl = plan_lowrank(desc, s, P ? k : 0);
  if (!workspace || ws_bytes < pl.step_total) return ACC_ERR_WORKSPACE;
  if ((rc = check_device()) != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  char* ws = (char*)workspace;
  const bool w_oi = (desc->flags & ACC_FLAG_W_OUT_IN) != 0;
  AdamParams h{};
  h.beta1 = hyper->beta1; h.beta2 = hyper->beta2; h.eps = hyper->eps;
  h.inv_c1 = (float)(1.0 / (1.0 - pow((double)hyper->beta1, (double)hyper->step)));
  h.inv_c2 = (float)(1.0 / (1.0 - pow((double)hyper->beta2, (double)hyper->step)));
  const int64_t kk = P ? k : s.r;            // rows of the moments
  const int64_t count = kk * s.d_out;
  const unsigned blocks = (unsigned)ceil_div(count, 1024);
  void* nrm = ws + pl.off_n;
  const bool fb = desc->factor_dtype == ACC_BF16;
  if (!P) {  // the left factor is the projector: the small factor is the projected gradient
    if (fb) L(adam_factor_kernel<bf16, bf16>, dim3(blocks), dim3(256), (const bf16*)Gr, M, V, (bf16*)nrm, count, h);
    else L(adam_factor_kernel<float, float>, dim3(blocks), dim3(256), (const float*)Gr, M, V, (float*)nrm, count, h);
  } else {
    // T1 [k, r] = P^T . left over the input channels (fp32, channel range split), then the projected gradient
    // R = T1 . Gr [k, d_out] (or Gr . T1^T [d_out, k]) in fp32
    float* t1 = (float*)(ws + pl.off_t1);
    float* proj = (float*)(ws + pl.off_r);
    {
      GemmParams p{};
      p.A = P; p.B = left; p.C = ws + pl.off_part;
      p.M = k; p.N = s.r; p.K = s.d_in;
      p.a_sm = 1; p.a_sk = k; p.b_sk = s.r; p.b_sn = 1; p.c_sm = s.r; p.c_sn = 1;
      p.k_per_split = pl.t1_k_per_split;
      p.c_split_stride = k * s.r;
      rsvd_gemm(desc->factor_dtype, desc->factor_dtype, ACC_F32, p, pl.t1_splits, L);
      L(sum_parts_kernel, dim3((unsigned)ceil_div(k * s.r, 64)), dim3(1024), (const float*)(ws + pl.off_part),
        pl.t1_splits, k * s.r, t1);
    }
    if (fb) {  // projected gradient, moments and normalised step in one launch
      ProjectAdamParams q{};
      q.T1 = t1; q.Gr = (const bf16*)Gr; q.M = M; q.V = V; q.N = (bf16*)nrm;
      q.k = k; q.r = s.r; q.d_out = s.d_out;
      q.b_sk = w_oi ? 1 : s.d_out; q.b_sn = w_oi ? s.r : 1;
      q.c_sm = w_oi ? 1 : s.d_out; q.c_sn = w_oi ? k : 1;
      q.h = h;
      L(project_adam_kernel, dim3((unsigned)ceil_div(k, 64), (unsigned)ceil_div(s.d_out, 64)), dim3(256), q);
    } else {
      GemmParams p{};
      p.C = proj; p.K = s.r;
      p.k_per_split = round_up(s.r, 32);
      if (w_oi) {  // R [d_out, k]: (o, a) = sum_j Gr[o, j] T1[a, j]
        p.A = Gr; p.B = t1; p.M = s.d_out; p.N = k;
        p.a_sm = s.r; p.a_sk = 1; p.b_sk = 1; p.b_sn = s.r; p.c_sm = k; p.c_sn = 1;
        rsvd_gemm(desc->factor_dtype, ACC_F32, ACC_F32, p, 1, L);
      } else {     // R [k, d_out]
        p.A = t1; p.B = Gr; p.M = k; p.N = s.d_out;
        p.a_sm = s.r; p.a_sk = 1; p.b_sk = s.d_out; p.b_sn = 1; p.c_sm = s.d_out; p.c_sn = 1;
        rsvd_gemm(ACC_F32, desc->factor_dtype, ACC_F32, p, 1, L);
      }
      L(adam_factor_kernel<float, float>, dim3(blocks), dim3(256), (const float*)proj, M, V, (float*)nrm, count, h);
    }
  }
  Shape sb = s;
  sb.r = kk;
  sb.ldf = kk;
  const FactorProductOut o{W, desc->io_dtype, s.ldw, true, -hyper->lr * hyper->scale,
                           1.f - hyper->lr * hyper->weight_decay};
  factor_product(desc, sb, P ? P : left, nrm, o, L);
  return L.status();
}

int acc_philox_dump_u32(uint64_t seed, uint64_t row_offset, int64_t n, int64_t r, uint32_t* out,
                        void* stream) {
  if (!out) return ACC_ERR_INVALID_ARG;
  if (n <= 0 || r <= 0 || row_offset % 4) return ACC_ERR_SHAPE;
  if (!aligned16(out)) return ACC_ERR_ALIGN;
  int rc = check_device();
  if (rc != ACC_OK) return rc;
  const int64_t nq = (n + 3) / 4;
  Launcher L{(hipStream_t)stream};
  L(philox_dump_kernel, dim3((unsigned)ceil_div(nq * r, 256)), dim3(256), (uint32_t)(seed & 0xFFFFFFFFu),
    (uint32_t)(seed >> 32), row_offset, nq, r, out);
  return L.status();
}

int acc_sketch_dump(const acc_linear_desc* desc, float* S, void* stream) {
  if (!desc || !S) return ACC_ERR_INVALID_ARG;
  if (!valid_dtype(desc->io_dtype)) return ACC_ERR_DTYPE;
  if (desc->n <= 0 || desc->r <= 0 || desc->row_offset % 4) return ACC_ERR_SHAPE;
  if (!aligned16(S)) return ACC_ERR_ALIGN;
  int rc = check_device();
  if (rc != ACC_OK) return rc;
  const int64_t nq = (desc->n + 3) / 4;
  const dim3 grid((unsigned)ceil_div(nq * desc->r, 256));
  const SketchParams sk = make_sketch_params(desc);
  Launcher L{(hipStream_t)stream};
  if (desc->io_dtype == ACC_F32) L(sketch_dump_kernel<true>, grid, dim3(256), sk, desc->n, desc->r, S);
  else L(sketch_dump_kernel<false>, grid, dim3(256), sk, desc->n, desc->r, S);
  return L.status();
}

int acc_probe_mfma(int shape, int waves_per_simd, int random_data, int64_t iters, float* sink, size_t sink_bytes,
                   double* flops, void* stream) {
  if (!sink || !flops) return ACC_ERR_INVALID_ARG;
  if (shape < 0 || shape > 2 || (waves_per_simd != 1 && waves_per_simd != 2) || iters < 1 || iters > (1 << 24))
    return ACC_ERR_SHAPE;
  if (!aligned16(sink)) return ACC_ERR_ALIGN;
  const unsigned threads = 256u * (unsigned)waves_per_simd, groups = 256;  // one work-group per compute unit
  if (sink_bytes < (size_t)groups * threads * sizeof(float)) return ACC_ERR_WORKSPACE;
  int rc = check_device();
  if (rc != ACC_OK) return rc;
  Launcher L{(hipStream_t)stream};
  if (shape == 0) L(mfma_probe_kernel<0>, dim3(groups), dim3(threads), random_data, iters, sink);
  else if (shape == 1) L(mfma_probe_kernel<1>, dim3(groups), dim3(threads), random_data, iters, sink);
  else L(mfma_probe_kernel<2>, dim3(groups), dim3(threads), random_data, iters, sink);
  *flops = (double)groups * (threads / 64) * (double)iters * 4.0 * (shape == 0 ? 32768.0 : shape == 1 ? 16384.0 : 65536.0);
  return L.status();
}

const char* acc_status_string(int status) {
  switch (status) {
    case ACC_OK: return "ACC_OK";
    case ACC_ERR_INVALID_ARG: return "ACC_ERR_INVALID_ARG: null descriptor/pointer or unknown flag";
    case ACC_ERR_SHAPE: return "ACC_ERR_SHAPE: unsupported size, stride or row_offset";
    case ACC_ERR_ALIGN: return "ACC_ERR_ALIGN: pointer not 16-byte aligned";
    case ACC_ERR_DTYPE: return "ACC_ERR_DTYPE: unknown dtype";
    case ACC_ERR_WORKSPACE: return "ACC_ERR_WORKSPACE: workspace missing or too small";
    case ACC_ERR_HIP: return "ACC_ERR_HIP: HIP runtime error or device is not gfx950";
    default: return "ACC_ERR_UNKNOWN";
  }
}

int acc_version(void) { return kVersion; }

}  // extern "C"
