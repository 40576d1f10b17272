// bf16 GEMM on the 16x16x32 matrix instruction for shapes with at least 192 output tiles of 256 x 256
// (steps F1, B1):  C[M, N] = A[M, K] . B, fp32 accumulate, bf16 output.
//
//   A is row-major with K contiguous (X, dY).
//   B_KMAJOR = true : B is given as Bt[N, K], K contiguous      (dX = dY . W^T reads W as is)
//   B_KMAJOR = false: B is given as  B[K, N], N contiguous      (Y = X . W); the operand is formed with
//                     transposing LDS reads (ds_read_b64_tr_b16).
//
// Work-group tile 256 x 256 x 64, four waves of 128 x 128 (one per SIMD), two 64 KB LDS stages filled global -> LDS
// directly, as in gemm_bf16_tile's large form; but a wave's tile is 8 x 8 blocks of 16 x 16 and a K tile is two
// k-steps of 32 with 64 matrix instructions each.  Why this instruction: it does the same multiply-adds per
// clock as 32x32x16 with half the accumulator traffic per multiply-add, and under the part's power limit it
// sustains about 12 % more on real data (register-only loop: 1.72 - 1.80 against 1.61 PFLOP/s); with it the GEMM
// runs at 2.0 GHz instead of 1.78 GHz.
//
// Registers: 256 accumulators (acc[i][j][e] = C[16 i + lane % 16][16 j + 4 (lane / 16) + e] of the wave's tile:
// the B operand goes first, so a lane holds four consecutive output columns); the eight A operands of a k-step
// are single-buffered (operand i is refilled for the next k-step as soon as block row i is done), the eight B
// operands double-buffered.
// One K tile = 128 slots (one matrix instruction each, at most a few other instructions beside it):
//   slots   0 ..  63  k-step 0; the A / B operands of k-step 1 are read from the same stage; the last four
//                     wave-loads of the next K tile go out (slots 2, 6, 10, 14)
//   slots  64 .. 127  k-step 1; before slot 64 + BAR_Q = 72 the barrier (next K tile landed for every wave, every
//                     wave done reading this stage); after it the operands of the next K tile's k-step 0 are read and
//                     the first twelve wave-loads of the K tile after next go into the stage just released, one
//                     every four slots.  Every transfer then has 70 to 110 slots (1100 to 1800 clocks) to land.
// Measured on the 3B-shaped projection (a step of the layer, same-box pairs): barrier before slot 72 0.547 - 0.552
// ms against 0.553 - 0.557 before slot 80; before slot 88 0.545 - 0.546 against 0.541 - 0.542 before slot 80; all
// sixteen wave-loads after the barrier, one every three slots, 0.565 against 0.553 - 0.557; eight after it and
// eight in the next k-step 0: equal; one wave-load every second slot: 0.561 against 0.550.  With M0 written a slot
// ahead (below) the same comparison again: sixteen after the barrier every three slots 0.574, fourteen every three
// 0.570, ten after it and six before 0.5588, eight and eight every six slots 0.5695 against 0.5585.  Spreading the wave-loads evenly (nine after the barrier, one every six
// slots, seven in the next k-step 0, one every six) 0.5545 against 0.5507; the last of them 14 slots before the
// barrier instead of 58: 0.584 (the transfers need their thousand clocks to land).
// What is left inside a K tile (in-kernel timestamps): 2924 clocks, of which the wait for the transfers is 8 and the
// barrier 67; the matrix instructions alone need 2048 back to back, about 2380 at the rate one wave issues them, and
// the rest is the issue of the sixteen 1 KB transfers per wave (a wave issues in order).  Two waves per SIMD (eight
// waves of 128 x 64) hide that but read 1.5 x the operand bytes from LDS: equal in time.
// A warning about builds, not about the hardware: the slot program indexes the register arrays (acc, a, b0, b1) with
// the slot number, so it is written as a compile-time loop (static_for).  As ordinary loops under #pragma unroll, two
// earlier variants of this kernel (denser wave-loads; four wave-loads sharing one LDS base in M0 through the
// instruction's immediate offset) came out with the arrays in scratch memory, the compiler having unrolled too late:
// same results, thirty times slower.  tests/test_kernel_resources.py checks that the scratch size stays zero.
#pragma once
#include <type_traits>

#include "acc_gemm.h"

namespace acc {

// Swizzle of an N-contiguous B tile for the 16-column operand blocks: the two 16-lane groups that read one
// 16-column block at k rows 8 apart are sent to different 32-byte bank groups as well.
__device__ __forceinline__ int swz_n16(int krow) { return ((krow & 3) << 2) | (((krow >> 3) & 1) << 1); }

// Persistent form: 256 work-groups (one per compute unit) walk over the output tiles b, b + 256, ...; the K pipeline
// runs across output tiles and the read-out of a finished tile rides in the slots of the matrix instructions that
// follow, so a new tile starts without a work-group launch, without a burst of first transfers from every compute
// unit at once and without the matrix pipe idling during an epilogue.
//   * K tile kt + 1 / kt + 2 of the slot program may belong to the next output tile: the transfers take their
//     buffer resources from a per-K-tile choice between the current and the next tile's, the LDS side does not
//     notice.  After the last output tile the "next" tile is the current one again: its first two K tiles are
//     fetched once more into stages nobody reads (branch-free), and drained before the kernel ends.
//   * The first k-step of an output tile multiplies onto zero (the accumulators are never cleared).
//   * In the last K tile block row i (16 x 128 outputs per wave) is final after slot 64 + 8 i + 7.  Its read-out
//     is 16 micro-operations: eight staging writes (convert to bf16, 8 bytes per lane, into one of two private
//     4 KB regions per wave, 16-byte chunk index XOR row) in the slots of block row i + 1, four 16-byte read-backs
//     and four 16-byte global stores (whole 256-byte rows) in the slots of block row i + 2.  Block row 7 is staged
//     behind the last matrix instruction, so no accumulator lives on into the next output tile; the read-backs and
//     stores of rows 6 and 7 ride in the first sixteen slots of the next output tile's first k-step.  (With row 7
//     staged in those slots instead the kernel measured the same, 0.5472 against 0.5509 ms per step; the compiler
//     then keeps two register assignments of the accumulators and 130 copies between them.)
// LDS: two 64 KB stages + 32 KB of staging regions = 160 KB.  Restrictions (host): bf16 output, no accumulation
// into C, no K split, K >= 192.
template <bool B_KMAJOR, int N1 = 12, int S1 = 4, int S0 = 4>
__global__ __launch_bounds__(256) void gemm16_persist_kernel(FastGemmParams p, int n_slots) {
  // schedule of k-step 1: the barrier sits before its slot BAR_Q; N1 wave-loads go out after it, one every S1
  // slots, the other 16 - N1 in the next K tile's k-step 0, one every S0 slots from slot 2
  constexpr int BAR_Q = 8;
  static_assert(BAR_Q + 2 + S1 * (N1 - 1) < 64 && 2 + S0 * (15 - N1) < 64, "wave-load slots");
  constexpr int AEARLY = BAR_Q / 8;  // A operands whose block row is done before the barrier
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = 4, WN = 2, TB = 8;
  constexpr int BM = 256, BN = 256, BK = 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW, NG = A_LOADS + B_LOADS;
  constexpr int BN_CHUNKS = BN / 8;
  constexpr int REGION = 16 * 256;  // one staged block row: 16 rows x 128 bf16
  static_assert(NG == 16, "the slot program places sixteen wave-loads per K tile");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int KT = (int)(p.K / BK);

  // ---- global -> LDS sources (relative to a tile's buffer resources) ----
  uint32_t a_src[A_LOADS], b_src[B_LOADS];
#pragma unroll
  for (int t = 0; t < A_LOADS; ++t) {
    const int row = (t * NW + wave) * 8 + (lane >> 3);
    a_src[t] = (uint32_t)(row * p.lda * 2 + (((lane & 7) ^ swz(row)) << 4));
  }
#pragma unroll
  for (int t = 0; t < B_LOADS; ++t) {
    if (B_KMAJOR) {
      const int row = (t * NW + wave) * 8 + (lane >> 3);
      b_src[t] = (uint32_t)(row * p.ldb * 2 + (((lane & 7) ^ swz(row)) << 4));
    } else {
      constexpr int ROWS = 64 / BN_CHUNKS;
      const int krow = (t * NW + wave) * ROWS + lane / BN_CHUNKS;
      b_src[t] = (uint32_t)(krow * p.ldb * 2 + (((lane % BN_CHUNKS) ^ swz_n16(krow)) << 4));
    }
  }
  const uint32_t b_kstep = B_KMAJOR ? BK * 2 : (uint32_t)(BK * p.ldb * 2);
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;

  struct TileRef {
    u32x4 a_rsrc, b_rsrc;
    int64_t m0, n0;
  };
  auto tile_ref = [&](int idx) -> TileRef {
    int tm, tn;
    xcd_tile(p, idx, tm, tn);
    TileRef r;
    r.m0 = (int64_t)tm * BM;
    r.n0 = (int64_t)tn * BN;
    r.a_rsrc = make_rsrc(p.A + r.m0 * p.lda, ((p.M - r.m0 - 1) * p.lda + p.K) * 2);
    r.b_rsrc = B_KMAJOR ? make_rsrc(p.B + r.n0 * p.ldb, ((p.N - r.n0 - 1) * p.ldb + p.K) * 2)
                        : make_rsrc(p.B + r.n0, ((p.K - 1) * p.ldb + (p.N - r.n0)) * 2);
    return r;
  };
  auto issue_one = [&](const TileRef& r, int g, int kt, uint32_t stage) {
    if (g < A_LOADS) buffer_to_lds_b128(r.a_rsrc, a_src[g], (uint32_t)kt * (BK * 2), stage + (g * NW + wave) * 1024);
    else buffer_to_lds_b128(r.b_rsrc, b_src[g - A_LOADS], (uint32_t)kt * b_kstep,
                            stage + A_BYTES + ((g - A_LOADS) * NW + wave) * 1024);
  };

  // The same transfer in two parts, as the slot program issues it: M0 (the LDS destination) is written at the end
  // of the slot before, so that the slot of the transfer holds the matrix instruction and the transfer alone (the
  // matrix instruction is the wait state the hardware asks for between a write of M0 and its use).  Against the
  // one-piece form (M0 write, s_nop, transfer in one slot): 0.5458 against 0.5502 ms per step, three same-box pairs.
  uint32_t m0_token = 0;
  auto set_m0 = [&](int g, uint32_t stage_wave) {  // stage_wave: the stage's LDS address + wave * 1024
    const int part = g < A_LOADS ? g * NW * 1024 : A_BYTES + (g - A_LOADS) * NW * 1024;  // a constant per wave-load
    asm volatile("s_add_u32 m0, %1, %2" : "={m0}"(m0_token) : "s"(stage_wave), "s"(part) : "scc");
  };
  auto issue_at_m0 = [&](const TileRef& r, int g, int kt) {
    if (g < A_LOADS)
      asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" ::"v"(a_src[g]), "s"(r.a_rsrc), "s"((uint32_t)kt * (BK * 2)), "{m0}"(m0_token) : "memory");
    else
      asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" ::"v"(b_src[g - A_LOADS]), "s"(r.b_rsrc), "s"((uint32_t)kt * b_kstep), "{m0}"(m0_token) : "memory");
  };

  // ---- LDS read offsets of the operands (see gemm16_tile) ----
  const int rswz = swz(l16);
  const int a_row = (wm * TB * 16 + l16) * 128;
  int kc[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) kc[s] = ((4 * s + g4) ^ rswz) << 4;
  auto read_a = [&](const char* st, int s, int i) -> bf16x8 { return lds_read_b128(st, a_row + i * 2048 + kc[s]); };
  int b_rd[TB];
#pragma unroll
  for (int j = 0; j < TB; ++j) {
    if (B_KMAJOR) {
      b_rd[j] = A_BYTES + (wn * TB * 16 + j * 16 + l16) * 128;
    } else {
      const int n_off = (wn * TB + j) * 16 + 4 * (l16 & 3);
      const int krow = 8 * g4 + (l16 >> 2);
      b_rd[j] = A_BYTES + krow * (BN * 2) + (((n_off >> 3) ^ swz_n16(krow)) << 4) + (n_off & 7) * 2;
    }
  }
  auto read_b = [&](const char* st, int s, int j) -> bf16x8 {
    if (B_KMAJOR) {
      return lds_read_b128(st, b_rd[j] + kc[s]);
    } else {
      const s16x4 lo = lds_read_tr16_b64(st, b_rd[j] + 32 * s * (BN * 2));
      const s16x4 hi = lds_read_tr16_b64(st, b_rd[j] + (32 * s + 4) * (BN * 2));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  // slots of the XCD tile map that hold no tile are skipped
  auto next_slot = [&](int idx) -> int {
    int tm, tn;
    for (idx += (int)gridDim.x; idx < n_slots && !xcd_tile(p, idx, tm, tn);) idx += (int)gridDim.x;
    return idx;
  };
  const int first_idx = next_slot((int)blockIdx.x - (int)gridDim.x);
  const bool has_tile = first_idx < n_slots;
  TileRef cur_t = tile_ref(has_tile ? first_idx : 0);

  // ---- read-out of a finished block row ----
  // acc[i][j][e] = C[16 i + l16][16 j + 4 g4 + e] of the wave's 128 x 128 tile.
  bf16* __restrict__ C = (bf16*)p.C;
  char* const regions = smem + 2 * STAGE + wave * (2 * REGION);
  // staging address of this lane's 8 bytes of block column j: chunk (2 j + g4 / 2) XOR row, half g4 % 2
  const uint32_t w_base = ((uint32_t)(uintptr_t)regions + l16 * 256 + (l16 << 4) + (g4 & 1) * 8) ^ (uint32_t)((g4 >> 1) << 4);
  // read-back t: row 4 t + g4, 16-byte chunk l16 (8 columns)
  const int r_addr = g4 * 256 + ((l16 ^ g4) << 4);
  const uint32_t c_row_bytes = (uint32_t)(p.ldc * 2);
  auto wave_fence = [&]() {  // lanes read what other lanes of the wave wrote
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  __amdgpu_buffer_rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc((void*)C, 0, 0, 0x00020000);  // empty: nothing to store yet
  uint32_t c_voff = 0xFFFFFFF0u;
  auto set_output = [&](const TileRef& t) {
    const int64_t gm_base = t.m0 + wm * TB * 16, gn_base = t.n0 + wn * TB * 16;
    int64_t c_rows = p.M - gm_base;
    if (c_rows > TB * 16) c_rows = TB * 16;
    const int64_t c_bytes = (c_rows > 0 && gn_base < p.N) ? ((c_rows - 1) * p.ldc + (p.N - gn_base)) * 2 : 0;
    c_rs = __builtin_amdgcn_make_buffer_rsrc((void*)(C + gm_base * p.ldc + gn_base), 0, (int)(uint32_t)c_bytes,
                                             0x00020000);
    c_voff = gn_base + l16 * 8 < p.N ? (uint32_t)((g4 * p.ldc + l16 * 8) * 2) : 0xFFFFFFF0u;  // columns past N: dropped
  };
  f32x4 acc[TB][TB];
  auto stage_write = [&](int i, int j) {
    bf16x4 v;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = (bf16)acc[i][j][t];
    typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
    *(lds_bf16x4_ptr)(uintptr_t)((w_base ^ (uint32_t)(j << 5)) + (i & 1) * REGION) = v;
  };
  auto read_back = [&](int i, int t) -> u32x4 {
    // row 4 t + g4: its chunk swizzle is (4 t + g4) & 15 = (4 t) ^ g4 (t < 4, g4 < 4: disjoint bits)
    return *(const u32x4*)(regions + (i & 1) * REGION + t * 1024 + (r_addr ^ (t << 6)));
  };
  auto store_back = [&](int i, int t, u32x4 v) {
    const uint32_t soff = (uint32_t)(i * 16 + t * 4) * c_row_bytes;
    __builtin_amdgcn_raw_buffer_store_b128(v, c_rs, c_voff, soff, 0);
  };
  u32x4 back[4];
  // What is left of the previous output tile's read-out, as work for slots 0 .. 15 of the next K tile: block rows 6
  // and 7 sit in the two staging regions when an output tile's last K tile ends (row 7 is staged behind that K
  // tile's last matrix instruction, so no accumulator lives on into the next output tile and the compiler keeps
  // one register assignment for all of them); their read-backs and global stores follow here.
  auto carry_slot = [&](int q) {
    if (q == 0) wave_fence();
    if (q < 4) back[q] = read_back(6, q);
    else if (q < 8) store_back(6, q - 4, back[q - 4]);
    else if (q < 12) back[q - 8] = read_back(7, q - 8);
    else store_back(7, q - 12, back[q - 12]);
  };

  bf16x8 a[TB], b0[TB], b1[TB];
  // A matrix instruction has no side effect, so nothing but heuristics keeps it in the slot it is written in (one
  // build of this kernel had the 72 of a K tile's first slots behind the barrier, all transfers and LDS reads of
  // those slots running with the matrix pipe idle: 15 % slower).  The empty statement below makes the result a value
  // the compiler must have at this point of the program order; it emits nothing.
  auto pin = [](f32x4& v) { asm volatile("" : "+a"(v)); };

  // One K tile (see the slot program at the top of this file).  sc: its stage.  ref1 / k1: the K tile that follows
  // (its wave-loads 12 .. 15 go out here), ref2 / k2: the one after that (wave-loads 0 .. 11).
  auto ktile = [&](int sc, const TileRef& ref1, int k1, const TileRef& ref2, int k2, auto zero, auto carry, auto fin) {
    constexpr bool ZERO = decltype(zero)::value, CARRY = decltype(carry)::value, FINAL = decltype(fin)::value;
    const char* cur = smem + sc * STAGE;
    const char* nxt = smem + (sc ^ 1) * STAGE;
    const uint32_t cur_lds = smem_lds + sc * STAGE, nxt_lds = smem_lds + (sc ^ 1) * STAGE;
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, 64>([&](auto slot) {  // k-step 0
      constexpr int q = decltype(slot)::value;
      constexpr int i = q >> 3, j = q & 7;
      if (q == 0) a[7] = read_a(cur, 0, 7);
      if constexpr (ZERO) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0[j], a[i], z, 0, 0, 0);
      } else {
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b0[j], a[i], acc[i][j], 0, 0, 0);
      }
      pin(acc[i][j]);
      if (q >= 2 && (q - 2) % S0 == 0 && (q - 2) / S0 < NG - N1) issue_at_m0(ref1, N1 + (q - 2) / S0, k1);
      if (j == 0 && i >= 1) a[i - 1] = read_a(cur, 1, i - 1);
      if (j == 4) b1[i] = read_b(cur, 1, i);
      if (CARRY && q < 16) carry_slot(q);
      if (q >= 1 && (q - 1) % S0 == 0 && (q - 1) / S0 < NG - N1) set_m0(N1 + (q - 1) / S0, nxt_lds + wave * 1024);
      __builtin_amdgcn_sched_barrier(0);
    });
    static_for<0, 64>([&](auto slot) {  // k-step 1
      constexpr int q = decltype(slot)::value;
      constexpr int i = q >> 3, j = q & 7;
      if (q == 0) a[7] = read_a(cur, 1, 7);
      if (q == BAR_Q) {
        wait_vmcnt0();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1[j], a[i], acc[i][j], 0, 0, 0);
      pin(acc[i][j]);
      if (q >= BAR_Q + 2 && (q - BAR_Q - 2) % S1 == 0 && (q - BAR_Q - 2) / S1 < N1)
        issue_at_m0(ref2, (q - BAR_Q - 2) / S1, k2);
      // operands of the next K tile's k-step 0: A operand i once block row i is done and the barrier is passed
      static_for<0, AEARLY>([&](auto early) {
        constexpr int e = decltype(early)::value;
        if (q == BAR_Q + 4 * e) a[e] = read_a(nxt, 0, e);
      });
      if (j == 0 && i >= AEARLY + 1) a[i - 1] = read_a(nxt, 0, i - 1);
      {
        constexpr int SP = (63 - BAR_Q - 1) / 8;  // B operands of the next K tile, spread over the rest of the k-step
        if (q >= BAR_Q + 1 && (q - BAR_Q - 1) % SP == 0 && (q - BAR_Q - 1) / SP < 8)
          b0[(q - BAR_Q - 1) / SP] = read_b(nxt, 0, (q - BAR_Q - 1) / SP);
      }
      if constexpr (FINAL) {
        if (i >= 2 && j == 0) wave_fence();
        if (i >= 1) stage_write(i - 1, j);
        if (i >= 2 && j < 4) back[j] = read_back(i - 2, j);
        if (i >= 2 && j >= 4) store_back(i - 2, j - 4, back[j - 4]);
      }
      if (q >= BAR_Q + 1 && (q - BAR_Q - 1) % S1 == 0 && (q - BAR_Q - 1) / S1 < N1)
        set_m0((q - BAR_Q - 1) / S1, cur_lds + wave * 1024);
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (FINAL) {
      static_for<0, TB>([&](auto col) { stage_write(TB - 1, decltype(col)::value); });
    }
  };

  // ---- prologue of the work-group's first tile ----
  if (has_tile) {
#pragma unroll
    for (int g = 0; g < NG; ++g) issue_one(cur_t, g, 0, smem_lds);
#pragma unroll
    for (int g = 0; g < N1; ++g) issue_one(cur_t, g, 1, smem_lds + STAGE);
  }
  if (p.red_count) {  // side job: this work-group's share of the pending partial sums (see gemm_bf16_tile)
    for (int64_t e = ((int64_t)blockIdx.x * (NW * 64) + tid) * 4; e < p.red_count; e += p.red_stride) {
      f32x4 sum = *(const f32x4*)(p.red_part + e);
#pragma unroll 8
      for (int g = 1; g < p.red_G; ++g) sum += *(const f32x4*)(p.red_part + (int64_t)g * p.red_count + e);
      const int64_t eo = p.red_ld == p.red_row ? e : (e / p.red_row) * p.red_ld + e % p.red_row;
      if (p.red_out_bf16) {
        bf16x4 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = (bf16)sum[t];
        *(bf16x4*)((bf16*)p.red_out + eo) = v;
      } else {
        *(f32x4*)((float*)p.red_out + eo) = sum;
      }
    }
  }
  if (!has_tile) return;
  wait_vmcnt0();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TB - 1; ++i) a[i] = read_a(smem, 0, i);
#pragma unroll
  for (int j = 0; j < TB; ++j) b0[j] = read_b(smem, 0, j);

  using T = std::true_type;
  using F = std::false_type;
  int par = 0;
  for (int idx = first_idx;;) {
    const int next_idx = next_slot(idx);
    const bool has_next = next_idx < n_slots;
    const TileRef next_t = has_next ? tile_ref(next_idx) : cur_t;
    // K tile 0: multiplies onto zero and finishes the previous read-out (before the first output tile the staging
    // regions hold nothing and the output resource is empty, so those stores are dropped)
    ktile(par, cur_t, 1, cur_t, 2, T{}, T{}, F{});
    // K tiles 1 .. KT - 2; the last of them already fetches the next output tile's first K tile
    for (int kt = 1; kt + 1 < KT; ++kt) {
      const bool wraps = kt + 2 >= KT;
      ktile((kt + par) & 1, cur_t, kt + 1, wraps ? next_t : cur_t, wraps ? 0 : kt + 2, F{}, F{}, F{});
    }
    const int kt = KT - 1;
    set_output(cur_t);
    ktile((kt + par) & 1, next_t, 0, next_t, 1, F{}, F{}, T{});       // last: the read-out starts
    if (!has_next) break;
    cur_t = next_t;
    par = (par + KT) & 1;
    idx = next_idx;
  }
  // no tile follows: block rows 6 and 7 are read out here
#pragma unroll
  for (int q = 0; q < 16; ++q) carry_slot(q);
  wait_vmcnt0();  // the surplus transfers of the last two K tiles must have landed before the LDS is released
}

}  // namespace acc
