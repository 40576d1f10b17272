// Tuned bf16 MFMA GEMM for gfx950 (steps F1, B1, B3):  C[M, N] = A[M, K] . B, fp32 accumulate.
//
//   A is row-major with K contiguous (X, dY, Xs).
//   B_KMAJOR = true : B is given as Bt[N, K], K contiguous      (dX = dY . W^T reads W as is)
//   B_KMAJOR = false: B is given as  B[K, N], N contiguous      (Y = X . W, dW = Xs . Gr); the MFMA
//                     operand is formed with transposing LDS reads (ds_read_b64_tr_b16).
//
// Work-group tile (WM*TM*32) x (WN*TN*32) x 64, WM x WN waves, each wave TM x TN MFMA 32x32x16 tiles.
// Tiles travel global -> LDS directly (global_load_lds_dwordx4, no staging registers); LDS is double
// buffered, one barrier per K tile, and the MFMAs run one k-step behind the LDS reads so that the
// reads after the barrier are covered by the last k-step of the previous tile.
// K % 64 == 0; M and N arbitrary (loads past the last row read zero through the buffer resource,
// stores are predicated); N % 8 == 0; every operand smaller than 4 GiB.
#pragma once
#include <type_traits>

#include "acc_common.h"

namespace acc {

struct FastGemmParams {
  const bf16* A;
  const bf16* B;
  void* C;
  int64_t M, N, K;
  int64_t lda, ldb, ldc;  // row strides in elements
  int tiles_m, tiles_n;   // work-group tiles along M and N
  int super_m, super_n;   // XCD super-tile shape (in tiles), super_m * super_n == 32
  int supers_n;           // super-tiles along N
  // Optional side job, done while the first tile's transfers are in flight: the reduction of the
  // split-token partials a sketch kernel left just before this launch,
  // red_out[e] = sum_g red_part[g * red_count + e] (same order as reduce_partials_kernel, so the same
  // bits).  red_count == 0: none.  red_count % 4 == 0.
  const float* red_part;
  void* red_out;
  int64_t red_count;
  int64_t red_stride;     // elements all work-groups of the launch cover per sweep: grid * threads * 4
  int red_G;
  int red_out_bf16;       // 1: red_out is bf16, 0: float
  int64_t red_row, red_ld;  // the result has rows of red_row elements (red_row % 4 == 0) stored red_ld apart
  int accumulate;         // 0: C = A . B;  1: C = beta C + alpha (A . B) (a bf16 C rounds the product, then the sum)
  float alpha, beta;      // used when accumulate; 1, 1 is the plain sum
  // Optional split of the K range over work-groups (skinny products whose M x N tiles alone do not fill
  // the chip): tile_blocks == 0 means no split.  Block b works on tile b % tile_blocks and K range
  // [s * k_per_split, min(K, (s + 1) * k_per_split)), s = b / tile_blocks, and stores its partial product
  // at C + s * c_split_stride.  k_per_split % 64 == 0.
  int tile_blocks;
  int64_t k_per_split;
  int64_t c_split_stride;
  int64_t kb_rows;        // N-contiguous B only: rows of B that exist (0 = K); K may exceed it when A is
                          // zero-padded along K, the missing rows of B then read as zero
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// LDS layout of a K-contiguous tile: 128-byte rows (64 bf16), 16-byte chunk c of row `row` stored at
// chunk position c ^ swz(row).  The LDS has 64 four-byte banks, so two consecutive rows cover the
// whole bank window; (row >> 1) & 7 makes 16 consecutive rows reading one logical chunk hit 16
// different bank groups (ds_read_b128 serves 16 lanes per clock).
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// LDS layout of an N-contiguous B tile: rows of BN bf16 (one k each), 16-byte chunk c of row k stored
// at chunk position c ^ ((k & 3) << 2): the 4 k-rows x 2 column groups that 32 lanes of a transposing
// read touch fall on 8 different 32-byte bank groups.
__device__ __forceinline__ int swz_n(int krow) { return (krow & 3) << 2; }

__device__ __forceinline__ bf16x8 lds_read_b128(const char* lds, int byte_off) {
  return *(const bf16x8*)(lds + byte_off);
}

// 4 x 16 transposed read (ds_read_b64_tr_b16): the 16 lanes of a group give 4 rows x 4 chunks of 4
// elements; lane l of the group receives element l of each of the 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr16_b64(const char* lds, int byte_off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(uintptr_t)(uint32_t)(uintptr_t)(lds + byte_off));
}

// Buffer resource over [base, base + bytes): loads beyond `bytes` return zero instead of faulting.
__device__ __forceinline__ u32x4 make_rsrc(const void* base, int64_t bytes) {
  const uint32_t n = bytes > 0xFFFFFFFFll ? 0xFFFFFFFFu : (bytes < 0 ? 0u : (uint32_t)bytes);
  const uint64_t a = (uint64_t)(uintptr_t)base;
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xFFFFu);  // 48-bit base, stride 0
  r[2] = __builtin_amdgcn_readfirstlane(n);                              // num_records in bytes
  r[3] = 0x00020000u;                                                    // raw buffer, 32-bit data format
  return r;
}

// 64 lanes x 16 bytes, global -> LDS without passing through registers (buffer_load_dwordx4 ... lds).
// Lane i reads rsrc[voffset_i + soffset] and lands at LDS byte (lds_wave_base + 16 * i); lds_wave_base
// and soffset are wave-uniform.  Counted by vmcnt.
// Written as inline assembly on purpose: when the compiler sees LDS-DMA it puts s_waitcnt vmcnt(0) in
// front of every LDS read it cannot prove disjoint (all transposing reads), which serialises the
// pipeline.  The caller therefore orders these transfers itself: wait_vmcnt0() + barrier before any
// read of the destination stage.
__device__ __forceinline__ void buffer_to_lds_b128(u32x4 rsrc, uint32_t voffset, uint32_t soffset,
                                                   uint32_t lds_wave_base) {
  // s_nop: one wait state between the scalar write of M0 (placed by the compiler right before this block) and
  // the transfer that reads it, as the ISA asks for
  asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
               :
               : "v"(voffset), "s"(rsrc), "s"(soffset), "{m0}"(lds_wave_base)  // M0 = LDS destination
               : "memory");
}

// s_waitcnt vmcnt(0) (expcnt / lgkmcnt untouched): all global -> LDS transfers of this wave landed.
__device__ __forceinline__ void wait_vmcnt0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Map the linear work-group id to an output tile so that the 32 tiles resident on one XCD
// (work-groups are dealt round-robin to the 8 XCDs) form a super_m x super_n block that shares
// A and B panels in that XCD's L2.  Returns false for padding work-groups.
__device__ __forceinline__ bool xcd_tile(const FastGemmParams& p, int b, int& tm, int& tn) {
  if (p.tile_blocks) {  // split-K launches of skinny products: few tiles, plain order, no padding blocks
    tm = b % p.tiles_m;
    tn = b / p.tiles_m;
    return tn < p.tiles_n;
  }
  const int xcd = b & 7, local = b >> 3;
  const int sid = (local >> 5) * 8 + xcd;  // super-tile id, N fastest
  const int in = local & 31;
  const int sm = sid / p.supers_n, sn = sid - sm * p.supers_n;
  tm = sm * p.super_m + in % p.super_m;
  tn = sn * p.super_n + in / p.super_m;
  return tm < p.tiles_m && tn < p.tiles_n;
}

// The work of one work-group: output tile number b (see xcd_tile), using the dynamic LDS at smem.
template <int WM, int WN, int TM, int TN, bool B_KMAJOR, typename TC>
__device__ __forceinline__ void gemm_bf16_tile(const FastGemmParams& p, int b, char* smem) {
  constexpr int NW = WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64;
  constexpr int A_BYTES = BM * BK * 2;
  constexpr int B_BYTES = BN * BK * 2;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW;  // 1 KB wave-loads per wave and K tile
  constexpr int B_LOADS = B_BYTES / 1024 / NW;
  constexpr int BN_CHUNKS = BN / 8;             // 16-byte chunks per row of an N-contiguous B tile
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile/waves");
  static_assert(B_KMAJOR || (BN_CHUNKS >= 16 && 64 % BN_CHUNKS == 0), "B tile shape");

  int tm, tn;
  int64_t k0 = 0, k1 = p.K;  // this work-group's K range
  int split = 0;
  if (p.tile_blocks) {
    split = b / p.tile_blocks;
    b -= split * p.tile_blocks;
    k0 = (int64_t)split * p.k_per_split;
    k1 = k0 + p.k_per_split < p.K ? k0 + p.k_per_split : p.K;
  }
  const bool has_tile = xcd_tile(p, b, tm, tn);
  if (!has_tile && p.red_count == 0) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  // ---- global source of every 16-byte chunk this lane moves ----
  // Wave-load t of wave w fills LDS bytes [(t * NW + w) * 1024, +1024) of the operand's tile: lane i
  // supplies the chunk that belongs at position i of that kilobyte.  Sources are byte offsets into
  // buffer resources that start at the tile's first row / column; rows past the end of the matrix
  // read as zero (their products are never stored).
  const int64_t am0 = m0, bn0 = n0;
  const int64_t kb = p.kb_rows ? p.kb_rows : p.K;
  const u32x4 a_rsrc = make_rsrc(p.A + am0 * p.lda + k0, ((p.M - am0 - 1) * p.lda + p.K - k0) * 2);
  const u32x4 b_rsrc =
      B_KMAJOR ? make_rsrc(p.B + bn0 * p.ldb + k0, ((p.N - bn0 - 1) * p.ldb + p.K - k0) * 2)
               : make_rsrc(p.B + k0 * p.ldb + bn0, kb > k0 ? ((kb - k0 - 1) * p.ldb + (p.N - bn0)) * 2 : 0);
  uint32_t a_src[A_LOADS];
#pragma unroll
  for (int t = 0; t < A_LOADS; ++t) {
    const int row = (t * NW + wave) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(row);
    a_src[t] = (uint32_t)(row * p.lda * 2 + c * 16);
  }
  uint32_t b_src[B_LOADS];
#pragma unroll
  for (int t = 0; t < B_LOADS; ++t) {
    if (B_KMAJOR) {
      const int row = (t * NW + wave) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz(row);
      b_src[t] = (uint32_t)(row * p.ldb * 2 + c * 16);
    } else {
      constexpr int ROWS = 64 / BN_CHUNKS;  // k-rows per wave-load
      const int krow = (t * NW + wave) * ROWS + lane / BN_CHUNKS;
      const int c = (lane % BN_CHUNKS) ^ swz_n(krow);
      b_src[t] = (uint32_t)(krow * p.ldb * 2 + c * 16);
    }
  }
  const uint32_t b_kstep = B_KMAJOR ? BK * 2 : (uint32_t)(BK * p.ldb * 2);  // bytes per K tile

  auto issue_loads = [&](int kt, uint32_t stage) {
#pragma unroll
    for (int t = 0; t < A_LOADS; ++t)
      buffer_to_lds_b128(a_rsrc, a_src[t], (uint32_t)kt * (BK * 2), stage + (t * NW + wave) * 1024);
#pragma unroll
    for (int t = 0; t < B_LOADS; ++t)
      buffer_to_lds_b128(b_rsrc, b_src[t], (uint32_t)kt * b_kstep, stage + A_BYTES + (t * NW + wave) * 1024);
  };

  // ---- LDS read offsets of this lane's MFMA operands ----
  const int lrow = lane & 31, kg = lane >> 5;
  int a_rd[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_rd[i] = (wm * TM * 32 + i * 32 + lrow) * 128;
  int b_rd[TN][2];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (B_KMAJOR) {
      b_rd[j][0] = b_rd[j][1] = A_BYTES + (wn * TN * 32 + j * 32 + lrow) * 128;
    } else {
      // 16-lane group g = lane / 16: columns 16 * (g & 1) .., k rows 8 * (g >> 1) ..; lane i of the
      // group reads k row i / 4 (+ 4 for the second half), 4-element chunk i % 4.
      const int g = lane >> 4, i16 = lane & 15;
      const int n_off = (wn * TN + j) * 32 + 16 * (g & 1) + 4 * (i16 & 3);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int krow = 8 * (g >> 1) + 4 * h + (i16 >> 2);
        b_rd[j][h] = A_BYTES + krow * (BN * 2) + (((n_off >> 3) ^ swz_n(krow)) << 4) + (n_off & 7) * 2;
      }
    }
  }
  const int a_swz = swz(lrow);  // rows i * 32 + lrow share swz(lrow)

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int KT = (int)((k1 - k0) / BK);
  bf16x8 af[2][TM], bfr[2][TN];

  auto read_a1 = [&](const char* st, int s, int i, bf16x8(&dst)[TM]) {
    dst[i] = lds_read_b128(st, a_rd[i] + (((2 * s + kg) ^ a_swz) << 4));
  };
  auto read_b1 = [&](const char* st, int s, int j, bf16x8(&dst)[TN]) {
    if (B_KMAJOR) {
      dst[j] = lds_read_b128(st, b_rd[j][0] + (((2 * s + kg) ^ a_swz) << 4));
    } else {
      const s16x4 lo = lds_read_tr16_b64(st, b_rd[j][0] + 16 * s * (BN * 2));
      const s16x4 hi = lds_read_tr16_b64(st, b_rd[j][1] + 16 * s * (BN * 2));
      dst[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };
  auto issue_one = [&](int g, int kt, uint32_t stage) {  // g-th wave-load of a K tile (A first, then B)
    if (g < A_LOADS) buffer_to_lds_b128(a_rsrc, a_src[g], (uint32_t)kt * (BK * 2), stage + (g * NW + wave) * 1024);
    else buffer_to_lds_b128(b_rsrc, b_src[g - A_LOADS], (uint32_t)kt * b_kstep,
                            stage + A_BYTES + ((g - A_LOADS) * NW + wave) * 1024);
  };

  // One k-step with a fixed instruction order: MFMA q of the step carries (at most) one operand read
  // for the next step and, every G_EVERY MFMAs, one global->LDS wave-load of a later tile.  Fences
  // keep the compiler from clustering the memory instructions, which stalls the wave in VMEM issue
  // while the texture path drains and starves the MFMA pipe.
  constexpr int NM = TM * TN;
  constexpr int NG_TOTAL = A_LOADS + B_LOADS;
  // The transfers of a tile are spread over the first two k-steps after the barrier that releases their
  // stage (the last k-step of one loop trip and the first of the next): they then have two to three
  // k-steps to land before the next barrier.  Spread over the three k-steps that end at that barrier, as
  // before, the last third had under one k-step (-1.9 % on a step, -8 % on a GEMM whose input comes from
  // HBM); all in one k-step, one per MFMA, stalls VMEM issue (+1 % step time).
  constexpr int G_STEPS = 2;                                   // k-steps that carry wave-loads
  constexpr int G_PER_STEP = (NG_TOTAL + G_STEPS - 1) / G_STEPS;
  constexpr int G_EVERY = NM / G_PER_STEP > 0 ? NM / G_PER_STEP : 1;
  auto kstep = [&](const bf16x8(&ca)[TM], const bf16x8(&cb)[TN], const char* rd_stage, int rd_s,
                   bf16x8(&na)[TM], bf16x8(&nb)[TN], int g_first, int g_count, int kt_next, uint32_t nxt) {
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      const int i = q / TN, j = q % TN;
      // B operand first: the product comes out transposed, lane = output row, 4 consecutive registers =
      // 4 consecutive output columns, which is what the epilogue packs
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cb[j], ca[i], acc[i][j], 0, 0, 0);
      if constexpr (NM >= 2 * (TM + TN)) {  // enough MFMAs: one read on every second one (+0.4 % on a step
                                            // against eight reads on the first eight MFMAs of sixteen)
        // in the order the next k-step consumes them (its MFMA i * TN + j needs a[i] and b[j]): a0, every b,
        // then the other a: each read is then at least ten MFMAs ahead of its use
        if (q % 2 == 0) {
          const int r = q / 2;
          if (r == 0) read_a1(rd_stage, rd_s, 0, na);
          else if (r <= TN) read_b1(rd_stage, rd_s, r - 1, nb);
          else if (r < TM + TN) read_a1(rd_stage, rd_s, r - TN, na);
        }
      } else if constexpr (NM >= TM + TN) {
        if (q < TM) read_a1(rd_stage, rd_s, q, na);
        else if (q < TM + TN) read_b1(rd_stage, rd_s, q - TM, nb);
      } else {  // small tiles: fewer MFMAs than operand reads, several reads per MFMA
#pragma unroll
        for (int i = q; i < TM + TN; i += NM) {
          if (i < TM) read_a1(rd_stage, rd_s, i, na);
          else read_b1(rd_stage, rd_s, i - TM, nb);
        }
      }
      if constexpr (NM < G_PER_STEP) {  // fewer MFMAs than wave-loads in a k-step: several loads per MFMA
#pragma unroll
        for (int i = q; i < G_PER_STEP; i += NM)
          if (i < g_count && g_first + i < NG_TOTAL) issue_one(g_first + i, kt_next, nxt);
      } else {
        if constexpr (NM >= 2 * (TM + TN) && G_EVERY == 2) {  // transfers on the odd MFMAs, reads on the even ones
          if (q % 2 == 1 && q / 2 < g_count && g_first + q / 2 < NG_TOTAL) issue_one(g_first + q / 2, kt_next, nxt);
        } else {
          if (q % G_EVERY == 0 && q / G_EVERY < g_count && g_first + q / G_EVERY < NG_TOTAL)
            issue_one(g_first + q / G_EVERY, kt_next, nxt);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // prologue: tile 0 -> stage 0, operands of its first k-step -> registers
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;  // LDS byte address of the dynamic segment
  if (has_tile) issue_loads(0, smem_lds);
  if (p.red_count) {  // side job: this work-group's share of the partial sums, 4 elements per lane
    for (int64_t e = ((int64_t)b * (NW * 64) + tid) * 4; e < p.red_count; e += p.red_stride) {
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
    if (!has_tile) return;
  }
  wait_vmcnt0();
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) read_a1(smem, 0, i, af[0]);
#pragma unroll
  for (int j = 0; j < TN; ++j) read_b1(smem, 0, j, bfr[0]);
  if (KT > 1) {  // first half of tile 1 (the loop's last k-step does this for the tiles after it)
#pragma unroll
    for (int g = 0; g < G_PER_STEP; ++g)
      if (g < NG_TOTAL) issue_one(g, 1, smem_lds + STAGE);
  }

  // One K tile.  `ahead` (a compile-time constant at each call below): the tile after next exists, so the last
  // k-step carries the first half of its transfers; the two last K tiles of the range are a second copy of the
  // body without them, which keeps eight uniform branches per K tile out of the steady-state loop.
  auto ktile = [&](int kt, auto ahead) {
    const char* cur = smem + (kt & 1) * STAGE;
    const char* nxt = smem + ((kt + 1) & 1) * STAGE;
    const uint32_t nxt_lds = smem_lds + ((kt + 1) & 1) * STAGE;
    // Branch-free first k-step: the last iteration re-loads half of its own tile into the idle stage, unused
    // (and waited for at the barrier below).
    const int kt_next = kt + 1 < KT ? kt + 1 : kt;
    __builtin_amdgcn_sched_barrier(0);
    kstep(af[0], bfr[0], cur, 1, af[1], bfr[1], G_PER_STEP, G_PER_STEP, kt_next, nxt_lds);  // second half of tile kt + 1
    kstep(af[1], bfr[1], cur, 2, af[0], bfr[0], 0, 0, kt_next, nxt_lds);
    kstep(af[0], bfr[0], cur, 3, af[1], bfr[1], 0, 0, kt_next, nxt_lds);
    // The next tile must have landed (every wave's transfers) before anyone reads it, and every
    // wave must be done reading `cur` before the tile after next is written over it.
    wait_vmcnt0();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // last k-step of this tile covers the latency of the first operand reads of the next one and carries the
    // first half of the transfers of the tile after next into the stage the barrier has just released (none
    // past the last tile: nothing may be in flight when the epilogue reuses the LDS)
    kstep(af[1], bfr[1], nxt, 0, af[0], bfr[0], 0, decltype(ahead)::value ? G_PER_STEP : 0, kt + 2,
          smem_lds + (kt & 1) * STAGE);
  };
  int kt = 0;
  for (; kt + 2 < KT; ++kt) ktile(kt, std::true_type{});

  for (; kt < KT; ++kt) ktile(kt, std::false_type{});

  // ---- epilogue ----
  // Lane holds output row (lane & 31) of each 32 x 32 block and columns 8 * (e / 4) + 4 * (lane >> 5) +
  // e % 4.  Each wave stages 32 rows of its tile in a private, padded LDS region (8- or 16-byte writes,
  // conflict-free), reads them back row-contiguous and stores 16 bytes per lane: full cache lines.
  constexpr int ES = sizeof(TC);
  constexpr int ROW_B = TN * 32 * ES;            // bytes of one staged row
  constexpr int PITCH = ROW_B + 8;               // +2 banks per row: 32 rows land on distinct banks
  constexpr int CH16 = ROW_B / 16;               // 16-byte chunks per row
  constexpr int WAVE_B = 32 * PITCH;
  static_assert(NW * WAVE_B <= 2 * STAGE, "epilogue staging exceeds the pipeline's LDS");
  __syncthreads();                               // every wave is done with the pipeline's LDS
  char* stage_w = smem + wave * WAVE_B;
  TC* __restrict__ C = (TC*)p.C + (int64_t)split * p.c_split_stride;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        char* dst = stage_w + lrow * PITCH + (j * 32 + g4 * 8 + kg * 4) * ES;
        if constexpr (ES == 2) {
          bf16x4 v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = (bf16)acc[i][j][g4 * 4 + t];
          *(bf16x4*)dst = v;
        } else {
          f32x4 v;
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] = acc[i][j][g4 * 4 + t];
          *(f32x4*)dst = v;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < 32 * CH16 / 64; ++t) {
      const int idx = t * 64 + lane, row = idx / CH16, ch = idx % CH16;
      const u32x4 v = *(const u32x4*)(stage_w + row * PITCH + ch * 16);
      const int64_t gm = m0 + (wm * TM + i) * 32 + row;
      const int64_t gn = n0 + wn * TN * 32 + ch * (16 / ES);
      if (gm < p.M && gn < p.N) {
        u32x4* dst = (u32x4*)(C + gm * p.ldc + gn);
        if (p.accumulate) {
          const u32x4 old = *dst;
          if constexpr (ES == 2) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, v), o = __builtin_bit_cast(bf16x8, old);
            bf16x8 sum;
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] = (bf16)(p.alpha * (float)a[t] + p.beta * (float)o[t]);
            *dst = __builtin_bit_cast(u32x4, sum);
          } else {
            *dst = __builtin_bit_cast(u32x4, p.alpha * __builtin_bit_cast(f32x4, v) + p.beta * __builtin_bit_cast(f32x4, old));
          }
        } else {
          *dst = v;
        }
      }
    }
  }
}

template <int WM, int WN, int TM, int TN, bool B_KMAJOR, typename TC>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(FastGemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  gemm_bf16_tile<WM, WN, TM, TN, B_KMAJOR, TC>(p, blockIdx.x, smem);
}

template <int WM, int WN, int TM, int TN>
constexpr int gemm_bf16_lds_bytes() {
  return 2 * (WM * TM * 32 + WN * TN * 32) * 64 * 2;
}

// Fill the tiling fields of p for a BM x BN work-group tile; returns the 1-D grid size.
static inline unsigned gemm_bf16_plan(FastGemmParams& p, int BM, int BN) {
  p.tiles_m = (int)ceil_div(p.M, BM);
  p.tiles_n = (int)ceil_div(p.N, BN);
  // 32 tiles per XCD at a time: prefer 8 x 4, shrink along a short dimension
  int sn = p.tiles_n >= 4 ? 4 : (p.tiles_n >= 2 ? 2 : 1);
  int sm = 32 / sn;
  p.super_m = sm;
  p.super_n = sn;
  p.supers_n = (int)ceil_div(p.tiles_n, sn);
  const int supers_m = (int)ceil_div(p.tiles_m, sm);
  const int supers = round_up((int64_t)supers_m * p.supers_n, 8);
  return (unsigned)(supers * 32);
}

}  // namespace acc
