// GEMM on 8-bit floating-point operands (fp8 e4m3, or bf8 e5m2 for A) with the 16x16x128 matrix instruction:
// C[M, N] = alpha * (A[M, K] . B), fp32 accumulate, bf16 output.  The exact products F1 / B1 of the layer when
// the caller holds 8-bit copies of their operands (twice the matrix rate of bf16, half the operand bytes).
//
//   A is row-major with K contiguous (X8, dY8), one byte per element.
//   B_KMAJOR = true : B is given as Bt[N, K], K contiguous
//   B_KMAJOR = false: B is given as  B[K, N], N contiguous; the operand is formed with transposing LDS reads
//                     (ds_read_b64_tr_b8: 16 lanes give 8 k-rows x 2 chunks of 8 columns, lane c receives column c
//                     of the 8 rows).
//
// Same frame as the bf16 kernel of acc_gemm16.h: 256 persistent work-groups of four waves walk over 256 x 256
// output tiles, K pipeline across output tiles, two 64 KB LDS stages filled global -> LDS directly, read-out of a
// finished block row under the matrix instructions that follow.  A K tile is 128 elements = 128 bytes per row, so
// the transfers, the LDS layout and the swizzle of a K-contiguous tile are those of the bf16 kernel; what differs:
//   * one instruction covers the whole K tile of a 16 x 16 block (each lane holds 32 k of its row: two 16-byte
//     LDS reads), so a K tile is 64 slots of one matrix instruction (8 passes, 32 clocks) each;
//   * both operand sets are single-buffered (128 registers): the 64 instructions run as two halves, block
//     columns 0..3 for all eight block rows, then block columns 4..7.  B operands 4..7 of a K tile are read
//     during its first half, B operands 0..3 of the next K tile during its second half (after the barrier),
//     and A operand i of the next K tile as soon as block row i of the second half is done;
//   * every instruction of an output tile's first K tile multiplies onto zero;
//   * the barrier sits before slot 32 (every wave has read its last operands of the stage: it can be refilled;
//     the next stage has landed), and the sixteen wave-loads of the K tile after next follow it, one every second
//     slot (64 clocks apart, the spacing of the bf16 kernel), which leaves each at least 1000 clocks to land.
// Restrictions (host): K % 128 == 0, K >= 384, N % 8 == 0, operands below 4 GiB.
#pragma once
#include <type_traits>

#include "acc_gemm.h"

namespace acc {

// Swizzle of an N-contiguous 8-bit B tile (rows of 256 bytes, one k each): 16-byte chunk c of row k is stored at
// chunk position c ^ swz_n8(k).  One transposing read touches rows 16 g + (0..7) (+ 8, + 64 or + 72) for the four
// lane groups g: the 8 rows and the parity of g select 16 different chunk positions.
__device__ __forceinline__ int swz_n8(int krow) { return (krow & 7) | (((krow >> 4) & 1) << 3); }

__device__ __forceinline__ u32x2 lds_read_tr8_b64(const char* lds, int byte_off) {
  typedef int v2i __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                                       (v2i __attribute__((address_space(3)))*)(uintptr_t)(uint32_t)(uintptr_t)(lds + byte_off)));
}

// A transfer as the slot program issues it, in two parts.  set_lds_dest writes M0 (the LDS destination) at the end
// of the slot before; transfer_at_m0 is the transfer alone, right behind its slot's matrix instruction, which also
// is the wait state the hardware asks for between a write of M0 and its use.  The vector offset is formed inside
// the block, lane part + a scalar: the sum needs one temporary register at the point of use and cannot be split up
// and kept per wave-load by the compiler; the whole byte offset is in the vector offset, so the resource's range
// check sees all of it.
__device__ __forceinline__ void set_lds_dest(uint32_t& m0_token, uint32_t lds_wave_base) {
  asm volatile("s_mov_b32 m0, %1" : "={m0}"(m0_token) : "s"(lds_wave_base));
}
__device__ __forceinline__ void transfer_at_m0(u32x4 rsrc, uint32_t voffset, uint32_t scalar_part, uint32_t m0_token) {
  uint32_t sum;
  asm volatile("v_add_u32 %0, %2, %1\n\tbuffer_load_dwordx4 %0, %3, 0 offen lds"
               : "=&v"(sum)
               : "v"(voffset), "s"(scalar_part), "s"(rsrc), "{m0}"(m0_token)
               : "memory");
}
// Both parts in one block (prologue).
__device__ __forceinline__ void buffer_to_lds_b128_sum(u32x4 rsrc, uint32_t voffset, uint32_t scalar_part,
                                                       uint32_t lds_wave_base) {
  uint32_t sum;
  asm volatile("v_add_u32 %0, %2, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %3, 0 offen lds"
               : "=&v"(sum)
               : "v"(voffset), "s"(scalar_part), "s"(rsrc), "{m0}"(lds_wave_base)
               : "memory");
}

// A_FMT: 0 = fp8 (e4m3), 1 = bf8 (e5m2) for the A operand; B is always fp8 (e4m3).
template <bool B_KMAJOR, int A_FMT>
__global__ __launch_bounds__(256) void gemm8_persist_kernel(FastGemmParams p, int n_slots) {
  // One barrier per K tile, before slot BAR_Q: every wave has read its last operands of this K tile's stage (it can
  // be refilled) and the next K tile's stage has landed.  The sixteen wave-loads of the K tile after next follow in
  // the odd slots DMA_Q, DMA_Q + 2, ...; the operand reads sit in even slots.  Measured against it on the 3B-shaped
  // projection: a barrier of its own for the release (before slot 21, transfers from slot 23, the landing barrier
  // waiting for all but the five youngest) 135.1 against 124.9 us; one wave-load per slot 146.6 against 140.1 us.
  constexpr int BAR_Q = 32, DMA_Q = 33, DMA_EVERY = 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = 4, WN = 2, TB = 8;
  constexpr int BM = 256, BN = 256, BK = 128;
  constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW, NG = A_LOADS + B_LOADS;
  constexpr int REGION = 16 * 256;  // one staged block row: 16 rows x 128 bf16
  static_assert(NG == 16 && DMA_Q + DMA_EVERY * (NG - 1) < 64 && DMA_Q > BAR_Q && BAR_Q > 20 && BAR_Q < 34, "the slot program places sixteen wave-loads per K tile");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int KT = (int)(p.K / BK);
  const char* const A8 = (const char*)p.A;
  const char* const B8 = (const char*)p.B;

  // ---- global -> LDS sources (relative to a tile's buffer resources) ----
  // Wave-load t of a wave covers rows (4 t + wave) * 8 + lane / 8 of a K-contiguous tile: the part that depends on
  // t (and on the K tile) is the same for all lanes, so one register holds the lane's part for all of them.  In an
  // N-contiguous B tile a wave-load is four k-rows of 256 bytes and the swizzle of a row depends on bit 0 of t.
  const int row0 = wave * 8 + (lane >> 3);
  const uint32_t a_voff = (uint32_t)(row0 * p.lda + (((lane & 7) ^ swz(row0)) << 4));
  uint32_t b_voff[2];
  if (B_KMAJOR) {
    b_voff[0] = b_voff[1] = (uint32_t)(row0 * p.ldb + (((lane & 7) ^ swz(row0)) << 4));
  } else {
    const int krow0 = wave * 4 + (lane >> 4);
#pragma unroll
    for (int u = 0; u < 2; ++u) b_voff[u] = (uint32_t)(krow0 * p.ldb + (((lane & 15) ^ swz_n8(krow0 + 16 * u)) << 4));
  }
  const uint32_t a_tstep = (uint32_t)(32 * p.lda), b_tstep = (uint32_t)((B_KMAJOR ? 32 : 16) * p.ldb);
  const uint32_t b_kstep = B_KMAJOR ? BK : (uint32_t)(BK * p.ldb);
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
    r.a_rsrc = make_rsrc(A8 + r.m0 * p.lda, (p.M - r.m0 - 1) * p.lda + p.K);
    r.b_rsrc = B_KMAJOR ? make_rsrc(B8 + r.n0 * p.ldb, (p.N - r.n0 - 1) * p.ldb + p.K)
                        : make_rsrc(B8 + r.n0, (p.K - 1) * p.ldb + (p.N - r.n0));
    return r;
  };
  auto issue_one = [&](const TileRef& r, int g, int kt, uint32_t stage) {
    if (g < A_LOADS)
      buffer_to_lds_b128_sum(r.a_rsrc, a_voff, (uint32_t)kt * BK + g * a_tstep, stage + (g * NW + wave) * 1024);
    else
      buffer_to_lds_b128_sum(r.b_rsrc, b_voff[(g - A_LOADS) & 1], (uint32_t)kt * b_kstep + (g - A_LOADS) * b_tstep,
                             stage + A_BYTES + ((g - A_LOADS) * NW + wave) * 1024);
  };

  uint32_t m0_token = 0;
  auto lds_dest = [&](int g, uint32_t stage) -> uint32_t {
    return g < A_LOADS ? stage + (g * NW + wave) * 1024 : stage + A_BYTES + ((g - A_LOADS) * NW + wave) * 1024;
  };
  auto issue_at_m0 = [&](const TileRef& r, int g, int kt) {
    if (g < A_LOADS) transfer_at_m0(r.a_rsrc, a_voff, (uint32_t)kt * BK + g * a_tstep, m0_token);
    else transfer_at_m0(r.b_rsrc, b_voff[(g - A_LOADS) & 1], (uint32_t)kt * b_kstep + (g - A_LOADS) * b_tstep, m0_token);
  };

  // ---- LDS read offsets of the operands ----
  // Lane (l16, g4) holds, for row / column l16, k = 16 g4 .. 16 g4 + 15 (16-byte chunk g4 of the row) in its first
  // four registers and k = 64 + 16 g4 .. (chunk 4 + g4) in the other four.  Which k a lane holds is free as long as
  // both operands agree (the instruction pairs register bytes, not k values); with this choice the four lane groups
  // of one 16-byte read take four neighbouring chunks, the pattern of the bf16 kernel, which its swizzle serves
  // without bank conflicts (chunks 2 g4 and 2 g4 + 1 per lane: conflicts in 49 % of the LDS-active cycles).
  const int rswz = swz(l16);
  const int a_row = (wm * TB * 16 + l16) * 128;
  int kc[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) kc[c] = ((4 * c + g4) ^ rswz) << 4;
  auto two_chunks = [&](const char* st, int row_off) -> i32x8 {
    const u32x4 lo = *(const u32x4*)(st + row_off + kc[0]);
    const u32x4 hi = *(const u32x4*)(st + row_off + kc[1]);
    return __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto read_a = [&](const char* st, int i) -> i32x8 { return two_chunks(st, a_row + i * 2048); };
  int b_rd[TB];
#pragma unroll
  for (int j = 0; j < TB; ++j) {
    if (B_KMAJOR) {
      b_rd[j] = A_BYTES + (wn * TB * 16 + j * 16 + l16) * 128;
    } else {
      const int n_off = (wn * TB + j) * 16 + 8 * (l16 & 1);
      const int krow = 16 * g4 + (l16 >> 1);
      b_rd[j] = A_BYTES + krow * BN + (((n_off >> 4) ^ swz_n8(krow)) << 4) + (n_off & 15);
    }
  }
  auto read_b = [&](const char* st, int j) -> i32x8 {
    if (B_KMAJOR) {
      return two_chunks(st, b_rd[j]);
    } else {
      // k rows 16 g4 + (0..7), + 8, + 64, + 72: the swizzle of a row is the same for the four
      const u32x2 r0 = lds_read_tr8_b64(st, b_rd[j]);
      const u32x2 r1 = lds_read_tr8_b64(st, b_rd[j] + 8 * BN);
      const u32x2 r2 = lds_read_tr8_b64(st, b_rd[j] + 64 * BN);
      const u32x2 r3 = lds_read_tr8_b64(st, b_rd[j] + 72 * BN);
      const u32x4 lo = __builtin_shufflevector(r0, r1, 0, 1, 2, 3);
      const u32x4 hi = __builtin_shufflevector(r2, r3, 0, 1, 2, 3);
      return __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
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

  // ---- read-out of a finished block row (as in acc_gemm16.h) ----
  // acc[i][j][e] = C[16 i + l16][16 j + 4 g4 + e] of the wave's 128 x 128 tile.
  bf16* __restrict__ C = (bf16*)p.C;
  const float alpha = p.alpha;
  char* const regions = smem + 2 * STAGE + wave * (2 * REGION);
  const uint32_t w_base = ((uint32_t)(uintptr_t)regions + l16 * 256 + (l16 << 4) + (g4 & 1) * 8) ^ (uint32_t)((g4 >> 1) << 4);
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
    for (int t = 0; t < 4; ++t) v[t] = (bf16)(alpha * acc[i][j][t]);
    typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
    *(lds_bf16x4_ptr)(uintptr_t)((w_base ^ (uint32_t)(j << 5)) + (i & 1) * REGION) = v;
  };
  auto read_back = [&](int i, int t) -> u32x4 {
    return *(const u32x4*)(regions + (i & 1) * REGION + t * 1024 + (r_addr ^ (t << 6)));
  };
  auto store_back = [&](int i, int t, u32x4 v) {
    const uint32_t soff = (uint32_t)(i * 16 + t * 4) * c_row_bytes;
    __builtin_amdgcn_raw_buffer_store_b128(v, c_rs, c_voff, soff, 2);  // aux 2: non-temporal (see the header)
  };
  u32x4 back[2];
  // What is left of the previous output tile's read-out: block rows 6 and 7 sit in the two staging regions when
  // its last K tile ends (row 7 is staged after that tile's last matrix instruction, so no accumulator lives on
  // into the next output tile); their read-backs and global stores ride in slots 33 .. 40 of the next K tile,
  // behind its barrier, so that the barrier's wait for the transfers does not also wait for stores just issued.
  auto carry_store = [&](int q) {  // q = 0 .. 7
    if (q == 0) wave_fence();
    const int row = 6 + (q >> 2), t = q & 2;
    if ((q & 1) == 0) { back[0] = read_back(row, t); back[1] = read_back(row, t + 1); }
    else { store_back(row, t, back[0]); store_back(row, t + 1, back[1]); }
  };

  i32x8 a[TB], b[TB];

  // One K tile.  sc: its stage; ref2 / k2: the K tile after next, whose wave-loads go out here.
  auto ktile = [&](int sc, const TileRef& ref2, int k2, auto zero, auto carry, auto fin) {
    constexpr bool ZERO = decltype(zero)::value, CARRY = decltype(carry)::value, FINAL = decltype(fin)::value;
    const char* cur = smem + sc * STAGE;
    const char* nxt = smem + (sc ^ 1) * STAGE;
    const uint32_t cur_lds = smem_lds + sc * STAGE;
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, 64>([&](auto slot) {
      constexpr int q = decltype(slot)::value;
      constexpr int h = q >> 5, i = (q >> 2) & 7, jj = q & 3, j = 4 * h + jj;
      if (q == 0) a[7] = read_a(cur, 7);
      if (q == BAR_Q) {
        wait_vmcnt0();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (ZERO) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], z, 0, A_FMT, 0, 0, 0, 0);
      } else {
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], acc[i][j], 0, A_FMT, 0, 0, 0, 0);
      }
      if (q >= DMA_Q && (q - DMA_Q) % DMA_EVERY == 0 && (q - DMA_Q) / DMA_EVERY < NG)
        issue_at_m0(ref2, (q - DMA_Q) / DMA_EVERY, k2);
      if (h == 0) {
        // B operands 4 .. 7 of this K tile (slots 2, 8, 14, 20)
        if (q >= 2 && (q - 2) % 6 == 0 && (q - 2) / 6 < 4) b[4 + (q - 2) / 6] = read_b(cur, 4 + (q - 2) / 6);
      } else {
        // operands of the next K tile: A operand i once block row i is done, B operands 0 .. 3 at slots 34, 42, 50, 58
        if (jj == 0 && i >= 1) a[i - 1] = read_a(nxt, i - 1);
        if (q >= BAR_Q + 2 && (q - BAR_Q - 2) % 8 == 0) b[(q - BAR_Q - 2) / 8] = read_b(nxt, (q - BAR_Q - 2) / 8);
        if (CARRY && q >= BAR_Q + 1 && q < BAR_Q + 9) carry_store(q - BAR_Q - 1);
        if constexpr (FINAL) {
          // block row i - 1 is final: staged in the slots of row i; read back and stored in those of row i + 1
          if (i >= 2 && jj == 0) wave_fence();
          if (i >= 1) { stage_write(i - 1, 2 * jj); stage_write(i - 1, 2 * jj + 1); }
          if (i >= 2 && (jj & 1) == 0) { back[0] = read_back(i - 2, jj); back[1] = read_back(i - 2, jj + 1); }
          if (i >= 2 && (jj & 1) == 1) { store_back(i - 2, jj - 1, back[0]); store_back(i - 2, jj, back[1]); }
        }
      }
      if (q + 1 >= DMA_Q && (q + 1 - DMA_Q) % DMA_EVERY == 0 && (q + 1 - DMA_Q) / DMA_EVERY < NG)
        set_lds_dest(m0_token, lds_dest((q + 1 - DMA_Q) / DMA_EVERY, cur_lds));
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (FINAL) {
      static_for<0, TB>([&](auto j) { stage_write(TB - 1, decltype(j)::value); });
    }
  };

  // ---- prologue of the work-group's first tile ----
  if (has_tile) {
#pragma unroll
    for (int g = 0; g < NG; ++g) issue_one(cur_t, g, 0, smem_lds);
#pragma unroll
    for (int g = 0; g < NG; ++g) issue_one(cur_t, g, 1, smem_lds + STAGE);
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
  for (int i = 0; i < TB - 1; ++i) a[i] = read_a(smem, i);
#pragma unroll
  for (int j = 0; j < 4; ++j) b[j] = read_b(smem, j);

  using T = std::true_type;
  using F = std::false_type;
  int par = 0;
  for (int idx = first_idx;;) {
    const int next_idx = next_slot(idx);
    const bool has_next = next_idx < n_slots;
    const TileRef next_t = has_next ? tile_ref(next_idx) : cur_t;
    // K tile 0: multiplies onto zero and finishes the previous read-out (before the first output tile the
    // accumulators hold nothing and the output resource is empty, so those stores are dropped)
    ktile(par, cur_t, 2, T{}, T{}, F{});
    // K tiles 1 .. KT - 2; the last of them already fetches the next output tile's first K tile
    for (int kt = 1; kt + 1 < KT; ++kt) {
      const bool wraps = kt + 2 >= KT;
      ktile((kt + par) & 1, wraps ? next_t : cur_t, wraps ? 0 : kt + 2, F{}, F{}, F{});
    }
    const int kt = KT - 1;
    set_output(cur_t);
    ktile((kt + par) & 1, next_t, 1, F{}, F{}, T{});  // last: the read-out starts
    if (!has_next) break;
    cur_t = next_t;
    par = (par + KT) & 1;
    idx = next_idx;
  }
  // no tile follows: block rows 6 and 7 are read out here
#pragma unroll
  for (int q = 0; q < 8; ++q) carry_store(q);
  wait_vmcnt0();  // the surplus transfers of the last two K tiles must have landed before the LDS is released
}

}  // namespace acc
