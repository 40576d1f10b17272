// Persistent form of the tuned bf16 GEMM (steps F1, B1) for shapes with several rounds of 256 x 256 tiles:
// 256 work-groups (one per compute unit) walk over the output tiles b, b + 256, b + 512, ... and the K
// pipeline runs across the tile boundary.  The last K tile of a tile carries the read-out of the finished
// accumulators (as in gemm_bf16_tile's FOLD path); the first K tile of the next output tile is requested in the
// cadence of any other K tile (first half in the last k-step of the last but one K tile, second half in the
// first k-step of the last), half of its second K tile goes into the stage the last K tile frees itself, so a
// new tile starts with its operands in LDS: no launch of a new work-group, no burst of first
// transfers from every compute unit at once, no wait for them.
//
// LDS: two 64 KB stages + 32 KB of staging regions for the read-out (two 4 KB regions per wave, rows of
// 128 bytes with the 16-byte chunk index XOR-ed with the row so that writes and read-backs spread over the banks).
// The first k-step of every tile multiplies onto zero, so the accumulators are never cleared; it also carries the
// read-out of the previous tile's last two units, which were final only after that tile's last MFMA.
// Restrictions (the host checks them): bf16 output, no accumulation into C, no K split, K >= 192.
#pragma once
#include "acc_gemm.h"

namespace acc {

template <bool B_KMAJOR>
__global__ __launch_bounds__(256) void gemm_bf16_persist_kernel(FastGemmParams p, int n_slots) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int WN = 2, TM = 4, TN = 4, NW = 4;
  constexpr int BM = 256, BN = 256, BK = 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW;
  constexpr int BN_CHUNKS = BN / 8;
  constexpr int NM = TM * TN, NG_TOTAL = A_LOADS + B_LOADS, G_PER_STEP = NG_TOTAL / 2;
  static_assert(NM == 16 && NG_TOTAL == 16 && G_PER_STEP == 8, "schedule below is written for 16 MFMAs and 16 wave-loads");
  constexpr int UNIT_B = 32 * 128;  // one staged 32 x 64 bf16 unit

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int lrow = lane & 31, kg = lane >> 5;
  const int KT = (int)(p.K / BK);

  // ---- per-lane sources of the global -> LDS transfers (relative to a tile's buffer resources) ----
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
      b_src[t] = (uint32_t)(krow * p.ldb * 2 + (((lane % BN_CHUNKS) ^ swz_n(krow)) << 4));
    }
  }
  const uint32_t b_kstep = B_KMAJOR ? BK * 2 : (uint32_t)(BK * p.ldb * 2);

  // ---- per-tile state: buffer resources of the operands, origin of the output tile ----
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
  auto issue_one = [&](const TileRef& r, int g, int kt, uint32_t stage) {  // g-th wave-load of a K tile
    if (g < A_LOADS) buffer_to_lds_b128(r.a_rsrc, a_src[g], (uint32_t)kt * (BK * 2), stage + (g * NW + wave) * 1024);
    else buffer_to_lds_b128(r.b_rsrc, b_src[g - A_LOADS], (uint32_t)kt * b_kstep,
                            stage + A_BYTES + ((g - A_LOADS) * NW + wave) * 1024);
  };

  // ---- LDS read offsets of this lane's MFMA operands ----
  int a_rd[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_rd[i] = (wm * TM * 32 + i * 32 + lrow) * 128;
  int b_rd[TN];  // N-contiguous B: first of the two transposing reads; the second is 4 k-rows further (same swizzle)
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (B_KMAJOR) {
      b_rd[j] = A_BYTES + (wn * TN * 32 + j * 32 + lrow) * 128;
    } else {
      const int g = lane >> 4, i16 = lane & 15;
      const int n_off = (wn * TN + j) * 32 + 16 * (g & 1) + 4 * (i16 & 3);
      const int krow = 8 * (g >> 1) + (i16 >> 2);
      b_rd[j] = A_BYTES + krow * (BN * 2) + (((n_off >> 3) ^ swz_n(krow)) << 4) + (n_off & 7) * 2;
    }
  }
  const int a_swz = swz(lrow);
  auto read_a = [&](const char* st, int s, int i) -> bf16x8 {
    return lds_read_b128(st, a_rd[i] + (((2 * s + kg) ^ a_swz) << 4));
  };
  auto read_b = [&](const char* st, int s, int j) -> bf16x8 {
    if (B_KMAJOR) {
      return lds_read_b128(st, b_rd[j] + (((2 * s + kg) ^ a_swz) << 4));
    } else {
      const s16x4 lo = lds_read_tr16_b64(st, b_rd[j] + 16 * s * (BN * 2));
      const s16x4 hi = lds_read_tr16_b64(st, b_rd[j] + (16 * s + 4) * (BN * 2));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  f32x16 acc[TM][TN];
  bf16x8 af[2][TM], bfr[2][TN];
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;

  // slots of the XCD tile map that hold no tile (the map is padded to whole super-tiles) are skipped
  auto next_slot = [&](int idx) -> int {
    int tm, tn;
    for (idx += (int)gridDim.x; idx < n_slots && !xcd_tile(p, idx, tm, tn);) idx += (int)gridDim.x;
    return idx;
  };
  const int first_idx = next_slot((int)blockIdx.x - (int)gridDim.x);
  const bool has_tile = first_idx < n_slots;
  TileRef cur_t = tile_ref(has_tile ? first_idx : 0);

  // ---- read-out of a finished 32 x 64 unit (see gemm_bf16_tile) ----
  bf16* __restrict__ C = (bf16*)p.C;
  const int e_row = lane >> 3, e_ch = lane & 7;
  char* const region = smem + 2 * STAGE + wave * (2 * UNIT_B);
  // staging address of 16-byte chunk c of this lane's row: w_base ^ (c << 4) (the region is 4 KB aligned and the
  // chunk index sits in bits 4 .. 6, so the XOR of the swizzle can be applied to the whole address)
  const uint32_t w_base = (uint32_t)(uintptr_t)region + lrow * 128 + ((lrow & 7) << 4) + kg * 8;
  const int r_addr = e_row * 128 + ((e_ch ^ e_row) << 4);
  const uint32_t c_row_bytes = (uint32_t)(p.ldc * 2);
  auto wave_fence = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  // output addressing of the tile that is being read out (set by final_tile, still used in the first k-step
  // of the next tile, which carries the end of the read-out)
  __amdgpu_buffer_rsrc_t c_rs;
  uint32_t c_voff[2];
  auto set_output = [&](const TileRef& t) {
    const int64_t gm_base = t.m0 + wm * TM * 32, gn_base = t.n0 + wn * TN * 32;
    int64_t c_rows = p.M - gm_base;
    if (c_rows > TM * 32) c_rows = TM * 32;
    const int64_t c_bytes = (c_rows > 0 && gn_base < p.N) ? ((c_rows - 1) * p.ldc + (p.N - gn_base)) * 2 : 0;
    c_rs = __builtin_amdgcn_make_buffer_rsrc((void*)(C + gm_base * p.ldc + gn_base), 0, (int)(uint32_t)c_bytes,
                                             0x00020000);
#pragma unroll
    for (int jh = 0; jh < 2; ++jh)
      c_voff[jh] = gn_base + jh * 64 + e_ch * 8 < p.N ? (uint32_t)((e_row * p.ldc + jh * 64 + e_ch * 8) * 2)
                                                      : 0xFFFFFFF0u;  // columns past N: out of range, dropped
  };
  auto stage_write = [&](int u, int k) {  // unit u = 2 * i + jh; write k: block column k / 4, register group k % 4
    const int i = u >> 1, j = 2 * (u & 1) + (k >> 2), g4 = k & 3;
    bf16x4 v;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = (bf16)acc[i][j][g4 * 4 + t];
    typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
    *(lds_bf16x4_ptr)(uintptr_t)((w_base ^ (uint32_t)(((k >> 2) * 4 + g4) << 4)) + (u & 1) * UNIT_B) = v;
  };
  auto read_back = [&](int u, int t) -> u32x4 {
    return *(const u32x4*)(region + (u & 1) * UNIT_B + t * 1024 + r_addr);
  };
  auto store_back = [&](int u, int t, u32x4 v) {
    const uint32_t soff = (uint32_t)((u >> 1) * 32 + t * 8) * c_row_bytes;
    __builtin_amdgcn_raw_buffer_store_b128(v, c_rs, c_voff[u & 1], soff, 0);
  };
  u32x4 back[4];
  // End of the read-out of a tile (units 6 and 7), as work for the sixteen slots of the next tile's first k-step:
  // unit 7's accumulators (block row 3, columns 2 and 3) are read before that k-step's MFMAs 14 and 15 restart them.
  auto drain_slot = [&](int q) {
    if (q == 0) wave_fence();
    if (q < 8) stage_write(7, q);
    if (q < 4) back[q] = read_back(6, q);
    else if (q < 8) store_back(6, q - 4, back[q - 4]);
    if (q == 8) wave_fence();
    if (q >= 8 && q < 12) back[q - 8] = read_back(7, q - 8);
    if (q >= 12) store_back(7, q - 12, back[q - 12]);
  };
  auto no_extra = [](int) {};

  // One k-step (same order as gemm_bf16_tile's): MFMA q carries one operand read of the next k-step on even q and
  // one wave-load on odd q.  zero: the products start the accumulators instead of adding to them.
  auto kstep = [&](const bf16x8(&ca)[TM], const bf16x8(&cb)[TN], const char* rd_stage, int rd_s, bf16x8(&na)[TM],
                   bf16x8(&nb)[TN], const TileRef& tr, int g_first, int g_count, int kt_next, uint32_t nxt, auto zero,
                   auto&& extra) {
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      const int i = q / TN, j = q % TN;
      if constexpr (decltype(zero)::value) {
        const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cb[j], ca[i], z, 0, 0, 0);
      } else {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cb[j], ca[i], acc[i][j], 0, 0, 0);
      }
      if (q % 2 == 0) {
        const int r = q / 2;
        if (r == 0) na[0] = read_a(rd_stage, rd_s, 0);
        else if (r <= TN) nb[r - 1] = read_b(rd_stage, rd_s, r - 1);
        else na[r - TN] = read_a(rd_stage, rd_s, r - TN);
      } else if (q / 2 < g_count) {
        issue_one(tr, g_first + q / 2, kt_next, nxt);
      }
      extra(q);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // One K tile in the steady state; par: stage of this tile's K tile 0.  ahead: what the last k-step requests
  // into the stage this K tile frees: 1 = first half of K tile kt + 2, 2 = first half of K tile 0 of the next
  // output tile (kt is then the last but one K tile), 0 = nothing.  first: K tile 0 of an output tile.  carry:
  // the first k-step also finishes the read-out of the previous output tile.
  auto ktile = [&](int kt, int par, auto ahead, auto first, auto carry, const TileRef& next_t, int next_count) {
    constexpr int AHEAD = decltype(ahead)::value;
    const int sc = (kt + par) & 1;
    const char* cur = smem + sc * STAGE;
    const char* nxt = smem + (sc ^ 1) * STAGE;
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(carry)::value)
      kstep(af[0], bfr[0], cur, 1, af[1], bfr[1], cur_t, G_PER_STEP, G_PER_STEP, kt + 1, smem_lds + (sc ^ 1) * STAGE, first,
            drain_slot);
    else
      kstep(af[0], bfr[0], cur, 1, af[1], bfr[1], cur_t, G_PER_STEP, G_PER_STEP, kt + 1, smem_lds + (sc ^ 1) * STAGE, first,
            no_extra);
    kstep(af[1], bfr[1], cur, 2, af[0], bfr[0], cur_t, 0, 0, 0, 0u, std::false_type{}, no_extra);
    kstep(af[0], bfr[0], cur, 3, af[1], bfr[1], cur_t, 0, 0, 0, 0u, std::false_type{}, no_extra);
    wait_vmcnt0();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (AHEAD == 2)  // next_count: G_PER_STEP, or 0 when no output tile follows
      kstep(af[1], bfr[1], nxt, 0, af[0], bfr[0], next_t, 0, next_count, 0, smem_lds + sc * STAGE, std::false_type{}, no_extra);
    else
      kstep(af[1], bfr[1], nxt, 0, af[0], bfr[0], cur_t, 0, AHEAD == 1 ? G_PER_STEP : 0, kt + 2, smem_lds + sc * STAGE,
            std::false_type{}, no_extra);
  };

  // Last K tile of an output tile.  prefetch: another output tile (next_t) follows.
  auto final_tile = [&](int kt, int par, const TileRef& next_t, auto prefetch) {
    constexpr bool PF = decltype(prefetch)::value;
    const int sc = (kt + par) & 1;
    const char* cur = smem + sc * STAGE;
    const char* other = smem + (sc ^ 1) * STAGE;
    const uint32_t cur_lds = smem_lds + sc * STAGE, other_lds = smem_lds + (sc ^ 1) * STAGE;
    set_output(cur_t);
    bf16x8 aq[2][4], bq[4][TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bq[0][j] = bfr[0][j];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 1; ks < 4; ++ks) {
      aq[0][ks] = read_a(cur, ks, 0);
      bq[ks][0] = read_b(cur, ks, 0);
      bq[ks][1] = read_b(cur, ks, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const int i = h >> 1, jh = h & 1;
      if (h >= 2) wave_fence();
      if (PF && h == 6) {
        // The next tile's K tile 0 (requested in the last k-step of the K tile before this one and in this one's
        // first eight slots) has landed for this wave: everything but the sixteen stores issued since is complete.  After the barrier it has landed for every wave,
        // and every wave has read all it needs from `cur`, which then takes half of the next K tile 1.
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int ks = k >> 1, j = 2 * jh + (k & 1);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[ks][j], ks == 0 ? af[0][i] : aq[i & 1][ks],
                                                            acc[i][j], 0, 0, 0);
        if (h == 0 && k < 6) bq[1 + k / 2][2 + (k & 1)] = read_b(cur, 1 + k / 2, 2 + (k & 1));
        if (jh == 0 && i < 3 && k >= 5) aq[(i + 1) & 1][k - 4] = read_a(cur, k - 4, i + 1);
        if (PF && h == 0) issue_one(next_t, G_PER_STEP + k, 0, other_lds);  // second half; the first went out a k-step ago
        if (PF && h == 6) issue_one(next_t, k, 1, cur_lds);
        if (PF && h == 6 && k < 4) af[1][k] = read_a(other, 0, k);
        if (PF && h == 6 && k >= 4) bfr[1][k - 4] = read_b(other, 0, k - 4);
        if (h >= 1) stage_write(h - 1, k);
        if (h >= 2 && k < 4) back[k] = read_back(h - 2, k);
        if (h >= 2 && k >= 4) store_back(h - 2, k - 4, back[k - 4]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (!PF) {  // no tile follows: units 6 and 7 are read out here (else in the next tile's first k-step)
#pragma unroll
      for (int q = 0; q < 16; ++q) drain_slot(q);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- prologue of the work-group's first tile ----
  if (has_tile) {
#pragma unroll
    for (int g = 0; g < NG_TOTAL; ++g) issue_one(cur_t, g, 0, smem_lds);
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
  for (int i = 0; i < TM; ++i) af[0][i] = read_a(smem, 0, i);
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = read_b(smem, 0, j);
#pragma unroll
  for (int g = 0; g < G_PER_STEP; ++g) issue_one(cur_t, g, 1, smem_lds + STAGE);

  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  int par = 0;
  for (int idx = first_idx;;) {
    const int next_idx = next_slot(idx);
    const bool has_next = next_idx < n_slots;
    const TileRef next_t = has_next ? tile_ref(next_idx) : cur_t;
    if (idx == first_idx) ktile(0, par, I1{}, std::true_type{}, std::false_type{}, next_t, 0);
    else ktile(0, par, I1{}, std::true_type{}, std::true_type{}, next_t, 0);  // carries the end of the last read-out
    int kt = 1;
    for (; kt + 2 < KT; ++kt) ktile(kt, par, I1{}, std::false_type{}, std::false_type{}, next_t, 0);
    ktile(kt, par, I2{}, std::false_type{}, std::false_type{}, next_t, has_next ? G_PER_STEP : 0);
    ++kt;
    if (!has_next) {
      final_tile(kt, par, cur_t, std::false_type{});
      break;
    }
    final_tile(kt, par, next_t, std::true_type{});
    // the next tile's k-step 0 operands were read into the second register set
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = af[1][i];
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = bfr[1][j];
    cur_t = next_t;
    par = (par + KT) & 1;
    idx = next_idx;
  }
}

}  // namespace acc
