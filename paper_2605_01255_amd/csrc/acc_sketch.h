// Tuned bf16 sketch kernel for gfx950 (steps F0 + F2 and F0 + B2):
//
//   part[g][c][j] = sum over the tokens t of split g of  A[t, c] * S[t, j]          (TRANSPOSED = false, Xs)
//   part[g][j][c] = the same value stored transposed                                 (TRANSPOSED = true,  Gr)
//
// A is X [n, d_in] or dY [n, d_out] (row-major, channels contiguous); S[t, j] is regenerated from the
// Philox counter (token, column) in registers, directly in MFMA operand layout, and never stored.
//
// Work-group = WC x WJ waves; output tile (WC * CWB * 32) channels x (WJ * 32) sketch columns, fp32
// accumulators in registers for the whole token range of the split (CWB * 16 registers per lane).
// Tokens stream through LDS in stages of 16 rows (one MFMA k-step), global -> LDS directly, in a ring of
// NSTAGE stages with NSTAGE - 1 stages in flight: the input is read once from HBM, so enough bytes
// must be outstanding per CU to cover DRAM latency.  The channel-major MFMA operand is formed from
// the token-major tile with transposing LDS reads.
// The contraction runs over tokens, so one Philox call (4 tokens of one column) feeds half an
// operand register set; every wave generates only the 32 columns it multiplies.
#pragma once
#include "acc_common.h"
#include "acc_gemm.h"
#include "acc_rng.h"

namespace acc {

struct SketchFastParams {
  const bf16* A;       // [n, lda]
  float* part;         // [G][C][r] or [G][r][C]
  int64_t n, C, lda;
  int r;
  int tokens_per_split;  // multiple of 32
  int n_cslab, n_js, G;  // channel slabs, column slices, token splits
  SketchParams sk;
};

// Store one wave's fp32 partial tile (CWB blocks of 32 x 32) with buffer stores: the lane part of the
// address is computed once, the (block, register) part is a scalar offset, and elements past the end
// of the matrix fall outside the buffer resource and are dropped by the hardware.
//   lane holds MFMA column (lane & 31) and rows 8 * (e / 4) + 4 * (lane >> 5) + e % 4 of each block;
//   !TRANSPOSED: rows = channels, columns = sketch columns, out[c * r + j]
//    TRANSPOSED: rows = sketch columns, columns = channels, out[j * C + c]
// cb0 = first channel of the wave's blocks, j0 = first sketch column of the wave.
template <bool TRANSPOSED, int CWB>
__device__ __forceinline__ void store_partial_tile(const f32x16 (&acc)[CWB], float* out, int64_t C, int r,
                                                   int64_t cb0, int j0, int lane) {
  const int lcol = lane & 31, kg = lane >> 5;
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc((void*)out, 0, (int)(uint32_t)(C * r * 4), 0x00020000);
  uint32_t voff;
  if (!TRANSPOSED) voff = (uint32_t)(((cb0 + kg * 4) * r + j0 + lcol) * 4);
  else voff = (uint32_t)((((int64_t)(j0 + kg * 4)) * C + cb0 + lcol) * 4);
#pragma unroll
  for (int mb = 0; mb < CWB; ++mb) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int rowi = (e >> 2) * 8 + (e & 3);
      const uint32_t soff = !TRANSPOSED ? (uint32_t)((mb * 32 + rowi) * r * 4)
                                        : (uint32_t)((rowi * C + mb * 32) * 4);
      const float v = acc[mb][e];
      // transposed: a channel past the end would land in the next row, so it is sent out of range
      // !transposed: a sketch column past r (rank not a multiple of the tile's columns) would land in the
      // next channel's row; transposed, such rows fall behind the end of the buffer by themselves
      const uint32_t vo = ((TRANSPOSED && cb0 + mb * 32 + lcol >= C) || (!TRANSPOSED && j0 + lcol >= r))
                              ? 0xFFFFFFF0u : voff;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, vo, soff, 0);
    }
  }
}

template <int WC, int WJ, int CWB, bool TRANSPOSED>
__global__ __launch_bounds__(WC* WJ * 64) void sketch_bf16_kernel(SketchFastParams p) {
  constexpr int NW = WC * WJ;
  constexpr int CH = WC * CWB * 32, RC = WJ * 32, BT = 16;
  constexpr int ROW_BYTES = CH * 2;
  constexpr int STAGE = BT * ROW_BYTES;
  constexpr int NSTAGE = 128 * 1024 / STAGE;    // ring of stages in 128 KB of LDS
  constexpr int DEPTH = NSTAGE - 1;             // stages in flight
  constexpr int PARTS = ROW_BYTES / 1024;       // 1 KB wave-loads per token row
  constexpr int LOADS = BT * PARTS / NW;        // wave-loads per wave and stage
  static_assert(BT * PARTS % NW == 0, "stage/waves");
  static_assert(CH % 512 == 0, "channel slab must be a multiple of 512");
  static_assert(CWB % 4 == 0, "the row swizzle permutes groups of four 32-channel blocks");
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // ---- which tile: pairs of column slices of one (split, slab) share an XCD (blockIdx % 8) ----
  const int b = blockIdx.x;
  const int js = (b >> 3) % p.n_js;
  const int pair = (b & 7) + 8 * ((b >> 3) / p.n_js);
  if (pair >= p.n_cslab * p.G) return;
  const int slab = pair % p.n_cslab, g = pair / p.n_cslab;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave / WJ, wj = wave % WJ;
  const int64_t t_begin = (int64_t)g * p.tokens_per_split;
  const int64_t c0 = (int64_t)slab * CH;
  int64_t t_end = t_begin + p.tokens_per_split;
  if (t_end > p.n) t_end = p.n;
  const int NS = t_end > t_begin ? (int)((t_end - t_begin + BT - 1) / BT) : 0;  // stages = k-steps

  // ---- global -> LDS: wave-load L = t * NW + wave covers token row L / PARTS, kilobyte L % PARTS ----
  const u32x4 rsrc = make_rsrc(p.A + t_begin * p.lda + c0, ((p.n - t_begin - 1) * p.lda + (p.C - c0)) * 2);
  uint32_t src[LOADS];
  uint32_t dst[LOADS];
#pragma unroll
  for (int t = 0; t < LOADS; ++t) {
    const int L = t * NW + wave, row = L / PARTS, part = L % PARTS;
    const int chunk = (part * 64 + lane) ^ swz_n(row);   // 16-byte chunk of the row this lane fetches
    src[t] = (uint32_t)(row * p.lda * 2 + chunk * 16);
    dst[t] = (uint32_t)(row * ROW_BYTES + part * 1024);
  }
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;
  auto issue_stage = [&](int st, uint32_t stage_lds) {
    const uint32_t soff = (uint32_t)st * (uint32_t)(BT * p.lda * 2);
#pragma unroll
    for (int t = 0; t < LOADS; ++t) buffer_to_lds_b128(rsrc, src[t], soff, stage_lds + dst[t]);
  };

  // ---- LDS addresses of the transposing operand reads ----
  // 16-lane group gq = lane / 16 reads channels 16 * (gq & 1) .. and tokens 8 * (gq >> 1) ..; lane i of
  // the group reads token i / 4 (+ 4 for the second half), 4-channel chunk i % 4.  The row swizzle only
  // touches bits 2..3 of the 16-byte chunk index, i.e. the 32-channel block index modulo 4.
  const int gq = lane >> 4, i16 = lane & 15;
  const int xr = (i16 >> 2) & 3;
  int rd_base[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int row = 8 * (gq >> 1) + (i16 >> 2);
    const int col16 = 2 * (gq & 1) + ((i16 & 3) >> 1);  // 16-byte chunk within the 32-channel block
    rd_base[v] = row * ROW_BYTES + (((((wc * CWB) & 3) ^ v ^ xr) & 3) << 6) + (col16 << 4) + ((i16 & 1) << 3) +
                 (((wc * CWB) >> 2) << 8);
  }
  // operand of channel block mb (0 .. CWB-1) from stage `st`
  auto read_block = [&](const char* st, int mb) -> bf16x8 {
    const int off = (mb >> 2) * 256;
    const s16x4 lo = lds_read_tr16_b64(st, rd_base[mb & 3] + off);
    const s16x4 hi = lds_read_tr16_b64(st, rd_base[mb & 3] + off + 4 * ROW_BYTES);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // ---- S operand: lane holds column j, tokens 8 * (lane >> 5) .. + 7 of the k-step ----
  const uint32_t jcol = (uint32_t)(js * RC + wj * 32 + (lane & 31));
  const uint64_t q_lane = ((p.sk.row_offset + (uint64_t)t_begin) >> 2) + 2 * (uint64_t)(lane >> 5);
  auto make_s = [&](int kstep) -> bf16x8 {  // kstep counts 16-token steps from t_begin (prologue only)
    uint32_t w0[4], w1[4];
    float z0[4], z1[4];
    const uint64_t q = q_lane + 4 * (uint64_t)kstep;
    sketch_words(p.sk.key0, p.sk.key1, q, jcol, w0);
    sketch_words(p.sk.key0, p.sk.key1, q + 1, jcol, w1);
    normals_from_words<false>(w0, p.sk.inv_sqrt_r, p.sk.neg2_ln2_over_r, z0);
    normals_from_words<false>(w1, p.sk.inv_sqrt_r, p.sk.neg2_ln2_over_r, z1);
    bf16x8 s;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      s[t] = (bf16)z0[t];
      s[4 + t] = (bf16)z1[t];
    }
    return s;
  };

  f32x16 acc[CWB];
#pragma unroll
  for (int i = 0; i < CWB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // One k-step (16 tokens) in CWB slots.  Slot mb issues MFMA mb on operands already in registers, the
  // two transposing reads of operand mb of the following k-step, and one slice of the generation of
  // the S operand of the following k-step (10 Philox rounds on two counters, 4 Box-Muller pairs, pack).
  // Fences between slots keep this order: the matrix pipe and the vector ALU then run concurrently
  // instead of one after the other, and every LDS read has a whole k-step to return.
  static_assert(CWB >= 16 || CWB == 8, "the S generation is spread over 16 slots, or packed into 8");
  struct SGen {
    uint32_t c[2][4];
    float z[8];
  };
  auto sgen_slot = [&](SGen& g, int slot, int kstep, bf16x8& out) {
    if (slot == 0) {
      const uint64_t q = q_lane + 4 * (uint64_t)kstep;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        g.c[h][0] = (uint32_t)(q + h); g.c[h][1] = jcol; g.c[h][2] = 0u; g.c[h][3] = (uint32_t)((q + h) >> 32);
      }
    }
    if constexpr (CWB >= 16) {
      if (slot < 10) {
        philox_round(g.c[0], p.sk.key0, p.sk.key1, slot);
        philox_round(g.c[1], p.sk.key0, p.sk.key1, slot);
      } else if (slot < 14) {
        const int pr = slot - 10, h = pr >> 1, a = (pr & 1) * 2;
        box_muller_fast(g.c[h][a], g.c[h][a + 1], p.sk.neg2_ln2_over_r, g.z[4 * h + a], g.z[4 * h + a + 1]);
      } else if (slot == 14) {
#pragma unroll
        for (int t = 0; t < 8; ++t) out[t] = (bf16)g.z[t];
      }
    } else {  // 8 slots: two rounds, then two Box-Muller pairs per slot
      if (slot < 5) {
#pragma unroll
        for (int rr = 2 * slot; rr < 2 * slot + 2; ++rr) {
          philox_round(g.c[0], p.sk.key0, p.sk.key1, rr);
          philox_round(g.c[1], p.sk.key0, p.sk.key1, rr);
        }
      } else if (slot < 7) {
        const int h = slot - 5;
        box_muller_fast(g.c[h][0], g.c[h][1], p.sk.neg2_ln2_over_r, g.z[4 * h], g.z[4 * h + 1]);
        box_muller_fast(g.c[h][2], g.c[h][3], p.sk.neg2_ln2_over_r, g.z[4 * h + 2], g.z[4 * h + 3]);
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) out[t] = (bf16)g.z[t];
      }
    }
  };
  auto kstep_slots = [&](const bf16x8(&af)[CWB], bf16x8 sf, const char* rd_stage, bf16x8(&nf)[CWB], SGen& g,
                         int gen_kstep, bf16x8& s_next) {
#pragma unroll
    for (int mb = 0; mb < CWB; ++mb) {
      if (TRANSPOSED) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, af[mb], acc[mb], 0, 0, 0);
      else acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mb], sf, acc[mb], 0, 0, 0);
      nf[mb] = read_block(rd_stage, mb);
      sgen_slot(g, mb, gen_kstep, s_next);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // s_waitcnt vmcnt((DEPTH - 1) * LOADS): everything but the DEPTH - 1 youngest stages has landed
  auto wait_oldest_stage = [&]() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 1) * LOADS) : "memory");
  };
  // One iteration = one k-step t: start the transfer of stage t + DEPTH into the slot stage t - 1 used,
  // make sure stage t + 1 has landed for every wave, then multiply k-step t while reading t + 1.
  // Branch-free: past the end the last stage is fetched again into a slot nobody reads.
  auto iteration = [&](int t, const bf16x8(&af)[CWB], bf16x8 sf, bf16x8(&nf)[CWB], SGen& g, bf16x8& s_next) {
    const int t_load = t + DEPTH < NS ? t + DEPTH : NS - 1;
    __builtin_amdgcn_sched_barrier(0);
    issue_stage(t_load, smem_lds + ((t + DEPTH) % NSTAGE) * STAGE);
    wait_oldest_stage();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    kstep_slots(af, sf, smem + ((t + 1) % NSTAGE) * STAGE, nf, g, t + 1, s_next);
  };

  if (NS > 0) {
    bf16x8 fa[CWB], fb[CWB];
    SGen gen;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue_stage(d < NS ? d : NS - 1, smem_lds + d * STAGE);
    bf16x8 s_a = make_s(0), s_b = s_a;
    wait_oldest_stage();
    __syncthreads();
#pragma unroll
    for (int mb = 0; mb < CWB; ++mb) fa[mb] = read_block(smem, mb);
    int t = 0;
    for (; t + 1 < NS; t += 2) {
      iteration(t, fa, s_a, fb, gen, s_b);
      iteration(t + 1, fb, s_b, fa, gen, s_a);
    }
    if (t < NS) iteration(t, fa, s_a, fb, gen, s_b);
  }
  wait_vmcnt0();  // no transfer may still be in flight when the work-group's LDS is released

  // ---- store the fp32 partial tile ----
  store_partial_tile<TRANSPOSED, CWB>(acc, p.part + (int64_t)g * p.C * p.r, p.C, p.r, c0 + wc * CWB * 32,
                                      js * RC + wj * 32, lane);
}

template <int WC, int WJ, int CWB>
constexpr int sketch_bf16_lds_bytes() {
  return 128 * 1024;
}

}  // namespace acc
