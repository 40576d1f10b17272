// One launch for a whole pass of the layer's heavy work (F1 + F0 + F2, or B1 + F0 + B2), used when the
// caller sets ACC_FLAG_ONE_LAUNCH: the work-groups of the exact GEMM (Y = X.W or dX = dY.W^T, 256 x 256
// tiles) and the work-groups of the sketch (Xs / Gr partials) are interleaved in one grid.  A CU that
// finishes a GEMM tile picks up whatever comes next, and the sketch reads its input while the GEMM has
// it in L2 / Infinity Cache.  Measured on MI355X the CU-time of the two kinds of work simply adds up
// (both need the whole LDS of a CU, and the chip is power-limited while the GEMM runs), so this path
// saves a launch but no time; the default path keeps two launches.
//
// Both kinds of work-group use 512 threads (8 waves, at most 256 registers per lane) and 128 KB of LDS.
#pragma once
#include "acc_gemm.h"
#include "acc_sketch.h"

namespace acc {

// Where the sketch work-groups sit in the grid, in groups of 8 work-groups (one per XCD): after every
// `period` groups of GEMM tiles comes one unit of `unit` sketch groups (the column slices of one
// input panel, which land on the same XCD), `n_units` times; the remaining GEMM groups follow.
struct FuseMap {
  int period, unit, n_units;
};

// 8-wave sketch work-group: tile 512 channels x 128 sketch columns, waves 2 (channels) x 4 (columns),
// each wave 256 channels x 32 columns = 8 MFMA blocks.  The two waves that share 32 columns each
// generate one Philox call per lane (4 of the 8 tokens a lane's operand needs) and trade halves
// through LDS, so S is generated once per work-group, not once per wave.
template <bool TRANSPOSED>
__device__ __forceinline__ void sketch8_tile(const SketchFastParams& p, int b, char* smem) {
  constexpr int WJ = 4, CWB = 8, NW = 8;
  constexpr int CH = 512, RC = 128, BT = 16;
  constexpr int ROW_BYTES = CH * 2;
  constexpr int STAGE = BT * ROW_BYTES;          // 16 KB: one MFMA k-step of tokens
  constexpr int NSTAGE = 7, DEPTH = NSTAGE - 1;  // 112 KB ring, 6 stages in flight
  constexpr int LOADS = BT / NW;                 // 1 KB wave-loads per wave and stage (one per token row)
  constexpr int XBUF = NSTAGE * STAGE;           // S exchange: 2 slots x 4 column groups x 64 lanes x 16 B

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
  if (NS == 0) return;

  // ---- global -> LDS: wave-load t of wave w is token row t * NW + w of the stage ----
  const u32x4 rsrc = make_rsrc(p.A + t_begin * p.lda + c0, ((p.n - t_begin - 1) * p.lda + (p.C - c0)) * 2);
  uint32_t src[LOADS], dst[LOADS];
#pragma unroll
  for (int t = 0; t < LOADS; ++t) {
    const int row = t * NW + wave;
    src[t] = (uint32_t)(row * p.lda * 2 + ((lane ^ swz_n(row)) << 4));
    dst[t] = (uint32_t)(row * ROW_BYTES);
  }
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;
  auto issue_stage = [&](int st, uint32_t stage_lds) {
    const uint32_t soff = (uint32_t)st * (uint32_t)(BT * p.lda * 2);
#pragma unroll
    for (int t = 0; t < LOADS; ++t) buffer_to_lds_b128(rsrc, src[t], soff, stage_lds + dst[t]);
  };
  auto wait_oldest_stage = [&]() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 1) * LOADS) : "memory"); };

  // ---- transposing operand reads (same layout as the 4-wave kernel) ----
  const int gq = lane >> 4, i16 = lane & 15;
  const int xr = (i16 >> 2) & 3;
  int rd_base[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int row = 8 * (gq >> 1) + (i16 >> 2);
    const int col16 = 2 * (gq & 1) + ((i16 & 3) >> 1);
    rd_base[v] = row * ROW_BYTES + (((v ^ xr) & 3) << 6) + (col16 << 4) + ((i16 & 1) << 3) + wc * (CWB * 64);
  }
  auto read_block = [&](const char* st, int mb) -> bf16x8 {
    const int off = (mb >> 2) * 256;
    const s16x4 lo = lds_read_tr16_b64(st, rd_base[mb & 3] + off);
    const s16x4 hi = lds_read_tr16_b64(st, rd_base[mb & 3] + off + 4 * ROW_BYTES);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // ---- S operand: lane holds column j and tokens 8 * (lane >> 5) .. + 7 of the k-step; this wave
  //      generates tokens 4 * wc .. 4 * wc + 3 of them (one Philox call) ----
  const uint32_t jcol = (uint32_t)(js * RC + wj * 32 + (lane & 31));
  const uint64_t q_lane = ((p.sk.row_offset + (uint64_t)t_begin) >> 2) + 2 * (uint64_t)(lane >> 5) + (uint64_t)wc;
  char* xslot[2] = {smem + XBUF + wj * 1024 + lane * 16, smem + XBUF + 4096 + wj * 1024 + lane * 16};
  struct HalfGen {
    uint32_t c[4];
    float z[4];
  };
  auto gen_begin = [&](HalfGen& h, int kstep) {
    const uint64_t q = q_lane + 4 * (uint64_t)kstep;
    h.c[0] = (uint32_t)q; h.c[1] = jcol; h.c[2] = 0u; h.c[3] = (uint32_t)(q >> 32);
  };
  auto gen_store = [&](const HalfGen& h, int kstep) {
    bf16x4 v;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = (bf16)h.z[t];
    *(bf16x4*)(xslot[kstep & 1] + wc * 8) = v;
  };
  // slice `slot` (0 .. 7) of generating this wave's half of the operand of k-step `kstep`
  auto gen_slot = [&](HalfGen& h, int slot, int kstep) {
    if (slot == 0) gen_begin(h, kstep);
    if (slot < 5) {
      philox_round(h.c, p.sk.key0, p.sk.key1, 2 * slot);
      philox_round(h.c, p.sk.key0, p.sk.key1, 2 * slot + 1);
    } else if (slot == 5) {
      box_muller_fast(h.c[0], h.c[1], p.sk.neg2_ln2_over_r, h.z[0], h.z[1]);
    } else if (slot == 6) {
      box_muller_fast(h.c[2], h.c[3], p.sk.neg2_ln2_over_r, h.z[2], h.z[3]);
    } else {
      gen_store(h, kstep);
    }
  };

  f32x16 acc[CWB];
#pragma unroll
  for (int i = 0; i < CWB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // One iteration = k-step t.  Start the transfer of stage t + DEPTH into the slot stage t - 1 used,
  // make sure stage t + 1 (and the S halves of k-step t + 1) are there for every wave, then in 8 slots:
  // MFMA on the operands in registers, the reads of the operands of k-step t + 1, and a slice of this
  // wave's half of S for k-step t + 2.  Branch-free: past the end the last stage is fetched again.
  HalfGen hg;
  auto iteration = [&](int t, const bf16x8(&af)[CWB], bf16x8 sf, bf16x8(&nf)[CWB], bf16x8& s_next) {
    const int t_load = t + DEPTH < NS ? t + DEPTH : NS - 1;
    __builtin_amdgcn_sched_barrier(0);
    issue_stage(t_load, smem_lds + ((t + DEPTH) % NSTAGE) * STAGE);
    wait_oldest_stage();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    const char* rd_stage = smem + ((t + 1) % NSTAGE) * STAGE;
#pragma unroll
    for (int mb = 0; mb < CWB; ++mb) {
      if (TRANSPOSED) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, af[mb], acc[mb], 0, 0, 0);
      else acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mb], sf, acc[mb], 0, 0, 0);
      if (mb == 0) s_next = *(const bf16x8*)xslot[(t + 1) & 1];  // both halves of k-step t + 1
      nf[mb] = read_block(rd_stage, mb);
      gen_slot(hg, mb, t + 2);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  bf16x8 fa[CWB], fb[CWB];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) issue_stage(d < NS ? d : NS - 1, smem_lds + d * STAGE);
#pragma unroll
  for (int k = 0; k < 2; ++k) {  // this wave's halves of the operands of k-steps 0 and 1
#pragma unroll
    for (int slot = 0; slot < 8; ++slot) gen_slot(hg, slot, k);
  }
  wait_oldest_stage();
  __syncthreads();
#pragma unroll
  for (int mb = 0; mb < CWB; ++mb) fa[mb] = read_block(smem, mb);
  bf16x8 s_a = *(const bf16x8*)xslot[0], s_b = s_a;
  int t = 0;
  for (; t + 1 < NS; t += 2) {
    iteration(t, fa, s_a, fb, s_b);
    iteration(t + 1, fb, s_b, fa, s_a);
  }
  if (t < NS) iteration(t, fa, s_a, fb, s_b);
  wait_vmcnt0();  // no transfer may still be in flight when the work-group's LDS is released

  store_partial_tile<TRANSPOSED, CWB>(acc, p.part + (int64_t)g * p.C * p.r, p.C, p.r, c0 + wc * CWB * 32,
                                      js * RC + wj * 32, lane);
}

// The 8-wave sketch tile as a kernel of its own (grid as for sketch_bf16_kernel).
template <bool TRANSPOSED>
__global__ __launch_bounds__(512) void sketch8_kernel(SketchFastParams sp) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  sketch8_tile<TRANSPOSED>(sp, blockIdx.x, smem);
}

template <bool B_KMAJOR, bool TRANSPOSED>
__global__ __launch_bounds__(512) void fused_linear_kernel(FastGemmParams gp, SketchFastParams sp, FuseMap fm) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int gi = blockIdx.x >> 3, x8 = blockIdx.x & 7;
  const int cycle = fm.period + fm.unit;
  const int cyc = gi / cycle, pos = gi - cyc * cycle;
  if (cyc < fm.n_units) {
    if (pos < fm.period) {
      gemm_bf16_tile<2, 4, 4, 2, B_KMAJOR, bf16>(gp, (cyc * fm.period + pos) * 8 + x8, smem);
    } else {
      sketch8_tile<TRANSPOSED>(sp, (cyc * fm.unit + (pos - fm.period)) * 8 + x8, smem);
    }
  } else {
    gemm_bf16_tile<2, 4, 4, 2, B_KMAJOR, bf16>(gp, (gi - fm.n_units * fm.unit) * 8 + x8, smem);
  }
}

}  // namespace acc
