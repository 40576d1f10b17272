// Tuned bf16 sketch kernel for gfx950 (steps F0 + F2 and F0 + B2):
//
//   part[g][c][j] = sum over the tokens t of split g of  A[t, c] * S[t, j]          (TRANSPOSED = false, Xs)
//   part[g][j][c] = the same value stored transposed                                 (TRANSPOSED = true,  Gr)
//
// A is X [n, d_in] or dY [n, d_out] (row-major, channels contiguous); S[t, j] is regenerated from the
// Philox counter (token, column) in registers, directly in MFMA operand layout, and never stored.
//
// Work-group = 8 waves on a tile of 512 channels x 64 or 128 sketch columns, fp32 accumulators in registers
// for the whole token range of the split.  Tokens stream through LDS in stages of 16 or 32 rows, global ->
// LDS directly, in a ring with 96 KB in flight: the input is read once from HBM, so enough bytes must be
// outstanding per CU to cover DRAM latency.  The channel-major MFMA operand is formed from the token-major
// tile with transposing LDS reads.  The contraction runs over tokens, so one Philox call (4 tokens of one
// column) feeds half an operand register set.
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

// 8-wave sketch work-group: tile 512 channels x (WJ * 32) sketch columns, waves WC = 8 / WJ (channels) x WJ
// (columns), each wave (512 / WC) channels x 32 columns.  An iteration is eight MFMAs per wave:
//   WJ = 4: 512 x 128 tile, waves 2 x 4, 8 channel blocks x one 16-token k-step  (128 accumulators per lane)
//   WJ = 2: 512 x  64 tile, waves 4 x 2, 4 channel blocks x two 16-token k-steps ( 64 accumulators per lane)
// The WC waves that share 32 columns each generate one Philox call per lane and iteration (4 of the 8 * WC / 2
// tokens a lane's operands need) and trade them through LDS, so S is generated once per work-group, not
// once per wave.  The narrow tile keeps half as many accumulators per compute unit: a work-group covers
// twice the tokens and the launch writes (and the fold reads) half as many bytes of partial tiles.
template <bool TRANSPOSED, int WJ = 4>
__device__ __forceinline__ void sketch8_tile(const SketchFastParams& p, int b, char* smem) {
  static_assert(WJ == 4 || WJ == 2, "column groups");
  constexpr int NW = 8, WC = NW / WJ;
  constexpr int CH = 512, RC = WJ * 32;
  constexpr int CWB = CH / (WC * 32);            // channel blocks per wave: 8 or 4
  constexpr int KS = 8 / CWB;                    // k-steps per iteration: 1 or 2
  constexpr int BT = 16 * KS;                    // tokens per stage
  constexpr int ROW_BYTES = CH * 2;
  constexpr int STAGE = BT * ROW_BYTES;          // 16 or 32 KB
  constexpr int NSTAGE = KS == 1 ? 7 : 4;        // ring of 112 or 128 KB,
  constexpr int DEPTH = NSTAGE - 1;              // 96 KB in flight
  constexpr int LOADS = BT / NW;                 // 1 KB wave-loads per wave and stage (one per token row)
  constexpr int XBUF = NSTAGE * STAGE;           // S exchange: 2 slots x KS k-steps x WJ column groups x 64 lanes x 16 B
  constexpr int XSLOT = KS * WJ * 1024;          // 4 KB either way

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
  const int NS = t_end > t_begin ? (int)((t_end - t_begin + BT - 1) / BT) : 0;  // stages = iterations
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
    const int col16 = 2 * (gq & 1) + ((i16 & 3) >> 1);
    rd_base[v] = row * ROW_BYTES + (((v ^ xr) & 3) << 6) + (col16 << 4) + ((i16 & 1) << 3) + wc * (CWB * 64);
  }
  // operand of slot s = k-step (s / CWB) of the stage, channel block (s % CWB) of the wave
  auto read_block = [&](const char* st, int s) -> bf16x8 {
    const int mb = s % CWB, ks = s / CWB;
    const int off = (mb >> 2) * 256 + ks * (16 * ROW_BYTES);
    const s16x4 lo = lds_read_tr16_b64(st, rd_base[mb & 3] + off);
    const s16x4 hi = lds_read_tr16_b64(st, rd_base[mb & 3] + off + 4 * ROW_BYTES);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // ---- S operand: lane holds column j and tokens 8 * (lane >> 5) .. + 7 of a k-step; this wave generates
  //      tokens 4 * (wc & 1) .. + 3 of them for k-step (wc >> 1) of the iteration (one Philox call) ----
  const uint32_t jcol = (uint32_t)(js * RC + wj * 32 + (lane & 31));
  const uint64_t q_lane = ((p.sk.row_offset + (uint64_t)t_begin) >> 2) + 2 * (uint64_t)(lane >> 5) +
                          (uint64_t)(wc & 1) + 4 * (uint64_t)(wc >> 1);
  char* const xbase = smem + XBUF + wj * 1024 + lane * 16;  // + parity * XSLOT + k-step * WJ * 1024
  struct HalfGen {
    uint32_t c[4];
    float z[4];
  };
  auto gen_begin = [&](HalfGen& h, int it) {
    const uint64_t q = q_lane + (uint64_t)(4 * KS) * (uint64_t)it;
    h.c[0] = (uint32_t)q; h.c[1] = jcol; h.c[2] = 0u; h.c[3] = (uint32_t)(q >> 32);
  };
  auto gen_store = [&](const HalfGen& h, int it) {
    bf16x4 v;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = (bf16)h.z[t];
    *(bf16x4*)(xbase + (it & 1) * XSLOT + (wc >> 1) * (WJ * 1024) + (wc & 1) * 8) = v;
  };
  // slice `slot` (0 .. 7) of generating this wave's share of the operands of iteration `it`
  auto gen_slot = [&](HalfGen& h, int slot, int it) {
    if (slot == 0) gen_begin(h, it);
    if (slot < 5) {
      philox_round(h.c, p.sk.key0, p.sk.key1, 2 * slot);
      philox_round(h.c, p.sk.key0, p.sk.key1, 2 * slot + 1);
    } else if (slot == 5) {
      box_muller_fast(h.c[0], h.c[1], p.sk.neg2_ln2_over_r, h.z[0], h.z[1]);
    } else if (slot == 6) {
      box_muller_fast(h.c[2], h.c[3], p.sk.neg2_ln2_over_r, h.z[2], h.z[3]);
    } else {
      gen_store(h, it);
    }
  };
  struct SOps {
    bf16x8 s[KS];
  };
  auto read_s = [&](int it) -> SOps {  // all shares of the operands of iteration `it`
    SOps o;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) o.s[ks] = *(const bf16x8*)(xbase + (it & 1) * XSLOT + ks * (WJ * 1024));
    return o;
  };

  f32x16 acc[CWB];
#pragma unroll
  for (int i = 0; i < CWB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // One iteration = stage t.  Start the transfer of stage t + DEPTH into the slot stage t - 1 used,
  // make sure stage t + 1 (and the S shares of iteration t + 1) are there for every wave, then in 8 slots:
  // MFMA on the operands in registers, the reads of the operands of iteration t + 1, and a slice of this
  // wave's share of S for iteration t + 2.  Branch-free: past the end the last stage is fetched again.
  HalfGen hg;
  auto iteration = [&](int t, const bf16x8(&af)[8], const SOps& sf, bf16x8(&nf)[8], SOps& s_next) {
    const int t_load = t + DEPTH < NS ? t + DEPTH : NS - 1;
    __builtin_amdgcn_sched_barrier(0);
    issue_stage(t_load, smem_lds + ((t + DEPTH) % NSTAGE) * STAGE);
    wait_oldest_stage();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    const char* rd_stage = smem + ((t + 1) % NSTAGE) * STAGE;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int mb = s % CWB, ks = s / CWB;
      if (TRANSPOSED) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf.s[ks], af[s], acc[mb], 0, 0, 0);
      else acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s], sf.s[ks], acc[mb], 0, 0, 0);
      if (s == 0) s_next = read_s(t + 1);
      nf[s] = read_block(rd_stage, s);
      gen_slot(hg, s, t + 2);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  bf16x8 fa[8], fb[8];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) issue_stage(d < NS ? d : NS - 1, smem_lds + d * STAGE);
#pragma unroll
  for (int k = 0; k < 2; ++k) {  // this wave's shares of the operands of iterations 0 and 1
#pragma unroll
    for (int slot = 0; slot < 8; ++slot) gen_slot(hg, slot, k);
  }
  wait_oldest_stage();
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 8; ++s) fa[s] = read_block(smem, s);
  SOps s_a = read_s(0), s_b = s_a;
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

// The 8-wave sketch tile as a kernel of its own: grid = 8 * n_js * ceil(n_cslab * G / 8) work-groups.
template <bool TRANSPOSED, int WJ = 4>
__global__ __launch_bounds__(512) void sketch8_kernel(SketchFastParams sp) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  sketch8_tile<TRANSPOSED, WJ>(sp, blockIdx.x, smem);
}

// Dynamic LDS of sketch8_kernel: the stage ring plus the 8 KB S exchange.
template <int WJ>
constexpr int sketch8_lds_bytes() {
  return WJ == 4 ? 128 * 1024 : 136 * 1024;
}

}  // namespace acc
