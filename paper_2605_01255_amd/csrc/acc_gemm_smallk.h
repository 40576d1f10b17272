// Product of the two gradient factors, C[M, N] = A[M, K] . B with a SHORT contraction (K = the sketch rank, or the
// optimizer's projector rank: 64 ... 512), fp32 accumulate (steps B3 and the weight update of the optimizer step):
//
//   C = A . B                      dW = Xs . Gr   (Sec. 4, update strategy (i))
//   C = beta C + alpha (A . B)     dW += ..., W <- (1 - lr wd) W - lr scale (P . N)   (update strategy (ii))
//
//   A is row-major with K contiguous (Xs, P; Gr in the paper's orientation).
//   B_KMAJOR = false: B[K, N], N contiguous (Gr);  B_KMAJOR = true: Bt[N, K], K contiguous (Xs in the paper's
//   orientation).  C row-major, bf16 or fp32.
//
// With four to eight K tiles a work-group's time is the latency of its transfers, not its arithmetic: a kernel
// that asks for K tile k + 1 while it multiplies K tile k (gemm_bf16_tile) waits for memory once per K tile.  Here
// a work-group asks for its first three K tiles at once (three LDS stages of 48 KB: 192 x 64 of A and 64 x 192 of
// B each) and for tile k + 3 as soon as tile k is consumed, so one latency is exposed at the start and little
// after it.  The tile is 192 x 192: 16 x 16 = 256 work-groups for a 3072 x 3072 gradient, one round of the chip.
// Four waves of 96 x 96 = 6 x 6 blocks of the 16x16x32 matrix instruction (144 accumulators per lane); operands
// of a k-step are read while the previous k-step multiplies.  K % 64 == 0, N % 8 == 0, operands below 4 GiB.
#pragma once
#include "acc_gemm16.h"

namespace acc {

// Swizzle of the 192-column N-contiguous B tile (rows of 384 bytes = 24 chunks of 16 bytes; a row starts on
// alternating halves of the 64 banks): the XOR stays inside an aligned group of eight chunks and sends the four
// k rows x two 16-lane groups of a transposing read to eight different 32-byte bank groups.
__device__ __forceinline__ int swz_n192(int krow) { return (((krow >> 1) & 1) << 1) | (((krow >> 3) & 1) << 2); }

template <bool B_KMAJOR, typename TC>
__global__ __launch_bounds__(256) void gemm16_smallk_kernel(FastGemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int NW = 4, WN = 2, TB = 6;
  constexpr int BM = 192, BN = 192, BK = 64, NS = 3;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW, NG = A_LOADS + B_LOADS;  // 6 + 6
  constexpr int BN_CHUNKS = BN / 8;  // 24

  const int tm = (int)(blockIdx.x % (unsigned)p.tiles_m), tn = (int)(blockIdx.x / (unsigned)p.tiles_m);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int l16 = lane & 15, g4 = lane >> 4;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int KT = (int)(p.K / BK);

  // ---- global -> LDS: wave-load t of wave w fills LDS bytes [(t * NW + w) * 1024, +1024) of the operand tile ----
  const u32x4 a_rsrc = make_rsrc(p.A + m0 * p.lda, ((p.M - m0 - 1) * p.lda + p.K) * 2);
  const u32x4 b_rsrc = B_KMAJOR ? make_rsrc(p.B + n0 * p.ldb, ((p.N - n0 - 1) * p.ldb + p.K) * 2)
                                : make_rsrc(p.B + n0, ((p.K - 1) * p.ldb + (p.N - n0)) * 2);
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
      const int c = (t * NW + wave) * 64 + lane;  // 16-byte chunk of the tile in LDS order
      const int krow = c / BN_CHUNKS, pos = c % BN_CHUNKS;
      // columns past the end of the matrix: the chunk would fall into the next row of B, so it is sent out of
      // the buffer's range and reads as zero
      const int chunk = pos ^ swz_n192(krow);
      b_src[t] = n0 + chunk * 8 < p.N ? (uint32_t)(krow * p.ldb * 2 + (chunk << 4)) : 0xFFFFFFF0u;
    }
  }
  const uint32_t b_kstep = B_KMAJOR ? BK * 2 : (uint32_t)(BK * p.ldb * 2);
  const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;
  auto issue_tile = [&](int kt, int stage) {
    const uint32_t st = smem_lds + stage * STAGE;
#pragma unroll
    for (int g = 0; g < A_LOADS; ++g)
      buffer_to_lds_b128(a_rsrc, a_src[g], (uint32_t)kt * (BK * 2), st + (g * NW + wave) * 1024);
#pragma unroll
    for (int g = 0; g < B_LOADS; ++g)
      buffer_to_lds_b128(b_rsrc, b_src[g], (uint32_t)kt * b_kstep, st + A_BYTES + (g * NW + wave) * 1024);
  };

  // ---- LDS read offsets of this lane's operands (see gemm16_persist_kernel) ----
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
      b_rd[j] = A_BYTES + krow * (BN * 2) + (((n_off >> 3) ^ swz_n192(krow)) << 4) + (n_off & 7) * 2;
    }
  }
  auto read_b = [&](const char* st, int s, int j) -> bf16x8 {
    if (B_KMAJOR) {
      return lds_read_b128(st, b_rd[j] + kc[s]);
    } else {
      // k rows + 32 s and + 4: bits 1 and 3 of the row index, which the swizzle uses, do not change
      const s16x4 lo = lds_read_tr16_b64(st, b_rd[j] + 32 * s * (BN * 2));
      const s16x4 hi = lds_read_tr16_b64(st, b_rd[j] + (32 * s + 4) * (BN * 2));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  f32x4 acc[TB][TB];
#pragma unroll
  for (int i = 0; i < TB; ++i)
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  bf16x8 a[2][TB], b[2][TB];

#pragma unroll
  for (int s = 0; s < NS; ++s)
    if (s < KT) issue_tile(s, s);

  // Read-modify-write of a bf16 C (the optimizer's update of W): the old values are requested now, in the layout the
  // epilogue moves them in (block row i, 16-byte chunk t * 64 + lane of its 16 x 96 piece), so that they arrive
  // under the K loop instead of after it.  They are PREFETCH = 18 loads of this wave, issued after the first
  // three K tiles and before the fourth, which the waits below count.
  constexpr bool RMW_PREFETCH = sizeof(TC) == 2;
  constexpr int PREFETCH = RMW_PREFETCH ? TB * 3 : 0;
  u32x4 old_c[RMW_PREFETCH ? TB : 1][3];
  const bool prefetch = RMW_PREFETCH && p.accumulate;
  if constexpr (RMW_PREFETCH) {
    if (prefetch) {
      __builtin_amdgcn_sched_barrier(0);
      // buffer resource over this wave's 96 x 96 piece of C: offsets stay below 4 GiB whatever the size of C
      const int64_t gm_base = m0 + wm * TB * 16, gn_base = n0 + wn * TB * 16;
      int64_t c_rows = p.M - gm_base;
      if (c_rows > TB * 16) c_rows = TB * 16;
      const int64_t c_bytes = (c_rows > 0 && gn_base < p.N) ? ((c_rows - 1) * p.ldc + (p.N - gn_base)) * 2 : 0;
      const __amdgpu_buffer_rsrc_t c_rs = __builtin_amdgcn_make_buffer_rsrc(
          (void*)((const bf16*)p.C + gm_base * p.ldc + gn_base), 0, (int)(uint32_t)c_bytes, 0x00020000);
#pragma unroll
      for (int i = 0; i < TB; ++i)
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          const int idx = t * 64 + lane, row = idx / 12, ch = idx % 12;
          // rows or columns past the end: out of the buffer's range, the load returns zero (never stored)
          const uint32_t off = (gm_base + i * 16 + row < p.M && gn_base + ch * 8 < p.N)
                                   ? (uint32_t)(((i * 16 + row) * p.ldc + ch * 8) * 2) : 0xFFFFFFF0u;
          old_c[i][t] = __builtin_amdgcn_raw_buffer_load_b128(c_rs, off, 0, 0);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  for (int kt = 0; kt < KT; ++kt) {
    const char* cur = smem + (kt % NS) * STAGE;
    // K tile kt has landed when at most the wave-loads of the tiles requested after it (and, for the first three
    // K tiles, the prefetch of C, which was issued after them) are outstanding
    const int later = (kt + NS - 1 < KT ? kt + NS - 1 : KT - 1) - kt;
    if (prefetch && kt < NS) {
      if (later >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NG + PREFETCH) : "memory");
      else if (later == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NG + PREFETCH) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PREFETCH) : "memory");
    } else {
      if (later >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NG) : "memory");
      else if (later == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NG) : "memory");
      else wait_vmcnt0();
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TB; ++i) a[0][i] = read_a(cur, 0, i);
#pragma unroll
    for (int j = 0; j < TB; ++j) b[0][j] = read_b(cur, 0, j);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < TB * TB; ++q) {  // k-step 0, the operands of k-step 1 read beside it
      const int i = q / TB, j = q % TB;
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[0][j], a[0][i], acc[i][j], 0, 0, 0);
      if (q % 3 == 0) {
        const int r = q / 3;
        if (r < TB) a[1][r] = read_a(cur, 1, r);
        else b[1][r - TB] = read_b(cur, 1, r - TB);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < TB * TB; ++q) {  // k-step 1
      const int i = q / TB, j = q % TB;
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[1][j], a[1][i], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();  // every wave is done reading this stage
    if (kt + NS < KT) issue_tile(kt + NS, kt % NS);
  }

  // ---- epilogue: lane holds output row l16 of each 16 x 16 block and columns 4 g4 .. + 3; a wave stages one block
  //      row (16 x 96) in a private padded LDS region (the stages are free: the loop ended on a barrier with nothing
  //      in flight) and moves 16 bytes per lane ----
  constexpr int ES = sizeof(TC);
  constexpr int ROW_B = TB * 16 * ES, PITCH = ROW_B + 16, CH16 = ROW_B / 16;
  char* stage_w = smem + wave * (16 * PITCH);
  TC* __restrict__ C = (TC*)p.C;
#pragma unroll
  for (int i = 0; i < TB; ++i) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      char* dst = stage_w + l16 * PITCH + (j * 16 + g4 * 4) * ES;
      if constexpr (ES == 2) {
        bf16x4 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = (bf16)acc[i][j][t];
        *(bf16x4*)dst = v;
      } else {
        *(f32x4*)dst = acc[i][j];
      }
    }
#pragma unroll
    for (int t = 0; t < 16 * CH16 / 64; ++t) {
      const int idx = t * 64 + lane, row = idx / CH16, ch = idx % CH16;
      const u32x4 v = *(const u32x4*)(stage_w + row * PITCH + ch * 16);
      const int64_t gm = m0 + (wm * TB + i) * 16 + row;
      const int64_t gn = n0 + wn * TB * 16 + ch * (16 / ES);
      if (gm < p.M && gn < p.N) {
        u32x4* dst = (u32x4*)(C + gm * p.ldc + gn);
        if (p.accumulate) {
          u32x4 old;
          if constexpr (RMW_PREFETCH) old = old_c[i][t];
          else old = *dst;
          if constexpr (ES == 2) {
            const bf16x8 x = __builtin_bit_cast(bf16x8, v), o = __builtin_bit_cast(bf16x8, old);
            bf16x8 sum;
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] = (bf16)(p.alpha * (float)x[e] + p.beta * (float)o[e]);
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

}  // namespace acc
