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
