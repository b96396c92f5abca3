// Pieces shared by the LDS-tiled GEMM kernels (gemm_mfma.hip, gemm_mx.hip): the workgroup -> tile map,
// the direct global -> LDS loads with their hand-counted waits, and the column tiling plan.
#ifndef SERQ_GEMM_TILE_H_
#define SERQ_GEMM_TILE_H_
#include "serq_device.h"

namespace serq {
namespace {

// Workgroup id -> output tile.  Consecutive ids go to different XCDs (8 of
// them, each with its own L2), so ids are first regrouped into one contiguous
// range per XCD; inside a range, tiles are ordered in bands of `groupm` token
// tiles so that the tiles in flight on one XCD share weight and token panels.
__device__ __forceinline__ void map_block(int bid, int tm, int tn, int gm, int& tile_m, int& tile_n) {
  const int T = tm * tn;
  const int per = (T + 7) >> 3;
  const int tall = (T & 7) == 0 ? 8 : (T & 7);
  const int xcd = bid & 7, loc = bid >> 3;
  const int logical = xcd < tall ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
  const int gsize = gm * tn;
  const int grp = logical / gsize;
  const int first_m = grp * gm;
  const int gsz = (tm - first_m) < gm ? (tm - first_m) : gm;
  const int within = logical - grp * gsize;
  tile_m = first_m + within % gsz;
  tile_n = within / gsz;
}

// ---- the hand-counted waits of the direct-to-LDS loads (dma16, serq_device.h) ----------------
// all but the youngest N vector-memory operations of this wave have completed,
// this wave's LDS reads are complete, and every wave of the workgroup has got here
template <int N>
__device__ __forceinline__ void wait_dma_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(N) : "memory");
}
__device__ __forceinline__ void fence() { __builtin_amdgcn_sched_barrier(0); }

// Column tiling: C tiles of `wide` or wide-1 blocks of 32 channels.  Estimated time of a launch:
// tiles are dealt to the compute units round by round, a round costs as much as its widest tile,
// and a tile of b blocks costs b + kFixed (the token panel and the per-step overheads do not
// shrink with the tile).
inline void plan_columns(int tiles_m, int NB, int ncu, int& C_out, int& wide_out, int& nwide_out) {
  const float kFixed = 4.0f;
  float best = 0.0f;
  int bestC = 0;
  const int cmin = (NB + 7) / 8;
  for (int C = cmin; C <= NB; ++C) {
    const int wide = (NB + C - 1) / C;
    const int nwide = NB - C * (wide - 1);            // tiles with `wide` blocks (the first ones)
    const long long tiles = (long long)tiles_m * C;
    const long long wide_tiles = (long long)tiles_m * nwide;
    const long long rounds = (tiles + ncu - 1) / ncu;
    const long long wide_rounds = (wide_tiles + ncu - 1) / ncu;
    const float cost = wide_rounds * (wide + kFixed) + (rounds - wide_rounds) * (wide - 1 + kFixed);
    if (bestC == 0 || cost < best - 1e-6f) { best = cost; bestC = C; }
    if (wide <= 2) break;                             // narrower tiles only add overhead
  }
  C_out = bestC;
  wide_out = (NB + bestC - 1) / bestC;
  nwide_out = NB - bestC * (wide_out - 1);
}

}  // namespace
}  // namespace serq
#endif  // SERQ_GEMM_TILE_H_
