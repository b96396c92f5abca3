// Pieces shared by the LDS-tiled GEMM kernels (gemm_mfma.hip, gemm_mx.hip): the workgroup -> tile map,
// the direct global -> LDS loads with their hand-counted waits, the column tiling plan and the K-slice plan.
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

// ---- K slicing: when and how (host side) ---------------------------------------------------------
// A layer with few tokens gives few tiles: one token tile x the column tiles.  Narrow column tiles fill more
// compute units but every one of them walks all of K re-reading its whole token panel from LDS, so the step
// gets no cheaper; cutting K into S slices instead multiplies the workgroups by S at the price of parking
// S accumulator tiles (INT32, or fp32 in the MXFP4 kernel) per output tile and a second launch that adds them up.  The plan below prices both with a
// small model fitted to measurements (cycles of one 64-channel step of a tile of b channel blocks; 5 TB/s for
// the parked tiles, written and read once; 3 us for the second launch) and slices only when that wins.
struct SplitPlan { int C, wide, nwide, S; };

// `kind`: 8 / 4 = the integer kernel with 8- / 4-bit activations, 0 = the MXFP4 kernel (twice the MFMA rate,
// so the global -> LDS stream of a narrow tile, 8 KiB of token codes + b KiB of weights at 32 B/clk, shows)
inline float step_cycles(int b, int kind) {
  if (kind == 0) {
    const float mfma = 64.0f * b, lds = 40.0f * b + 192.0f, dma = 32.0f * b + 256.0f;
    const float m2 = mfma > lds ? mfma : lds;
    return 1.3f * (m2 > dma ? m2 : dma);
  }
  const float mfma = 128.0f * b, lds = kind == 8 ? 40.0f * b + 384.0f : 40.0f * b + 192.0f;
  return 1.3f * (mfma > lds ? mfma : lds);
}

inline SplitPlan plan_split(int M, int N, int K, int kind, int ncu, int forced) {
  const int NB = N / 32, tiles_m = (M + 255) / 256;   // both kernels: 256 tokens per tile
  const int CHh = kind == 8 ? 2 : 4;
  const int KT = (K / 64 + CHh - 1) / CHh;             // main tiles
  SplitPlan best;
  plan_columns(tiles_m, NB, ncu, best.C, best.wide, best.nwide);
  best.S = 1;
  if (forced == 1) return best;
  if (forced > 1) {
    best.S = forced < KT ? forced : KT;
    return best;
  }
  if ((long long)tiles_m * best.C * 4 >= 3LL * ncu || M > 512 || KT < 8) return best;   // the tiles fill the part well enough
  const float steps = (float)(K / 64);
  auto cost = [&](int C, int wide, int S) {
    const long long wg = (long long)tiles_m * C * S;
    const float rounds = (float)((wg + ncu - 1) / ncu);
    float us = rounds * (steps / S) * step_cycles(wide, kind) / 2000.0f;
    if (S > 1) us += 2.0f * ((float)S * M * N * 4.0f) / 5.0e6f + 3.0f;
    return us;
  };
  float bc = cost(best.C, best.wide, 1);
  const int cand[] = {2, 3, 4, 6, 8, 12, 16};
  for (int wide = 1; wide <= 8; ++wide) {
    const int C = (NB + wide - 1) / wide;
    const int w2 = (NB + C - 1) / C;                    // the width this many tiles really have
    for (int S : cand) {
      if (S * 2 > KT || (long long)tiles_m * C * S > 2LL * ncu) continue;
      const float c = cost(C, w2, S);
      if (c < bc * 0.9f) {                              // only for a clear win: the model is rough
        bc = c;
        best.C = C; best.wide = w2; best.nwide = NB - C * (w2 - 1); best.S = S;
      }
    }
  }
  return best;
}

inline int wave_blocks8(int wide) { const int h = (wide + 1) / 2; return 8 * (h < 1 ? 1 : h); }

}  // namespace
}  // namespace serq
#endif  // SERQ_GEMM_TILE_H_
