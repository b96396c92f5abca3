// SERQ linear layer for prefill-sized batches: LDS-tiled int8-MFMA GEMM over
// nibble-packed weights with the rank-r compensation and the dequantising
// epilogue fused in, so Y is written once (Eq. 2 + Eq. 7, first line):
//   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k] Wq[n,k] + sum_j Xq[m,S_j] R[j,n] )
//
// Workgroup: 8 waves = 2 along the output channels x 4 along the tokens.  A
// workgroup tile is 256 tokens x up to 256 output channels (1..8 blocks of 32);
// the host picks the number of column tiles so that the tiles fill the compute
// units in whole rounds, and the two channel halves of a tile are dealt to the
// waves so that every SIMD carries one wave of each half.  Each wave owns up to
// 4 channel blocks x 2 token blocks = 8 MFMA tiles of 32x32 (128 accumulator
// registers).  The weights are the MFMA "A" operand (rows = output channels)
// and the tokens the "B" operand (columns), so each lane ends up with runs of 4
// consecutive output channels of one token.
//
// The work of a workgroup is a sequence of tiles flowing through a ring of LDS
// stages (3 x 48 KiB for 8-bit activations, 2 x 64 KiB for 4-bit):
//   main tiles     : 128 (8-bit) or 256 (4-bit) input channels; a token row of
//                    the tile is 128 bytes either way.  Weights: the 1-KiB
//                    fragments of the packed blob, unchanged (lane-linear).
//                    Tokens: 256 rows x 128 B, the 16-byte piece c of row i
//                    stored at piece c ^ ((i >> 1) & 7): conflict-free reads.
//   low-rank tiles : 64 salient channels each, appended after the main tiles:
//                    32 KiB of packed R fragments plus the codes of the 256
//                    tokens for those channels.
// Tiles travel global -> LDS directly (global_load_lds_dwordx4: a lane's 16
// bytes land at M0 + 16*lane); the swizzle is applied on the source side.  These
// loads are issued from inline assembly and counted by hand with vmcnt, because
// the compiler would wait for every outstanding LDS-bound load before any LDS
// read it cannot disambiguate.  In the steady state the refill of a stage is
// spread over the MFMA groups of one 64-channel step.
//
// Inside a tile the operand fragments are double-buffered in registers: the LDS
// reads of the next 64-channel fragment are issued before the MFMAs of the
// current one (scheduling fences keep them there).
//
// Nibbles are widened only in registers, to 16*q (three VALU ops per packed
// dword); the accumulators hold 2^SH times the true sums and the epilogue folds
// 2^-SH into wscale (exact).  After the last main tile the integer accumulators
// are converted in place to fp32 (wscale[n] * acc) and the low-rank tiles are
// accumulated on top with 32x32x16 f16/bf16 MFMAs.  16-bit outputs are then
// transposed through LDS so that every store instruction writes whole 512-byte
// row segments.
#include <type_traits>

#include "gemm_tile.h"
#include "serq_device.h"

namespace serq {
namespace {

constexpr int BM = 256;
constexpr int kThreads = 512;
constexpr int kWaves = 8;

template <int ABITS>
struct Tile {
  static constexpr int BK = ABITS == 8 ? 128 : 256;   // channels per main tile
  static constexpr int CH = BK / 64;                  // 64-channel fragments per main tile
  static constexpr int W_BYTES = 8 * CH * 1024;
  static constexpr int X_BYTES = BM * 128;
  static constexpr int STAGE = W_BYTES + X_BYTES;
  static constexpr int NS = ABITS == 8 ? 3 : 2;       // ring depth
  static constexpr int SH = ABITS == 8 ? 4 : 8;
  static constexpr int NLW = CH;                      // direct loads per wave and main tile: weights
  static constexpr int NLX = 4;                       //                                      tokens
  static constexpr int NL = NLW + NLX;
  static constexpr int LR_R_BYTES = 8 * 4 * 1024;
  static constexpr int LR_XROW = 64 * ABITS / 8;      // bytes of one token's 64 salient codes
  static constexpr int LR_NLX = BM * LR_XROW / 16 / kThreads;
  static constexpr int NL_LR = 4 + LR_NLX;
  static constexpr int WS_OFF = NS * STAGE;           // 256 floats: the tile's weight scales
  static constexpr int RS_OFF = WS_OFF + 256 * 4;     // 256 floats: the scales of a 4-bit compensation matrix
  static constexpr int LDS_BYTES = RS_OFF + 256 * 4;
  static_assert(LR_R_BYTES + BM * LR_XROW <= STAGE, "a low-rank tile fits a stage");
  static_assert(NS == 2 || NL == NL_LR, "one vmcnt immediate serves both tile kinds");
  static_assert(BM * 512 <= NS * STAGE, "the 16-bit output tile fits the ring");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

struct MfmaParams {
  const uint8_t* Xq; const float* scale;
  const u4* Wq; const float* wscale;
  const u4* Rp; int r_dtype; int s_begin; int r;
  const float* rscale;    // r_dtype == SERQ_I4: per-channel scales of the 4-bit compensation matrix
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int32_t* acc_out; int64_t ldacc;
  int tiles_m, tiles_n, groupm;
  int wide, nwide;        // column tiles 0..nwide-1 have `wide` blocks of 32 channels, the rest wide-1
  // K slicing for layers whose tiles alone leave most compute units idle (two launches of this kernel):
  //   pass 1 (kslices > 1, reduce = 0): grid (tiles, kslices); workgroup (tile, s) multiplies slice s of K and
  //     parks its raw INT32 tile in `part`, in register order (every store a full 1-KiB wave row);
  //   pass 2 (reduce = 1): grid (tiles); no main tiles -- the accumulators start as the sum of the parked
  //     tiles (integer addition: the same bits as an unsliced run), then the usual epilogue.
  int kslices, reduce;
  int4* part;             // [kslices][tiles][8 waves][hm8][64 lanes]
  int hm8;                // 8 x the largest number of channel blocks a wave owns (wide rounded up to even, / 2)
};

// ---- operand fragments ---------------------------------------------------------
template <int ABITS>
struct Frag {                       // one 64-channel fragment of a main tile
  u4 w[4];                          // packed weights of the wave's channel blocks
  u4 x[ABITS == 8 ? 4 : 2];         // tokens: 8-bit: [2*j + half], 4-bit: [j] (packed)
};

__device__ __forceinline__ v4i widen(uint32_t d0, uint32_t d1) {
  int a, b, c, d;
  unpack16(d0, a, b);
  unpack16(d1, c, d);
  return v4i{a, b, c, d};
}

// LRT: form of the compensation matrix -- SERQ_BF16 / SERQ_F16 fragments, or SERQ_I4: the 4-bit blob,
// whose tiles run on the int8 units.  A compile-time choice: selected at run time inside the rank-r
// loop, the f16 and bf16 MFMAs leave the compiler merging their results with register copies after
// every MFMA.
template <int ABITS, int LRT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void serq_mfma_kernel(const MfmaParams p) {
  using T = Tile<ABITS>;
  constexpr int CH = T::CH;
  constexpr int NS = T::NS;
  constexpr int STAGE = T::STAGE;
  __shared__ __align__(16) uint8_t lds[T::LDS_BYTES];

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int wn = (w ^ (w >> 2)) & 1;                 // every SIMD gets one wave of each channel half
  const int wm = w >> 1;
  const int lm = l & 31, g = l >> 5;
  int tile_m, tile_n;
  map_block(blockIdx.x, p.tiles_m, p.tiles_n, p.groupm, tile_m, tile_n);
  const int m0 = tile_m * BM;
  const int nbt = tile_n < p.nwide ? p.wide : p.wide - 1;                       // blocks of 32 channels in this tile
  const int nb0 = tile_n < p.nwide ? tile_n * p.wide : p.nwide * p.wide + (tile_n - p.nwide) * (p.wide - 1);
  const int n0 = nb0 << 5;
  const int half = (nbt + 1) >> 1;
  const int blk0 = __builtin_amdgcn_readfirstlane(wn ? half : 0);              // this wave's first block in the tile
  const int nbw = __builtin_amdgcn_readfirstlane(wn ? nbt - half : half);      // and how many it owns (0..4)
  const int KBg = p.K >> 6;                          // fragments per channel block in memory
  // the main tiles [ta, tb) this workgroup multiplies: all of them, one K slice (pass 1), or none (pass 2)
  const bool part_out = p.kslices > 1 && !p.reduce;
  int ta = 0, tb = (KBg + CH - 1) / CH;
  if (part_out) {
    const int per = tb / p.kslices, rem = tb % p.kslices, sl = blockIdx.y;
    ta = sl * per + (sl < rem ? sl : rem);
    tb = ta + per + (sl < rem ? 1 : 0);
  } else if (p.reduce) {
    tb = 0;
  }
  const int KB = (tb * CH < KBg ? tb * CH : KBg) - ta * CH;   // this workgroup's fragments
  const uint32_t rowbytes = (uint32_t)p.K * ABITS / 8;
  const int mrows = p.M - m0 < BM ? p.M - m0 : BM;   // valid token rows of this tile

  const int KTF = KB / CH;                           // full main tiles
  const int KTAIL = KB - KTF * CH;                   // fragments of a last, partial main tile
  const int KT = KTF + (KTAIL ? 1 : 0);
  const int JB = (p.acc_out == nullptr && !part_out) ? (p.r >> 4) : 0;
  const int LT = (JB + 3) >> 2;                      // low-rank tiles of 64 salient channels (16-bit R: up to 4 x 16)
  constexpr bool lr_int = LRT == SERQ_I4;            // one weight-like fragment per tile and block
  const int TT = KT + LT;

  // the tile's weight scales, times 2^-SH (exact), for the int -> float conversion
  constexpr float kInv = 1.0f / (float)(1 << T::SH);
  float* lws = reinterpret_cast<float*>(lds + T::WS_OFF);
  if (tid < 256 && p.wscale != nullptr) lws[tid] = tid < 32 * nbt ? p.wscale[n0 + tid] * kInv : 0.0f;
  float* lrs = reinterpret_cast<float*>(lds + T::RS_OFF);
  if (tid < 256 && lr_int && LT > 0) lrs[tid] = tid < 32 * nbt ? p.rscale[n0 + tid] * kInv : 0.0f;

  const int wu = __builtin_amdgcn_readfirstlane(w);
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr(lds));

  // ---- per-lane source offsets of the direct loads ------------------------------
  // weights: wave w fetches fragments f = 8*i + w of the stage, f = nbl*CH + ch
  uint32_t wv[T::NLW];
#pragma unroll
  for (int i = 0; i < T::NLW; ++i) {
    const int f = i * kWaves + wu;
    int nbl = f / CH;
    nbl = nbl < nbt ? nbl : nbt - 1;                 // blocks past the tile: duplicates, never read
    wv[i] = (uint32_t)((nbl * KBg + (f % CH)) * 1024 + l * 16);
  }
  // tokens: LDS piece pc = 512*i + tid -> row pc/8, slot pc%8 holds global piece slot ^ swizzle(row)
  uint32_t xv[T::NLX];
#pragma unroll
  for (int i = 0; i < T::NLX; ++i) {
    const int pc = i * kThreads + tid;
    int row = pc >> 3;
    const int c = (pc & 7) ^ ((row >> 1) & 7);
    row = row < mrows ? row : mrows - 1;             // rows past M: duplicates, never stored
    xv[i] = (uint32_t)row * rowbytes + 16u * c;
  }
  const uint8_t* wbase = (const uint8_t*)p.Wq + ((size_t)nb0 * KBg + (size_t)ta * CH) * 1024;
  const uint8_t* xbase = p.Xq + (size_t)m0 * rowbytes;
  const uint8_t* xmain = xbase + (size_t)ta * 128;     // token codes of this workgroup's first main tile

  // k-th direct load of main tile t into stage st (k < NL)
  auto issue_main_one = [&](int t, int st, int k) {
    const uint32_t sb = lds0 + (uint32_t)st * STAGE + (uint32_t)wu * 1024;
    if (k < T::NLW) dma16(wbase + (size_t)t * CH * 1024, wv[k], sb + kWaves * 1024 * k);
    else dma16(xmain + (size_t)t * 128, xv[k - T::NLW], sb + T::W_BYTES + kWaves * 1024 * (k - T::NLW));
  };
  // a main tile whose fragments / pieces may run past K: clamp them into the tile's first fragment
  auto issue_main_tail = [&](int t, int st) {
    const uint32_t sb = lds0 + (uint32_t)st * STAGE + (uint32_t)wu * 1024;
    const int nf = KB - t * CH;                      // 1 .. CH-1 valid fragments
#pragma unroll
    for (int i = 0; i < T::NLW; ++i) {
      const int f = i * kWaves + wu;
      int nbl = f / CH, ch = f % CH;
      nbl = nbl < nbt ? nbl : nbt - 1;
      ch = ch < nf ? ch : 0;
      dma16(wbase + (size_t)t * CH * 1024, (uint32_t)((nbl * KBg + ch) * 1024 + l * 16), sb + kWaves * 1024 * i);
    }
    const int npc = nf * (ABITS == 8 ? 4 : 2);       // valid 16-byte pieces of a token row
#pragma unroll
    for (int i = 0; i < T::NLX; ++i) {
      const int pc = i * kThreads + tid;
      int row = pc >> 3;
      int c = (pc & 7) ^ ((row >> 1) & 7);
      c = c < npc ? c : 0;
      row = row < mrows ? row : mrows - 1;
      dma16(xmain + (size_t)t * 128, (uint32_t)row * rowbytes + 16u * c, sb + T::W_BYTES + kWaves * 1024 * i);
    }
  };
  // low-rank tile lt (4 x 16 salient channels) into stage st
  auto issue_lr = [&](int lt, int st) {
    const uint32_t sb = lds0 + (uint32_t)st * STAGE + (uint32_t)wu * 1024;
    // opaque copy of the thread index: the per-lane offsets below are recomputed here instead of
    // being carried in registers through the main loop, where every register is taken
    int tl = tid;
    asm volatile("" : "+v"(tl));
    if constexpr (lr_int) {
      // wave w brings the fragment of block w to slot w; the other three loads of a wave repeat it
      // into unused slots so that every tile kind issues the same number of loads
      const uint8_t* rbase = (const uint8_t*)p.Rp + ((size_t)nb0 * LT + lt) * 1024;
      const int nbl = wu < nbt ? wu : nbt - 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) dma16(rbase, (uint32_t)(nbl * LT * 1024 + l * 16), sb + kWaves * 1024 * i);
    } else {
      const int njb = JB - 4 * lt < 4 ? JB - 4 * lt : 4;
      const uint8_t* rbase = (const uint8_t*)p.Rp + ((size_t)nb0 * JB + 4 * lt) * 1024;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int f = i * kWaves + wu;               // f = nbl*4 + jbl
        int nbl = f >> 2, jbl = f & 3;
        nbl = nbl < nbt ? nbl : nbt - 1;
        jbl = jbl < njb ? jbl : 0;
        dma16(rbase, (uint32_t)((nbl * JB + jbl) * 1024 + l * 16), sb + kWaves * 1024 * i);
      }
    }
    if constexpr (ABITS == 8) {
      const uint8_t* cbase = xbase + p.s_begin + 64 * lt;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        int row = (tl + kThreads * i) >> 2;
        int c = (tl & 3) ^ ((row >> 2) & 3);
        c = (64 * lt + 16 * c + 16 <= p.r) ? c : 0;  // a piece past the salient block is never read
        row = row < mrows ? row : mrows - 1;
        dma16(cbase, (uint32_t)row * rowbytes + 16u * c, sb + T::LR_R_BYTES + kWaves * 1024 * i);
      }
    } else {
      const uint8_t* cbase = xbase + ((p.s_begin + 64 * lt) >> 1);
      int row = tl >> 1;
      int c = (tl & 1) ^ ((row >> 3) & 1);
      c = (64 * lt + 32 * c < p.r) ? c : 0;
      row = row < mrows ? row : mrows - 1;
      dma16(cbase, (uint32_t)row * rowbytes + 16u * c, sb + T::LR_R_BYTES);
    }
  };
  auto issue = [&](int t, int st) {                  // whole tile t of the sequence
    if (t < KTF) {
#pragma unroll
      for (int k = 0; k < T::NL; ++k) issue_main_one(t, st, k);
    } else if (t < KT) {
      issue_main_tail(t, st);
    } else {
      issue_lr(t - KT, st);
    }
  };

  // ---- per-lane offsets of the fragment reads -----------------------------------
  const int wfrag_off = (blk0 * CH * 64 + l) * 16;
  const int lr_r_off = (blk0 * 4 * 64 + l) * 16;
  int xrow_off[2], xswz[2], lr_x_off[2], lr_x_swz[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 64 * wm + 32 * j + lm;
    xrow_off[j] = T::W_BYTES + row * 128;
    xswz[j] = (row >> 1) & 7;
    lr_x_off[j] = T::LR_R_BYTES + row * T::LR_XROW;
    lr_x_swz[j] = ABITS == 8 ? ((row >> 2) & 3) : ((row >> 3) & 1);
  }

  auto load_frags = [&](const uint8_t* st, int ch, Frag<ABITS>& f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f.w[i] = *(const u4*)(st + wfrag_off + (i * CH + ch) * 1024);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if constexpr (ABITS == 8) {
        const int c = 4 * ch + 2 * g;
        f.x[2 * j] = *(const u4*)(st + xrow_off[j] + 16 * (c ^ xswz[j]));
        f.x[2 * j + 1] = *(const u4*)(st + xrow_off[j] + 16 * ((c + 1) ^ xswz[j]));
      } else {
        const int c = 2 * ch + g;
        f.x[j] = *(const u4*)(st + xrow_off[j] + 16 * (c ^ xswz[j]));
      }
    }
  };
  auto load_lr_r = [&](const uint8_t* st, int jb4, u4 (&r)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = *(const u4*)(st + lr_r_off + (i * 4 + jb4) * 1024);
  };
  auto load_lr_x = [&](const uint8_t* st, int jb4, u2 (&x)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if constexpr (ABITS == 8) {
        x[j] = *(const u2*)(st + lr_x_off[j] + 16 * (jb4 ^ lr_x_swz[j]) + 8 * g);
      } else {
        x[j].x = *(const uint32_t*)(st + lr_x_off[j] + 16 * ((jb4 >> 1) ^ lr_x_swz[j]) + 8 * (jb4 & 1) + 4 * g);
        x[j].y = 0;
      }
    }
  };

  // Everything from here on is specialised on the number of channel blocks this wave owns, so that
  // the MFMA groups carry no run-time tests.  Both halves of a tile run the same sequence of
  // barriers whatever their block counts.
  auto body = [&](auto nbw_c) {
    constexpr int NBW = decltype(nbw_c)::value;
    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    // the 16 (or fewer) MFMAs of one 64-channel fragment; REFILL: spread the NL direct
    // loads of main tile `rt` into stage `rst` over the 8 groups
    auto mfma_frag = [&](auto refill_c, const Frag<ABITS>& f, int rt, int rst) {
      constexpr bool REFILL = decltype(refill_c)::value;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        v4i xb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          if constexpr (ABITS == 8) xb[j] = as_v4i(f.x[2 * j + t]);
          else xb[j] = t == 0 ? widen(f.x[j].x, f.x[j].y) : widen(f.x[j].z, f.x[j].w);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (i < NBW) {
            const v4i wa = t == 0 ? widen(f.w[i].x, f.w[i].y) : widen(f.w[i].z, f.w[i].w);
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa, xb[j], acc[i][j], 0, 0, 0);
          }
          if constexpr (REFILL) {
            const int gi = t * 4 + i;
#pragma unroll
            for (int k = 0; k < T::NL; ++k)
              if (k * 8 / T::NL == gi) issue_main_one(rt, rst, k);
          }
          fence();
        }
      }
    };

    // ---- prologue: fill the ring ---------------------------------------------------
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (s < TT) issue(s, s);
    if (NS == 3 && TT >= 3) wait_dma_barrier<2 * T::NL>();
    else wait_dma_barrier<0>();

    int t = 0;                                          // tile being computed
    int st = 0;                                         // its stage
    Frag<ABITS> F[2];
    auto stage_ptr = [&](int s) { return (const uint8_t*)lds + s * STAGE; };
    // Tile t has been read completely (its last fragment is in registers): make sure tile
    // t+1 is in LDS and let every wave catch up; after that stage `st` may be refilled.
    auto handoff_wait = [&]() {
      if (t + 1 < TT) {
        if (NS == 3 && t + 2 < TT) wait_dma_barrier<T::NL>();
        else wait_dma_barrier<0>();
      }
    };
    auto advance = [&]() {
      st = st + 1 == NS ? 0 : st + 1;
      ++t;
    };
    auto prefetch_first = [&]() {                       // first fragment of main tile t (already advanced)
      if (t < KT) load_frags(stage_ptr(st), 0, F[0]);
    };

    load_frags(stage_ptr(0), 0, F[0]);

    // steady state: full main tiles whose refill (tile t+NS) is another full main tile
    for (; t + NS < KTF; ) {
#pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        if (ch + 1 < CH) {
          load_frags(stage_ptr(st), ch + 1, F[(ch + 1) & 1]);
          fence();
          mfma_frag(std::false_type{}, F[ch & 1], 0, 0);
        } else {
          handoff_wait();
          const int rt = t + NS, rst = st;
          advance();
          load_frags(stage_ptr(st), 0, F[0]);
          fence();
          mfma_frag(std::true_type{}, F[ch & 1], rt, rst);
        }
      }
    }
    // remaining full main tiles
    for (; t < KTF; ) {
#pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
        if (ch + 1 < CH) {
          load_frags(stage_ptr(st), ch + 1, F[(ch + 1) & 1]);
        } else {
          handoff_wait();
          if (t + NS < TT) issue(t + NS, st);
          advance();
          prefetch_first();
        }
        fence();
        mfma_frag(std::false_type{}, F[ch & 1], 0, 0);
      }
    }
    if (KTAIL) {                                        // last main tile with 1 .. CH-1 fragments
#pragma unroll
      for (int ch = 0; ch < CH - 1; ++ch) {
        if (ch < KTAIL) {
          if (ch + 1 < KTAIL) {
            load_frags(stage_ptr(st), ch + 1, F[(ch + 1) & 1]);
          } else {
            handoff_wait();
            if (t + NS < TT) issue(t + NS, st);
            advance();
            prefetch_first();
          }
          fence();
          mfma_frag(std::false_type{}, F[ch & 1], 0, 0);
        }
      }
    }

    // ---- epilogue ---------------------------------------------------------------
    // register e of lane l in tile (i,j): channel n0 + 32*(blk0+i) + 8*(e/4) + 4*g + e%4,
    //                                     token   m0 + 64*wm + 32*j + lm.
    const int mbase = m0 + 64 * wm + lm;

    if (p.kslices > 1) {
      // register (i, j, q4) of lane l <-> int4 ((w * hm8 + (2*i + j) * 4 + q4) * 64 + l) of the tile's slot
      const size_t slot = (size_t)kWaves * p.hm8 * 64;
      int4* mine = p.part + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * slot + (size_t)w * p.hm8 * 64 + l;
      if (part_out) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < NBW)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4)
                mine[((2 * i + j) * 4 + q4) * 64] = make_int4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2],
                                                             acc[i][j][4 * q4 + 3]);
        return;
      }
      // pass 2: the accumulators are the sum of the slices' tiles (blockIdx.y is 0 here)
      for (int sl = 0; sl < p.kslices; ++sl) {
        const int4* src = mine + (size_t)sl * gridDim.x * slot;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < NBW)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const int4 v = src[((2 * i + j) * 4 + q4) * 64];
                acc[i][j][4 * q4] += v.x; acc[i][j][4 * q4 + 1] += v.y;
                acc[i][j][4 * q4 + 2] += v.z; acc[i][j][4 * q4 + 3] += v.w;
              }
      }
    }

    if (p.acc_out) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int m = mbase + 32 * j;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + 32 * (blk0 + i) + 8 * q4 + 4 * g;
            if (m < p.M && i < NBW && blk0 + i < nbt) {
              int4 o;
              o.x = acc[i][j][4 * q4 + 0] >> T::SH;
              o.y = acc[i][j][4 * q4 + 1] >> T::SH;
              o.z = acc[i][j][4 * q4 + 2] >> T::SH;
              o.w = acc[i][j][4 * q4 + 3] >> T::SH;
              *(int4*)(p.acc_out + (size_t)m * p.ldacc + n) = o;
            }
          }
        }
      return;
    }

    v16f accf[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int cl = 32 * (blk0 + i) + 8 * q4 + 4 * g;          // channel within the tile
        const float4 ws = *(const float4*)(lws + (cl < 256 ? cl : 0));
        const float s4[4] = {ws.x, ws.y, ws.z, ws.w};
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) accf[i][j][4 * q4 + e] = s4[e] * (float)acc[i][j][4 * q4 + e];
      }
      fence();                                       // at most one block's scales in flight: the registers are full here
    }

    // low-rank tiles: the last one may hold fewer than 4 blocks of 16 channels
    using bf_t = std::integral_constant<bool, LRT != SERQ_F16>;
    // 16-bit R: the 8 codes a lane holds for one block of 16 salient channels, as exact 16-bit floats
    auto lr_codes = [&](auto bf_c, const u2 (&x)[2], u4 (&xf)[2]) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        int c[8];
        if constexpr (ABITS == 8) codes_from_a8(x[j].x, x[j].y, c);
        else codes_from_a4(x[j].x, c);
        xf[j] = codes8_to_16bit(c, decltype(bf_c)::value);
      }
    };
    auto mfma_lr = [&](auto bf_c, const u4 (&r)[4], const u4 (&xf)[2]) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < NBW) {
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            if constexpr (decltype(bf_c)::value)
              accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, r[i]),
                                                                   __builtin_bit_cast(v8bf, xf[j]), accf[i][j], 0, 0, 0);
            else
              accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, r[i]),
                                                                  __builtin_bit_cast(v8h, xf[j]), accf[i][j], 0, 0, 0);
          }
        }
      }
    };
    // A tile of a 4-bit compensation matrix: per channel block one weight-like fragment of 64 ranks,
    // multiplied on the int8 units against the tile's token codes into a scratch INT32 tile that is
    // scaled by rscale[n] * 2^-SH and added to the fp32 accumulators.
    auto lr_tile_int = [&](const uint8_t* stp) {
      // the scales are the same for every tile; an opaque offset keeps the compiler from holding all
      // 64 of them in registers across the tiles
      int rs_off = 0;
      asm volatile("" : "+v"(rs_off));
      const float* lrs_t = lrs + rs_off;
      // the two MFMAs of (token block j, channel block i) into a scratch tile
      auto product = [&](int i, const v4i& xb0, const v4i& xb1) {
        const u4 rq = *(const u4*)(stp + (blk0 + i) * 1024 + l * 16);
        v16i tq;
#pragma unroll
        for (int e = 0; e < 16; ++e) tq[e] = 0;
        tq = __builtin_amdgcn_mfma_i32_32x32x32_i8(widen(rq.x, rq.y), xb0, tq, 0, 0, 0);
        tq = __builtin_amdgcn_mfma_i32_32x32x32_i8(widen(rq.z, rq.w), xb1, tq, 0, 0, 0);
        return tq;
      };
      // accf[i][j] += rscale * 2^-SH * scratch tile
      auto add_scaled = [&](auto i_c, auto j_c, const v16i& tq) {
        constexpr int i = decltype(i_c)::value, j = decltype(j_c)::value;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int cl = 32 * (blk0 + i) + 8 * q4 + 4 * g;
          const float4 rs = *(const float4*)(lrs_t + (cl < 256 ? cl : 0));
          const float r4[4] = {rs.x, rs.y, rs.z, rs.w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            accf[i][j][4 * q4 + e] = __builtin_fmaf(r4[e], (float)tq[4 * q4 + e], accf[i][j][4 * q4 + e]);
        }
        // pin the update here: left alone, the compiler sinks it below the hand-off and keeps
        // every scratch tile and all the scales alive until then
        asm volatile("" : "+v"(accf[i][j]));
      };
      v4i xb0[2], xb1[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (ABITS == 8) {
          xb0[j] = *(const v4i*)(stp + lr_x_off[j] + 16 * ((2 * g) ^ lr_x_swz[j]));
          xb1[j] = *(const v4i*)(stp + lr_x_off[j] + 16 * ((2 * g + 1) ^ lr_x_swz[j]));
        } else {
          const u4 xp = *(const u4*)(stp + lr_x_off[j] + 16 * (g ^ lr_x_swz[j]));
          xb0[j] = widen(xp.x, xp.y);
          xb1[j] = widen(xp.z, xp.w);
        }
      }
      // software pipeline over the 2*NBW products: the MFMAs of the next one are issued before the
      // current scratch tile is converted, so the matrix unit works while the VALU scales
      v16i cur = product(0, xb0[0], xb1[0]);
      fence();
      auto stage = [&](auto p_c) {
        constexpr int pidx = decltype(p_c)::value;            // product pidx = (i = pidx / 2, j = pidx % 2)
        if constexpr (pidx < 2 * NBW) {
          v16i nxt = cur;
          if constexpr (pidx + 1 < 2 * NBW) nxt = product((pidx + 1) / 2, xb0[(pidx + 1) % 2], xb1[(pidx + 1) % 2]);
          fence();
          add_scaled(std::integral_constant<int, pidx / 2>{}, std::integral_constant<int, pidx % 2>{}, cur);
          fence();
          cur = nxt;
        }
      };
      stage(std::integral_constant<int, 0>{}); stage(std::integral_constant<int, 1>{});
      stage(std::integral_constant<int, 2>{}); stage(std::integral_constant<int, 3>{});
      stage(std::integral_constant<int, 4>{}); stage(std::integral_constant<int, 5>{});
      stage(std::integral_constant<int, 6>{}); stage(std::integral_constant<int, 7>{});
    };
    // low-rank tiles; during them every refill is another low-rank tile
    fence();
    for (int lt = 0; lt < LT; ++lt) {
      if constexpr (lr_int) {
        lr_tile_int(stage_ptr(st));
        fence();
      } else {
        // per block of 16 channels: R fragments from LDS, 8 MFMAs, and -- while those run -- the
        // conversion of the next block's token codes
        const int njb = (JB - 4 * lt) < 4 ? (JB - 4 * lt) : 4;
        u2 xr[2];
        u4 xf[2];
        load_lr_x(stage_ptr(st), 0, xr);
        lr_codes(bf_t{}, xr, xf);
        for (int jb4 = 0; jb4 < njb; ++jb4) {
          u4 rr[4];
          load_lr_r(stage_ptr(st), jb4, rr);
          const bool more = jb4 + 1 < njb;
          if (more) load_lr_x(stage_ptr(st), jb4 + 1, xr);
          fence();
          mfma_lr(bf_t{}, rr, xf);
          if (more) lr_codes(bf_t{}, xr, xf);
          fence();
        }
      }
      handoff_wait();
      if (t + NS < TT) issue_lr(t + NS - KT, st);
      advance();
    }

    if (p.y_dtype == SERQ_F32) {
      // fp32 rows do not fit the LDS transpose: 16-byte stores straight from the accumulators
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = mbase + 32 * j;
        if (m >= p.M) continue;
        const float sm = p.scale[m];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (i >= NBW || blk0 + i >= nbt) continue;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + 32 * (blk0 + i) + 8 * q4 + 4 * g;
            *(float4*)((float*)p.Y + (size_t)m * p.ldy + n) =
                make_float4(sm * accf[i][j][4 * q4 + 0], sm * accf[i][j][4 * q4 + 1], sm * accf[i][j][4 * q4 + 2],
                            sm * accf[i][j][4 * q4 + 3]);
          }
        }
      }
      return;
    }

    // 16-bit output: y = scale[m] * accf, cast, transpose through LDS (rows of 512 B; the 16-byte
    // piece pc of row r sits at piece pc ^ (r & 31)), then whole-row-segment stores
    __syncthreads();                                    // every wave is done with the ring
    const bool ybf = p.y_dtype == SERQ_BF16;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = 64 * wm + 32 * j + lm;
      const int m = m0 + r;
      const float sm = p.scale[m < p.M ? m : p.M - 1];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i >= NBW) continue;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int pc = 4 * (blk0 + i) + q4;
          const float y0 = sm * accf[i][j][4 * q4 + 0], y1 = sm * accf[i][j][4 * q4 + 1];
          const float y2 = sm * accf[i][j][4 * q4 + 2], y3 = sm * accf[i][j][4 * q4 + 3];
          u2 o;
          if (ybf) o = u2{f32x2_to_bf16x2(y0, y1), f32x2_to_bf16x2(y2, y3)};
          else o = u2{f32x2_to_f16x2(y0, y1), f32x2_to_f16x2(y2, y3)};
          *(u2*)(lds + r * 512 + 16 * (pc ^ (r & 31)) + 8 * g) = o;
        }
      }
    }
    __syncthreads();
    const int npc = 4 * nbt;                            // 16-byte pieces of an output row segment
#pragma unroll 4
    for (int rr = 0; rr < BM / 16; ++rr) {
      const int r = rr * 16 + (tid >> 5);
      const int pc = tid & 31;
      if (r < mrows && pc < npc) {
        const u4 v = *(const u4*)(lds + r * 512 + 16 * (pc ^ (r & 31)));
        *(u4*)((uint16_t*)p.Y + (size_t)(m0 + r) * p.ldy + n0 + 8 * pc) = v;
      }
    }

  };
  switch (nbw) {
    case 4: body(std::integral_constant<int, 4>{}); break;
    case 3: body(std::integral_constant<int, 3>{}); break;
    case 2: body(std::integral_constant<int, 2>{}); break;
    default: body(std::integral_constant<int, 1>{}); break;   // a wave without blocks computes a duplicate it never stores
  }
}

}  // namespace

// bytes of workspace the sliced path needs for this call (0: not sliced); `forced` as LinearArgs::splitk
size_t mfma_split_workspace_bytes(int M, int N, int K, int abits, int forced) {
  if (M <= 0) return 0;
  const SplitPlan pl = plan_split(M, N, K, abits, device_cu_count(), forced);
  if (pl.S <= 1) return 0;
  const size_t tiles = (size_t)((M + BM - 1) / BM) * pl.C;
  return (size_t)pl.S * tiles * kWaves * wave_blocks8(pl.wide) * 64 * sizeof(int4);
}

int launch_mfma(const LinearArgs& a, hipStream_t st) {
  const int ncu = device_cu_count();
  MfmaParams p;
  p.Xq = a.Xq; p.scale = a.scale; p.Wq = a.Wq; p.wscale = a.wscale;
  p.Rp = a.Rp; p.r_dtype = a.r_dtype; p.s_begin = a.s_begin; p.r = a.Rp ? a.r : 0;
  p.rscale = a.rscale;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.acc_out = a.acc_out; p.ldacc = a.ldacc;
  p.tiles_m = (a.M + BM - 1) / BM;
  // K slices need their part of the workspace (it lies behind the decode path's words); without it, none
  const size_t ws_skip = skinny_workspace_bytes(a.N);
  const size_t ws_have = (a.workspace && a.workspace_bytes > ws_skip) ? a.workspace_bytes - ws_skip : 0;
  SplitPlan pl = plan_split(a.M, a.N, a.K, a.abits, ncu, a.coltiles > 0 && a.splitk == 0 ? 1 : a.splitk);
  if (pl.S > 1) {
    const size_t need = (size_t)pl.S * p.tiles_m * pl.C * kWaves * wave_blocks8(pl.wide) * 64 * sizeof(int4);
    if (need > ws_have) {
      if (a.splitk > 1) return SERQ_EWORKSPACE;         // an explicit request cannot be honoured
      pl = plan_split(a.M, a.N, a.K, a.abits, ncu, 1);
    }
  }
  p.tiles_n = pl.C; p.wide = pl.wide; p.nwide = pl.nwide;
  if (a.coltiles > 0) {                               // caller's override of the column tiling
    const int NB = a.N / 32;
    int C = a.coltiles < (NB + 7) / 8 ? (NB + 7) / 8 : (a.coltiles > NB ? NB : a.coltiles);
    p.tiles_n = C;
    p.wide = (NB + C - 1) / C;
    p.nwide = NB - C * (p.wide - 1);
  }
  p.groupm = a.groupm > 0 ? a.groupm : 4;
  p.kslices = pl.S; p.reduce = 0;
  p.hm8 = wave_blocks8(p.wide);
  p.part = pl.S > 1 ? (int4*)((char*)a.workspace + ws_skip) : nullptr;
  const long long tiles = (long long)p.tiles_m * p.tiles_n;
  if (tiles > 0x7fffffffLL) return SERQ_ESHAPE;
  if (pl.S > 1) {
    const size_t need = (size_t)pl.S * tiles * kWaves * p.hm8 * 64 * sizeof(int4);
    if (need > ws_have) return SERQ_EWORKSPACE;         // (a column-tiling override can change the size)
  }
  dim3 block(kThreads);
  const bool has_lr = p.r > 0 && p.acc_out == nullptr;
  const int lrt = !has_lr ? SERQ_BF16 : p.r_dtype;     // without a compensation matrix any instantiation will do
#define SERQ_MFMA_LAUNCH(AB, LRT) hipLaunchKernelGGL((serq_mfma_kernel<AB, LRT>), grid, block, 0, st, p)
  auto launch = [&](dim3 grid) {
    if (a.abits == 8) {
      if (lrt == SERQ_I4) SERQ_MFMA_LAUNCH(8, SERQ_I4);
      else if (lrt == SERQ_F16) SERQ_MFMA_LAUNCH(8, SERQ_F16);
      else SERQ_MFMA_LAUNCH(8, SERQ_BF16);
    } else {
      if (lrt == SERQ_I4) SERQ_MFMA_LAUNCH(4, SERQ_I4);
      else if (lrt == SERQ_F16) SERQ_MFMA_LAUNCH(4, SERQ_F16);
      else SERQ_MFMA_LAUNCH(4, SERQ_BF16);
    }
  };
  if (pl.S > 1) {
    launch(dim3((unsigned)tiles, (unsigned)pl.S));     // pass 1: the slices park their INT32 tiles
    p.reduce = 1;
  }
  launch(dim3((unsigned)tiles));                       // the whole layer, or pass 2
#undef SERQ_MFMA_LAUNCH
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // namespace serq
