// SERQ linear layer for prefill-sized batches: LDS-tiled int8-MFMA GEMM over
// nibble-packed weights with the rank-r compensation and the dequantising
// epilogue fused in, so Y is written once (Eq. 2 + Eq. 7, first line):
//   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k] Wq[n,k] + sum_j Xq[m,S_j] R[j,n] )
//
// Workgroup tile: 256 tokens x 256 output channels, 8 waves (2 along N x 4
// along M), each wave 128 channels x 64 tokens = 4 x 2 MFMA tiles of 32x32
// (128 accumulator registers).  The weights are the MFMA "A" operand (rows =
// output channels) and the tokens the "B" operand (columns), so that each
// lane ends up with runs of 4 consecutive output channels of one token -- a
// contiguous 8-byte piece of a bf16 row of Y.
//
// K is consumed in tiles of 128 (8-bit activations) or 256 (4-bit) channels;
// either way a token row of the tile is 128 bytes.  LDS holds two stages:
//   weights : the 1-KiB fragments of the blob, unchanged (lane-linear, so the
//             16-byte fragment reads of a wave are one contiguous KiB);
//   tokens  : 256 rows x 128 B, the 16-byte piece c of row i stored at piece
//             c ^ ((i >> 1) & 7), which makes both the row-wise stores and the
//             column-wise fragment reads bank-conflict free.
// Nibbles are widened only in registers, to 16*q (two VALU ops per dword); the
// accumulators therefore hold 2^SH times the true sums and the epilogue folds
// 2^-SH into wscale (exact).  After the K loop the integer accumulators are
// converted in place to fp32 (wscale[n] * acc) and the r/16 low-rank steps are
// accumulated on top with 32x32x16 f16/bf16 MFMAs, reading the packed R
// fragments and the salient codes straight from global memory (L2).
#include "serq_device.h"

namespace serq {
namespace {

constexpr int BM = 256;
constexpr int BN = 256;
constexpr int kThreads = 512;

template <int ABITS>
struct Tile {
  static constexpr int BK = ABITS == 8 ? 128 : 256;   // channels per K tile
  static constexpr int CH = BK / 64;                  // weight fragments per 32 channels per K tile
  static constexpr int W_BYTES = (BN / 32) * CH * 1024;
  static constexpr int A_BYTES = BM * 128;
  static constexpr int STAGE = W_BYTES + A_BYTES;
  static constexpr int SH = ABITS == 8 ? 4 : 8;
};

struct MfmaParams {
  const uint8_t* Xq; const float* scale;
  const u4* Wq; const float* wscale;
  const u4* Rp; int r_dtype; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int32_t* acc_out; int64_t ldacc;
  int tiles_m, tiles_n, groupm;
};

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

template <int ABITS>
__global__ __launch_bounds__(kThreads) void serq_mfma_kernel(const MfmaParams p) {
  using T = Tile<ABITS>;
  constexpr int CH = T::CH;
  __shared__ __align__(16) uint8_t lds[2 * T::STAGE];

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int wn = w & 1, wm = w >> 1;
  const int lm = l & 31, g = l >> 5;

  int tile_m, tile_n;
  map_block(blockIdx.x, p.tiles_m, p.tiles_n, p.groupm, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int nb0 = n0 >> 5;
  const int NB = p.N >> 5;
  const int KB = p.K >> 6;
  const int KT = (KB + CH - 1) / CH;
  const size_t rowbytes = (size_t)p.K * ABITS / 8;

  // ---- global -> register -> LDS staging assignments ------------------------
  // tokens: 4 pieces of 16 B per thread; 8 consecutive threads cover one 128-B row
  const int a_c = tid & 7;
  const uint8_t* a_src[4];
  int a_dst[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 3) + 64 * i;
    int gm = m0 + row;
    gm = gm < p.M ? gm : p.M - 1;                        // rows past M are never stored
    a_src[i] = p.Xq + (size_t)gm * rowbytes;
    a_dst[i] = T::W_BYTES + row * 128 + 16 * (a_c ^ ((row >> 1) & 7));
  }
  // weights: CH pieces per thread, a straight copy of 8*CH KiB of blob fragments
  const u4* w_src[CH];
  bool w_ok[CH];
  int w_ch[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int q = tid + kThreads * i;
    const int nbl = q / (64 * CH);
    const int within = q % (64 * CH);
    w_ch[i] = within >> 6;
    w_ok[i] = (nb0 + nbl) < NB;
    const int nbc = w_ok[i] ? nb0 + nbl : NB - 1;
    w_src[i] = p.Wq + ((size_t)nbc * KB) * 64 + within;
  }

  u4 ra[4];
  u4 rw[CH];
  auto gload = [&](int kt) {
    size_t aoff = (size_t)kt * 128 + 16 * a_c;
    if (aoff + 16 > rowbytes) aoff = 0;                  // K tail: stay inside the row (the weights there are zero)
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *(const u4*)(a_src[i] + aoff);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const bool ok = w_ok[i] && (kt * CH + w_ch[i]) < KB;
      rw[i] = u4{0u, 0u, 0u, 0u};
      if (ok) rw[i] = w_src[i][(size_t)kt * CH * 64];
    }
  };
  auto lstore = [&](int buf) {
    uint8_t* base = lds + buf * T::STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u4*)(base + a_dst[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u4*)(base + (tid + kThreads * i) * 16) = rw[i];
  };

  v16i acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

  // fragment read offsets inside a stage
  int xrow_off[2], xswz[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 64 * wm + 32 * j + lm;
    xrow_off[j] = T::W_BYTES + row * 128;
    xswz[j] = (row >> 1) & 7;
  }
  const int wfrag_off = (4 * wn * CH * 64 + l) * 16;

  gload(0);
  lstore(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
    const uint8_t* base = lds + cur * T::STAGE;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      v4i wa[4][2], xb[2][2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const u4 wp = *(const u4*)(base + wfrag_off + (i * CH + ch) * 1024);
        unpack_frag(wp, wa[i][0], wa[i][1]);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (ABITS == 8) {
          const int c = 4 * ch + 2 * g;
          xb[j][0] = as_v4i(*(const u4*)(base + xrow_off[j] + 16 * (c ^ xswz[j])));
          xb[j][1] = as_v4i(*(const u4*)(base + xrow_off[j] + 16 * ((c + 1) ^ xswz[j])));
        } else {
          const int c = 2 * ch + g;
          const u4 xp = *(const u4*)(base + xrow_off[j] + 16 * (c ^ xswz[j]));
          unpack_frag(xp, xb[j][0], xb[j][1]);
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa[i][t], xb[j][t], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) lstore(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue ---------------------------------------------------------------
  // register e of lane l in tile (i,j): channel n0 + 128*wn + 32*i + 8*(e/4) + 4*g + e%4,
  //                                     token   m0 + 64*wm + 32*j + lm.
  const int nbase = n0 + 128 * wn + 4 * g;
  const int mbase = m0 + 64 * wm + lm;

  if (p.acc_out) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = mbase + 32 * j;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int n = nbase + 32 * i + 8 * q4;
          if (m < p.M && n < p.N) {
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
  constexpr float kInv = 1.0f / (float)(1 << T::SH);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int n = nbase + 32 * i + 8 * q4;
      float4 ws = make_float4(0.f, 0.f, 0.f, 0.f);
      if (n < p.N) ws = *(const float4*)(p.wscale + n);
      const float s4[4] = {ws.x * kInv, ws.y * kInv, ws.z * kInv, ws.w * kInv};
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) accf[i][j][4 * q4 + e] = s4[e] * (float)acc[i][j][4 * q4 + e];
    }

  if (p.r > 0) {
    const int JB = p.r >> 4;
    const bool bf = p.r_dtype == SERQ_BF16;
    const u4* rsrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int nb = nb0 + 4 * wn + i;
      nb = nb < NB ? nb : NB - 1;
      rsrc[i] = p.Rp + (size_t)nb * JB * 64 + l;
    }
    const uint8_t* xsrc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int gm = mbase + 32 * j;
      gm = gm < p.M ? gm : p.M - 1;
      xsrc[j] = p.Xq + (size_t)gm * rowbytes + (((size_t)p.s_begin + 8 * g) * ABITS / 8);
    }
    u4 rf[4];
    u2 xc[2];
    auto lr_load = [&](int jb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) rf[i] = rsrc[i][(size_t)jb * 64];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (ABITS == 8) xc[j] = *(const u2*)(xsrc[j] + jb * 16);
        else { xc[j].x = *(const uint32_t*)(xsrc[j] + jb * 8); xc[j].y = 0; }
      }
    };
    lr_load(0);
    for (int jb = 0; jb < JB; ++jb) {
      u4 rcur[4];
      u4 xf[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) rcur[i] = rf[i];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        int c[8];
        if constexpr (ABITS == 8) codes_from_a8(xc[j].x, xc[j].y, c);
        else codes_from_a4(xc[j].x, c);
        xf[j] = codes8_to_16bit(c, bf);
      }
      if (jb + 1 < JB) lr_load(jb + 1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          if (bf)
            accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, rcur[i]),
                                                                 __builtin_bit_cast(v8bf, xf[j]), accf[i][j], 0, 0, 0);
          else
            accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, rcur[i]),
                                                                __builtin_bit_cast(v8h, xf[j]), accf[i][j], 0, 0, 0);
        }
    }
  }

#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = mbase + 32 * j;
    if (m >= p.M) continue;
    const float sm = p.scale[m];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = nbase + 32 * i + 8 * q4;
        if (n >= p.N) continue;
        const float y0 = sm * accf[i][j][4 * q4 + 0], y1 = sm * accf[i][j][4 * q4 + 1];
        const float y2 = sm * accf[i][j][4 * q4 + 2], y3 = sm * accf[i][j][4 * q4 + 3];
        const size_t o = (size_t)m * p.ldy + n;
        if (p.y_dtype == SERQ_BF16) {
          *(u2*)((uint16_t*)p.Y + o) = u2{f32x2_to_bf16x2(y0, y1), f32x2_to_bf16x2(y2, y3)};
        } else if (p.y_dtype == SERQ_F16) {
          *(u2*)((uint16_t*)p.Y + o) = u2{f32x2_to_f16x2(y0, y1), f32x2_to_f16x2(y2, y3)};
        } else {
          *(float4*)((float*)p.Y + o) = make_float4(y0, y1, y2, y3);
        }
      }
  }
}

}  // namespace

int launch_mfma(const LinearArgs& a, hipStream_t st) {
  MfmaParams p;
  p.Xq = a.Xq; p.scale = a.scale; p.Wq = a.Wq; p.wscale = a.wscale;
  p.Rp = a.Rp; p.r_dtype = a.r_dtype; p.s_begin = a.s_begin; p.r = a.Rp ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.acc_out = a.acc_out; p.ldacc = a.ldacc;
  p.tiles_m = (a.M + BM - 1) / BM;
  p.tiles_n = (a.N + BN - 1) / BN;
  p.groupm = a.groupm > 0 ? a.groupm : 4;
  const long long tiles = (long long)p.tiles_m * p.tiles_n;
  if (tiles > 0x7fffffffLL) return SERQ_ESHAPE;
  dim3 grid((unsigned)tiles), block(kThreads);
  if (a.abits == 8) hipLaunchKernelGGL(serq_mfma_kernel<8>, grid, block, 0, st, p);
  else hipLaunchKernelGGL(serq_mfma_kernel<4>, grid, block, 0, st, p);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // namespace serq
