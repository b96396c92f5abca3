// SERQ linear layer with MXFP4 operands (the 4-bit Microscaling format of the paper's W4A4 runs,
// Sec. 4.1; Eq. 7, second line, with Q = MXFP4 for weights, activations and the compensation matrix):
//   Y[m,n] = sum_k X^[m,k] W^[n,k] + sum_{j<r} X^[m,s_begin+j] R^[n,j]
// where every ^ operand stands for E2M1 code * 2^(E-127) with one E per block of 32 along k (or j).
//
// The contraction runs on the block-scaled FP4 MFMA (32x32x64: a lane's 16 bytes are the 32 codes
// of one block, a byte of a lane's scale register is that block's E), so the inner loop has no
// unpacking and no scaling arithmetic at all and the accumulators are fp32 from the start; there are
// no per-token or per-channel scales left for the epilogue.  The compensation product has the same
// form as the main one (codes x codes with block scales), so its tiles are simply appended to the
// tile sequence, reading the salient columns of X once more against R.
//
// Workgroup, output tile, wave layout and column tiling are those of the integer kernel: 8 waves =
// 2 along the output channels x 4 along the tokens, 256 tokens x up to 256 output channels, each
// wave up to 4 x 2 MFMA tiles of 32x32 (128 fp32 accumulator registers); weights are the "A"
// operand.  A tile of the sequence is 256 input channels (4 fragments of 64):
//   weights  8 blocks x 4 fragments x 1 KiB, lane-linear as stored,
//   tokens   256 rows x 128 B, the 16-byte piece c of row i at piece c ^ ((i >> 1) & 7),
//   scales   256 rows x 8 B (tokens), 8 blocks x 64 lanes x 4 B (weights): 4 KiB,
// two stages of 68 KiB, filled by direct global -> LDS loads (source-side swizzle) that are counted
// by hand; the refill of a stage is spread over the MFMAs of the tile's last fragment.  The LDS reads
// of the next fragment's operands are issued among the MFMAs of the current one.
#include <type_traits>

#include "gemm_tile.h"
#include "serq_device.h"

namespace serq {
namespace {

constexpr int BM = 256;
constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int CH = 4;                               // 64-channel fragments per tile
constexpr int W_BYTES = 8 * CH * 1024;
constexpr int X_BYTES = BM * 128;
constexpr int XS_OFF = W_BYTES + X_BYTES;           // token scales of the tile: [256][8]
constexpr int WS_OFF = XS_OFF + BM * 8;             // weight scales of the tile: [8][64][4]
constexpr int STAGE = WS_OFF + 8 * 256;
constexpr int NS = 2;
constexpr int LDS_BYTES = NS * STAGE;
static_assert(BM * 512 <= LDS_BYTES, "the 16-bit output tile fits the ring");
static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");

struct MxParams {
  const uint8_t* Xq; const uint8_t* xsc;
  const u4* Wq; const uint8_t* wsc;
  const u4* Rq; const uint8_t* rsc; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int tiles_m, tiles_n, groupm;
  int wide, nwide;
  // K slicing for layers whose tiles alone leave most compute units idle (two launches of this kernel):
  //   pass 1 (kslices > 1, reduce = 0): grid (tiles, kslices); workgroup (tile, s) multiplies slice s of the main
  //     tiles and parks its fp32 tile in `part`, in register order (every store a full 1-KiB wave row);
  //   pass 2 (reduce = 1): grid (tiles); no main tiles -- the accumulators start as the sum of the parked tiles,
  //     added in slice order (the result depends on the number of slices, not on the run), then the
  //     compensation tiles and the usual epilogue.
  int kslices, reduce;
  float4* part;           // [kslices][tiles][8 waves][hm8][64 lanes]
  int hm8;                // 8 x the largest number of channel blocks a wave owns
};


__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void serq_mx_kernel(const MxParams p) {
  __shared__ __align__(16) uint8_t lds[LDS_BYTES];

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int wn = (w ^ (w >> 2)) & 1;                 // every SIMD gets one wave of each channel half
  const int wm = w >> 1;
  const int lm = l & 31, g = l >> 5;
  int tile_m, tile_n;
  map_block(blockIdx.x, p.tiles_m, p.tiles_n, p.groupm, tile_m, tile_n);
  const int m0 = tile_m * BM;
  const int nbt = tile_n < p.nwide ? p.wide : p.wide - 1;
  const int nb0 = tile_n < p.nwide ? tile_n * p.wide : p.nwide * p.wide + (tile_n - p.nwide) * (p.wide - 1);
  const int n0 = nb0 << 5;
  const int half = (nbt + 1) >> 1;
  const int blk0 = __builtin_amdgcn_readfirstlane(wn ? half : 0);
  const int nbw = __builtin_amdgcn_readfirstlane(wn ? nbt - half : half);
  const int KB = p.K >> 6;                           // weight fragments per channel block
  const int KTg = (KB + CH - 1) / CH;                // main tiles of the layer (the last one may be partial)
  // the main tiles [ta, tb) this workgroup multiplies: all of them, one K slice (pass 1), or none (pass 2)
  const bool part_out = p.kslices > 1 && !p.reduce;
  int ta = 0, tb = KTg;
  if (part_out) {
    const int per = KTg / p.kslices, rem = KTg % p.kslices, sl = blockIdx.y;
    ta = sl * per + (sl < rem ? sl : rem);
    tb = ta + per + (sl < rem ? 1 : 0);
  } else if (p.reduce) {
    tb = 0;
  }
  const int KT = tb - ta;                            // this workgroup's main tiles
  const int KTF = (tb < KB / CH ? tb : KB / CH) - ta;   // the full ones among them (all but, possibly, the layer's last)
  const int FR = part_out ? 0 : (p.r + 63) >> 6;     // fragments of the compensation matrix per channel block
  const int LT = (FR + CH - 1) / CH;
  const int TT = KT + LT;
  const uint32_t rowbytes = (uint32_t)p.K >> 1;
  const int mrows = p.M - m0 < BM ? p.M - m0 : BM;
  const int Mp = (p.M + 1) & ~1;                     // rows of a tile of the token-scale array

  const int wu = __builtin_amdgcn_readfirstlane(w);
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr(lds));
  const uint8_t* xbase = p.Xq + (size_t)m0 * rowbytes;
  const uint8_t* wbase = (const uint8_t*)p.Wq + (size_t)nb0 * KB * 1024;

  const uint8_t* xsbase = p.xsc + (size_t)m0 * 8;
  const uint8_t* wsbase = p.wsc + (size_t)nb0 * KTg * 256;

  // k-th direct load (k < 9; the 9th brings the scales) of tile t of the sequence into
  // stage st.  FULL: a main tile with all four fragments.  Otherwise every fragment / piece past the
  // tile's valid fragments is clamped into the first one (loaded, never used).  All per-lane offsets
  // are rebuilt here from an opaque copy of the thread index instead of being carried in registers
  // through the main loop, where every register is taken; everything else is wave-uniform.
  auto issue_one = [&](auto full_c, int t, int st, int k) {
    constexpr bool FULL = decltype(full_c)::value;
    const uint32_t sb = lds0 + (uint32_t)st * STAGE + (uint32_t)wu * 1024;
    int tl = tid;
    asm volatile("" : "+v"(tl));
    const int ll = tl & 63;
    const bool lr = !FULL && t >= KT;
    const int lt = t - KT;
    const int KBs = lr ? FR : KB;                    // fragments per channel block in the source
    const int tg = ta + t;                           // a main tile's index in the layer
    const int f0 = lr ? CH * lt : CH * tg;           // first fragment of the tile
    const int nf = FULL ? CH : (KBs - f0 < CH ? KBs - f0 : CH);
    if (k < 4) {
      // weights: wave w fetches slots f = 8*k + w of the stage, f = nbl*CH + ch
      const uint8_t* wsrc = lr ? (const uint8_t*)p.Rq + ((size_t)nb0 * FR + f0) * 1024 : wbase + (size_t)f0 * 1024;
      const int f = k * kWaves + wu;
      int nbl = f / CH, ch = f % CH;
      nbl = nbl < nbt ? nbl : nbt - 1;               // blocks past the tile: duplicates, never read
      ch = ch < nf ? ch : 0;
      dma16(wsrc + (size_t)(nbl * KBs + ch) * 1024, (uint32_t)ll * 16u, sb + kWaves * 1024 * k);
    } else if (k < 8) {
      // tokens: LDS piece pc = 512*(k-4) + tid -> row pc/8, slot pc%8 holds global piece slot ^ swizzle(row)
      const uint8_t* xsrc = lr ? xbase + (p.s_begin >> 1) + (size_t)lt * 128 : xbase + (size_t)tg * 128;
      const int pc = (k - 4) * kThreads + tl;
      int row = pc >> 3;
      int c = (pc & 7) ^ ((row >> 1) & 7);
      if (!FULL) c = c < 2 * nf ? c : 0;
      row = row < mrows ? row : mrows - 1;           // rows past M: duplicates, never stored
      dma16(xsrc, (uint32_t)row * rowbytes + 16u * c, sb + W_BYTES + kWaves * 1024 * (k - 4));
    } else {
      // scales, without a branch (control flow inside the main loop lets the compiler sink the MFMAs
      // past it): waves 0,1 (and 4,5 once more) bring the token scales, 16 bytes = two rows; waves
      // 2,3 (and 6,7) the weight scales, 16 bytes = four lanes of one block
      // (both candidates are computed and then selected: a conditional expression over anything
      // costlier would be compiled into a branch)
      const int q = wu & 3;
      const bool tok = q < 2;
      const int tx = lr ? (p.s_begin >> 8) + lt : tg; // 256-channel tile of the token-scale array
      int rp = 64 * q + ll;
      const int rplast = (mrows - 1) >> 1;
      rp = rp < rplast ? rp : rplast;
      const int Ts = lr ? LT : KTg;                  // scale tiles per channel block in the source
      const uint8_t* wsrc_main = wsbase + (size_t)tg * 256;
      const uint8_t* wsrc_lr = p.rsc + ((size_t)nb0 * LT + lt) * 256;
      const uint8_t* wssrc = lr ? wsrc_lr : wsrc_main;
      const uint8_t* xssrc = xsbase + (size_t)tx * Mp * 8;
      const int o = (q - 2) * 1024 + 16 * ll;
      int nbl = o >> 8;
      const int nblast = nbt - 1;
      nbl = nbl < nblast ? nbl : nblast;
      const uint32_t xoff = (uint32_t)rp * 16u;
      const uint32_t woff = (uint32_t)nbl * 256u * (uint32_t)Ts + (uint32_t)(o & 255);
      const uint8_t* src = tok ? xssrc : wssrc;
      const uint32_t off = tok ? xoff : woff;
      dma16(src, off, lds0 + (uint32_t)st * STAGE + XS_OFF + (uint32_t)q * 1024);   // XS_OFF + 2048 = WS_OFF
    }
  };
  auto issue_any = [&](int t, int st) {
#pragma unroll
    for (int k = 0; k < 9; ++k) issue_one(std::false_type{}, t, st, k);
  };
  auto frags_of = [&](int t) {                       // valid fragments of tile t
    const int left = t < KT ? KB - CH * (ta + t) : FR - CH * (t - KT);
    return left < CH ? left : CH;
  };

  // ---- per-lane offsets of the fragment reads -----------------------------------
  // A token row is 128 bytes and the stage size a multiple of 128, so the swizzled piece address of
  // fragment ch, row_base + 16*((2*ch + g) ^ swz), equals (stage + row_base + 16*(g ^ swz)) ^ (32*ch):
  // one register per token block instead of one per block and fragment.
  const int wfrag_off = (blk0 * CH * 64 + l) * 16;
  const int wsc_off = WS_OFF + blk0 * 256 + 4 * l;   // blk0 + 3 <= 7: always inside the 8 blocks of a stage
  int xa[2], xsc_off[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 64 * wm + 32 * j + lm;
    xa[j] = W_BYTES + row * 128 + 16 * (g ^ ((row >> 1) & 7));
    xsc_off[j] = XS_OFF + row * 8;
  }
  const uint32_t xsel = g ? 0x07050301u : 0x06040200u;   // bytes g, 2+g, 4+g, 6+g of a token's 8 scales
  static_assert(STAGE % 128 == 0, "stage offsets keep the low address bits free for the xor");

  // `so`: byte offset of the stage in LDS
  auto load_w = [&](int so, int ch, int i) { return *(const u4*)(lds + so + wfrag_off + (i * CH + ch) * 1024); };
  auto load_x = [&](int so, int ch, u4 (&x)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) x[j] = *(const u4*)(lds + ((so + xa[j]) ^ (32 * ch)));
  };
  // byte c of a scale register: E of the lane's block in fragment c of the tile
  auto load_ws = [&](int so, int i) { return *(const uint32_t*)(lds + so + wsc_off + i * 256); };
  auto load_xs = [&](int so, uint32_t (&xs)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const u2 e = *(const u2*)(lds + so + xsc_off[j]);
      xs[j] = __builtin_amdgcn_perm(e.y, e.x, xsel);
    }
  };

  auto body = [&](auto nbw_c) {
    constexpr int NBW = decltype(nbw_c)::value;
    v16f acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    // register (i, j, q4) of lane l <-> float4 ((w * hm8 + (2*i + j) * 4 + q4) * 64 + l) of the tile's slot
    // (the address is rebuilt where it is used, from an opaque copy of the thread index: nothing of it is
    // carried through the main loop)
    auto my_slot = [&]() {
      int tp = tid;
      asm volatile("" : "+v"(tp));
      const size_t slot = (size_t)kWaves * p.hm8 * 64;
      return p.part + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * slot + (size_t)(tp >> 6) * p.hm8 * 64 + (tp & 63);
    };
    if (p.reduce) {                                     // pass 2: start from the slices' tiles, in slice order
      const float4* mine = my_slot();
      const size_t slot = (size_t)kWaves * p.hm8 * 64;
      for (int sl = 0; sl < p.kslices; ++sl) {
        const float4* src = mine + (size_t)sl * gridDim.x * slot;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (i < NBW)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const float4 v = src[((2 * i + j) * 4 + q4) * 64];
                acc[i][j][4 * q4] += v.x; acc[i][j][4 * q4 + 1] += v.y;
                acc[i][j][4 * q4 + 2] += v.z; acc[i][j][4 * q4 + 3] += v.w;
              }
      }
    }

    // Operand registers.  The token fragments are double-buffered (X[parity]); a weight fragment and
    // a weight scale are replaced in place as soon as the MFMAs that read them have been issued, one
    // channel block at a time, which is early enough for the next fragment and halves their registers.
    u4 W[4], X[2][2];
    uint32_t ws[4], xs[2];

    // The 2*NBW MFMAs of fragment CHI of the current tile, whose token operands are X[PAR].
    // NEXT = 1: fetch fragment CHI+1 of the same stage meanwhile; 2: fragment 0 and the scales of the
    // tile in stage `nst`; 0: nothing.  REFILL: spread the direct loads of full main tile `rt` into
    // stage `rst` over the MFMA groups.
    auto run_frag = [&](auto ch_c, auto par_c, auto next_c, auto refill_c, int nst, int rt, int rst) {
      constexpr int CHI = decltype(ch_c)::value;
      constexpr int PAR = decltype(par_c)::value;
      constexpr int NEXT = decltype(next_c)::value;
      constexpr bool REFILL = decltype(refill_c)::value;
      constexpr int NCH = NEXT == 1 ? CHI + 1 : 0;
      uint32_t xsn[2] = {0u, 0u};
      if constexpr (NEXT != 0) load_x(nst, NCH, X[PAR ^ 1]);
      if constexpr (NEXT == 2) load_xs(nst, xsn);
      fence();
      v8i xb[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) xb[j] = fp4_operand(X[PAR][j]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < NBW) {
          const v8i wa = fp4_operand(W[i]);
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wa, xb[j], acc[i][j], 4, 4, CHI, (int)ws[i],
                                                                        CHI, (int)xs[j]);
          if constexpr (NEXT != 0) W[i] = load_w(nst, NCH, i);
          if constexpr (NEXT == 2) ws[i] = load_ws(nst, i);
        }
        if constexpr (REFILL) {
          issue_one(std::true_type{}, rt, rst, 2 * i);
          issue_one(std::true_type{}, rt, rst, 2 * i + 1);
          if (i == 3) issue_one(std::true_type{}, rt, rst, 8);
        }
        fence();
      }
      if constexpr (NEXT == 2) {
        xs[0] = xsn[0];
        xs[1] = xsn[1];
      }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // ---- prologue: fill the ring ---------------------------------------------------
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (s < TT) issue_any(s, s);
    wait_dma_barrier<0>();

    int t = 0;                                          // tile being computed
    int st = 0;                                         // its stage
    auto stage_ptr = [&](int s) { return s * STAGE; };   // byte offset of stage s
    // Tile t has been read completely (its last fragment is in registers): make sure tile
    // t+1 is in LDS and let every wave catch up; after that stage `st` may be refilled.
    auto handoff_wait = [&]() {
      if (t + 1 < TT) wait_dma_barrier<0>();
    };
    auto advance = [&]() {
      st = st + 1 == NS ? 0 : st + 1;
      ++t;
    };

#pragma unroll
    for (int i = 0; i < 4; ++i) {
      W[i] = load_w(stage_ptr(0), 0, i);
      ws[i] = load_ws(stage_ptr(0), i);
    }
    load_x(stage_ptr(0), 0, X[0]);
    load_xs(stage_ptr(0), xs);

    // steady state: full main tiles whose refill (tile t+NS) is another full main tile
    for (; t + NS < KTF; ) {
      run_frag(I0{}, I0{}, I1{}, std::false_type{}, stage_ptr(st), 0, 0);
      run_frag(I1{}, I1{}, I1{}, std::false_type{}, stage_ptr(st), 0, 0);
      run_frag(I2{}, I0{}, I1{}, std::false_type{}, stage_ptr(st), 0, 0);
      wait_dma_barrier<0>();                            // hand-off, unconditional here: no control flow in this loop
      const int rt = t + NS, rst = st;
      advance();
      run_frag(I3{}, I1{}, I2{}, std::true_type{}, stage_ptr(st), rt, rst);
    }
    // Every other tile (the last main tiles, a partial one, the low-rank tiles): nf = 1..4 valid
    // fragments, refilled by whatever comes NS tiles later.  One code path for every fragment: the
    // current token operands are X[0], and byte 0 of the scale registers is the current fragment's
    // (the registers are reloaded for every fragment and shifted), so the loop can run over a
    // run-time fragment index.
    auto run_frag_any = [&](int nso, int nch) {
      // fetch fragment nch of the stage at nso (after the last fragment of all: anything) meanwhile
      uint32_t xsn[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) X[1][j] = *(const u4*)(lds + ((nso + xa[j]) ^ (32 * nch)));
      load_xs(nso, xsn);
      fence();
      v8i xb[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) xb[j] = fp4_operand(X[0][j]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i < NBW) {
          const v8i wa = fp4_operand(W[i]);
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wa, xb[j], acc[i][j], 4, 4, 0, (int)ws[i], 0,
                                                                        (int)xs[j]);
          W[i] = *(const u4*)(lds + nso + wfrag_off + (i * CH) * 1024 + nch * 1024);
          ws[i] = load_ws(nso, i) >> (8 * nch);
        }
        fence();
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        xs[j] = xsn[j] >> (8 * nch);
        X[0][j] = X[1][j];
      }
      // pin the results here: the MFMAs have no side effects, so left alone the compiler sinks them
      // below the control flow that follows and keeps the operands of several fragments alive
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < NBW) {
          asm volatile("" : "+v"(acc[i][0]));
          asm volatile("" : "+v"(acc[i][1]));
        }
    };
    while (t < TT) {
      const int nf = frags_of(t);
      for (int ch = 0; ch < nf; ++ch) {
        int nch = ch + 1;
        if (nch == nf) {                                // last fragment of the tile: it is in registers already
          handoff_wait();
          if (t + NS < TT) issue_any(t + NS, st);
          advance();
          nch = 0;
        }
        run_frag_any(stage_ptr(st), nch);
      }
    }

    // ---- epilogue ---------------------------------------------------------------
    if (part_out) {                                     // pass 1: park the slice's tile
      float4* mine = my_slot();
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < NBW)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
              mine[((2 * i + j) * 4 + q4) * 64] = make_float4(acc[i][j][4 * q4], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2],
                                                              acc[i][j][4 * q4 + 3]);
      return;
    }
    // register e of lane l in tile (i,j): channel n0 + 32*(blk0+i) + 8*(e/4) + 4*g + e%4,
    //                                     token   m0 + 64*wm + 32*j + lm.
    // (lane indices rebuilt from an opaque copy of the thread index: nothing of them is carried
    // through the main loop)
    int te = tid;
    asm volatile("" : "+v"(te));
    const int lm = te & 31, g = (te >> 5) & 1, wm = te >> 7;
    const int mbase = m0 + 64 * wm + lm;
    if (p.y_dtype == SERQ_F32) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = mbase + 32 * j;
        if (m >= p.M) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (i >= NBW || blk0 + i >= nbt) continue;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + 32 * (blk0 + i) + 8 * q4 + 4 * g;
            *(float4*)((float*)p.Y + (size_t)m * p.ldy + n) =
                make_float4(acc[i][j][4 * q4 + 0], acc[i][j][4 * q4 + 1], acc[i][j][4 * q4 + 2], acc[i][j][4 * q4 + 3]);
          }
        }
      }
      return;
    }
    // 16-bit output: cast, transpose through LDS (rows of 512 B; the 16-byte piece pc of row r sits
    // at piece pc ^ (r & 31)), then whole-row-segment stores
    __syncthreads();                                    // every wave is done with the ring
    const bool ybf = p.y_dtype == SERQ_BF16;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = 64 * wm + 32 * j + lm;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (i >= NBW) continue;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int pc = 4 * (blk0 + i) + q4;
          const float y0 = acc[i][j][4 * q4 + 0], y1 = acc[i][j][4 * q4 + 1];
          const float y2 = acc[i][j][4 * q4 + 2], y3 = acc[i][j][4 * q4 + 3];
          u2 o;
          if (ybf) o = u2{f32x2_to_bf16x2(y0, y1), f32x2_to_bf16x2(y2, y3)};
          else o = u2{f32x2_to_f16x2(y0, y1), f32x2_to_f16x2(y2, y3)};
          *(u2*)(lds + r * 512 + 16 * (pc ^ (r & 31)) + 8 * g) = o;
        }
      }
    }
    __syncthreads();
    const int npc = 4 * nbt;
#pragma unroll 4
    for (int rr = 0; rr < BM / 16; ++rr) {
      const int r = rr * 16 + (te >> 5);
      const int pc = te & 31;
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

// bytes of workspace the sliced path needs for this call (0: not sliced); `forced` as MxLinearArgs::splitk
size_t mx_split_workspace_bytes(int M, int N, int K, int forced) {
  if (M <= 0) return 0;
  const SplitPlan pl = plan_split(M, N, K, 0, device_cu_count(), forced);
  if (pl.S <= 1) return 0;
  const size_t tiles = (size_t)((M + BM - 1) / BM) * pl.C;
  return (size_t)pl.S * tiles * kWaves * wave_blocks8(pl.wide) * 64 * sizeof(float4);
}

int launch_mx_linear(const MxLinearArgs& a, hipStream_t st) {
  const int ncu = device_cu_count();
  MxParams p;
  p.Xq = a.Xq; p.xsc = a.xsc; p.Wq = a.Wq; p.wsc = a.wsc;
  p.Rq = a.Rq; p.rsc = a.rsc; p.s_begin = a.s_begin; p.r = a.Rq ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.tiles_m = (a.M + BM - 1) / BM;
  const int NB = a.N / 32;
  // K slices need their part of the workspace (it lies behind the decode kernel's words); without it, none
  const size_t ws_skip = skinny_mx_workspace_bytes(a.N);
  const size_t ws_have = (a.workspace && a.workspace_bytes > ws_skip) ? a.workspace_bytes - ws_skip : 0;
  SplitPlan pl = plan_split(a.M, a.N, a.K, 0, ncu, a.coltiles > 0 && a.splitk == 0 ? 1 : a.splitk);
  if (pl.S > 1) {
    const size_t need = (size_t)pl.S * p.tiles_m * pl.C * kWaves * wave_blocks8(pl.wide) * 64 * sizeof(float4);
    if (need > ws_have) {
      if (a.splitk > 1) return SERQ_EWORKSPACE;         // an explicit request cannot be honoured
      pl = plan_split(a.M, a.N, a.K, 0, ncu, 1);
    }
  }
  p.tiles_n = pl.C; p.wide = pl.wide; p.nwide = pl.nwide;
  if (a.coltiles > 0) {
    int C = a.coltiles < (NB + 7) / 8 ? (NB + 7) / 8 : (a.coltiles > NB ? NB : a.coltiles);
    p.tiles_n = C;
    p.wide = (NB + C - 1) / C;
    p.nwide = NB - C * (p.wide - 1);
  }
  p.groupm = 4;
  p.kslices = pl.S; p.reduce = 0;
  p.hm8 = wave_blocks8(p.wide);
  p.part = pl.S > 1 ? (float4*)((char*)a.workspace + ws_skip) : nullptr;
  const long long tiles = (long long)p.tiles_m * p.tiles_n;
  if (tiles > 0x7fffffffLL) return SERQ_ESHAPE;
  if (pl.S > 1) {
    const size_t need = (size_t)pl.S * tiles * kWaves * p.hm8 * 64 * sizeof(float4);
    if (need > ws_have) return SERQ_EWORKSPACE;         // (a column-tiling override can change the size)
    hipLaunchKernelGGL(serq_mx_kernel, dim3((unsigned)tiles, (unsigned)pl.S), dim3(kThreads), 0, st, p);   // pass 1
    p.reduce = 1;
  }
  hipLaunchKernelGGL(serq_mx_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, st, p);   // the whole layer, or pass 2
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // namespace serq
