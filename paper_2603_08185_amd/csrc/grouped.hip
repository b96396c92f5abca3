// The layer in the paper's accuracy-table setting (Sec. 4.1, implementation details): weights quantised
// in groups of 128 input channels (round-to-nearest, symmetric INT4, one 16-bit scale per output channel
// and group), activations per token with round-to-nearest ASYMMETRIC integer quantisation:
//
//   x^[m,k] = scale[m] (Xq[m,k] - zero[m]),      w^[n,k] = gscale[n, k/128] Wq[n,k],
//   Y[m,n]  = sum_k x^[m,k] w^[n,k] + sum_{j<r} x^[m,S_j] R[j,n]                      (Eq. 2 + Eq. 7, first line)
//           = scale[m] ( sum_g gscale[n,g] acc_g[m,n] - zero[m] wsum[n] + sum_j (Xq[m,S_j] - zero[m]) R[j,n] ),
//   acc_g[m,n] = sum_{k in group g} Xq[m,k] Wq[n,k]  (exact, INT32),   wsum[n] = sum_k w^[n,k]  (offline).
//
// The integer sums run on the int8 MFMA exactly as in the per-channel path; what changes is that the
// INT32 tile is folded into an fp32 tile after every group of 128 channels (one convert and one fused
// multiply-add per element and group -- the vector unit works about as long as the matrix unit), and the
// zero point becomes a rank-one term of the epilogue.  The rank-r term takes the re-centred codes
// (Xq - zero, at most 255 in magnitude: exact in bf16 and fp16).
//
// This file holds the whole variant: the asymmetric quantiser, the offline preparation, a
// weight-streaming kernel for M <= 32 and an LDS-tiled kernel above, and their C entry points.
// Weight codes use the fragment layout of the per-channel path (serq_unpack_weights reads them back);
// group scales: [N/32][K/128][32 channels] fp16.
#include "gemm_tile.h"
#include "serq_device.h"

namespace serq {
namespace {

constexpr int kGroup = 128;

__device__ __forceinline__ float f16bits_to_f32(uint16_t u) { return (float)__builtin_bit_cast(_Float16, u); }

// ---------------------------------------------------------------------------------------------------
// asymmetric per-token quantiser: lo = min(0, min v), hi = max(0, max v), scale = (hi - lo) / (2^n - 1),
// z = rne(-lo / scale), code = clip(rne(v / scale) + z, 0, 2^n - 1); stored re-centred by 2^(n-1).
// Every decision is IEEE fp32, as in the oracle.  One workgroup per token, the row kept in registers.
// ---------------------------------------------------------------------------------------------------
constexpr int kQT = 256;

__device__ __forceinline__ void block_minmax(float& lo, float& hi, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, off, 64));
    hi = fmaxf(hi, __shfl_xor(hi, off, 64));
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[2 * w] = lo; red[2 * w + 1] = hi; }
  __syncthreads();
  lo = red[0]; hi = red[1];
#pragma unroll
  for (int i = 1; i < kQT / 64; ++i) { lo = fminf(lo, red[2 * i]); hi = fmaxf(hi, red[2 * i + 1]); }
}

// codes of 8 values: rne(v / sc) + z, clamped to [0, top], re-centred.  t = v * rcp(sc) decides unless it
// lies within 1.25 * 2^-22 max(|t|, 1) of a half-integer (then, and for tiny scales, the divisions are done).
template <int ABITS>
__device__ __forceinline__ void asym_codes8(const float v[8], float sc, float rsc, float z, int c[8]) {
  constexpr float top = (float)((1 << ABITS) - 1);
  constexpr float kMagic = 12582912.0f;
  float r[8], maxd = 0.0f, maxt = 1.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float t = v[i] * rsc;
    r[i] = (t + kMagic) - kMagic;                       // round-half-to-even for |t| < 2^22
    maxd = fmaxf(maxd, fabsf(t - r[i]));
    maxt = fmaxf(maxt, fabsf(t));
  }
  if (sc < 1e-30f || !(maxt < 4194304.0f) || 0.5f - maxd < 2.98023223876953125e-07f * maxt) {
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = rintf(v[i] / sc);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) c[i] = (int)fminf(fmaxf(r[i] + z, 0.0f), top) - (1 << (ABITS - 1));
}

template <int ABITS>
__device__ __forceinline__ void store_codes8(const int c[8], void* xq_row, int chunk) {
  if constexpr (ABITS == 8) {
    const uint32_t d0 = (c[0] & 0xff) | ((c[1] & 0xff) << 8) | ((c[2] & 0xff) << 16) | ((uint32_t)(c[3] & 0xff) << 24);
    const uint32_t d1 = (c[4] & 0xff) | ((c[5] & 0xff) << 8) | ((c[6] & 0xff) << 16) | ((uint32_t)(c[7] & 0xff) << 24);
    ((uint2*)xq_row)[chunk] = make_uint2(d0, d1);
  } else {
    uint32_t o = 0;                                     // byte j: code j (low nibble), code 4+j (high nibble)
#pragma unroll
    for (int j = 0; j < 4; ++j) o |= ((uint32_t)(c[j] & 0xf) | ((uint32_t)(c[4 + j] & 0xf) << 4)) << (8 * j);
    ((uint32_t*)xq_row)[chunk] = o;
  }
}

__device__ __forceinline__ void flat8(const float* s_inv, int chunk, float v[8]) {
  if (s_inv) {
    const float4* p = (const float4*)s_inv + 2 * (size_t)chunk;
    const float4 a = p[0], b = p[1];
    v[0] *= a.x; v[1] *= a.y; v[2] *= a.z; v[3] *= a.w;
    v[4] *= b.x; v[5] *= b.y; v[6] *= b.z; v[7] *= b.w;
  }
}

// NC = 16-byte pieces a thread keeps in registers (0: any K, the row is read twice)
template <int XDT, int ABITS, int NC>
__global__ __launch_bounds__(kQT) void quantize_act_asym_kernel(const void* __restrict__ X, const float* __restrict__ s_inv,
                                                                 int K, int64_t ldx, void* __restrict__ Xq,
                                                                 float* __restrict__ scale, int32_t* __restrict__ zero) {
  __shared__ float red[2 * kQT / 64];
  const int64_t m = blockIdx.x;
  const int nchunk = K >> 3;
  constexpr size_t esz = (XDT == SERQ_F32) ? 4 : 2;
  const char* row = (const char*)X + (size_t)m * (size_t)ldx * esz;
  char* xq_row = (char*)Xq + (size_t)m * ((size_t)K * ABITS / 8);
  constexpr float top = (float)((1 << ABITS) - 1);
  float lo = 0.0f, hi = 0.0f;                           // the range always contains 0
  float v[NC > 0 ? NC : 1][8];
  if constexpr (NC > 0) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int chunk = threadIdx.x + c * kQT;
      if (chunk < nchunk) {
        load8<XDT>(row, chunk, v[c]);
        flat8(s_inv, chunk, v[c]);
#pragma unroll
        for (int i = 0; i < 8; ++i) { lo = fminf(lo, v[c][i]); hi = fmaxf(hi, v[c][i]); }
      }
    }
  } else {
    for (int chunk = threadIdx.x; chunk < nchunk; chunk += kQT) {
      load8<XDT>(row, chunk, v[0]);
      flat8(s_inv, chunk, v[0]);
#pragma unroll
      for (int i = 0; i < 8; ++i) { lo = fminf(lo, v[0][i]); hi = fmaxf(hi, v[0][i]); }
    }
  }
  block_minmax(lo, hi, red);
  const float span = hi - lo;
  const float sc = span > 0.0f ? span / top : 1.0f;
  const float z = rintf(-lo / sc);
  if (threadIdx.x == 0) {
    scale[m] = sc;
    zero[m] = (int)z - (1 << (ABITS - 1));
  }
  const float rsc = __builtin_amdgcn_rcpf(sc);
  int c8[8];
  if constexpr (NC > 0) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int chunk = threadIdx.x + c * kQT;
      if (chunk < nchunk) {
        asym_codes8<ABITS>(v[c], sc, rsc, z, c8);
        store_codes8<ABITS>(c8, xq_row, chunk);
      }
    }
  } else {
    for (int chunk = threadIdx.x; chunk < nchunk; chunk += kQT) {
      load8<XDT>(row, chunk, v[0]);
      flat8(s_inv, chunk, v[0]);
      asym_codes8<ABITS>(v[0], sc, rsc, z, c8);
      store_codes8<ABITS>(c8, xq_row, chunk);
    }
  }
}

template <int XDT, int ABITS>
int launch_asym_t(const void* X, const float* s_inv, int64_t M, int K, int64_t ldx, void* Xq, float* scale,
                  int32_t* zero, hipStream_t st) {
  const int per = ((K >> 3) + kQT - 1) / kQT;
  dim3 grid((unsigned)M), block(kQT);
#define SERQ_QAA(NC) hipLaunchKernelGGL((quantize_act_asym_kernel<XDT, ABITS, NC>), grid, block, 0, st, X, s_inv, K, ldx, Xq, scale, zero)
  if (per <= 1) SERQ_QAA(1);
  else if (per <= 2) SERQ_QAA(2);
  else if (per <= 4) SERQ_QAA(4);
  else if (per <= 8) SERQ_QAA(8);
  else SERQ_QAA(0);
#undef SERQ_QAA
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

// ---------------------------------------------------------------------------------------------------
// offline preparation (not timed; written for clarity)
// ---------------------------------------------------------------------------------------------------
constexpr int kT = 256;

__device__ __forceinline__ float folded_w(const void* W, int w_dtype, const float* s, size_t n, int K, int k_orig) {
  float w = ld_any(W, w_dtype, n * (size_t)K + k_orig);
  if (s) w = w * s[k_orig];
  return w;
}
__device__ __forceinline__ int quant7(float w, float gs) {
  float t = rintf(w / gs);
  t = fminf(fmaxf(t, -7.0f), 7.0f);
  return (int)t;
}
__device__ __forceinline__ size_t gscale_index(size_t n, int g, int G) { return ((n >> 5) * G + g) * 32 + (n & 31); }

// one wave per (output channel, group): gscale = fp16(max |w| / 7) kept inside fp16's positive range; 1 for a zero group
__global__ __launch_bounds__(kT) void group_scale_kernel(const void* __restrict__ W, int w_dtype, const float* __restrict__ s,
                                                         const int32_t* __restrict__ perm, int N, int K,
                                                         uint16_t* __restrict__ gsc) {
  const int G = K / kGroup;
  const size_t gw = (size_t)blockIdx.x * (kT / 64) + (threadIdx.x >> 6);
  if (gw >= (size_t)N * G) return;
  const size_t n = gw / G;
  const int g = (int)(gw % G);
  const int l = threadIdx.x & 63;
  float m = fmaxf(fabsf(folded_w(W, w_dtype, s, n, K, perm[g * kGroup + l])),
                  fabsf(folded_w(W, w_dtype, s, n, K, perm[g * kGroup + 64 + l])));
  m = wave_max(m);
  if (l == 0) {
    float f = 1.0f;
    if (m > 0.0f) {
      f = (float)(_Float16)(m / 7.0f);
      f = fminf(fmaxf(f, 5.9604644775390625e-08f), 65504.0f);
    }
    gsc[gscale_index(n, g, G)] = __builtin_bit_cast(uint16_t, (_Float16)f);
  }
}

// one thread per packed dword of the weight blob (the fragment layout of the per-channel path)
__global__ __launch_bounds__(kT) void quant_pack_grouped_kernel(const void* __restrict__ W, int w_dtype,
                                                                const float* __restrict__ s, const int32_t* __restrict__ perm,
                                                                const uint16_t* __restrict__ gsc, int N, int K,
                                                                uint32_t* __restrict__ blob) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)N * K / 8) return;
  const int d = idx & 3;
  const int lane = (idx >> 2) & 63;
  const size_t frag = idx >> 8;
  const int KB = K >> 6;
  const int kb = frag % KB;
  const size_t n = (frag / KB) * 32 + (lane & 31);
  const int k0 = kb * 64 + (lane >> 5) * 32 + d * 8;
  const float gs = f16bits_to_f32(gsc[gscale_index(n, k0 / kGroup, K / kGroup)]);
  uint32_t out = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int lo = quant7(folded_w(W, w_dtype, s, n, K, perm[k0 + j]), gs);
    const int hi = quant7(folded_w(W, w_dtype, s, n, K, perm[k0 + 4 + j]), gs);
    out |= ((uint32_t)(lo & 0xf) | ((uint32_t)(hi & 0xf) << 4)) << (8 * j);
  }
  blob[idx] = out;
}

// wsum[n] = sum_k gscale[n, k/128] * Wq[n,k], accumulated in fp64 (one workgroup per output channel)
__global__ __launch_bounds__(kT) void wsum_kernel(const void* __restrict__ W, int w_dtype, const float* __restrict__ s,
                                                  const int32_t* __restrict__ perm, const uint16_t* __restrict__ gsc,
                                                  int K, float* __restrict__ wsum) {
  __shared__ double red[kT];
  const size_t n = blockIdx.x;
  const int G = K / kGroup;
  double a = 0.0;
  for (int k = threadIdx.x; k < K; k += kT) {
    const float gs = f16bits_to_f32(gsc[gscale_index(n, k / kGroup, G)]);
    a += (double)gs * (double)quant7(folded_w(W, w_dtype, s, n, K, perm[k]), gs);
  }
  red[threadIdx.x] = a;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) wsum[n] = (float)red[0];
}

// R[j,n] = W^[n,j] - gscale[n, j/128] * Wq[n,j] for the r leading channels (canonical and/or packed)
__global__ __launch_bounds__(kT) void residual_grouped_kernel(const void* __restrict__ W, int w_dtype, const float* __restrict__ s,
                                                              const int32_t* __restrict__ perm, const uint16_t* __restrict__ gsc,
                                                              int N, int K, int r, void* __restrict__ R_out, int r_dtype,
                                                              uint16_t* __restrict__ Rp_out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)r * N) return;
  const int j = idx / N;
  const size_t n = idx % N;
  const float gs = f16bits_to_f32(gsc[gscale_index(n, j / kGroup, K / kGroup)]);
  const float w = folded_w(W, w_dtype, s, n, K, perm[j]);
  const float res = __fmaf_rn(-gs, (float)quant7(w, gs), w);
  uint16_t h = 0;
  if (r_dtype == SERQ_BF16) h = f32_to_bf16_rne(res);
  else if (r_dtype == SERQ_F16) h = f32_to_f16_rne(res);
  if (R_out) {
    if (r_dtype == SERQ_F32) ((float*)R_out)[idx] = res;
    else ((uint16_t*)R_out)[idx] = h;
  }
  if (Rp_out) {
    const int JB = r >> 4;
    const int jb = j >> 4, g = (j >> 3) & 1, p = j & 7;
    Rp_out[(((n >> 5) * JB + jb) * 64 + (int)(n & 31) + 32 * g) * 8 + p] = h;
  }
}

__global__ __launch_bounds__(kT) void unpack_gscale_kernel(const uint16_t* __restrict__ gsc, int N, int G, float* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)N * G) return;
  out[idx] = f16bits_to_f32(gsc[gscale_index(idx / G, (int)(idx % G), G)]);
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + kT - 1) / kT); }

// ---------------------------------------------------------------------------------------------------
// the layer
// ---------------------------------------------------------------------------------------------------
struct GParams {
  const uint8_t* Xq; const float* scale; const int32_t* zero;
  const u4* Wq; const uint16_t* gsc; const float* wsum;
  const u4* Rp; int r_dtype; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
};

__device__ __forceinline__ void store_y(const GParams& p, int m, int n, const float y[4]) {
  const size_t o = (size_t)m * p.ldy + n;
  if (p.y_dtype == SERQ_F32) *(float4*)((float*)p.Y + o) = make_float4(y[0], y[1], y[2], y[3]);
  else if (p.y_dtype == SERQ_BF16) *(u2*)((uint16_t*)p.Y + o) = u2{f32x2_to_bf16x2(y[0], y[1]), f32x2_to_bf16x2(y[2], y[3])};
  else *(u2*)((uint16_t*)p.Y + o) = u2{f32x2_to_f16x2(y[0], y[1]), f32x2_to_f16x2(y[2], y[3])};
}

// the 16 group scales a lane needs for one 32-channel block: channels 8i + 4g + 0..3, i = 0..3, as stored
// (fp16: the fold below widens them inside a mixed-precision fused multiply-add)
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
struct GS16 { h4 v[4]; };
// accf += gscale * acc for one 32 x 32 tile (register e: channel 8*(e/4) + 4g + e%4)
__device__ __forceinline__ void fold_tile(const GS16& gs, const v16i& acc, v16f& accf) {
#pragma unroll
  for (int e = 0; e < 16; ++e) accf[e] = __builtin_fmaf((float)gs.v[e >> 2][e & 3], (float)acc[e], accf[e]);
}

// 8 re-centred codes (code - zero) of one lane as exact 16-bit floats; all zero for a lane without a token
// (in two steps, so that a loop can have the loads of several fragments in flight before it converts the first)
template <int ABITS>
__device__ __forceinline__ u2 lr_load(const uint8_t* xrow, int col) {
  if constexpr (ABITS == 8) return *(const u2*)(xrow + col);
  else return u2{*(const uint32_t*)(xrow + (col >> 1)), 0u};
}
template <int ABITS>
__device__ __forceinline__ u4 lr_convert(const u2& x, int zm, bool valid, bool bf) {
  int c[8];
  if constexpr (ABITS == 8) codes_from_a8(x.x, x.y, c);
  else codes_from_a4(x.x, c);
#pragma unroll
  for (int i = 0; i < 8; ++i) c[i] = valid ? c[i] - zm : 0;
  return codes8_to_16bit(c, bf);
}
// The same for a lane that always has a token (or a duplicate of one whose results are never stored: the columns
// of the MFMA are independent), in fewer vector operations: the codes are turned into unsigned bytes by flipping
// their sign bit, converted straight from the packed bytes, and re-centred by one subtraction (zero + the flipped
// bit's worth).  |code - zero| <= 255, so the fp32 values are whole numbers that both 16-bit formats hold exactly.
template <int ABITS>
__device__ __forceinline__ u4 lr_convert_packed(const u2& x, int zm, bool bf) {
  float f[8];
  if constexpr (ABITS == 8) {
    const uint32_t t0 = x.x ^ 0x80808080u, t1 = x.y ^ 0x80808080u;
    const float off = (float)(128 + zm);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f[k] = (float)((t0 >> (8 * k)) & 0xffu) - off;
      f[4 + k] = (float)((t1 >> (8 * k)) & 0xffu) - off;
    }
  } else {
    // byte j of the dword: code j in the low nibble, code 4 + j in the high nibble
    const uint32_t t = x.x ^ 0x88888888u;
    const uint32_t lo = t & 0x0f0f0f0fu, hi = (t >> 4) & 0x0f0f0f0fu;
    const float off = (float)(8 + zm);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f[k] = (float)((lo >> (8 * k)) & 0xffu) - off;
      f[4 + k] = (float)((hi >> (8 * k)) & 0xffu) - off;
    }
  }
  u4 o;
  if (bf) {
    o.x = f32x2_to_bf16x2(f[0], f[1]); o.y = f32x2_to_bf16x2(f[2], f[3]);
    o.z = f32x2_to_bf16x2(f[4], f[5]); o.w = f32x2_to_bf16x2(f[6], f[7]);
  } else {
    o.x = f32x2_to_f16x2(f[0], f[1]); o.y = f32x2_to_f16x2(f[2], f[3]);
    o.z = f32x2_to_f16x2(f[4], f[5]); o.w = f32x2_to_f16x2(f[6], f[7]);
  }
  return o;
}
template <int ABITS>
__device__ __forceinline__ u4 lr_operand(const uint8_t* xrow, int col, int zm, bool valid, bool bf) {
  return lr_convert<ABITS>(lr_load<ABITS>(xrow, col), zm, valid, bf);
}

__device__ __forceinline__ v16f mfma_lr16(const u4& r, const u4& x, v16f acc, bool bf) {
  if (bf) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, r), __builtin_bit_cast(v8bf, x), acc, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, r), __builtin_bit_cast(v8h, x), acc, 0, 0, 0);
}

// ---- M <= 32: one workgroup of 8 waves per block of 32 output channels, weights streamed once ----------
// Wave w takes the groups w, w+8, ... NG at a time (2, or 4 for K >= 8192, where a wave still has two rounds
// of them: measured better from there on, worse below): the 1-KiB weight fragments, the groups' scales and
// the token codes are all requested before the first is used.  The tokens are the MFMA's row operand
// and the weights its column operand, so a lane holds ONE output channel (one group scale per lane) and
// its registers are tokens: register e of lane (c, g) is token 8*(e/4) + 4g + e%4 of channel c.  With M <= 8
// tokens only registers 0..3 carry anything, with M <= 16 registers 0..7, ...: the fold of a group's INT32
// tile into the fp32 tile touches 4*MQ registers (MQ = ceil(M/8)), not 16.  The wave adds its share of the
// rank-r term, and the eight waves are added through LDS in a fixed order (run-to-run identical).
constexpr int kPitch = 33;
constexpr int kSkinnyWaves = 8;
template <int ABITS, int MQ, int NG>
__global__ __launch_bounds__(64 * kSkinnyWaves) void serq_g128_skinny_kernel(const GParams p) {
  constexpr int SH = ABITS == 8 ? 4 : 8;
  constexpr float kInv = 1.0f / (float)(1 << SH);
  constexpr int NE = 4 * MQ;                                // live accumulator registers
  __shared__ float red[kSkinnyWaves][8 * MQ * kPitch];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, m = l & 31, g = l >> 5;
  const int nb = blockIdx.x;
  const int KB = p.K >> 6, G = p.K >> 7;
  const size_t rowbytes = (size_t)p.K * ABITS / 8;
  const bool mv = m < p.M;
  const uint8_t* xrow = p.Xq + (size_t)(mv ? m : 0) * rowbytes;
  const u4* wfr = p.Wq + (size_t)nb * KB * 64 + l;
  const uint16_t* gsl = p.gsc + (size_t)nb * G * 32 + m;    // this lane's channel (lane & 31)
  const int zm = (p.zero && mv) ? p.zero[m] : 0;
  const v16i kZero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  float accf[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) accf[e] = 0.0f;
  // the token operands of fragment fr: two int8x16 pieces (8-bit) or one packed piece (4-bit); zero without a token
  auto load_x = [&](int fr, u4& x0, u4& x1) {
    x0 = u4{0u, 0u, 0u, 0u};
    x1 = x0;
    if (mv) {
      if constexpr (ABITS == 8) {
        const uint8_t* xp = xrow + (size_t)fr * 64 + 32 * g;
        x0 = *(const u4*)xp;
        x1 = *(const u4*)(xp + 16);
      } else {
        x0 = *(const u4*)(xrow + (size_t)fr * 32 + 16 * g);
      }
    }
  };
  auto group_mfma = [&](const u4& wa, const u4& wb, const u4 (&x)[4], _Float16 gs) {
    v16i acc;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      v4i a0, a1, b0, b1;
      unpack_frag(u ? wb : wa, a0, a1);
      if constexpr (ABITS == 8) {
        b0 = as_v4i(x[2 * u]);
        b1 = as_v4i(x[2 * u + 1]);
      } else {
        unpack_frag(x[2 * u], b0, b1);
      }
      // tokens first: rows of the result are tokens, columns (lanes) are channels; the group starts from zero
      if (u == 0) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a0, kZero16, 0, 0, 0);
      else acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(b0, a0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(b1, a1, acc, 0, 0, 0);
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) accf[e] = __builtin_fmaf((float)gs, (float)acc[e], accf[e]);
  };
#pragma unroll 1
  for (int grp = w; grp < G; grp += NG * kSkinnyWaves) {
    u4 wv[NG][2], xv[NG][4];
    _Float16 gsv[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) {
      const int gq = grp + q * kSkinnyWaves;
      const int gb = gq < G ? gq : grp;                   // a wave without a q-th group repeats the first (unused)
      wv[q][0] = __builtin_nontemporal_load(&wfr[(size_t)(2 * gb) * 64]);
      wv[q][1] = __builtin_nontemporal_load(&wfr[(size_t)(2 * gb + 1) * 64]);
      load_x(2 * gb, xv[q][0], xv[q][1]);
      load_x(2 * gb + 1, xv[q][2], xv[q][3]);
      gsv[q] = __builtin_bit_cast(_Float16, gsl[(size_t)gb * 32]);
    }
#pragma unroll
    for (int q = 0; q < NG; ++q)
      if (grp + q * kSkinnyWaves < G) group_mfma(wv[q][0], wv[q][1], xv[q], gsv[q]);   // uniform over the wave
  }
  // rank-r term on the re-centred codes, added to the wave's tile
  const bool has_lr = p.r > 0 && p.Rp != nullptr;
  const bool bf = p.r_dtype == SERQ_BF16;
  if (has_lr) {
    v16f accl;
#pragma unroll
    for (int e = 0; e < 16; ++e) accl[e] = 0.0f;
    const int JB = p.r >> 4;
    const u4* rfr = p.Rp + (size_t)nb * JB * 64 + l;
    for (int jb = w; jb < JB; jb += kSkinnyWaves) {
      const u4 rr = rfr[(size_t)jb * 64];
      const u4 xf = lr_operand<ABITS>(xrow, p.s_begin + 16 * jb + 8 * g, zm, mv, bf);
      accl = mfma_lr16(xf, rr, accl, bf);
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) accf[e] = __builtin_fmaf(accf[e], kInv, accl[e]);   // 2^-SH: exact
  } else {
#pragma unroll
    for (int e = 0; e < NE; ++e) accf[e] *= kInv;
  }
  // combine: register 4i+e of lane (c,g) is token 8i + 4g + e of channel c
#pragma unroll
  for (int e = 0; e < NE; ++e) red[w][(8 * (e >> 2) + 4 * g + (e & 3)) * kPitch + m] = accf[e];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 256 * MQ / (64 * kSkinnyWaves) + (256 * MQ % (64 * kSkinnyWaves) ? 1 : 0); ++q) {
    const int id = tid + q * 64 * kSkinnyWaves;
    const int nl = id & 31, mt = id >> 5;
    if (mt >= p.M) continue;
    float tot = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kSkinnyWaves; ++ww) tot += red[ww][mt * kPitch + nl];
    const int n = nb * 32 + nl;
    const float zf = p.zero ? (float)p.zero[mt] : 0.0f;
    const float y = p.scale[mt] * (tot - zf * p.wsum[n]);
    const size_t o = (size_t)mt * p.ldy + n;
    if (p.y_dtype == SERQ_F32) ((float*)p.Y)[o] = y;
    else if (p.y_dtype == SERQ_BF16) ((uint16_t*)p.Y)[o] = f32_to_bf16_rne(y);
    else ((uint16_t*)p.Y)[o] = f32_to_f16_rne(y);
  }
}

// ---- M > 32: LDS-tiled kernel, 128 tokens x 128 channels per workgroup of 4 waves (2 x 2) ----------------
// One stage = one group of 128 input channels: 4 blocks x 2 weight fragments (8 KiB), 128 token rows
// (16 KiB at 8 bits, 8 KiB at 4 bits; 16-byte pieces xor-swizzled per row so that the operand reads are
// free of bank conflicts) and the group's 128 scales (256 B).  The stages form a ring (3 deep at 8 bits,
// 4 at 4 bits) filled by direct global -> LDS loads (no staging registers) that run two or three groups
// ahead of the arithmetic and are counted by hand with vmcnt; one barrier per group.  Two workgroups
// share a compute unit, so the barrier of one is covered by the other.
// Each wave owns 2 x 2 MFMA tiles: 64 INT32 accumulators, folded into 64 fp32 accumulators after every
// group.  The four MFMAs of a group run tile by tile, and the convert-and-FMA pairs that fold the tile
// finished before are issued between them, so that the vector unit works in the shadow of the matrix
// unit (a group costs as many cycles on the one as on the other).
template <int ABITS>
struct GTile {
  static constexpr int XROW = 128 * ABITS / 8;       // bytes of a token's 128 codes
  static constexpr int P = XROW / 16;                // 16-byte pieces per token row: 8 or 4
  static constexpr int WB = 4 * 2 * 1024;
  static constexpr int XB = 128 * XROW;
  static constexpr int SC_OFF = WB + XB;             // 4 blocks x 32 fp16 scales
  static constexpr int STAGE = SC_OFF + 256;
  static constexpr int NS = ABITS == 8 ? 3 : 4;      // ring depth
  static constexpr int NLX = 128 * P / 256;          // token loads per thread and group: 4 or 2
  static constexpr int NL = 2 + NLX + 1;             // direct loads per wave and group
  static __device__ __forceinline__ int swz(int row) { return ABITS == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
  static_assert(2 * NS * STAGE <= 160 * 1024, "two workgroups per compute unit");
};

template <int ABITS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void serq_g128_tiled_kernel(const GParams p) {
  using T = GTile<ABITS>;
  constexpr int SH = ABITS == 8 ? 4 : 8;
  constexpr float kInv = 1.0f / (float)(1 << SH);
  constexpr int NS = T::NS;
  __shared__ __align__(16) uint8_t lds[NS * T::STAGE];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lm = l & 31, g = l >> 5;
  const int wn = w & 1, wm = w >> 1;
  const int NB = p.N >> 5, KB = p.K >> 6, G = p.K >> 7;
  // workgroup id -> tile: one contiguous range of tiles per XCD, in bands of 8 token tiles, so that the
  // tiles in flight on one XCD share their weight and token panels in its L2
  int tile_m, tile_n;
  map_block(blockIdx.x, (p.M + 127) >> 7, (NB + 3) >> 2, 8, tile_m, tile_n);
  const int nb0 = tile_n * 4;
  const int nbt = NB - nb0 < 4 ? NB - nb0 : 4;
  const int m0 = tile_m * 128;
  const int mrows = p.M - m0 < 128 ? p.M - m0 : 128;
  const size_t rowbytes = (size_t)p.K * ABITS / 8;

  // ---- what this wave sends from global memory into a stage ---------------------------------------
  // A direct load puts the 16 bytes of lane l at (wave-uniform LDS base) + 16 l, so the swizzle of the
  // token pieces is applied on the source side.  Per group and wave: 2 weight fragments, NLX x 64 token
  // pieces, and (4 lanes) the 64 bytes of scales of block w.
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_addr(lds));
  uint32_t wv[2], xv[T::NLX];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pc = tid + 256 * i;                     // [block][fragment][lane]
    int b = pc >> 7;
    b = b < nbt ? b : nbt - 1;                        // blocks past the tile: duplicates, never stored
    wv[i] = (uint32_t)((b * KB + ((pc >> 6) & 1)) * 1024 + (pc & 63) * 16);
  }
#pragma unroll
  for (int i = 0; i < T::NLX; ++i) {
    const int q = tid + 256 * i;                      // LDS piece: row q / P, slot q % P
    const int row = q / T::P;
    const int c = (q % T::P) ^ T::swz(row);           // the global piece that lives in that slot
    const int rr = row < mrows ? row : mrows - 1;     // rows past M: duplicates, never stored
    xv[i] = (uint32_t)((size_t)rr * rowbytes) + 16u * c;
  }
  const uint32_t sv = (uint32_t)((wu < nbt ? wu : nbt - 1) * G * 64 + (l & 3) * 16);
  const uint8_t* wbase = (const uint8_t*)p.Wq + (size_t)nb0 * KB * 1024;
  const uint8_t* xbase = p.Xq + (size_t)m0 * rowbytes;
  const uint8_t* sbase = (const uint8_t*)p.gsc + (size_t)nb0 * G * 64;
  // The sequence of stages: the G groups of the layer, then -- for the rank-r term -- once more the LG groups whose
  // token codes are the salient block (only their token rows are read then; the loads are the same so that every
  // stage counts the same number of them).
  const bool has_lr = p.r > 0 && p.Rp != nullptr;
  const int lg0 = p.s_begin >> 7;
  const int LG = has_lr ? ((p.s_begin + p.r + 127) >> 7) - lg0 : 0;
  const int GT = G + LG;
  auto issue = [&](int q, int st) {
    const int gi = q < G ? q : lg0 + (q - G);
    const uint32_t sb = lds0 + (uint32_t)st * T::STAGE;
#pragma unroll
    for (int i = 0; i < 2; ++i) dma16(wbase + (size_t)gi * 2048, wv[i], sb + 1024 * wu + 4096 * i);
#pragma unroll
    for (int i = 0; i < T::NLX; ++i) dma16(xbase + (size_t)gi * T::XROW, xv[i], sb + T::WB + 1024 * wu + 4096 * i);
    if (l < 4) dma16(sbase + (size_t)gi * 64, sv, sb + T::SC_OFF + 64 * wu);
  };

  // this wave's blocks 2*wn + i and token rows 32*(2*wm + j) + lm
  int xoff[2], xsw[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 32 * (2 * wm + j) + lm;
    xoff[j] = T::WB + row * T::XROW;
    xsw[j] = T::swz(row);
  }
  int bi[2];                                          // block index in the layer, clamped for the loads of the epilogue
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int b = 2 * wn + i;
    bi[i] = nb0 + (b < nbt ? b : nbt - 1);
  }

  v16i acc[2][2];
  v16f accf[2][2];
  const v16i kZero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { acc[i][j][e] = 0; accf[i][j][e] = 0.0f; }
  GS16 gprev;                                         // scales of the tiles whose fold is still owed: block 1 of the group before
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) gprev.v[q4] = h4{0, 0, 0, 0};

  // the four MFMAs of tile (i,j) of a group, each followed by a quarter of the fold of tile `fa` into `ff`
  auto tile = [&](const v4i (&a)[4], const v4i (&b)[4], v16i& t_acc, const GS16& fg, const v16i& fa, v16f& ff) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      // the first product of a group starts from zero (a constant operand, no registers to clear)
      if (t == 0) t_acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t], b[t], kZero16, 0, 0, 0);
      else t_acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t], b[t], t_acc, 0, 0, 0);
#pragma unroll
      for (int e = 4 * t; e < 4 * t + 4; ++e) ff[e] = __builtin_fmaf((float)fg.v[e >> 2][e & 3], (float)fa[e], ff[e]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < GT) issue(s, s);
  int st = 0, sti = NS - 1;
#pragma unroll 1
  for (int gi = 0; gi < G; ++gi) {
    // group gi has landed (this wave's loads: all but those of the NS-2 groups behind it), every wave has
    // got here, so everybody's loads have landed and the stage read last round may be refilled
    const int last = gi + NS - 2 < GT - 1 ? gi + NS - 2 : GT - 1;
    if (last - gi == NS - 2) wait_dma_barrier<(NS - 2) * T::NL>();
    else wait_dma_barrier<0>();
    if (gi + NS - 1 < GT) issue(gi + NS - 1, sti);
    sti = sti + 1 == NS ? 0 : sti + 1;
    const uint8_t* s = lds + st * T::STAGE;
    st = st + 1 == NS ? 0 : st + 1;
    v4i a[2][4], b[2][4];                             // operands of the group's four 32-channel steps
    GS16 gs[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int f = 0; f < 2; ++f)
        unpack_frag(*(const u4*)(s + (((2 * wn + i) * 2 + f) * 64 + l) * 16), a[i][2 * f], a[i][2 * f + 1]);
      const int j = i;
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        if constexpr (ABITS == 8) {
          const int c = 4 * f + 2 * g;
          b[j][2 * f] = *(const v4i*)(s + xoff[j] + 16 * (c ^ xsw[j]));
          b[j][2 * f + 1] = *(const v4i*)(s + xoff[j] + 16 * ((c + 1) ^ xsw[j]));
        } else {
          unpack_frag(*(const u4*)(s + xoff[j] + 16 * ((2 * f + g) ^ xsw[j])), b[j][2 * f], b[j][2 * f + 1]);
        }
      }
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) gs[i].v[q4] = *(const h4*)(s + T::SC_OFF + 64 * (2 * wn + i) + 2 * (8 * q4 + 4 * g));
    }
    // each tile's MFMAs shadow the fold of the tile finished two tiles earlier (its results have long arrived);
    // the two tiles of block 1 are folded during the first half of the next group
    tile(a[0], b[0], acc[0][0], gprev, acc[1][0], accf[1][0]);
    tile(a[0], b[1], acc[0][1], gprev, acc[1][1], accf[1][1]);
    tile(a[1], b[0], acc[1][0], gs[0], acc[0][0], accf[0][0]);
    tile(a[1], b[1], acc[1][1], gs[0], acc[0][1], accf[0][1]);
    gprev = gs[1];
  }
  fold_tile(gprev, acc[1][0], accf[1][0]);
  fold_tile(gprev, acc[1][1], accf[1][1]);

  // ---- epilogue: zero point, rank-r term on the re-centred codes, token scale, one store ----------------
  const bool bf = p.r_dtype == SERQ_BF16;
  int mrow[2], zm[2];
  float sm[2];
  bool rv[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = m0 + 32 * (2 * wm + j) + lm;
    rv[j] = m < p.M;
    mrow[j] = rv[j] ? m : p.M - 1;
    zm[j] = p.zero ? p.zero[mrow[j]] : 0;
    sm[j] = p.scale[mrow[j]];
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float ws[16];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float4 t = *(const float4*)(p.wsum + (size_t)bi[i] * 32 + 8 * q4 + 4 * g);
      ws[4 * q4] = t.x; ws[4 * q4 + 1] = t.y; ws[4 * q4 + 2] = t.z; ws[4 * q4 + 3] = t.w;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) accf[i][j][e] = __builtin_fmaf(accf[i][j][e], kInv, -(float)zm[j] * ws[e]);   // 2^-SH: exact
  }
  if (has_lr) {
    // The token codes of the salient block come back through the ring (they ran ahead of the last main groups,
    // like any stage); the R fragments come straight from L2, four 16-rank fragments requested before the first
    // is used.
    const int JB = p.r >> 4;
    constexpr int NJ = 4;
#pragma unroll 1
    for (int lg = 0; lg < LG; ++lg) {
      const int q = G + lg;
      const int last = q + NS - 2 < GT - 1 ? q + NS - 2 : GT - 1;
      if (last - q == NS - 2) wait_dma_barrier<(NS - 2) * T::NL>();
      else wait_dma_barrier<0>();
      if (q + NS - 1 < GT) issue(q + NS - 1, sti);
      sti = sti + 1 == NS ? 0 : sti + 1;
      const uint8_t* s = lds + st * T::STAGE;
      st = st + 1 == NS ? 0 : st + 1;
      const int c0 = 128 * (lg0 + lg);                    // first channel of this group of token codes
      const int jb_lo = c0 > p.s_begin ? (c0 - p.s_begin) >> 4 : 0;
      const int jb_end = (c0 + 128 - p.s_begin) >> 4;
      const int jb_hi = jb_end < JB ? jb_end : JB;
#pragma unroll 1
      for (int jb0 = jb_lo; jb0 < jb_hi; jb0 += NJ) {
        u4 rr[NJ][2];
#pragma unroll
        for (int q4 = 0; q4 < NJ; ++q4) {
          const int jb = jb0 + q4 < jb_hi ? jb0 + q4 : jb_hi - 1;   // past the end: a duplicate, never used
#pragma unroll
          for (int i = 0; i < 2; ++i) rr[q4][i] = p.Rp[((size_t)bi[i] * JB + jb) * 64 + l];
        }
#pragma unroll
        for (int q4 = 0; q4 < NJ; ++q4) {
          if (jb0 + q4 < jb_hi) {                         // uniform
            const int col = p.s_begin + 16 * (jb0 + q4) + 8 * g - c0;   // this lane's first channel within the group
            u4 xf[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              u2 xr;
              if constexpr (ABITS == 8) {
                xr = *(const u2*)(s + xoff[j] + 16 * ((col >> 4) ^ xsw[j]) + (col & 15));
              } else {
                const int byte = col >> 1;
                xr = u2{*(const uint32_t*)(s + xoff[j] + 16 * ((byte >> 4) ^ xsw[j]) + (byte & 15)), 0u};
              }
              xf[j] = lr_convert_packed<ABITS>(xr, zm[j], bf);   // rows past M: duplicates, never stored
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j) accf[i][j] = mfma_lr16(rr[q4][i], xf[j], accf[i][j], bf);
          }
        }
      }
    }
  }
  if (p.y_dtype != SERQ_F32) {
    // 16-bit output: cast, transpose through LDS (the ring is free now; rows of 256 B, the 16-byte piece pc of
    // row r at piece pc ^ (r & 15)), then stores of whole row segments: 16 lanes write 256 contiguous bytes
    __syncthreads();                                    // every wave is done with the ring
    const bool ybf = p.y_dtype == SERQ_BF16;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int r = 32 * (2 * wm + j) + lm;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int pc = 4 * (2 * wn + i) + q4;
          const float y0 = sm[j] * accf[i][j][4 * q4], y1 = sm[j] * accf[i][j][4 * q4 + 1];
          const float y2 = sm[j] * accf[i][j][4 * q4 + 2], y3 = sm[j] * accf[i][j][4 * q4 + 3];
          u2 o;
          if (ybf) o = u2{f32x2_to_bf16x2(y0, y1), f32x2_to_bf16x2(y2, y3)};
          else o = u2{f32x2_to_f16x2(y0, y1), f32x2_to_f16x2(y2, y3)};
          *(u2*)(lds + r * 256 + 16 * (pc ^ (r & 15)) + 8 * g) = o;
        }
      }
    __syncthreads();
    const int npc = 4 * nbt;                            // 16-byte pieces of a row that belong to the layer
#pragma unroll 2
    for (int rr = 0; rr < 128 / 16; ++rr) {
      const int r = rr * 16 + (tid >> 4);
      const int pc = tid & 15;
      if (r < mrows && pc < npc) {
        const u4 v = *(const u4*)(lds + r * 256 + 16 * (pc ^ (r & 15)));
        *(u4*)((uint16_t*)p.Y + (size_t)(m0 + r) * p.ldy + nb0 * 32 + 8 * pc) = v;
      }
    }
    return;
  }
  // fp32 output: 16-byte stores straight from the accumulators
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (2 * wn + i >= nbt) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (!rv[j]) continue;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float y[4] = {sm[j] * accf[i][j][4 * q4], sm[j] * accf[i][j][4 * q4 + 1], sm[j] * accf[i][j][4 * q4 + 2],
                            sm[j] * accf[i][j][4 * q4 + 3]};
        store_y(p, mrow[j], bi[i] * 32 + 8 * q4 + 4 * g, y);
      }
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool dtype_ok(int dt) { return dt == SERQ_F32 || dt == SERQ_F16 || dt == SERQ_BF16; }
inline int check_nk128(int64_t N, int64_t K) {
  if (K < 128 || K > 131072 || (K % 128) != 0) return SERQ_ESHAPE;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24)) return SERQ_ESHAPE;
  return SERQ_OK;
}
inline int hip_ok() { return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP; }

}  // namespace
}  // namespace serq

using namespace serq;

extern "C" {

size_t serq_g128_scale_bytes(int64_t N, int64_t K) {
  if (check_nk128(N, K) != SERQ_OK) return 0;
  return (size_t)N * (size_t)(K / kGroup) * 2;
}

int serq_quantize_act_asym(const void* X, int x_dtype, const float* s_inv, int64_t M, int64_t K, int64_t ldx, int abits,
                           void* Xq_out, float* scale_out, int32_t* zero_out, void* stream) {
  if (abits != 4 && abits != 8) return SERQ_EDTYPE;
  if (!dtype_ok(x_dtype)) return SERQ_EDTYPE;
  if (M < 0 || M > (1 << 30) || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (ldx < K) return SERQ_ESHAPE;
  if ((ldx % 8) != 0) return SERQ_EALIGN;
  if (M == 0) return SERQ_OK;
  if (!X || !Xq_out || !scale_out || !zero_out) return SERQ_ENULL;
  if (!aligned16(X) || !aligned16(Xq_out) || !aligned16(s_inv) || (reinterpret_cast<uintptr_t>(scale_out) & 3u) ||
      (reinterpret_cast<uintptr_t>(zero_out) & 3u))
    return SERQ_EALIGN;
  hipStream_t st = (hipStream_t)stream;
#define SERQ_QAA_DT(DT)                                                                                              \
  (abits == 4 ? launch_asym_t<DT, 4>(X, s_inv, M, (int)K, ldx, Xq_out, scale_out, zero_out, st)                      \
              : launch_asym_t<DT, 8>(X, s_inv, M, (int)K, ldx, Xq_out, scale_out, zero_out, st))
  if (x_dtype == SERQ_F32) return SERQ_QAA_DT(SERQ_F32);
  if (x_dtype == SERQ_F16) return SERQ_QAA_DT(SERQ_F16);
  return SERQ_QAA_DT(SERQ_BF16);
#undef SERQ_QAA_DT
}

int serq_g128_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int64_t N, int64_t K, int r,
                           void* Wq_out, void* gscale_out, float* wsum_out, int32_t* perm_out, float* s_inv_out,
                           void* R_out, int r_dtype, void* Rp_out, void* stream) {
  if (!W || !Wq_out || !gscale_out || !wsum_out || !perm_out || !s_inv_out) return SERQ_ENULL;
  if (!dtype_ok(w_dtype)) return SERQ_EDTYPE;
  int rc = check_nk128(N, K);
  if (rc != SERQ_OK) return rc;
  if (r < 0 || (r % 16) != 0 || r > K) return SERQ_ESHAPE;
  if (r > 0 && (R_out || Rp_out)) {
    if (!dtype_ok(r_dtype)) return SERQ_EDTYPE;
    if (Rp_out && r_dtype != SERQ_F16 && r_dtype != SERQ_BF16) return SERQ_EDTYPE;
  }
  if (!aligned16(W) || !aligned16(Wq_out) || !aligned16(gscale_out) || !aligned16(wsum_out) || !aligned16(perm_out) ||
      !aligned16(s_inv_out) || !aligned16(R_out) || !aligned16(Rp_out) || !aligned16(s) || !aligned16(perm_in))
    return SERQ_EALIGN;
  hipStream_t st = (hipStream_t)stream;
  rc = prepare_perm_impl(W, w_dtype, s, perm_in, (int)N, (int)K, perm_out, s_inv_out, st);
  if (rc != SERQ_OK) return rc;
  const int G = (int)(K / kGroup);
  uint16_t* gsc = (uint16_t*)gscale_out;
  hipLaunchKernelGGL(group_scale_kernel, dim3(blocks_for((size_t)N * G * 64)), dim3(kT), 0, st, W, w_dtype, s, perm_out,
                     (int)N, (int)K, gsc);
  hipLaunchKernelGGL(quant_pack_grouped_kernel, dim3(blocks_for((size_t)N * K / 8)), dim3(kT), 0, st, W, w_dtype, s,
                     perm_out, gsc, (int)N, (int)K, (uint32_t*)Wq_out);
  hipLaunchKernelGGL(wsum_kernel, dim3((unsigned)N), dim3(kT), 0, st, W, w_dtype, s, perm_out, gsc, (int)K, wsum_out);
  if (r > 0 && (R_out || Rp_out))
    hipLaunchKernelGGL(residual_grouped_kernel, dim3(blocks_for((size_t)r * N)), dim3(kT), 0, st, W, w_dtype, s, perm_out,
                       gsc, (int)N, (int)K, r, R_out, r_dtype, (uint16_t*)Rp_out);
  return hip_ok();
}

int serq_g128_unpack_scales(const void* gscale, int64_t N, int64_t K, float* out, void* stream) {
  if (!gscale || !out) return SERQ_ENULL;
  const int rc = check_nk128(N, K);
  if (rc != SERQ_OK) return rc;
  const int G = (int)(K / kGroup);
  hipLaunchKernelGGL(unpack_gscale_kernel, dim3(blocks_for((size_t)N * G)), dim3(kT), 0, (hipStream_t)stream,
                     (const uint16_t*)gscale, (int)N, G, out);
  return hip_ok();
}

int serq_g128_linear(const void* Xq, const float* scale, const int32_t* zero, int abits,
                     const void* Wq, const void* gscale, const float* wsum,
                     int s_begin, int r, const void* Rp, int r_dtype,
                     int64_t M, int64_t N, int64_t K, void* Y, int y_dtype, int64_t ldy, int flags, void* stream) {
  if (abits != 4 && abits != 8) return SERQ_EDTYPE;
  if (!dtype_ok(y_dtype)) return SERQ_EDTYPE;
  int rc = check_nk128(N, K);
  if (rc != SERQ_OK) return rc;
  if (M < 0 || M > (1 << 22)) return SERQ_ESHAPE;
  if (r < 0 || (r % 16) != 0 || s_begin < 0 || (s_begin % 32) != 0 || (int64_t)s_begin + r > K) return SERQ_ESHAPE;
  if (r > 0 && Rp && r_dtype != SERQ_F16 && r_dtype != SERQ_BF16) return SERQ_EDTYPE;
  if (ldy < N) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!Xq || !scale || !Wq || !gscale || !wsum || !Y) return SERQ_ENULL;
  if ((ldy % 8) != 0 || !aligned16(Y) || !aligned16(Xq) || !aligned16(Wq) || !aligned16(gscale) || !aligned16(wsum) ||
      !aligned16(Rp) || (reinterpret_cast<uintptr_t>(scale) & 3u) || (reinterpret_cast<uintptr_t>(zero) & 3u))
    return SERQ_EALIGN;
  const int path = flags & 0xff;
  if (path != SERQ_PATH_AUTO && path != SERQ_PATH_SKINNY && path != SERQ_PATH_MFMA) return SERQ_EUNSUPPORTED;
  if (path == SERQ_PATH_SKINNY && M > 32) return SERQ_ESHAPE;
  GParams p;
  p.Xq = (const uint8_t*)Xq; p.scale = scale; p.zero = zero;
  p.Wq = (const u4*)Wq; p.gsc = (const uint16_t*)gscale; p.wsum = wsum;
  p.Rp = (r > 0 ? (const u4*)Rp : nullptr); p.r_dtype = r_dtype; p.s_begin = s_begin; p.r = Rp ? r : 0;
  p.M = (int)M; p.N = (int)N; p.K = (int)K;
  p.Y = Y; p.y_dtype = y_dtype; p.ldy = ldy;
  hipStream_t st = (hipStream_t)stream;
  const bool skinny = path == SERQ_PATH_SKINNY || (path == SERQ_PATH_AUTO && M <= 32);
  if (skinny) {
    dim3 grid((unsigned)(N / 32));
    // specialised on ceil(M / 8): the number of accumulator register quads that hold tokens
#define SERQ_G128_SKINNY(AB, MQ)                                                                                   \
  do {                                                                                                             \
    if (deep) hipLaunchKernelGGL((serq_g128_skinny_kernel<AB, MQ, 4>), grid, dim3(64 * kSkinnyWaves), 0, st, p);   \
    else hipLaunchKernelGGL((serq_g128_skinny_kernel<AB, MQ, 2>), grid, dim3(64 * kSkinnyWaves), 0, st, p);        \
  } while (0)
    const int mq = (int)((M + 7) / 8);
    const bool deep = K / kGroup >= 64;                   // four groups in flight per wave pay once a wave has two rounds of them
    if (abits == 8) {
      if (mq == 1) SERQ_G128_SKINNY(8, 1); else if (mq == 2) SERQ_G128_SKINNY(8, 2);
      else if (mq == 3) SERQ_G128_SKINNY(8, 3); else SERQ_G128_SKINNY(8, 4);
    } else {
      if (mq == 1) SERQ_G128_SKINNY(4, 1); else if (mq == 2) SERQ_G128_SKINNY(4, 2);
      else if (mq == 3) SERQ_G128_SKINNY(4, 3); else SERQ_G128_SKINNY(4, 4);
    }
#undef SERQ_G128_SKINNY
  } else {
    const long long tiles = (long long)((N / 32 + 3) / 4) * ((M + 127) / 128);
    if (tiles > 0x7fffffffLL) return SERQ_ESHAPE;
    dim3 grid((unsigned)tiles);
    if (abits == 8) hipLaunchKernelGGL(serq_g128_tiled_kernel<8>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(serq_g128_tiled_kernel<4>, grid, dim3(256), 0, st, p);
  }
  return hip_ok();
}

}  // extern "C"
