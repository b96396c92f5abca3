// MXFP4 front end: per-token activation quantisation, offline weight / compensation-matrix packing
// and the canonical views for parity checks.
//
// Format (the 4-bit Microscaling format of the paper's W4A4 latency runs, Sec. 4.1 and the appendix on
// the MX format; arithmetic per the OCP Microscaling specification): blocks of 32 consecutive input
// channels share one E8M0 scale 2^(E-127) with E - 127 = max(floor(log2(max|v|)) - 2, -127) (127 for
// an all-zero block); elements are E2M1 codes (sign bit 8, magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6),
// round to nearest with ties to the even mantissa bit, magnitudes above 6 saturating.  Scaling by a
// power of two is exact in fp32, so every code is decided exactly: by comparisons against the
// midpoints (the offline pack) or by the part's conversion instruction (the online quantiser).
//
// Layouts: codes use the INT4 layouts (activations: [M][K/2] bytes, a dword = 8 consecutive
// channels, byte j = channel j in the low and channel 4+j in the high nibble; weights: [N/32][K/64]
// lane-linear fragments).  A lane's 16 bytes are then exactly one operand of the 32x32x64 scaled
// MFMA and its 32 channels exactly one block.  Scales are stored per 256-channel tile of the GEMM:
//   activations  xsc [ceil(K/256)][Mp][8]           byte b = block 8*tile + b of the token; Mp = M rounded
//                                                   up to even (the GEMM fetches rows in pairs)
//   weights      wsc [N/32][ceil(K/256)][64][4]     byte c of lane l = block 2*(4*tile + c) + l/32
//                                                   of channel 32*nb + l%32
// (bytes of blocks past K hold 127).  The compensation matrix is packed like a weight matrix with
// the rank index in the place of the input channel.
#include "serq_device.h"

namespace serq {
namespace {

constexpr int kT = 256;
inline unsigned blocks_for(size_t n) { return (unsigned)((n + kT - 1) / kT); }
inline int ok() { return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP; }

// shared exponent byte of a block whose largest magnitude is amax
__device__ __forceinline__ int mx_exponent(float amax) {
  if (!(amax > 0.0f)) return 127;
  const int ef = (int)((__float_as_uint(amax) >> 23) & 0xffu);      // 0 for subnormals: clipped below anyway
  int se = ef - 127 - 2;
  se = se < -127 ? -127 : se;
  return se + 127;
}
// v * 2^-(E-127): exact unless the result is subnormal, and then it is far below the smallest midpoint
__device__ __forceinline__ float mx_scale_down(float v, int E) {
  return ldexpf(v, 127 - E);
}
// nearest E2M1 code of t (exact comparisons against the midpoints; ties to the even code)
__device__ __forceinline__ uint32_t e2m1_code(float t) {
  const float a = fabsf(t);
  uint32_t idx = (a > 0.25f) + (a >= 0.75f) + (a > 1.25f) + (a >= 1.75f) + (a > 2.5f) + (a >= 3.5f) + (a > 5.0f);
  return (t < 0.0f && idx != 0) ? idx + 8u : idx;
}
__device__ __forceinline__ float e2m1_value(uint32_t code) {
  const uint32_t i = code & 7u;
  // 0, .5, 1, 1.5, 2, 3, 4, 6
  const float v = i < 2 ? 0.5f * (float)i : ldexpf(1.0f + 0.5f * (float)(i & 1u), (int)(i >> 1) - 1);
  return (code & 8u) ? -v : v;
}
// The same eight codes from the part's own conversion instruction (two fp32 values divided by the
// power of two in the scale operand's exponent field, rounded to nearest even on the E2M1 grid and
// saturated, packed into one byte: low nibble first operand, high nibble second), already in the
// interleaved nibble layout.  The instruction keeps the sign of a value that rounds to zero; codes are
// canonical here (zero has sign 0), so the sign bit of every nibble without magnitude bits is cleared.
// Checked against the comparison form above on a million random pairs, every tie, saturation and the
// ends of the exponent range: identical.
__device__ __forceinline__ uint32_t mx_codes8(const float v[8], int E) {
  const float sc = __uint_as_float((uint32_t)E << 23);
  uint32_t d = 0;
  d = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(d, v[0], v[4], sc, 0);
  d = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(d, v[1], v[5], sc, 1);
  d = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(d, v[2], v[6], sc, 2);
  d = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(d, v[3], v[7], sc, 3);
  const uint32_t nz = ((d & 0x77777777u) + 0x77777777u) & 0x88888888u;   // bit 3 of a nibble: its magnitude is not zero
  return d & (0x77777777u | nz);
}
// eight codes (channels k0 .. k0+7) -> one dword in the interleaved nibble layout
__device__ __forceinline__ uint32_t pack8(const uint32_t c[8]) {
  uint32_t d = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) d |= (c[j] | (c[4 + j] << 4)) << (8 * j);
  return d;
}

// ---- activations ----------------------------------------------------------------------------------
// One workgroup per token; a thread owns 8 consecutive channels, four neighbouring threads a block.
// (One 16-byte piece per thread on a two-dimensional grid, with the exponent bytes of a 256-channel
// tile gathered by shuffles into one 8-byte store, measured 10 % slower.)
// GLU: the row is the gated product silu(X) * U formed in fp32 (the input of the down projection,
// quantised where it is made; Sec. 3.2, the decoder-layer flow of Fig. 2(b)).
template <int XDT, bool GLU>
__global__ __launch_bounds__(kT) void mx_quantize_act_kernel(const void* __restrict__ X, const void* __restrict__ U,
                                                             const float* __restrict__ s_inv, int K, int64_t ldx,
                                                             int64_t ldu, int64_t M, uint32_t* __restrict__ Xq,
                                                             uint8_t* __restrict__ xsc) {
  const int64_t m = blockIdx.x;
  constexpr size_t esz = (XDT == SERQ_F32) ? 4 : 2;
  const char* row = (const char*)X + (size_t)m * (size_t)ldx * esz;
  const char* urow = GLU ? (const char*)U + (size_t)m * (size_t)ldu * esz : nullptr;
  const int nchunk = K >> 3;
  const size_t Mp = (size_t)((M + 1) & ~(int64_t)1);
  const int nround = (nchunk + kT - 1) / kT;                          // kT is a multiple of 4: blocks never straddle rounds
  for (int rd = 0; rd < nround; ++rd) {
    const int chunk = rd * kT + threadIdx.x;
    const bool live = chunk < nchunk;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    if (live) {
      load8<XDT>(row, chunk, v);
      if constexpr (GLU) {
        float u[8];
        load8<XDT>(urow, chunk, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = silu_mul(v[i], u[i]);
      }
      if (s_inv) {
        const float4* p = (const float4*)s_inv + 2 * (size_t)chunk;
        const float4 a = p[0], b = p[1];
        v[0] *= a.x; v[1] *= a.y; v[2] *= a.z; v[3] *= a.w; v[4] *= b.x; v[5] *= b.y; v[6] *= b.z; v[7] *= b.w;
      }
    }
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
    const int E = mx_exponent(amax);
    if (live) {
      Xq[(size_t)m * nchunk + chunk] = mx_codes8(v, E);
      if ((chunk & 3) == 0) {
        const int blk = chunk >> 2;
        xsc[((size_t)(blk >> 3) * Mp + (size_t)m) * 8 + (blk & 7)] = (uint8_t)E;
      }
    }
  }
  // scale bytes of the blocks that the last 256-channel tile does not have
  const int nblk = K >> 5;
  const int nblk8 = (nblk + 7) & ~7;
  if ((int)threadIdx.x < nblk8 - nblk) {
    const int blk = nblk + threadIdx.x;
    xsc[((size_t)(blk >> 3) * Mp + (size_t)m) * 8 + (blk & 7)] = 127;
  }
  // the padding row of an odd M
  if (m == M - 1 && (size_t)M < Mp)
    for (int blk = threadIdx.x; blk < nblk8; blk += kT) xsc[((size_t)(blk >> 3) * Mp + (size_t)M) * 8 + (blk & 7)] = 127;
}

// ---- weights and compensation matrix ------------------------------------------------------------------
// folded weight of (output channel n, permuted input channel kp)
__device__ __forceinline__ float folded(const void* W, int w_dtype, const float* s, const int32_t* perm, size_t n,
                                        int K, int kp) {
  const int k = perm[kp];
  float w = ld_any(W, w_dtype, n * (size_t)K + k);
  if (s) w = w * s[k];
  return w;
}
__device__ __forceinline__ void store_block(uint32_t* frag_blob, uint8_t* sc_blob, size_t n, int blk, int KB,
                                            const uint32_t c[32], int E) {
  const int kb = blk >> 1, g = blk & 1;
  const int T = (KB + 3) >> 2;
  const size_t nb = n >> 5;
  const int lane = (int)(n & 31) + 32 * g;
  uint32_t* dst = frag_blob + ((nb * KB + kb) * 64 + lane) * 4;
#pragma unroll
  for (int d = 0; d < 4; ++d) dst[d] = pack8(c + 8 * d);
  sc_blob[((nb * T + (kb >> 2)) * 64 + lane) * 4 + (kb & 3)] = (uint8_t)E;
}

// one thread per (output channel, block of 32 input channels)
__global__ __launch_bounds__(kT) void mx_pack_weights_kernel(const void* __restrict__ W, int w_dtype,
                                                             const float* __restrict__ s,
                                                             const int32_t* __restrict__ perm, int N, int K,
                                                             uint32_t* __restrict__ Wq, uint8_t* __restrict__ wsc) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const int nblk = K >> 5;
  if (idx >= (size_t)N * nblk) return;
  const size_t n = idx / nblk;
  const int blk = (int)(idx % nblk);
  float v[32];
  float amax = 0.0f;
  for (int i = 0; i < 32; ++i) {
    v[i] = folded(W, w_dtype, s, perm, n, K, 32 * blk + i);
    amax = fmaxf(amax, fabsf(v[i]));
  }
  const int E = mx_exponent(amax);
  uint32_t c[32];
  for (int i = 0; i < 32; ++i) c[i] = e2m1_code(mx_scale_down(v[i], E));
  store_block(Wq, wsc, n, blk, K >> 6, c, E);
}

// the compensation matrix: residual of the r leading (salient) channels, itself in MXFP4 along the rank
// index; one thread per (output channel, block of 32 ranks); ranks r .. 64*ceil(r/64)-1 are zero
__global__ __launch_bounds__(kT) void mx_pack_residual_kernel(const void* __restrict__ W, int w_dtype,
                                                              const float* __restrict__ s,
                                                              const int32_t* __restrict__ perm, int N, int K, int r,
                                                              uint32_t* __restrict__ Rq, uint8_t* __restrict__ rsc) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const int FR = (r + 63) >> 6;
  if (idx >= (size_t)N * FR * 2) return;
  const size_t n = idx / (FR * 2);
  const int blk = (int)(idx % (FR * 2));
  float res[32];
  float amax = 0.0f;
  if (32 * blk < r) {
    float v[32];
    float wmax = 0.0f;
    for (int i = 0; i < 32; ++i) {
      v[i] = folded(W, w_dtype, s, perm, n, K, 32 * blk + i);
      wmax = fmaxf(wmax, fabsf(v[i]));
    }
    const int Ew = mx_exponent(wmax);
    for (int i = 0; i < 32; ++i) {
      const float deq = ldexpf(e2m1_value(e2m1_code(mx_scale_down(v[i], Ew))), Ew - 127);
      res[i] = v[i] - deq;                                           // one fp32 subtraction
      amax = fmaxf(amax, fabsf(res[i]));
    }
  } else {
    for (int i = 0; i < 32; ++i) res[i] = 0.0f;
  }
  const int E = mx_exponent(amax);
  uint32_t c[32];
  for (int i = 0; i < 32; ++i) c[i] = e2m1_code(mx_scale_down(res[i], E));
  store_block(Rq, rsc, n, blk, FR, c, E);
}

// scale bytes of fragments that the last 256-channel tile does not have
__global__ __launch_bounds__(kT) void mx_pad_scales_kernel(uint8_t* __restrict__ sc, int N, int KB) {
  const int T = (KB + 3) >> 2;
  const int pad = 4 * T - KB;
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (pad == 0 || idx >= (size_t)(N / 32) * 64 * pad) return;
  const int c = KB % 4 + (int)(idx % pad);
  const size_t rest = idx / pad;
  const int lane = (int)(rest % 64);
  const size_t nb = rest / 64;
  sc[((nb * T + (T - 1)) * 64 + lane) * 4 + c] = 127;
}

// ---- canonical views --------------------------------------------------------------------------------
__global__ __launch_bounds__(kT) void mx_unpack_weights_kernel(const uint32_t* __restrict__ Wq,
                                                               const uint8_t* __restrict__ wsc, int N, int K,
                                                               uint8_t* __restrict__ codes, uint8_t* __restrict__ E) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const int nblk = K >> 5, KB = K >> 6, T = (KB + 3) >> 2;
  if (idx >= (size_t)N * nblk) return;
  const size_t n = idx / nblk;
  const int blk = (int)(idx % nblk);
  const int kb = blk >> 1, g = blk & 1;
  const size_t nb = n >> 5;
  const int lane = (int)(n & 31) + 32 * g;
  const uint32_t* src = Wq + ((nb * KB + kb) * 64 + lane) * 4;
  for (int d = 0; d < 4; ++d) {
    const uint32_t w = src[d];
    for (int j = 0; j < 4; ++j) {
      codes[n * (size_t)K + 32 * blk + 8 * d + j] = (uint8_t)((w >> (8 * j)) & 0xf);
      codes[n * (size_t)K + 32 * blk + 8 * d + 4 + j] = (uint8_t)((w >> (8 * j + 4)) & 0xf);
    }
  }
  E[n * (size_t)nblk + blk] = wsc[((nb * T + (kb >> 2)) * 64 + lane) * 4 + (kb & 3)];
}

__global__ __launch_bounds__(kT) void mx_unpack_act_kernel(const uint32_t* __restrict__ Xq, const uint8_t* __restrict__ xsc,
                                                           int64_t M, int K, uint8_t* __restrict__ codes,
                                                           uint8_t* __restrict__ E) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const int nchunk = K >> 3;
  if (idx >= (size_t)M * nchunk) return;
  const size_t m = idx / nchunk;
  const int chunk = (int)(idx % nchunk);
  const uint32_t w = Xq[idx];
  for (int j = 0; j < 4; ++j) {
    codes[m * (size_t)K + 8 * chunk + j] = (uint8_t)((w >> (8 * j)) & 0xf);
    codes[m * (size_t)K + 8 * chunk + 4 + j] = (uint8_t)((w >> (8 * j + 4)) & 0xf);
  }
  if ((chunk & 3) == 0) {
    const int blk = chunk >> 2;
    const size_t Mp = (size_t)((M + 1) & ~(int64_t)1);
    E[m * (size_t)(K >> 5) + blk] = xsc[((size_t)(blk >> 3) * Mp + m) * 8 + (blk & 7)];
  }
}

}  // namespace

int launch_mx_quantize_act(const void* X, const void* U, int x_dtype, const float* s_inv, int64_t M, int K, int64_t ldx,
                           int64_t ldu, void* Xq, uint8_t* xsc, hipStream_t st) {
  dim3 grid((unsigned)M), block(kT);
#define SERQ_MXQ_LAUNCH(XDT)                                                                                          \
  do {                                                                                                                \
    if (U) hipLaunchKernelGGL((mx_quantize_act_kernel<XDT, true>), grid, block, 0, st, X, U, s_inv, K, ldx, ldu, M,   \
                              (uint32_t*)Xq, xsc);                                                                    \
    else hipLaunchKernelGGL((mx_quantize_act_kernel<XDT, false>), grid, block, 0, st, X, U, s_inv, K, ldx, ldu, M,    \
                            (uint32_t*)Xq, xsc);                                                                      \
  } while (0)
  if (x_dtype == SERQ_F32) SERQ_MXQ_LAUNCH(SERQ_F32);
  else if (x_dtype == SERQ_F16) SERQ_MXQ_LAUNCH(SERQ_F16);
  else SERQ_MXQ_LAUNCH(SERQ_BF16);
#undef SERQ_MXQ_LAUNCH
  return ok();
}

int mx_pack_weights_impl(const void* W, int w_dtype, const float* s, const int32_t* perm, int N, int K, int r,
                         void* Wq, uint8_t* wsc, void* Rq, uint8_t* rsc, hipStream_t st) {
  hipLaunchKernelGGL(mx_pack_weights_kernel, dim3(blocks_for((size_t)N * (K / 32))), dim3(kT), 0, st, W, w_dtype, s,
                     perm, N, K, (uint32_t*)Wq, wsc);
  hipLaunchKernelGGL(mx_pad_scales_kernel, dim3(blocks_for((size_t)(N / 32) * 64 * 3)), dim3(kT), 0, st, wsc, N, K / 64);
  if (r > 0 && Rq && rsc) {
    const int FR = (r + 63) / 64;
    hipLaunchKernelGGL(mx_pack_residual_kernel, dim3(blocks_for((size_t)N * FR * 2)), dim3(kT), 0, st, W, w_dtype, s,
                       perm, N, K, r, (uint32_t*)Rq, rsc);
    hipLaunchKernelGGL(mx_pad_scales_kernel, dim3(blocks_for((size_t)(N / 32) * 64 * 3)), dim3(kT), 0, st, rsc, N, FR);
  }
  return ok();
}

int mx_unpack_weights_impl(const void* Wq, const uint8_t* wsc, int N, int K, uint8_t* codes, uint8_t* E, hipStream_t st) {
  hipLaunchKernelGGL(mx_unpack_weights_kernel, dim3(blocks_for((size_t)N * (K / 32))), dim3(kT), 0, st,
                     (const uint32_t*)Wq, wsc, N, K, codes, E);
  return ok();
}

int mx_unpack_act_impl(const void* Xq, const uint8_t* xsc, int64_t M, int K, uint8_t* codes, uint8_t* E, hipStream_t st) {
  if (M == 0) return SERQ_OK;
  hipLaunchKernelGGL(mx_unpack_act_kernel, dim3(blocks_for((size_t)M * (K / 8))), dim3(kT), 0, st, (const uint32_t*)Xq,
                     xsc, M, K, codes, E);
  return ok();
}

}  // namespace serq
