// Per-token activation flattening + symmetric quantisation + packing.
//
// Sec. 3.2 Eq. 4 (X~ = X diag(1/s)) followed by Sec. 2.1 Eq. 1 per token:
//   scale[m] = max_k |x~| / qmax,  code = clip(rne(x~ / scale), -qmax, qmax).
// One 256-thread workgroup per token; the row is read from HBM once, in
// 16-byte pieces, and kept in registers between the absmax pass and the
// quantise pass.  (Variants that walk several tokens per workgroup or per wave,
// with the next row prefetched and the flattening factors kept in registers,
// measured slower: thousands of small independent workgroups overlap their
// phases better than any hand-made pipeline here.)  Every code equals what IEEE
// fp32 arithmetic gives for one multiply, one division and one
// round-to-nearest-even (codes8 below avoids most of the divisions without
// changing any result), so the codes do not depend on how the reduction is
// scheduled.
//
// GLU variants: the token row is the gated product silu(gate) * up of two inputs (the input of the
// down projection, quantised where it is made instead of being stored in 16 bits and read back;
// Sec. 3.2, the decoder-layer flow of Fig. 2(b)).  The product is formed in fp32 (hardware exp2 and
// reciprocal, an ulp each) and never rounded to the storage type.
#include "serq_device.h"

namespace serq {
namespace {

constexpr int kThreads = 256;

// v <- silu(v) * u, elementwise
template <int XDT>
__device__ __forceinline__ void glu8(const void* urow, int chunk, float v[8]) {
  float u[8];
  load8<XDT>(urow, chunk, u);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = serq::silu_mul(v[i], u[i]);
}

__device__ __forceinline__ void flatten8(const float* s_inv, int chunk, float v[8]) {
  if (s_inv) {
    const float4* p = (const float4*)s_inv + 2 * (size_t)chunk;
    float4 a = p[0], b = p[1];
    v[0] *= a.x; v[1] *= a.y; v[2] *= a.z; v[3] *= a.w;
    v[4] *= b.x; v[5] *= b.y; v[6] *= b.z; v[7] *= b.w;
  }
}

__device__ __forceinline__ float absmax8(const float v[8], float m) {
#pragma unroll
  for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(v[i]));
  return m;
}

// Codes of 8 flattened values, bit-identical to clip(rne(v / sc)) in IEEE fp32, at the price of
// a multiplication per value.  t = v * rcp(sc) is within 2^-22 |t| of the correctly rounded
// quotient (one ulp from the reciprocal, half an ulp from the product, half an ulp from the
// quotient's own rounding), so the two round to the same integer unless t lies within that distance
// of a half-integer; only then (the ties of synthetic inputs, and about one piece in a hundred
// otherwise) are the divisions carried out.  The margin used is 1.25 * 2^-22 max(|t|, 1) over the piece.
// A token whose scale is tiny (below 1e-30, a wave-uniform test: the reciprocal of a subnormal scale is
// not finite, and neither estimate above holds near the bottom of the exponent range) always takes the
// divisions.
// (The bookkeeping of this check -- four VALU operations per value -- costs about a tenth of the
// kernel's time; the fallback itself is too rare to show.)
// Clamping before rounding equals rounding before clamping for integer bounds, and adding
// 1.5 * 2^23 rounds to nearest-even and leaves the two's-complement code in the low mantissa bits.
template <int ABITS>
__device__ __forceinline__ void codes8(const float v[8], float sc, float rsc, uint32_t u[8]) {
  constexpr float q = (float)((1 << (ABITS - 1)) - 1);
  constexpr float kMagic = 12582912.0f;
  float maxd = 0.0f, maxt = 1.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float tc = __builtin_amdgcn_fmed3f(v[i] * rsc, -q, q);
    const float uf = tc + kMagic;
    u[i] = __float_as_uint(uf);
    maxd = fmaxf(maxd, fabsf(tc - (uf - kMagic)));
    maxt = fmaxf(maxt, fabsf(tc));
  }
  if (sc < 1e-30f || 0.5f - maxd < 2.98023223876953125e-07f * maxt) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float t = rintf(v[i] / sc);          // IEEE division, then round-half-to-even
      t = fminf(fmaxf(t, -q), q);
      u[i] = __float_as_uint(t + kMagic);
    }
  }
}

template <int ABITS>
__device__ __forceinline__ void quant_store8(const float v[8], float sc, void* xq_row, int chunk) {
  const float rsc = __builtin_amdgcn_rcpf(sc);
  uint32_t u[8];
  codes8<ABITS>(v, sc, rsc, u);
  if constexpr (ABITS == 8) {
    // low bytes of u[0..3] and u[4..7]
    const uint32_t d0 = __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u) | __builtin_amdgcn_perm(u[3], u[2], 0x04000c0cu);
    const uint32_t d1 = __builtin_amdgcn_perm(u[5], u[4], 0x0c0c0400u) | __builtin_amdgcn_perm(u[7], u[6], 0x04000c0cu);
    ((uint2*)xq_row)[chunk] = make_uint2(d0, d1);
  } else {
    // byte j = code j in the low nibble, code 4+j in the high nibble
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = (u[4 + j] << 4) | (u[j] & 0xfu);
    ((uint32_t*)xq_row)[chunk] =
        __builtin_amdgcn_perm(w[1], w[0], 0x0c0c0400u) | __builtin_amdgcn_perm(w[3], w[2], 0x04000c0cu);
  }
}

__device__ __forceinline__ float block_max(float m, float* red) {
  m = wave_max(m);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = m;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int i = 1; i < kThreads / 64; ++i) r = fmaxf(r, red[i]);
  return r;
}

// NC = 16-byte pieces (8 channels each) a thread keeps in registers; NC = 0 is
// the any-K variant that reads the row a second time (from L2).
template <int XDT, int ABITS, int NC, bool GLU>
__global__ __launch_bounds__(kThreads) void quantize_act_kernel(
    const void* __restrict__ X, const void* __restrict__ U, const float* __restrict__ s_inv, int K, int64_t ldx,
    int64_t ldu, void* __restrict__ Xq, float* __restrict__ scale) {
  __shared__ float red[kThreads / 64];
  const int64_t m = blockIdx.x;
  const int nchunk = K >> 3;
  constexpr size_t esz = (XDT == SERQ_F32) ? 4 : 2;
  const char* row = (const char*)X + (size_t)m * (size_t)ldx * esz;
  const char* urow = GLU ? (const char*)U + (size_t)m * (size_t)ldu * esz : nullptr;
  char* xq_row = (char*)Xq + (size_t)m * ((size_t)K * ABITS / 8);
  constexpr float q = (float)((1 << (ABITS - 1)) - 1);

  if constexpr (NC > 0) {
    float v[NC][8];
    float amax = 0.0f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int chunk = threadIdx.x + c * kThreads;
      if (chunk < nchunk) {
        load8<XDT>(row, chunk, v[c]);
        if constexpr (GLU) glu8<XDT>(urow, chunk, v[c]);
        flatten8(s_inv, chunk, v[c]);
        amax = absmax8(v[c], amax);
      }
    }
    amax = block_max(amax, red);
    const float sc = amax > 0.0f ? amax / q : 1.0f;
    if (threadIdx.x == 0) scale[m] = sc;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int chunk = threadIdx.x + c * kThreads;
      if (chunk < nchunk) quant_store8<ABITS>(v[c], sc, xq_row, chunk);
    }
  } else {
    float amax = 0.0f;
    for (int chunk = threadIdx.x; chunk < nchunk; chunk += kThreads) {
      float v[8];
      load8<XDT>(row, chunk, v);
      if constexpr (GLU) glu8<XDT>(urow, chunk, v);
      flatten8(s_inv, chunk, v);
      amax = absmax8(v, amax);
    }
    amax = block_max(amax, red);
    const float sc = amax > 0.0f ? amax / q : 1.0f;
    if (threadIdx.x == 0) scale[m] = sc;
    for (int chunk = threadIdx.x; chunk < nchunk; chunk += kThreads) {
      float v[8];
      load8<XDT>(row, chunk, v);
      if constexpr (GLU) glu8<XDT>(urow, chunk, v);
      flatten8(s_inv, chunk, v);
      quant_store8<ABITS>(v, sc, xq_row, chunk);
    }
  }
}

template <int XDT, int ABITS, bool GLU>
int launch_t(const void* X, const void* U, const float* s_inv, int64_t M, int K, int64_t ldx, int64_t ldu, void* Xq,
             float* scale, hipStream_t st) {
  const int nchunk = K >> 3;
  const int per = (nchunk + kThreads - 1) / kThreads;
  dim3 grid((unsigned)M), block(kThreads);
#define SERQ_QA_LAUNCH(NC) \
  hipLaunchKernelGGL((quantize_act_kernel<XDT, ABITS, NC, GLU>), grid, block, 0, st, X, U, s_inv, K, ldx, ldu, Xq, scale)
  if (per <= 1) SERQ_QA_LAUNCH(1);
  else if (per <= 2) SERQ_QA_LAUNCH(2);
  else if (per <= 4) SERQ_QA_LAUNCH(4);
  else if (per <= 8) SERQ_QA_LAUNCH(8);
  else SERQ_QA_LAUNCH(0);
#undef SERQ_QA_LAUNCH
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

template <int XDT>
int launch_b(const void* X, const void* U, const float* s_inv, int64_t M, int K, int64_t ldx, int64_t ldu, int abits,
             void* Xq, float* scale, hipStream_t st) {
  if (U) {
    return abits == 4 ? launch_t<XDT, 4, true>(X, U, s_inv, M, K, ldx, ldu, Xq, scale, st)
                      : launch_t<XDT, 8, true>(X, U, s_inv, M, K, ldx, ldu, Xq, scale, st);
  }
  return abits == 4 ? launch_t<XDT, 4, false>(X, nullptr, s_inv, M, K, ldx, 0, Xq, scale, st)
                    : launch_t<XDT, 8, false>(X, nullptr, s_inv, M, K, ldx, 0, Xq, scale, st);
}

}  // namespace

// U != nullptr: the row is silu(X) * U (same dtype, row stride ldu)
int launch_quantize_act(const void* X, const void* U, int x_dtype, const float* s_inv, int64_t M, int K, int64_t ldx,
                        int64_t ldu, int abits, void* Xq, float* scale, hipStream_t st) {
  // the grid's x dimension carries the token index
  for (int64_t m0 = 0; m0 < M; m0 += (1 << 30)) {
    const int64_t mc = (M - m0) < (1 << 30) ? (M - m0) : (1 << 30);
    const size_t esz = x_dtype == SERQ_F32 ? 4 : 2;
    const void* Xs = (const char*)X + (size_t)m0 * (size_t)ldx * esz;
    const void* Us = U ? (const char*)U + (size_t)m0 * (size_t)ldu * esz : nullptr;
    void* Xqs = (char*)Xq + (size_t)m0 * ((size_t)K * abits / 8);
    int rc;
    if (x_dtype == SERQ_F32) rc = launch_b<SERQ_F32>(Xs, Us, s_inv, mc, K, ldx, ldu, abits, Xqs, scale + m0, st);
    else if (x_dtype == SERQ_F16) rc = launch_b<SERQ_F16>(Xs, Us, s_inv, mc, K, ldx, ldu, abits, Xqs, scale + m0, st);
    else rc = launch_b<SERQ_BF16>(Xs, Us, s_inv, mc, K, ldx, ldu, abits, Xqs, scale + m0, st);
    if (rc != SERQ_OK) return rc;
  }
  return SERQ_OK;
}

}  // namespace serq
