// Experiment: the exact INT32 sums of the W4A4 layer (Eq. 2; first term of Eq. 7) computed on the
// block-scaled matrix instruction with both operands in FP6 (E2M3) at unit scale, instead of on the int8
// instruction.  Every INT4 code -7..7 is an E2M3 value (0, 1, 2, 3 = 2*1.5, 4, 5 = 4*1.25, 6 = 4*1.5,
// 7 = 4*1.75), every product is exact, and an fp32 sum of integers stays exact below 2^24 (49 * K for
// K <= 131072 is below it up to K = 342 000), so the result is the same integer -- if the instruction's own
// accumulation is exact, which the parity test establishes.  gfx950 has no INT4 matrix instruction; the
// FP6 form of v_mfma_scale_f32_32x32x64_f8f6f4 has a higher peak rate than the int8 one, at 6 instead of 4
// bits per operand element through LDS.
//
// To compare the two routes at equal kernel quality, one plain LDS-tiled kernel (128 tokens x 128 channels
// per workgroup of 4 waves, 2 x 2 MFMA tiles per wave, one stage = 128 input channels, global -> registers
// -> LDS double buffering) is instantiated twice: with the 4-bit operands of the production layout, widened
// in registers and fed to the int8 instruction, and with FP6 operands fed to the scaled instruction as they
// are.  Both store the INT32 sums.
//
// FP6 layouts: weights [N/32][K/64] fragments of 1536 bytes, lane l owning 24 bytes = the 32 codes of
// channel 32*nb + (l & 31) and input channels 64*kb + 32*(l >> 5) + i, code i in bits 6i .. 6i+5;
// activations [M][K * 3 / 4] bytes, the 32 codes of every block of 32 consecutive channels in 24 bytes.
#include "serq_device.h"
#include "../../include/serq_fp6.h"

namespace serq {
namespace {

constexpr int kT = 256;

// E2M3 bit pattern of an integer code -7..7
__device__ __forceinline__ uint32_t e2m3_of(int c) {
  const int a = c < 0 ? -c : c;
  // 0, 1.0, 2.0, 3.0, 4.0, 5.0, 6.0, 7.0 -> exponent/mantissa fields
  const uint32_t mag = a == 0 ? 0u : a == 1 ? 8u : a == 2 ? 16u : a == 3 ? 20u : a == 4 ? 24u : a == 5 ? 26u : a == 6 ? 28u : 30u;
  return mag | (c < 0 ? 32u : 0u);
}

// 32 int8 codes -> 24 bytes (six dwords), code i in bits 6i .. 6i+5
__device__ __forceinline__ void pack32(const int8_t* c, uint32_t out[6]) {
#pragma unroll
  for (int d = 0; d < 6; ++d) out[d] = 0;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const uint32_t v = e2m3_of(c[i]);
    const int bit = 6 * i, d = bit >> 5, sh = bit & 31;
    out[d] |= v << sh;
    if (sh > 26) out[d + 1] |= v >> (32 - sh);
  }
}

// canonical int8 codes [N][K] -> FP6 weight fragments; one thread per (fragment, lane)
__global__ __launch_bounds__(kT) void fp6_pack_weights_kernel(const int8_t* __restrict__ codes, int N, int K,
                                                              uint32_t* __restrict__ blob) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const int KB = K >> 6;
  if (idx >= (size_t)(N >> 5) * KB * 64) return;
  const int lane = idx & 63;
  const size_t frag = idx >> 6;
  const int kb = frag % KB;
  const size_t n = (frag / KB) * 32 + (lane & 31);
  int8_t c[32];
  const int8_t* src = codes + n * (size_t)K + kb * 64 + (lane >> 5) * 32;
#pragma unroll
  for (int i = 0; i < 32; ++i) c[i] = src[i];
  uint32_t o[6];
  pack32(c, o);
#pragma unroll
  for (int d = 0; d < 6; ++d) blob[idx * 6 + d] = o[d];
}

// canonical int8 codes [M][K] -> FP6 rows; one thread per block of 32 channels
__global__ __launch_bounds__(kT) void fp6_pack_act_kernel(const int8_t* __restrict__ codes, size_t blocks,
                                                          uint32_t* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= blocks) return;
  int8_t c[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) c[i] = codes[idx * 32 + i];
  uint32_t o[6];
  pack32(c, o);
#pragma unroll
  for (int d = 0; d < 6; ++d) out[idx * 6 + d] = o[d];
}

struct ProtoParams {
  const uint8_t* X; const uint8_t* W;
  int M, N, K;
  int32_t* acc; int64_t ldacc;
};

// MODE 0: 4-bit operands (production layouts), widened to int8 in registers, int8 MFMA.
// MODE 1: FP6 operands, block-scaled MFMA with both formats E2M3 and both scales 2^0.
template <int MODE>
struct PTile {
  static constexpr int FRAG = MODE == 0 ? 1024 : 1536;         // bytes of a 32-channel x 64-channel weight fragment
  static constexpr int XROW = MODE == 0 ? 64 : 96;             // bytes of a token's 128 codes
  static constexpr int WB = 4 * 2 * FRAG;
  static constexpr int XB = 128 * XROW;
  static constexpr int STAGE = WB + XB;
  static constexpr int NW = WB / 16 / kT;                      // 16-byte pieces per thread: 2 or 3
  static constexpr int NX = XB / 16 / kT;                      //                            2 or 3
  static constexpr int P = XROW / 16;                          // pieces per token row: 4 or 6
  // 4-bit rows of 64 bytes: xor the piece index so that 8 consecutive rows hit 8 different bank groups;
  // FP6 rows of 96 bytes need none (a stride of 24 banks spreads 8 rows over all 64)
  static __device__ __forceinline__ int swz(int row) { return MODE == 0 ? ((row >> 2) & 3) : 0; }
};

template <int MODE>
__global__ __launch_bounds__(kT) __attribute__((amdgpu_waves_per_eu(2, 2))) void proto_gemm_kernel(const ProtoParams p) {
  using T = PTile<MODE>;
  __shared__ __align__(16) uint8_t lds[2 * T::STAGE];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, lm = l & 31, g = l >> 5;
  const int wn = w & 1, wm = w >> 1;
  const int NB = p.N >> 5, KB = p.K >> 6, G = p.K >> 7;
  const int nb0 = blockIdx.x * 4;
  const int nbt = NB - nb0 < 4 ? NB - nb0 : 4;
  const int m0 = blockIdx.y * 128;
  const int mrows = p.M - m0 < 128 ? p.M - m0 : 128;
  const size_t rowbytes = (size_t)p.K * (MODE == 0 ? 4 : 6) / 8;

  const uint8_t* wsrc[T::NW];
  const uint8_t* xsrc[T::NX];
  int wdst[T::NW], xdst[T::NX];
#pragma unroll
  for (int i = 0; i < T::NW; ++i) {
    const int pc = tid + kT * i;                         // 16-byte piece of the stage's weights: [block][2 fragments]
    int b = pc / (2 * T::FRAG / 16);
    const int off = (pc % (2 * T::FRAG / 16)) * 16;      // byte offset inside the block's two consecutive fragments
    b = b < nbt ? b : nbt - 1;                           // blocks past the tile: duplicates, never stored
    wsrc[i] = p.W + ((size_t)(nb0 + b) * KB) * T::FRAG + off;
    wdst[i] = pc * 16;
  }
#pragma unroll
  for (int i = 0; i < T::NX; ++i) {
    const int q = tid + kT * i;
    const int row = q / T::P, c = q % T::P;
    const int rr = row < mrows ? row : mrows - 1;        // rows past M: duplicates, never stored
    xsrc[i] = p.X + (size_t)(m0 + rr) * rowbytes + 16 * c;
    xdst[i] = T::WB + row * T::XROW + 16 * (c ^ T::swz(row));
  }
  u4 wreg[T::NW], xreg[T::NX];
  auto fetch = [&](int gi) {
#pragma unroll
    for (int i = 0; i < T::NW; ++i) wreg[i] = *(const u4*)(wsrc[i] + (size_t)gi * 2 * T::FRAG);
#pragma unroll
    for (int i = 0; i < T::NX; ++i) xreg[i] = *(const u4*)(xsrc[i] + (size_t)gi * T::XROW);
  };
  auto park = [&](int st) {
    uint8_t* s = lds + st * T::STAGE;
#pragma unroll
    for (int i = 0; i < T::NW; ++i) *(u4*)(s + wdst[i]) = wreg[i];
#pragma unroll
    for (int i = 0; i < T::NX; ++i) *(u4*)(s + xdst[i]) = xreg[i];
  };
  int xoff[2], xsw[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 32 * (2 * wm + j) + lm;
    xoff[j] = T::WB + row * T::XROW;
    xsw[j] = T::swz(row);
  }

  v16i acc[2][2];
  v16f accf[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { acc[i][j][e] = 0; accf[i][j][e] = 0.0f; }

  fetch(0);
  park(0);
  __syncthreads();
#pragma unroll 1
  for (int gi = 0; gi < G; ++gi) {
    const bool more = gi + 1 < G;
    if (more) fetch(gi + 1);
    const uint8_t* s = lds + (gi & 1) * T::STAGE;
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      if constexpr (MODE == 0) {
        v4i a0[2], a1[2], b0[2], b1[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) unpack_frag(*(const u4*)(s + ((2 * wn + i) * 2 + f) * 1024 + l * 16), a0[i], a1[i]);
#pragma unroll
        for (int j = 0; j < 2; ++j) unpack_frag(*(const u4*)(s + xoff[j] + 16 * ((2 * f + g) ^ xsw[j])), b0[j], b1[j]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
          }
      } else {
        v8i a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const uint2* q = (const uint2*)(s + ((2 * wn + i) * 2 + f) * 1536 + l * 24);
          const uint2 q0 = q[0], q1 = q[1], q2 = q[2];
          a[i] = v8i{(int)q0.x, (int)q0.y, (int)q1.x, (int)q1.y, (int)q2.x, (int)q2.y, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint2* q = (const uint2*)(s + xoff[j] + 48 * f + 24 * g);
          const uint2 q0 = q[0], q1 = q[1], q2 = q[2];
          b[j] = v8i{(int)q0.x, (int)q0.y, (int)q1.x, (int)q1.y, (int)q2.x, (int)q2.y, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            accf[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], accf[i][j], 2, 2, 0, 127, 0, 127);
      }
    }
    if (more) park((gi + 1) & 1);
    __syncthreads();
  }

  // register e of lane (lm, g) in tile (i, j): channel 32*(block) + 8*(e/4) + 4*g + e%4, token 32*(2*wm+j) + lm
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (2 * wn + i >= nbt) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int m = m0 + 32 * (2 * wm + j) + lm;
      if (m >= p.M) continue;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        int4 o;
        if constexpr (MODE == 0) {
          o = make_int4(acc[i][j][4 * q4] >> 8, acc[i][j][4 * q4 + 1] >> 8, acc[i][j][4 * q4 + 2] >> 8, acc[i][j][4 * q4 + 3] >> 8);
        } else {
          o = make_int4((int)accf[i][j][4 * q4], (int)accf[i][j][4 * q4 + 1], (int)accf[i][j][4 * q4 + 2], (int)accf[i][j][4 * q4 + 3]);
        }
        *(int4*)(p.acc + (size_t)m * p.ldacc + (nb0 + 2 * wn + i) * 32 + 8 * q4 + 4 * g) = o;
      }
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline unsigned blocks_for(size_t n) { return (unsigned)((n + kT - 1) / kT); }

}  // namespace
}  // namespace serq

using namespace serq;

extern "C" {

size_t serq_fp6_weight_bytes(int64_t N, int64_t K) {
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || K < 128 || K > 131072 || (K % 128) != 0) return 0;
  return (size_t)N * (size_t)K * 3 / 4;
}

size_t serq_fp6_act_bytes(int64_t M, int64_t K) {
  if (M < 0 || K < 128 || K > 131072 || (K % 128) != 0) return 0;
  return (size_t)M * (size_t)K * 3 / 4;
}

int serq_fp6_pack_weights(const int8_t* codes, int64_t N, int64_t K, void* W6_out, void* stream) {
  if (!codes || !W6_out) return SERQ_ENULL;
  if (serq_fp6_weight_bytes(N, K) == 0) return SERQ_ESHAPE;
  if (!aligned16(W6_out)) return SERQ_EALIGN;
  hipLaunchKernelGGL(fp6_pack_weights_kernel, dim3(blocks_for((size_t)N * K / 32)), dim3(kT), 0, (hipStream_t)stream, codes,
                     (int)N, (int)K, (uint32_t*)W6_out);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

int serq_fp6_pack_act(const int8_t* codes, int64_t M, int64_t K, void* X6_out, void* stream) {
  if (M < 0 || K < 128 || K > 131072 || (K % 128) != 0) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!codes || !X6_out) return SERQ_ENULL;
  if (!aligned16(X6_out)) return SERQ_EALIGN;
  const size_t blocks = (size_t)M * K / 32;
  hipLaunchKernelGGL(fp6_pack_act_kernel, dim3(blocks_for(blocks)), dim3(kT), 0, (hipStream_t)stream, codes, blocks,
                     (uint32_t*)X6_out);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

int serq_proto_gemm_i32(const void* X, const void* W, int fp6, int64_t M, int64_t N, int64_t K, int32_t* acc_out,
                        int64_t ldacc, void* stream) {
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || K < 128 || K > 131072 || (K % 128) != 0) return SERQ_ESHAPE;
  if (M < 0 || M > (1 << 22) || ldacc < N) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!X || !W || !acc_out) return SERQ_ENULL;
  if (!aligned16(X) || !aligned16(W) || !aligned16(acc_out) || (ldacc % 4) != 0) return SERQ_EALIGN;
  ProtoParams p;
  p.X = (const uint8_t*)X; p.W = (const uint8_t*)W;
  p.M = (int)M; p.N = (int)N; p.K = (int)K;
  p.acc = acc_out; p.ldacc = ldacc;
  dim3 grid((unsigned)((N / 32 + 3) / 4), (unsigned)((M + 127) / 128));
  if (fp6) hipLaunchKernelGGL(proto_gemm_kernel<1>, grid, dim3(kT), 0, (hipStream_t)stream, p);
  else hipLaunchKernelGGL(proto_gemm_kernel<0>, grid, dim3(kT), 0, (hipStream_t)stream, p);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // extern "C"
