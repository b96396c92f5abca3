// Offline weight preparation and the canonical <-> packed layout converters.
//
// Sec. 3.2: fold the flattening vector into the weights (Eq. 4), order the
// input channels by saliency (text before Eq. 5), quantise every output
// channel to symmetric INT4 (Sec. 2.1 Eq. 1), extract the residual of the r
// leading channels as the single compensation matrix R (Eq. 5), and lay the
// codes out in the fragment order the GEMM kernels read.
// None of this is on the timed path; the kernels favour clarity.
#include "serq_device.h"

namespace serq {
namespace {

constexpr int kT = 256;

// wscale[n] = max_k |W[n,k]*s[k]| / 7   (one workgroup per output channel)
__global__ __launch_bounds__(kT) void row_scale_kernel(const void* __restrict__ W, int w_dtype,
                                                       const float* __restrict__ s, int K,
                                                       float* __restrict__ wscale) {
  __shared__ float red[kT / 64];
  const size_t n = blockIdx.x;
  float m = 0.0f;
  for (int k = threadIdx.x; k < K; k += kT) {
    float w = ld_any(W, w_dtype, n * (size_t)K + k);
    if (s) w = w * s[k];
    m = fmaxf(m, fabsf(w));
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = red[0];
    for (int i = 1; i < kT / 64; ++i) r = fmaxf(r, red[i]);
    wscale[n] = r > 0.0f ? r / 7.0f : 1.0f;
  }
}

__global__ __launch_bounds__(kT) void zero_floats_kernel(float* __restrict__ p, int n) {
  const int i = blockIdx.x * kT + threadIdx.x;
  if (i < n) p[i] = 0.0f;
}

// sal[k] = max_n |W[n,k]*s[k]|: a thread takes one input channel (coalesced over k) and a slab of
// kSalRows output channels (blockIdx.y); the slabs meet in an integer maximum of the bit patterns,
// which orders non-negative floats as the floats themselves and does not depend on the order of
// arrival.  sal must be zero on entry.
constexpr int kSalRows = 128;
__global__ __launch_bounds__(kT) void col_saliency_kernel(const void* __restrict__ W, int w_dtype,
                                                          const float* __restrict__ s, int N, int K,
                                                          float* __restrict__ sal) {
  const int k = blockIdx.x * kT + threadIdx.x;
  if (k >= K) return;
  const float sk = s ? s[k] : 1.0f;
  const int n0 = blockIdx.y * kSalRows;
  const int n1 = n0 + kSalRows < N ? n0 + kSalRows : N;
  float m = 0.0f;
  for (int n = n0; n < n1; ++n) {
    float w = ld_any(W, w_dtype, (size_t)n * K + k);
    if (s) w = w * sk;
    m = fmaxf(m, fabsf(w));
  }
  atomicMax(reinterpret_cast<unsigned int*>(sal) + k, __float_as_uint(m));
}

// Stable descending order by counting: position of k = number of channels that
// come before it (larger saliency, or equal saliency and lower index).
__global__ __launch_bounds__(kT) void rank_perm_kernel(const float* __restrict__ sal, int K,
                                                       int32_t* __restrict__ perm) {
  const int k = blockIdx.x * kT + threadIdx.x;
  if (k >= K) return;
  const float mine = sal[k];
  int pos = 0;
  for (int j = 0; j < K; ++j) {
    const float o = sal[j];
    pos += (o > mine) || (o == mine && j < k);
  }
  perm[pos] = k;
}

// a caller's order is trusted to be a permutation; indices are clamped into [0, K) all the same, so that a bad one
// cannot make the kernels below read outside W and s (it still gives a wrong layer)
__global__ __launch_bounds__(kT) void copy_perm_kernel(const int32_t* __restrict__ in, int K,
                                                       int32_t* __restrict__ out) {
  const int k = blockIdx.x * kT + threadIdx.x;
  if (k < K) {
    const int v = in[k];
    out[k] = v < 0 ? 0 : (v >= K ? K - 1 : v);
  }
}

__global__ __launch_bounds__(kT) void sinv_kernel(const float* __restrict__ s, const int32_t* __restrict__ perm,
                                                  int K, float* __restrict__ s_inv) {
  const int kp = blockIdx.x * kT + threadIdx.x;
  if (kp >= K) return;
  s_inv[kp] = s ? 1.0f / s[perm[kp]] : 1.0f;
}

__device__ __forceinline__ int quant_w(const void* W, int w_dtype, const float* s, size_t n, int K, int k_orig,
                                       float ws, float* folded) {
  float w = ld_any(W, w_dtype, n * (size_t)K + k_orig);
  if (s) w = w * s[k_orig];
  *folded = w;
  float t = rintf(w / ws);
  t = fminf(fmaxf(t, -7.0f), 7.0f);
  return (int)t;
}

// one thread per packed dword of the weight blob
__global__ __launch_bounds__(kT) void quant_pack_kernel(const void* __restrict__ W, int w_dtype,
                                                        const float* __restrict__ s,
                                                        const int32_t* __restrict__ perm,
                                                        const float* __restrict__ wscale, int N, int K,
                                                        uint32_t* __restrict__ blob) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const size_t total = (size_t)N * K / 8;
  if (idx >= total) return;
  const int d = idx & 3;
  const int lane = (idx >> 2) & 63;
  const size_t frag = idx >> 8;
  const int KB = K >> 6;
  const int kb = frag % KB;
  const size_t nb = frag / KB;
  const size_t n = nb * 32 + (lane & 31);
  const int k0 = kb * 64 + (lane >> 5) * 32 + d * 8;
  const float ws = wscale[n];
  uint32_t out = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float f;
    const int lo = quant_w(W, w_dtype, s, n, K, perm[k0 + j], ws, &f);
    const int hi = quant_w(W, w_dtype, s, n, K, perm[k0 + 4 + j], ws, &f);
    out |= ((uint32_t)(lo & 0xf) | ((uint32_t)(hi & 0xf) << 4)) << (8 * j);
  }
  blob[idx] = out;
}

// R[j,n] = W^[n,j] - wscale[n]*Wq[n,j]  for the r leading (salient) channels
__global__ __launch_bounds__(kT) void residual_kernel(const void* __restrict__ W, int w_dtype,
                                                      const float* __restrict__ s,
                                                      const int32_t* __restrict__ perm,
                                                      const float* __restrict__ wscale, int N, int K, int r,
                                                      void* __restrict__ R_out, int r_dtype,
                                                      uint16_t* __restrict__ Rp_out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)r * N) return;
  const int j = idx / N;
  const size_t n = idx % N;
  const float ws = wscale[n];
  float folded;
  const int q = quant_w(W, w_dtype, s, n, K, perm[j], ws, &folded);
  const float res = __fmaf_rn(-ws, (float)q, folded);
  uint16_t h = 0;
  if (r_dtype == SERQ_BF16) h = f32_to_bf16_rne(res);
  else if (r_dtype == SERQ_F16) h = f32_to_f16_rne(res);
  if (R_out) {
    if (r_dtype == SERQ_F32) ((float*)R_out)[idx] = res;
    else ((uint16_t*)R_out)[idx] = h;
  }
  if (Rp_out) {
    const int JB = r >> 4;
    const size_t nb = n >> 5;
    const int jb = j >> 4, g = (j >> 3) & 1, p = j & 7;
    const int lane = (int)(n & 31) + 32 * g;
    Rp_out[((nb * JB + jb) * 64 + lane) * 8 + p] = h;
  }
}

// canonical R [r,N]  <->  fragment-ordered Rp
__global__ __launch_bounds__(kT) void pack_lowrank_kernel(uint16_t* __restrict__ R, int N, int r,
                                                          uint16_t* __restrict__ Rp, bool unpack) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)r * N) return;
  const int j = idx / N;
  const size_t n = idx % N;
  const int JB = r >> 4;
  const size_t nb = n >> 5;
  const int jb = j >> 4, g = (j >> 3) & 1, p = j & 7;
  const int lane = (int)(n & 31) + 32 * g;
  const size_t pidx = ((nb * JB + jb) * 64 + lane) * 8 + p;
  if (unpack) R[idx] = Rp[pidx];
  else Rp[pidx] = R[idx];
}

// ---- the 4-bit compensation matrix Q(R) (Eq. 7, second line) -------------------
// Blob: [N/32][ceil(r/64)] fragments of 1 KiB in the weight-fragment layout with the rank index j in
// the place of the input channel (ranks past r hold zero codes), then rscale [N] fp32.

// rscale[n] = max_j |R[j,n]| / 7   (Eq. 1 per output channel; 1.0 for a zero column)
__global__ __launch_bounds__(kT) void lowrank_scale_kernel(const void* __restrict__ R, int r_dtype, int N, int r,
                                                           float* __restrict__ rscale) {
  const int n = blockIdx.x * kT + threadIdx.x;
  if (n >= N) return;
  float m = 0.0f;
  for (int j = 0; j < r; ++j) m = fmaxf(m, fabsf(ld_any(R, r_dtype, (size_t)j * N + n)));
  rscale[n] = m > 0.0f ? m / 7.0f : 1.0f;
}

// one thread per packed dword
__global__ __launch_bounds__(kT) void lowrank_q4_pack_kernel(const void* __restrict__ R, int r_dtype, int N, int r,
                                                             const float* __restrict__ rscale,
                                                             uint32_t* __restrict__ blob) {
  const int FR = (r + 63) >> 6;
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)(N / 32) * FR * 256) return;
  const int d = idx & 3;
  const int lane = (idx >> 2) & 63;
  const size_t frag = idx >> 8;
  const int fb = frag % FR;
  const size_t n = (frag / FR) * 32 + (lane & 31);
  const int j0 = fb * 64 + (lane >> 5) * 32 + d * 8;
  const float rs = rscale[n];
  auto code = [&](int j) {
    if (j >= r) return 0;
    float t = rintf(ld_any(R, r_dtype, (size_t)j * N + n) / rs);
    return (int)fminf(fmaxf(t, -7.0f), 7.0f);
  };
  uint32_t out = 0;
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
    out |= ((uint32_t)(code(j0 + jj) & 0xf) | ((uint32_t)(code(j0 + 4 + jj) & 0xf) << 4)) << (8 * jj);
  blob[idx] = out;
}

// canonical view: codes int8 [r,N]; one thread per packed dword
__global__ __launch_bounds__(kT) void lowrank_q4_unpack_kernel(const uint32_t* __restrict__ blob, int N, int r,
                                                               int8_t* __restrict__ out) {
  const int FR = (r + 63) >> 6;
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (size_t)(N / 32) * FR * 256) return;
  const int d = idx & 3;
  const int lane = (idx >> 2) & 63;
  const size_t frag = idx >> 8;
  const int fb = frag % FR;
  const size_t n = (frag / FR) * 32 + (lane & 31);
  const int j0 = fb * 64 + (lane >> 5) * 32 + d * 8;
  int c[8];
  codes_from_a4(blob[idx], c);
#pragma unroll
  for (int jj = 0; jj < 8; ++jj)
    if (j0 + jj < r) out[(size_t)(j0 + jj) * N + n] = (int8_t)c[jj];
}

__global__ __launch_bounds__(kT) void unpack_weights_kernel(const uint32_t* __restrict__ blob, int N, int K,
                                                            int8_t* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  const size_t total = (size_t)N * K / 8;
  if (idx >= total) return;
  const int d = idx & 3;
  const int lane = (idx >> 2) & 63;
  const size_t frag = idx >> 8;
  const int KB = K >> 6;
  const int kb = frag % KB;
  const size_t nb = frag / KB;
  const size_t n = nb * 32 + (lane & 31);
  const int k0 = kb * 64 + (lane >> 5) * 32 + d * 8;
  int c[8];
  codes_from_a4(blob[idx], c);
  uint32_t d0 = (c[0] & 0xff) | ((c[1] & 0xff) << 8) | ((c[2] & 0xff) << 16) | ((uint32_t)(c[3] & 0xff) << 24);
  uint32_t d1 = (c[4] & 0xff) | ((c[5] & 0xff) << 8) | ((c[6] & 0xff) << 16) | ((uint32_t)(c[7] & 0xff) << 24);
  *(uint2*)(out + n * (size_t)K + k0) = make_uint2(d0, d1);
}

__global__ __launch_bounds__(kT) void unpack_act4_kernel(const uint32_t* __restrict__ xq, size_t total,
                                                         int8_t* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= total) return;
  int c[8];
  codes_from_a4(xq[idx], c);
  uint32_t d0 = (c[0] & 0xff) | ((c[1] & 0xff) << 8) | ((c[2] & 0xff) << 16) | ((uint32_t)(c[3] & 0xff) << 24);
  uint32_t d1 = (c[4] & 0xff) | ((c[5] & 0xff) << 8) | ((c[6] & 0xff) << 16) | ((uint32_t)(c[7] & 0xff) << 24);
  ((uint2*)out)[idx] = make_uint2(d0, d1);
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + kT - 1) / kT); }
inline int ok() { return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP; }

}  // namespace

int pack_weights_impl(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int N, int K, int r,
                      void* Wq_out, float* wscale_out, int32_t* perm_out, float* s_inv_out, void* R_out,
                      int r_dtype, void* Rp_out, hipStream_t st) {
  hipLaunchKernelGGL(row_scale_kernel, dim3(N), dim3(kT), 0, st, W, w_dtype, s, K, wscale_out);
  const int prc = prepare_perm_impl(W, w_dtype, s, perm_in, N, K, perm_out, s_inv_out, st);
  if (prc != SERQ_OK) return prc;
  hipLaunchKernelGGL(quant_pack_kernel, dim3(blocks_for((size_t)N * K / 8)), dim3(kT), 0, st, W, w_dtype, s,
                     perm_out, wscale_out, N, K, (uint32_t*)Wq_out);
  if (r > 0 && (R_out || Rp_out)) {
    hipLaunchKernelGGL(residual_kernel, dim3(blocks_for((size_t)r * N)), dim3(kT), 0, st, W, w_dtype, s, perm_out,
                       wscale_out, N, K, r, R_out, r_dtype, (uint16_t*)Rp_out);
  }
  return ok();
}

// saliency order (or the caller's) and the reciprocal flattening vector in that order
int prepare_perm_impl(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int N, int K,
                      int32_t* perm_out, float* s_inv_out, hipStream_t st) {
  if (perm_in) {
    hipLaunchKernelGGL(copy_perm_kernel, dim3(blocks_for(K)), dim3(kT), 0, st, perm_in, K, perm_out);
  } else {
    float* sal = s_inv_out;  // borrowed until sinv_kernel overwrites it
    hipLaunchKernelGGL(zero_floats_kernel, dim3(blocks_for(K)), dim3(kT), 0, st, sal, K);
    hipLaunchKernelGGL(col_saliency_kernel, dim3(blocks_for(K), (unsigned)((N + kSalRows - 1) / kSalRows)), dim3(kT), 0, st,
                       W, w_dtype, s, N, K, sal);
    hipLaunchKernelGGL(rank_perm_kernel, dim3(blocks_for(K)), dim3(kT), 0, st, sal, K, perm_out);
  }
  hipLaunchKernelGGL(sinv_kernel, dim3(blocks_for(K)), dim3(kT), 0, st, s, perm_out, K, s_inv_out);
  return ok();
}

int pack_lowrank_impl(void* R, int N, int r, void* Rp, bool unpack, hipStream_t st) {
  if (r == 0) return SERQ_OK;
  hipLaunchKernelGGL(pack_lowrank_kernel, dim3(blocks_for((size_t)r * N)), dim3(kT), 0, st, (uint16_t*)R, N, r,
                     (uint16_t*)Rp, unpack);
  return ok();
}

size_t lowrank_q4_frag_bytes(int N, int r) { return (size_t)(N / 32) * ((r + 63) / 64) * 1024; }

int pack_lowrank_q4_impl(const void* R, int r_dtype, int N, int r, void* Rq, hipStream_t st) {
  if (r == 0) return SERQ_OK;
  const size_t fb = lowrank_q4_frag_bytes(N, r);
  float* rscale = (float*)((char*)Rq + fb);
  hipLaunchKernelGGL(lowrank_scale_kernel, dim3(blocks_for(N)), dim3(kT), 0, st, R, r_dtype, N, r, rscale);
  hipLaunchKernelGGL(lowrank_q4_pack_kernel, dim3(blocks_for(fb / 4)), dim3(kT), 0, st, R, r_dtype, N, r, rscale,
                     (uint32_t*)Rq);
  return ok();
}

int unpack_lowrank_q4_impl(const void* Rq, int N, int r, int8_t* codes, float* rscale, hipStream_t st) {
  if (r == 0) return SERQ_OK;
  const size_t fb = lowrank_q4_frag_bytes(N, r);
  if (codes)
    hipLaunchKernelGGL(lowrank_q4_unpack_kernel, dim3(blocks_for(fb / 4)), dim3(kT), 0, st, (const uint32_t*)Rq, N, r,
                       codes);
  if (rscale &&
      hipMemcpyAsync(rscale, (const char*)Rq + fb, (size_t)N * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
    return SERQ_EHIP;
  return ok();
}

int unpack_weights_impl(const void* Wq, int N, int K, int8_t* out, hipStream_t st) {
  hipLaunchKernelGGL(unpack_weights_kernel, dim3(blocks_for((size_t)N * K / 8)), dim3(kT), 0, st,
                     (const uint32_t*)Wq, N, K, out);
  return ok();
}

int unpack_act_impl(const void* Xq, int abits, int64_t M, int K, int8_t* out, hipStream_t st) {
  if (M == 0) return SERQ_OK;
  if (abits == 8) {
    return hipMemcpyAsync(out, Xq, (size_t)M * K, hipMemcpyDeviceToDevice, st) == hipSuccess ? SERQ_OK : SERQ_EHIP;
  }
  const size_t total = (size_t)M * K / 8;
  hipLaunchKernelGGL(unpack_act4_kernel, dim3(blocks_for(total)), dim3(kT), 0, st, (const uint32_t*)Xq, total, out);
  return ok();
}

}  // namespace serq
