// SERQ linear layer for decode-sized batches (M <= 32): an HBM-bound kernel
// that streams every packed weight fragment exactly once.
//
// Computes, for up to 32 tokens, Eq. 2 + Eq. 7 (first line):
//   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k] Wq[n,k] + sum_j Xq[m,S_j] R[j,n] )
//
// Work decomposition: a workgroup of 8 waves owns one block of 32 output
// channels and one slice of K (split-K when N alone gives too few workgroups).
// Each wave walks its share of the 1-KiB weight fragments with one coalesced
// 16-byte load per lane, widens the nibbles to int8 (x16) in two VALU ops per
// dword, and feeds two 32x32x32 int8 MFMAs whose B operand is the token block
// (rows >= M are zero).  The rank-r term runs through 32x32x16 f16/bf16 MFMAs
// on the packed R fragments into a second, fp32 accumulator.  The 8 waves are
// combined through LDS; with split-K the slices are combined in a fixed order
// by the last workgroup to arrive (integer sums: order-free; the fp32 low-rank
// sums: fixed order, so results are run-to-run identical).
#include "serq_device.h"

namespace serq {
namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kUnroll = 4;

struct SkinnyParams {
  const uint8_t* Xq; const float* scale;
  const u4* Wq; const float* wscale;
  const u4* Rp; int r_dtype; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int32_t* acc_out; int64_t ldacc;
  int splitk;
  int32_t* counters; int32_t* part_i; float* part_f;
};

template <int ABITS>
__global__ __launch_bounds__(kThreads) void serq_skinny_kernel(const SkinnyParams p) {
  __shared__ int red_i[kWaves][1024];
  __shared__ float red_f[kWaves][1024];
  __shared__ int is_last;

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int m = l & 31, g = l >> 5;
  const int nb = blockIdx.x / p.splitk;
  const int ks = blockIdx.x % p.splitk;
  const int KB = p.K >> 6;
  const int kb0 = (int)(((int64_t)KB * ks) / p.splitk);
  const int kb1 = (int)(((int64_t)KB * (ks + 1)) / p.splitk);
  constexpr int SH = (ABITS == 8) ? 4 : 8;
  const size_t rowbytes = (size_t)p.K * ABITS / 8;

  const bool mv = m < p.M;
  const uint8_t* xrow = p.Xq + (size_t)(mv ? m : 0) * rowbytes;
  const u4* wfr = p.Wq + (size_t)nb * KB * 64 + l;

  v16i acc;
  v16f accf;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[e] = 0; accf[e] = 0.0f; }

  // ---- main integer contraction over this workgroup's K slice -------------
  for (int kb = kb0 + w; kb < kb1; kb += kWaves * kUnroll) {
    u4 wp[kUnroll];
    u4 x0[kUnroll];
    u4 x1[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int kbu = kb + u * kWaves;
      const bool ok = kbu < kb1;
      const int kc = ok ? kbu : kb0;                    // always a valid fragment
      wp[u] = wfr[(size_t)kc * 64];
      if (!ok) wp[u] = u4{0u, 0u, 0u, 0u};              // zero weights contribute nothing
      if constexpr (ABITS == 8) {
        const u4* xp = (const u4*)(xrow + (size_t)kc * 64 + g * 32);
        x0[u] = xp[0];
        x1[u] = xp[1];
      } else {
        x0[u] = *(const u4*)(xrow + (size_t)kc * 32 + g * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      v4i a0, a1, b0, b1;
      unpack_frag(wp[u], a0, a1);
      if constexpr (ABITS == 8) {
        b0 = as_v4i(x0[u]);
        b1 = as_v4i(x1[u]);
      } else {
        unpack_frag(x0[u], b0, b1);
      }
      if (!mv) { b0 = (v4i){0, 0, 0, 0}; b1 = (v4i){0, 0, 0, 0}; }
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc, 0, 0, 0);
    }
  }

  // ---- rank-r compensation: blocks of 16 salient channels ------------------
  if (p.r > 0 && p.acc_out == nullptr) {
    const int JB = p.r >> 4;
    const bool bf = p.r_dtype == SERQ_BF16;
    const u4* rfr = p.Rp + (size_t)nb * JB * 64 + l;
    for (int jb = ks * kWaves + w; jb < JB; jb += kWaves * p.splitk) {
      const u4 rf = rfr[(size_t)jb * 64];
      const int col = p.s_begin + jb * 16 + g * 8;      // first of this lane's 8 channels
      int c[8];
      if constexpr (ABITS == 8) {
        const u2 d = *(const u2*)(xrow + col);
        codes_from_a8(d.x, d.y, c);
      } else {
        const uint32_t d = *(const uint32_t*)(xrow + (col >> 1));
        codes_from_a4(d, c);
      }
      u4 xf = codes8_to_16bit(c, bf);
      if (!mv) xf = u4{0u, 0u, 0u, 0u};
      if (bf)
        accf = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, rf), __builtin_bit_cast(v8bf, xf),
                                                       accf, 0, 0, 0);
      else
        accf = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, rf), __builtin_bit_cast(v8h, xf),
                                                      accf, 0, 0, 0);
    }
  }

  // ---- combine the 8 waves --------------------------------------------------
  // accumulator register e of lane l holds channel 8*(e/4) + 4*(l/32) + e%4 of
  // the block and token l%32.
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    red_i[w][e * 64 + l] = acc[e];
    red_f[w][e * 64 + l] = accf[e];
  }
  __syncthreads();

  int tot_i[2];
  float tot_f[2];
  int mm[2], nn[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int nl = tid & 31;                 // channel within the block: consecutive threads, consecutive n
    const int mt = (tid >> 5) + 16 * h;      // token
    const int e = 4 * (nl >> 3) + (nl & 3);
    const int ll = mt + 32 * ((nl >> 2) & 1);
    int si = 0;
    float sf = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) {
      si += red_i[ww][e * 64 + ll];
      sf += red_f[ww][e * 64 + ll];
    }
    tot_i[h] = si; tot_f[h] = sf; mm[h] = mt; nn[h] = nb * 32 + nl;
  }

  if (p.splitk > 1) {
    const size_t base = (size_t)blockIdx.x * 1024;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      p.part_i[base + tid + 512 * h] = tot_i[h];
      p.part_f[base + tid + 512 * h] = tot_f[h];
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      const int old = atomicAdd(&p.counters[nb], 1);
      is_last = (old == p.splitk - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      int si = 0;
      float sf = 0.0f;
      for (int s = 0; s < p.splitk; ++s) {
        const size_t o = ((size_t)nb * p.splitk + s) * 1024 + tid + 512 * h;
        si += __hip_atomic_load(&p.part_i[o], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sf += __hip_atomic_load(&p.part_f[o], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      tot_i[h] = si; tot_f[h] = sf;
    }
    if (tid == 0) p.counters[nb] = 0;        // leave the workspace ready for the next call
  }

#pragma unroll
  for (int h = 0; h < 2; ++h) {
    if (mm[h] >= p.M) continue;
    const int a = tot_i[h] >> SH;            // exact: the sum is a multiple of 2^SH
    if (p.acc_out) {
      p.acc_out[(size_t)mm[h] * p.ldacc + nn[h]] = a;
    } else {
      const float y = p.scale[mm[h]] * (p.wscale[nn[h]] * (float)a + tot_f[h]);
      const size_t o = (size_t)mm[h] * p.ldy + nn[h];
      if (p.y_dtype == SERQ_F32) ((float*)p.Y)[o] = y;
      else if (p.y_dtype == SERQ_BF16) ((uint16_t*)p.Y)[o] = f32_to_bf16_rne(y);
      else ((uint16_t*)p.Y)[o] = f32_to_f16_rne(y);
    }
  }
}

}  // namespace

int skinny_splitk_auto(int M, int N, int K) {
  (void)M;
  const int nblk = N / 32;
  const int KB = K / 64;
  int s = (1024 + nblk - 1) / nblk;          // aim for >= 1024 workgroups (4 per CU)
  const int smax = KB / kWaves > 0 ? KB / kWaves : 1;   // keep >= 1 fragment per wave
  if (s > smax) s = smax;
  if (s > 32) s = 32;
  if (s < 1) s = 1;
  return s;
}

size_t skinny_workspace_bytes(int N, int splitk) {
  const size_t nblk = (size_t)N / 32;
  size_t counters = (nblk * 4 + 255) & ~(size_t)255;
  if (splitk <= 1) return counters;
  return counters + nblk * (size_t)splitk * 1024 * 8;
}

int launch_skinny(const LinearArgs& a, hipStream_t st) {
  SkinnyParams p;
  p.Xq = a.Xq; p.scale = a.scale; p.Wq = a.Wq; p.wscale = a.wscale;
  p.Rp = a.Rp; p.r_dtype = a.r_dtype; p.s_begin = a.s_begin; p.r = a.Rp ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.acc_out = a.acc_out; p.ldacc = a.ldacc;
  int splitk = a.splitk > 0 ? a.splitk : skinny_splitk_auto(a.M, a.N, a.K);
  const int KB = a.K / 64;
  if (splitk > KB) splitk = KB;
  const size_t nblk = (size_t)a.N / 32;
  if (splitk > 1) {
    if (a.workspace == nullptr || a.workspace_bytes < skinny_workspace_bytes(a.N, splitk)) {
      if (a.splitk > 0) return SERQ_EWORKSPACE;      // an explicit request cannot be honoured
      splitk = 1;                                     // auto: fall back to no split
    }
  }
  p.splitk = splitk;
  const size_t coff = (nblk * 4 + 255) & ~(size_t)255;
  p.counters = (int32_t*)a.workspace;
  p.part_i = splitk > 1 ? (int32_t*)((char*)a.workspace + coff) : nullptr;
  p.part_f = splitk > 1 ? (float*)((char*)a.workspace + coff + nblk * (size_t)splitk * 1024 * 4) : nullptr;
  dim3 grid((unsigned)(nblk * splitk)), block(kThreads);
  if (a.abits == 8) hipLaunchKernelGGL(serq_skinny_kernel<8>, grid, block, 0, st, p);
  else hipLaunchKernelGGL(serq_skinny_kernel<4>, grid, block, 0, st, p);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // namespace serq
