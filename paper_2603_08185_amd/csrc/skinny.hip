// SERQ linear layer for decode-sized batches (M <= 32): an HBM-bound kernel
// that streams every packed weight fragment exactly once.
//
// Computes, for up to 32 tokens, Eq. 2 + Eq. 7 (first line):
//   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k] Wq[n,k] + sum_j Xq[m,S_j] R[j,n] )
//
// Work decomposition: a workgroup of 4 or 8 waves owns one block of 32 output
// channels and one slice of K (the host splits K only when N alone gives too
// few workgroups to fill the chip).  The 1-KiB weight fragments of the block
// are contiguous in memory; wave w of W takes fragments w, w+W, ... of the slice,
// four at a time: one coalesced 16-byte load per lane and fragment, all four in
// flight before the first is used.  The nibbles are widened to int8 (x16) in
// registers and fed to two 32x32x32 int8 MFMAs per fragment whose B operand is
// the token block (rows >= M are zero) -- the matrix unit is nearly idle, the
// point is that it costs no VALU work to reduce over K.  The rank-r term runs
// through 32x32x16 f16/bf16 MFMAs on the packed R fragments (one fragment per
// wave) into a second, fp32 accumulator.
//
// The waves are combined through LDS in a fixed order.  With a split K the
// workgroup stores its partial sums (INT32 for the main term, fp32 for the
// low-rank term, which only slice 0 computes) to the workspace and a second,
// small kernel adds the slices in a fixed order and applies the epilogue -- the
// kernel boundary is the only synchronisation, so no device-wide fences or
// atomics are needed and results are run-to-run identical.
#include "serq_device.h"

namespace serq {
namespace {



struct SkinnyParams {
  const uint8_t* Xq; const float* scale;
  const u4* Wq; const float* wscale;
  const u4* Rp; int r_dtype; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int32_t* acc_out; int64_t ldacc;
  int splitk;
  int32_t* part_i; float* part_f;       // [N/32][splitk][1024] each
#ifdef SERQ_SKINNY_DBG
  unsigned long long* dbg;
#endif
};

// y for (token m, channel n) from the two sums; one store
__device__ __forceinline__ void finish(const SkinnyParams& p, int m, int n, int acc_scaled, float lr, float sm, float wn) {
  if (m >= p.M) return;
  if (p.acc_out) {
    p.acc_out[(size_t)m * p.ldacc + n] = acc_scaled;
    return;
  }
  const float y = sm * (wn * (float)acc_scaled + lr);
  const size_t o = (size_t)m * p.ldy + n;
  if (p.y_dtype == SERQ_F32) ((float*)p.Y)[o] = y;
  else if (p.y_dtype == SERQ_BF16) ((uint16_t*)p.Y)[o] = f32_to_bf16_rne(y);
  else ((uint16_t*)p.Y)[o] = f32_to_f16_rne(y);
}

template <int ABITS, int kWaves, int kUnroll>
__global__ __launch_bounds__(kWaves * 64) void serq_skinny_kernel(const SkinnyParams p) {
  constexpr int kThreads = kWaves * 64;
  constexpr int kPitch = 65;                            // words per accumulator register row: an odd pitch spreads the gather over the banks
  __shared__ int red[kWaves][16 * kPitch];              // used for the INT32, then the fp32 partials

#ifdef SERQ_SKINNY_DBG
  const unsigned long long dbg_t0 = wall_clock64();
#endif
  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int m = l & 31, g = l >> 5;
  const int nb = blockIdx.x / p.splitk;
  const int ks = blockIdx.x - nb * p.splitk;
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

  // Everything this wave will need is requested before anything is used, so that the
  // workgroup pays the memory latency once: the operands of the rank-r term (blocks of
  // 16 salient channels, slice 0 only; up to kLrMax blocks per wave are prefetched) ...
  const bool has_lr = p.r > 0 && p.acc_out == nullptr;
  const bool lr_here = has_lr && ks == 0;
  const int JB = p.r >> 4;
  const bool bf = p.r_dtype == SERQ_BF16;
  constexpr int kLrMax = 2;
  u4 rf[kLrMax];
  u2 xc[kLrMax];
  const u4* rfr = p.Rp + (size_t)nb * JB * 64 + l;
  auto lr_load = [&](int jb, u4& r_out, u2& x_out) {
    r_out = __builtin_nontemporal_load(&rfr[(size_t)jb * 64]);
    const int col = p.s_begin + jb * 16 + g * 8;        // first of this lane's 8 channels
    if constexpr (ABITS == 8) x_out = *(const u2*)(xrow + col);
    else { x_out.x = *(const uint32_t*)(xrow + (col >> 1)); x_out.y = 0; }
  };
  auto lr_mfma = [&](const u4& r_in, const u2& x_in) {
    int c[8];
    if constexpr (ABITS == 8) codes_from_a8(x_in.x, x_in.y, c);
    else codes_from_a4(x_in.x, c);
    u4 xf = codes8_to_16bit(c, bf);
    if (!mv) xf = u4{0u, 0u, 0u, 0u};
    if (bf)
      accf = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, r_in), __builtin_bit_cast(v8bf, xf),
                                                     accf, 0, 0, 0);
    else
      accf = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, r_in), __builtin_bit_cast(v8h, xf),
                                                    accf, 0, 0, 0);
  };
  if (lr_here) {
#pragma unroll
    for (int q = 0; q < kLrMax; ++q)
      if (w + q * kWaves < JB) lr_load(w + q * kWaves, rf[q], xc[q]);
  }
  // ... the scales of the outputs this thread will finish ...
  constexpr int NQ = 1024 / kThreads;
  float sc_m[NQ], sc_n[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    sc_m[q] = sc_n[q] = 0.0f;
    if (p.acc_out == nullptr && p.splitk == 1 && (id >> 5) < p.M) {
      sc_m[q] = p.scale[id >> 5];
      sc_n[q] = p.wscale[nb * 32 + (id & 31)];
    }
  }

  // ... and the main integer contraction over this workgroup's K slice, in batches of kUnroll
  // fragments per wave.  Registers are kept few on purpose: many resident waves hide the latency.
  struct Batch { u4 wp[kUnroll]; u4 x0[kUnroll]; u4 x1[ABITS == 8 ? kUnroll : 1]; };
  auto load_batch = [&](int kb, Batch& B) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int kbu = kb + u * kWaves;
      const bool ok = kbu < kb1;
      const int kc = ok ? kbu : kb0;                    // always a valid fragment
      B.wp[u] = __builtin_nontemporal_load(&wfr[(size_t)kc * 64]);   // streamed once: do not keep it in the caches
      if (!ok) B.wp[u] = u4{0u, 0u, 0u, 0u};            // zero weights contribute nothing
      if constexpr (ABITS == 8) {
        const u4* xp = (const u4*)(xrow + (size_t)kc * 64 + g * 32);
        B.x0[u] = xp[0];
        B.x1[u] = xp[1];
      } else {
        B.x0[u] = *(const u4*)(xrow + (size_t)kc * 32 + g * 16);
      }
    }
  };
  auto mul_batch = [&](const Batch& B) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      v4i a0, a1, b0, b1;
      unpack_frag(B.wp[u], a0, a1);
      if constexpr (ABITS == 8) {
        b0 = as_v4i(B.x0[u]);
        b1 = as_v4i(B.x1[u]);
      } else {
        unpack_frag(B.x0[u], b0, b1);
      }
      if (!mv) { b0 = (v4i){0, 0, 0, 0}; b1 = (v4i){0, 0, 0, 0}; }
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc, 0, 0, 0);
    }
  };
  for (int kb = kb0 + w; kb < kb1; kb += kWaves * kUnroll) {
    Batch B;
    load_batch(kb, B);
    __builtin_amdgcn_sched_barrier(0);                  // every load of the batch is in flight before the first use
    mul_batch(B);
  }

  if (lr_here) {
#pragma unroll
    for (int q = 0; q < kLrMax; ++q)
      if (w + q * kWaves < JB) lr_mfma(rf[q], xc[q]);
    for (int jb = w + kLrMax * kWaves; jb < JB; jb += kWaves) {   // ranks beyond the prefetched blocks
      u4 r1; u2 x1;
      lr_load(jb, r1, x1);
      lr_mfma(r1, x1);
    }
  }

#ifdef SERQ_SKINNY_DBG
  const unsigned long long dbg_t1 = wall_clock64();
#endif
  // ---- combine the waves ----------------------------------------------------
  // accumulator register e of lane l holds channel 8*(e/4) + 4*(l/32) + e%4 of
  // the block and token l%32; only tokens < M are exchanged.
  // Thread tid finishes (token q/32, channel q%32) for q = tid, tid + kThreads, ...
  const int nwl = JB < kWaves ? JB : kWaves;              // waves that hold low-rank sums
  if (mv) {
#pragma unroll
    for (int e = 0; e < 16; ++e) red[w][e * kPitch + l] = acc[e];
  }
  __syncthreads();
  int tot_i[NQ];
  float tot_f[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    const int nl = id & 31, mt = id >> 5;
    const int e_src = 4 * (nl >> 3) + (nl & 3);
    const int l_src = mt + 32 * ((nl >> 2) & 1);
    tot_i[q] = 0;
    tot_f[q] = 0.0f;
    if (mt < p.M) {
#pragma unroll
      for (int ww = 0; ww < kWaves; ++ww) tot_i[q] += red[ww][e_src * kPitch + l_src];
    }
  }
  if (has_lr) {                                           // uniform over the grid
    __syncthreads();
    float* redf = reinterpret_cast<float*>(&red[0][0]);
    if (mv && w < nwl && lr_here) {
#pragma unroll
      for (int e = 0; e < 16; ++e) redf[w * 16 * kPitch + e * kPitch + l] = accf[e];
    }
    __syncthreads();
    if (lr_here) {
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int id = tid + q * kThreads;
        const int nl = id & 31, mt = id >> 5;
        const int e_src = 4 * (nl >> 3) + (nl & 3);
        const int l_src = mt + 32 * ((nl >> 2) & 1);
        if (mt < p.M)
          for (int ww = 0; ww < nwl; ++ww) tot_f[q] += redf[ww * 16 * kPitch + e_src * kPitch + l_src];
      }
    }
  }

#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    const int nl = id & 31, mt = id >> 5;
    if (mt >= p.M) continue;
    if (p.splitk > 1) {
      // partial sums of this slice; the reduce kernel finishes the job
      p.part_i[((size_t)nb * p.splitk + ks) * 1024 + id] = tot_i[q];
      if (lr_here) p.part_f[(size_t)nb * 1024 + id] = tot_f[q];
    } else {
      finish(p, mt, nb * 32 + nl, tot_i[q] >> SH, tot_f[q], sc_m[q], sc_n[q]);   // exact shift: the sum is a multiple of 2^SH
    }
  }
#ifdef SERQ_SKINNY_DBG
  if (p.dbg && tid == 0) { p.dbg[blockIdx.x * 3] = dbg_t0; p.dbg[blockIdx.x * 3 + 1] = dbg_t1; p.dbg[blockIdx.x * 3 + 2] = wall_clock64(); }
#endif
}

// second kernel of a split-K launch: one workgroup per block of 32 channels
template <int ABITS>
__global__ __launch_bounds__(1024) void serq_skinny_reduce_kernel(const SkinnyParams p) {
  constexpr int SH = (ABITS == 8) ? 4 : 8;
  const int tid = threadIdx.x;
  const int nb = blockIdx.x;
  const int mt = tid >> 5;
  if (mt >= p.M) return;
  int tot_i = 0;
  for (int s = 0; s < p.splitk; ++s) tot_i += p.part_i[((size_t)nb * p.splitk + s) * 1024 + tid];
  const bool has_lr = p.r > 0 && p.acc_out == nullptr;
  const float tot_f = has_lr ? p.part_f[(size_t)nb * 1024 + tid] : 0.0f;
  const int n = nb * 32 + (tid & 31);
  const bool scaled = p.acc_out == nullptr;
  finish(p, mt, n, tot_i >> SH, tot_f, scaled ? p.scale[mt] : 0.0f, scaled ? p.wscale[n] : 0.0f);
}

}  // namespace

int skinny_splitk_auto(int M, int N, int K) {
  (void)M;
  const int nblk = N / 32;
  const int KB = K / 64;
  int s = (256 + nblk - 1) / nblk;           // aim for one workgroup per compute unit; splitting further only adds passes
  const int smax = KB / 16 > 0 ? KB / 16 : 1;          // keep >= 2 fragments per wave of an 8-wave workgroup
  if (s > smax) s = smax;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return s;
}

size_t skinny_workspace_bytes(int N, int splitk) {
  const size_t nblk = (size_t)N / 32;
  if (splitk <= 1) return 256;
  return nblk * (size_t)splitk * 1024 * 4 + nblk * 1024 * 4;
}

int launch_skinny(const LinearArgs& a, hipStream_t st) {
  SkinnyParams p;
  p.Xq = a.Xq; p.scale = a.scale; p.Wq = a.Wq; p.wscale = a.wscale;
  p.Rp = a.Rp; p.r_dtype = a.r_dtype; p.s_begin = a.s_begin; p.r = a.Rp ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.acc_out = a.acc_out; p.ldacc = a.ldacc;
#ifdef SERQ_SKINNY_DBG
  p.dbg = (unsigned long long*)a.dbg;
#endif
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
  p.part_i = splitk > 1 ? (int32_t*)a.workspace : nullptr;
  p.part_f = splitk > 1 ? (float*)((char*)a.workspace + nblk * (size_t)splitk * 1024 * 4) : nullptr;
  // waves per workgroup: 8 when the slice is long enough to give each of them several batches,
  // else 4 -- launching and combining waves costs more than it hides on a short slice
  int nw = a.skinny_waves;
  if (nw != 4 && nw != 8) nw = (KB / splitk >= 128) ? 8 : 4;
  dim3 grid((unsigned)(nblk * splitk)), block((unsigned)nw * 64);
#define SERQ_SKINNY_LAUNCH(AB, NW) hipLaunchKernelGGL((serq_skinny_kernel<AB, NW, 4>), grid, block, 0, st, p)
  if (a.abits == 8) {
    if (nw == 4) SERQ_SKINNY_LAUNCH(8, 4); else SERQ_SKINNY_LAUNCH(8, 8);
  } else {
    if (nw == 4) SERQ_SKINNY_LAUNCH(4, 4); else SERQ_SKINNY_LAUNCH(4, 8);
  }
#undef SERQ_SKINNY_LAUNCH
  if (hipGetLastError() != hipSuccess) return SERQ_EHIP;
  if (splitk > 1) {
    dim3 grid2((unsigned)nblk), block2(1024);
    if (a.abits == 8) hipLaunchKernelGGL(serq_skinny_reduce_kernel<8>, grid2, block2, 0, st, p);
    else hipLaunchKernelGGL(serq_skinny_reduce_kernel<4>, grid2, block2, 0, st, p);
    if (hipGetLastError() != hipSuccess) return SERQ_EHIP;
  }
  return SERQ_OK;
}

}  // namespace serq
