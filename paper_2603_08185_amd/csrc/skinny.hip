// SERQ linear layer for decode-sized batches (M <= 32): an HBM-bound kernel
// that streams every packed weight fragment exactly once.
//
// Computes, for up to 32 tokens, Eq. 2 + Eq. 7 (first line):
//   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k] Wq[n,k] + sum_j Xq[m,S_j] R[j,n] )
//
// Work decomposition: a workgroup of 4 or 8 waves owns one block of 32 output
// channels and all of K, or one slice of it when N alone gives fewer workgroups
// than there are CUs.  (Cutting only the blocks that do not deal out evenly --
// 344 blocks on 256 CUs: 256 whole blocks and 88 in slices -- was tried and
// measured no faster than leaving 88 CUs with two blocks.)  The 1-KiB weight
// fragments of a block are contiguous in
// memory; wave w of W takes the groups w, w+W, ... of four or eight consecutive
// fragments: one coalesced 16-byte load per lane and fragment, the whole group
// in flight before its first fragment is used.
//
// The token operand of a group (M rows of 4*64 or 8*64 channels) is what limits
// a naive version: read per lane in MFMA operand order it touches 32 cache
// lines per load instruction and the CU's L1 spends more cycles on it than on
// the weights.  Here a wave fetches it with whole-line direct-to-LDS loads
// (8, 4 or 2 rows of 128/256/512 contiguous bytes per instruction, no staging
// registers) into a wave-private LDS region -- piece order xor-swizzled per
// row, so the per-token operand reads are bank-conflict free -- and reads the
// operands back from there.  Loads retire in order, so the token loads are
// issued before the weight loads of the group (cache hits must not queue behind
// the HBM stream) and one hand-counted wait on "all but the weight loads"
// covers them.  No barrier is needed in the main loop.
//
// The nibbles are widened to int8 (x16) in registers and fed to two 32x32x32
// int8 MFMAs per fragment whose B operand is the token block (rows >= M are
// zero) -- the matrix unit is nearly idle, the point is that it costs no VALU
// work to reduce over K.  The rank-r term runs through 32x32x16 f16/bf16 MFMAs
// on the packed R fragments (one fragment per wave) into a second, fp32
// accumulator.
//
// The waves are combined through LDS in a fixed order (each wave parks its
// partial sums in its own region: one barrier per workgroup).  The workgroups
// of a sliced block meet in the workspace, one 64-bit word per output: a thread
// adds 2^40 + (its INT32 partial sum) with one returning agent-scope atomic; the
// old value tells it how many slices had arrived (bits 40 and up; the signed sum
// below stays within +-2^39) and what they summed to.  The thread that finds all
// the others there has the total in hand, applies the epilogue and stores zero
// back (the workspace is clean again for the next launch).  One round trip, no
// barrier, no counter -- three dependent round trips (add, ticket, fetch)
// measured slower than the imbalance they were meant to cure, because under a
// saturated memory system each costs microseconds -- and only read-modify-write
// atomics touch that memory, so no cache write-back or invalidate is needed
// (device-wide fences cost an L2 write-back each on this part and made an earlier
// version 10-30x slower).  Every slice computes the rank-r term itself (8 KiB of
// R per slice, a few per cent more traffic) so that whichever slice arrives last
// can finish alone.  Integer addition is associative and every slice computes
// the same rank-r sums, so results are run-to-run identical.
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
  int region;                           // bytes of LDS per wave
  int lrx_off;                          // where in its region a wave keeps the token codes of a 4-bit R fragment
  const float* rscale;                  // scales of a 4-bit compensation matrix (r_dtype == SERQ_I4)
  unsigned long long* ws;               // [N/32][1024]: where the slices of a block meet, all zero between launches
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


constexpr int kRedPitch = 36;           // words per token row of a wave's parked partial sums


// Geometry of the token staging for one group of kGroup consecutive fragments (4 or 8).
template <int ABITS, int kGroup>
struct Stage {
  static constexpr int FB = 8 * ABITS;                  // bytes of one token's 64 channels
  static constexpr int P = kGroup * FB / 16;            // 16-byte pieces per token row: 8, 16 or 32
  static constexpr int RPI = 64 / P;                    // token rows one load instruction covers: 8, 4 or 2
  static constexpr int NI = 32 / RPI < 8 ? 32 / RPI : 8; // load instructions the kernel provides for: at most 8 KiB of token rows per group
  static constexpr int ROWB = P * 16;                   // 128, 256 or 512 bytes
  // xor applied to the piece index of row m: spreads 16 consecutive rows over the 16 bank groups
  // (rows of 128 bytes already alternate between two halves of the banks)
  static __device__ __forceinline__ int sw(int m) { return P >= 16 ? (m & 15) : ((m >> 1) & 7); }
};

template <int ABITS, int kWaves, int kGroup>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu((kGroup == 8 || kWaves == 4) ? 4 : 5, 8))) void serq_skinny_kernel(
    // needed before the first load is issued: passed one by one so that the dispatcher can preload them into SGPRs
    const uint8_t* hXq, const u4* hWq, int hK, int hM, int kb_per, int kb_rem, int hregion,
    const SkinnyParams p) {
  constexpr int kThreads = kWaves * 64;
  constexpr int SH = (ABITS == 8) ? 4 : 8;
  typedef Stage<ABITS, kGroup> S;
  extern __shared__ __align__(16) uint8_t lds[];        // per wave: token staging, then the partial sums

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int m = l & 31, g = l >> 5;
  // grid: (channel blocks, K slices); slices of kb_per fragments, the first kb_rem of them one longer
  const int nb = blockIdx.x, ks = blockIdx.y, ns = gridDim.y;
  const int KB = hK >> 6;
  const int kb0 = ks * kb_per + (ks < kb_rem ? ks : kb_rem);
  const int kb1 = kb0 + kb_per + (ks < kb_rem ? 1 : 0);
  const size_t rowbytes = (size_t)hK * ABITS / 8;

  const bool mv = m < hM;
  const uint8_t* xrow = hXq + (size_t)(mv ? m : 0) * rowbytes;
  const u4* wfr = hWq + (size_t)nb * KB * 64 + l;
  uint8_t* my = lds + (size_t)w * hregion;
  const uint32_t my_lds = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr(my));

  v16i acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0;

  // ---- cache-resident operands of the epilogue, requested first ---------------
  // the token codes of the rank-r term (slice 0 only; one fragment of R per wave is requested up front):
  // blocks of 16 salient channels for a 16-bit R, of 64 for a 4-bit one ...
  const bool has_lr = p.r > 0 && p.acc_out == nullptr;
  const bool lr_here = has_lr;                          // every slice computes it: whichever finishes the block needs it
  const bool lr_int = p.r_dtype == SERQ_I4;
  const int JB = lr_int ? (p.r + 63) >> 6 : p.r >> 4;  // fragments of R per channel block
  const bool bf = p.r_dtype == SERQ_BF16;
  const u4* rfr = p.Rp + (size_t)nb * JB * 64 + l;
  auto lr_load_x = [&](int jb) {
    u2 x = {0u, 0u};
    const int col = p.s_begin + jb * 16 + g * 8;        // first of this lane's 8 channels
    if (mv) {
      if constexpr (ABITS == 8) x = *(const u2*)(xrow + col);
      else x.x = *(const uint32_t*)(xrow + (col >> 1));
    }
    return x;
  };
  // 4-bit R: this lane's 32 (16) bytes of codes for fragment jf go straight to its own LDS slot
  auto lr_dma_x = [&](int jf) {
    const uint32_t off = (uint32_t)(mv ? m : 0) * (uint32_t)rowbytes +
                         (uint32_t)((p.s_begin + 64 * jf) * ABITS / 8 + g * (S::FB / 2));
    dma16(hXq, off, my_lds + (uint32_t)p.lrx_off);
    if constexpr (ABITS == 8) dma16(hXq, off + 16, my_lds + (uint32_t)p.lrx_off + 1024u);
  };
  const bool lr_first = lr_here && w < JB;
  u2 xc = {0u, 0u};
  if (lr_first) {
    if (lr_int) lr_dma_x(w);
    else xc = lr_load_x(w);
  }
  // ... and the scales of the outputs this thread will finish
  constexpr int NQ = 1024 / kThreads;
  float sc_m[NQ], sc_n[NQ], sc_r[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    sc_m[q] = sc_n[q] = sc_r[q] = 0.0f;
    if (p.acc_out == nullptr && (id >> 5) < hM) {       // any workgroup may be the one that finishes its block
      sc_m[q] = p.scale[id >> 5];
      sc_n[q] = p.wscale[nb * 32 + (id & 31)];
      if (has_lr && lr_int) sc_r[q] = p.rscale[nb * 32 + (id & 31)];
    }
  }
  u4 rf = {0u, 0u, 0u, 0u};
  if (lr_first) rf = __builtin_nontemporal_load(&rfr[(size_t)w * 64]);

  // ---- the integer contraction over this workgroup's K slice ------------------
  // staging role of this lane: row srow0 + RPI*j of instruction j, slot l % P of the row
  const int srow0 = l / S::P, slot = l % S::P;
  const int nfr = kb1 - kb0;                            // fragments in the slice
  const uint8_t* xslice = hXq + (size_t)kb0 * S::FB;
#pragma unroll 1
  for (int gi = w; gi * kGroup < nfr; gi += kWaves) {
    const int f0 = gi * kGroup;                         // first fragment of the group, relative to the slice
    // token rows of the group straight into LDS, whole lines, ahead of the weight loads
#pragma unroll
    for (int j = 0; j < S::NI; ++j) {
      if (S::RPI * j < hM) {                           // uniform
        const int row = srow0 + S::RPI * j;
        const int rowc = row < hM ? row : hM - 1;     // rows past M: any valid address, never read back
        int col = f0 * S::FB + ((slot ^ S::sw(row)) << 4);
        col = col < nfr * S::FB ? col : 0;              // pieces past a ragged slice likewise
        dma16(xslice, (uint32_t)rowc * (uint32_t)rowbytes + (uint32_t)col, my_lds + 1024u * j);
      }
    }
    u4 wp[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const bool ok = f0 + u < nfr;
      wp[u] = __builtin_nontemporal_load(&wfr[(size_t)(kb0 + (ok ? f0 + u : 0)) * 64]);   // streamed once: do not keep it in the caches
      if (!ok) wp[u] = u4{0u, 0u, 0u, 0u};              // zero weights contribute nothing
    }
    // the kGroup weight loads are the only vector-memory operations younger than the token rows
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kGroup) : "memory");
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      if (f0 + u >= kb1 - kb0) break;                   // uniform over the wave
      v4i a0, a1, b0, b1;
      unpack_frag(wp[u], a0, a1);
      b0 = (v4i){0, 0, 0, 0};
      b1 = (v4i){0, 0, 0, 0};
      if (mv) {
        const uint8_t* xr = my + m * S::ROWB;
        if constexpr (ABITS == 8) {
          b0 = *(const v4i*)(xr + (((4 * u + 2 * g) ^ S::sw(m)) << 4));
          b1 = *(const v4i*)(xr + (((4 * u + 2 * g + 1) ^ S::sw(m)) << 4));
        } else {
          unpack_frag(*(const u4*)(xr + (((2 * u + g) ^ S::sw(m)) << 4)), b0, b1);
        }
      }
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, acc, 0, 0, 0);
    }
  }

  // ---- the rank-r term ----------------------------------------------------------
  // its sums: fp32 bit patterns for a 16-bit R, INT32 (times 2^SH like the main sums) for a 4-bit one
  v16i accl;
#pragma unroll
  for (int e = 0; e < 16; ++e) accl[e] = 0;
  auto lr_mfma = [&](const u4& r_in, const u2& x_in) {
    int c[8];
    if constexpr (ABITS == 8) codes_from_a8(x_in.x, x_in.y, c);
    else codes_from_a4(x_in.x, c);
    u4 xf = codes8_to_16bit(c, bf);                     // zero codes for lanes without a token
    v16f af = __builtin_bit_cast(v16f, accl);
    if (bf)
      af = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, r_in), __builtin_bit_cast(v8bf, xf), af, 0, 0, 0);
    else
      af = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, r_in), __builtin_bit_cast(v8h, xf), af, 0, 0, 0);
    accl = __builtin_bit_cast(v16i, af);
  };
  auto lr_mfma_int = [&](const u4& r_in) {              // one 64-rank fragment of Q(R) against the parked codes
    v4i a0, a1, b0, b1;
    unpack_frag(r_in, a0, a1);
    b0 = (v4i){0, 0, 0, 0};
    b1 = (v4i){0, 0, 0, 0};
    if (mv) {
      const uint8_t* xp = my + p.lrx_off + l * 16;
      if constexpr (ABITS == 8) {
        b0 = *(const v4i*)xp;
        b1 = *(const v4i*)(xp + 1024);
      } else {
        unpack_frag(*(const u4*)xp, b0, b1);
      }
    }
    accl = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, accl, 0, 0, 0);
    accl = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, accl, 0, 0, 0);
  };
  if (lr_here && lr_int) {
    if (lr_first) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the parked codes (a wave without a group never waited)
      lr_mfma_int(rf);
    }
    for (int jf = w + kWaves; jf < JB; jf += kWaves) {  // fragments beyond the first of each wave
      lr_dma_x(jf);
      const u4 r1 = __builtin_nontemporal_load(&rfr[(size_t)jf * 64]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      lr_mfma_int(r1);
    }
  } else if (lr_here) {
    if (lr_first) lr_mfma(rf, xc);
    for (int jb = w + kWaves; jb < JB; jb += kWaves) {  // ranks beyond the first block of each wave
      const u4 r1 = __builtin_nontemporal_load(&rfr[(size_t)jb * 64]);
      lr_mfma(r1, lr_load_x(jb));
    }
  }

  // ---- combine the waves ----------------------------------------------------
  // accumulator registers 4i..4i+3 of lane l hold channels 8i + 4*(l/32) + 0..3 of
  // the block for token l%32; only tokens < M are exchanged.  A wave parks its
  // partials in its own region (dead as token staging by now) as [token][channel]
  // rows of kRedPitch words -- four 16-byte writes per lane, and a pitch of 9
  // bank groups keeps both the writes and the gather conflict-free -- with the
  // rank-r partials M rows further.
  // Thread tid finishes (token q/32, channel q%32) for q = tid, tid + kThreads, ...
  const int nwl = JB < kWaves ? JB : kWaves;              // waves that hold low-rank sums
  if (mv) {
    int* red = reinterpret_cast<int*>(my) + m * kRedPitch + 4 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<v4i*>(red + 8 * i) = (v4i){acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
    if (lr_here && w < nwl) {
      int* redl = red + hM * kRedPitch;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<v4i*>(redl + 8 * i) = (v4i){accl[4 * i], accl[4 * i + 1], accl[4 * i + 2], accl[4 * i + 3]};
    }
  }
  __syncthreads();
  int tot_i[NQ], tot_l[NQ];                               // rank-r sums as words: fp32 bits or INT32
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    const int nl = id & 31, mt = id >> 5;
    tot_i[q] = tot_l[q] = 0;
    if (mt >= hM) continue;
    const int src = mt * kRedPitch + nl;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) tot_i[q] += *reinterpret_cast<const int*>(lds + (size_t)ww * hregion + 4 * src);
    if (lr_here) {
      int li = 0;
      float lf = 0.0f;
      for (int ww = 0; ww < nwl; ++ww) {
        const int word = *reinterpret_cast<const int*>(lds + (size_t)ww * hregion + 4 * (hM * kRedPitch + src));
        if (lr_int) li += word;
        else lf += __int_as_float(word);
      }
      tot_l[q] = lr_int ? li : __float_as_int(lf);
    }
  }

  unsigned long long* wsb = p.ws + (size_t)nb * 1024;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    const int nl = id & 31, mt = id >> 5;
    if (mt >= hM) continue;
    int total = tot_i[q];
    if (ns > 1) {                                         // uniform over the workgroup
      const long long mine = (1ll << 40) + (long long)tot_i[q];
      const long long old = (long long)__hip_atomic_fetch_add(wsb + id, (unsigned long long)mine, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT);
      const long long arrived = (old + (1ll << 39)) >> 40;
      if (arrived != ns - 1) continue;                    // someone after us finishes this output
      total += (int)(old - (arrived << 40));
      __hip_atomic_store(wsb + id, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const float lr = !has_lr ? 0.0f : (lr_int ? sc_r[q] * (float)(tot_l[q] >> SH) : __int_as_float(tot_l[q]));
    finish(p, mt, nb * 32 + nl, total >> SH, lr, sc_m[q], sc_n[q]);   // exact shifts: the sums are multiples of 2^SH
  }
}

}  // namespace

size_t skinny_workspace_bytes(int N) {
  return (size_t)N / 32 * 1024 * 8;                      // one 64-bit word per output of a 32-token block
}

int launch_skinny(const LinearArgs& a, hipStream_t st) {
  const int ncu = device_cu_count();
  SkinnyParams p;
  p.Xq = a.Xq; p.scale = a.scale; p.Wq = a.Wq; p.wscale = a.wscale;
  p.Rp = a.Rp; p.r_dtype = a.r_dtype; p.s_begin = a.s_begin; p.r = a.Rp ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  p.acc_out = a.acc_out; p.ldacc = a.ldacc;
  p.rscale = a.rscale;
  const int KB = a.K / 64;
  const int nblk = a.N / 32;
  const bool have_ws = a.workspace != nullptr && a.workspace_bytes >= skinny_workspace_bytes(a.N);

  // K slices per block: as requested by the flags, else as many as it takes to have about one
  // workgroup per CU when there are fewer blocks than CUs (needs the workspace; without it, none).
  int nsplit = 1;
  if (a.splitk > 1) {
    if (!have_ws) return SERQ_EWORKSPACE;               // an explicit request cannot be honoured
    nsplit = a.splitk;
  } else if (a.splitk == 0 && have_ws && nblk < ncu) {
    nsplit = ncu / nblk;
    const int smax = KB / 8;                            // a slice keeps at least 8 fragments
    if (nsplit > smax) nsplit = smax;
    if (nsplit > 16) nsplit = 16;
  }
  if (nsplit > KB) nsplit = KB;
  if (nsplit < 1) nsplit = 1;
  p.ws = have_ws ? (unsigned long long*)a.workspace : nullptr;

  // Waves per workgroup: 8 once the longest piece gives each of them a group of fragments, else 4.
  // (16-wave workgroups measured slower: their registers and LDS allow one workgroup per CU where two
  // or three smaller ones overlap each other's start-up and epilogue.)
  const int KBs = (KB + nsplit - 1) / nsplit;           // longest slice, in fragments
  int nw = a.skinny_waves;
  if (nw != 4 && nw != 8) nw = KBs >= 32 ? 8 : 4;
  // Fragments per group: 8 when every wave gets a full group of 8 and the token rows of such a group
  // stay within 8 KiB of LDS per wave, else 4.
  const int rowb8 = 8 * 8 * a.abits / 16 * 16;          // bytes of a token row of a group of 8
  const int rpi8 = 1024 / rowb8;
  const bool can8 = (a.M + rpi8 - 1) / rpi8 * rpi8 * rowb8 <= 8192;
  const int grp = (KBs >= 8 * nw && can8) ? 8 : 4;
  // LDS per wave: the token rows of one group, later the wave's partial sums
  const int rowb = grp * 8 * a.abits / 16 * 16;
  const int rpi = 1024 / rowb;
  const int rows = (a.M + rpi - 1) / rpi * rpi;
  const bool has_lr = p.r > 0 && p.acc_out == nullptr;
  int region = rows * rowb;
  p.lrx_off = region;
  if (has_lr && a.r_dtype == SERQ_I4) region += a.abits == 8 ? 2048 : 1024;
  const int red = (has_lr ? 2 : 1) * a.M * kRedPitch * 4;
  if (red > region) region = red;
  region = (region + 15) & ~15;
  p.region = region;
  const size_t lds_bytes = (size_t)region * nw;

  dim3 grid((unsigned)nblk, (unsigned)nsplit), block((unsigned)nw * 64);
#define SERQ_SKINNY_LAUNCH(AB, NW, G) hipLaunchKernelGGL((serq_skinny_kernel<AB, NW, G>), grid, block, lds_bytes, st, p.Xq, p.Wq, p.K, p.M, KB / nsplit, KB % nsplit, p.region, p)
  if (a.abits == 8) {
    if (nw == 4) { if (grp == 4) SERQ_SKINNY_LAUNCH(8, 4, 4); else SERQ_SKINNY_LAUNCH(8, 4, 8); }
    else { if (grp == 4) SERQ_SKINNY_LAUNCH(8, 8, 4); else SERQ_SKINNY_LAUNCH(8, 8, 8); }
  } else {
    if (nw == 4) { if (grp == 4) SERQ_SKINNY_LAUNCH(4, 4, 4); else SERQ_SKINNY_LAUNCH(4, 4, 8); }
    else { if (grp == 4) SERQ_SKINNY_LAUNCH(4, 8, 4); else SERQ_SKINNY_LAUNCH(4, 8, 8); }
  }
#undef SERQ_SKINNY_LAUNCH
  if (hipGetLastError() != hipSuccess) return SERQ_EHIP;
  return SERQ_OK;
}

}  // namespace serq
