// MXFP4 layer for decode-sized batches (M <= 32): an HBM-bound kernel that streams every weight
// fragment and every block scale exactly once (the MXFP4 form of Eq. 7, second line; see gemm_mx.hip):
//   Y[m,n] = sum_k X^[m,k] W^[n,k] + sum_{j<r} X^[m,s_begin+j] R^[n,j]
//
// Same decomposition as the integer decode kernel: a workgroup of 4 or 8 waves owns one block of 32
// output channels and all of K; wave w takes the groups w, w+W, ... of four or eight consecutive
// 1-KiB weight fragments (one coalesced 16-byte load per lane and fragment, the whole group in flight
// before its first fragment is used); the token codes of a group travel by whole-line direct-to-LDS
// loads into a wave-private, xor-swizzled LDS region, issued before the weight loads, and one
// hand-counted wait on "all but the weight loads" covers them; no barrier in the main loop.
// A fragment is one block-scaled FP4 MFMA (32 channels x 32 tokens x 64 input channels; a lane's 16
// bytes are the operand as stored) whose B operand is the token block (rows >= M are zero codes).
// Scales: the weight scales of a 256-channel tile are one dword per lane (256 contiguous bytes per
// wave, streamed), the token scales 8 bytes per token and tile (from L2), reordered by one
// v_perm_b32 so that byte c belongs to fragment c of the tile.  The compensation fragments are
// further fragments of the same loop, dealt to the waves after the main ones, with the token codes
// of the salient block read straight from memory.  The sums are fp32 from the start; the waves are
// combined through LDS in a fixed order, so results are run-to-run identical.
//
// When N alone gives fewer workgroups than there are CUs and K is long, K is cut into slices of whole
// 256-channel scale tiles (blockIdx.y), and the slices of a block meet in the workspace.  fp32 sums cannot meet in
// one integer atomic as the integer kernel's do, so each output takes two dependent round trips, both
// returning read-modify-write atomics at agent scope (the only kind of access that needs no cache
// write-back or invalidate here): a slice publishes its partial sum with an exchange into its own
// slot, waits for the exchange to return, and takes a ticket from the output's counter; the slice that
// draws the last ticket exchanges every slot back to zero in slice order, adds what it gets in that
// fixed order (run-to-run identical results) and stores the output; it also clears the counter, so
// the workspace is clean for the next launch.  The compensation fragments belong to slice 0.
#include <type_traits>

#include "serq_device.h"

namespace serq {
namespace {

constexpr int kRedPitch = 36;           // words per token row of a wave's parked partial sums
constexpr int kMaxSlices = 16;


struct SkinnyMxParams {
  const uint8_t* Xq; const uint8_t* xsc;
  const u4* Wq; const uint8_t* wsc;
  const u4* Rq; const uint8_t* rsc; int s_begin; int r;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int region;                           // bytes of LDS per wave
  int unit_per, unit_rem;               // K slices in scale tiles (4 fragments): unit_per each, the first unit_rem one more
  uint32_t* cnt;                        // [N/32][1024] tickets, all zero between launches
  uint32_t* slots;                      // [N/32][slices][1024] published partial sums (fp32 bits), likewise
};

// Geometry of the token staging for one group of kGroup consecutive fragments (4 or 8): a token's
// 64 channels are 32 bytes.
template <int kGroup>
struct Stage {
  static constexpr int FB = 32;
  static constexpr int P = kGroup * FB / 16;            // 16-byte pieces per token row: 8 or 16
  static constexpr int RPI = 64 / P;                    // token rows one load instruction covers: 8 or 4
  static constexpr int NI = 32 / RPI;                   // load instructions for 32 rows: 4 or 8
  static constexpr int ROWB = P * 16;                   // 128 or 256 bytes
  static __device__ __forceinline__ int sw(int m) { return P >= 16 ? (m & 15) : ((m >> 1) & 7); }
};

template <int kWaves, int kGroup>
__global__ __launch_bounds__(kWaves * 64) void serq_skinny_mx_kernel(const SkinnyMxParams p) {
  constexpr int kThreads = kWaves * 64;
  typedef Stage<kGroup> S;
  constexpr int NT = kGroup / 4;                        // 256-channel scale tiles per group
  extern __shared__ __align__(16) uint8_t lds[];        // per wave: token staging, then the partial sums

  const int tid = threadIdx.x;
  const int w = tid >> 6, l = tid & 63;
  const int m = l & 31, g = l >> 5;
  const int nb = blockIdx.x, ks = blockIdx.y, ns = gridDim.y;
  const int hM = p.M;
  const int KB = p.K >> 6;
  const int T = (KB + 3) >> 2;                          // scale tiles of a channel block
  // this workgroup's fragments [kb0, kb1): whole scale tiles
  const int u0 = ks * p.unit_per + (ks < p.unit_rem ? ks : p.unit_rem);
  const int u1 = u0 + p.unit_per + (ks < p.unit_rem ? 1 : 0);
  const int kb0 = 4 * u0;
  const int kb1 = 4 * u1 < KB ? 4 * u1 : KB;
  const size_t rowbytes = (size_t)p.K >> 1;
  const size_t Mp = (size_t)((hM + 1) & ~1);

  const bool mv = m < hM;
  const int mc = mv ? m : 0;
  const u4* wfr = p.Wq + (size_t)nb * KB * 64 + l;
  const uint32_t* wsl = (const uint32_t*)p.wsc + (size_t)nb * T * 64 + l;
  uint8_t* my = lds + (size_t)w * p.region;
  const uint32_t my_lds = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr(my));
  const uint32_t xsel = g ? 0x07050301u : 0x06040200u;  // bytes g, 2+g, 4+g, 6+g of a token's 8 scales

  v16f acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.0f;

  // token scales of 256-channel tile t for this lane's token, byte c = fragment c of the tile
  auto token_scales = [&](int t) -> uint32_t {
    const u2 e = *(const u2*)(p.xsc + ((size_t)t * Mp + (size_t)mc) * 8);
    return __builtin_amdgcn_perm(e.y, e.x, xsel);
  };

  // ---- the main fragments ---------------------------------------------------------
  const int srow0 = l / S::P, slot = l % S::P;
#pragma unroll 1
  for (int gi = w; kb0 + gi * kGroup < kb1; gi += kWaves) {
    const int f0 = kb0 + gi * kGroup;                   // first fragment of the group (a multiple of 4)
    // token rows of the group straight into LDS, whole lines, ahead of the weight loads
#pragma unroll
    for (int j = 0; j < S::NI; ++j) {
      if (S::RPI * j < hM) {                           // uniform
        const int row = srow0 + S::RPI * j;
        const int rowc = row < hM ? row : hM - 1;     // rows past M: any valid address, never read back
        int col = f0 * S::FB + ((slot ^ S::sw(row)) << 4);
        col = col < kb1 * S::FB ? col : 0;              // pieces past the slice likewise
        dma16(p.Xq, (uint32_t)rowc * (uint32_t)rowbytes + (uint32_t)col, my_lds + 1024u * j);
      }
    }
    uint32_t xs[NT], wsd[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const int t = (f0 >> 2) + i;
      const int tc = t < T ? t : T - 1;
      xs[i] = token_scales(tc);
      wsd[i] = __builtin_nontemporal_load(&wsl[(size_t)tc * 64]);
    }
    u4 wp[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      const bool ok = f0 + u < kb1;
      wp[u] = __builtin_nontemporal_load(&wfr[(size_t)(ok ? f0 + u : 0) * 64]);   // streamed once: do not keep it in the caches
      if (!ok) wp[u] = u4{0u, 0u, 0u, 0u};              // zero codes contribute nothing
    }
    // at most the kGroup weight loads and the scale loads are younger than the token rows
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kGroup) : "memory");
    auto frag = [&](auto u_c) {
      constexpr int u = decltype(u_c)::value;
      if constexpr (u < kGroup) {
        if (f0 + u < kb1) {                             // uniform over the wave
          u4 xb = {0u, 0u, 0u, 0u};
          if (mv) xb = *(const u4*)(my + m * S::ROWB + (((2 * u + g) ^ S::sw(m)) << 4));
          acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(wp[u]), fp4_operand(xb), acc, 4, 4, u & 3,
                                                                (int)wsd[u >> 2], u & 3, (int)xs[u >> 2]);
        }
      }
    };
    frag(std::integral_constant<int, 0>{}); frag(std::integral_constant<int, 1>{});
    frag(std::integral_constant<int, 2>{}); frag(std::integral_constant<int, 3>{});
    frag(std::integral_constant<int, 4>{}); frag(std::integral_constant<int, 5>{});
    frag(std::integral_constant<int, 6>{}); frag(std::integral_constant<int, 7>{});
  }

  // ---- the compensation fragments: 64 ranks each, dealt to the waves one at a time ----------
  const int FR = (p.Rq && ks == 0) ? (p.r + 63) >> 6 : 0;
  const int TR = (FR + 3) >> 2;
#pragma unroll 1
  for (int jf = w; jf < FR; jf += kWaves) {
    const u4 rq = __builtin_nontemporal_load(&p.Rq[((size_t)nb * FR + jf) * 64 + l]);
    const uint32_t rs = ((const uint32_t*)p.rsc)[((size_t)nb * TR + (jf >> 2)) * 64 + l] >> (8 * (jf & 3));
    const uint32_t xs = token_scales((p.s_begin >> 8) + (jf >> 2)) >> (8 * (jf & 3));
    u4 xb = {0u, 0u, 0u, 0u};
    if (mv) xb = *(const u4*)(p.Xq + (size_t)m * rowbytes + ((p.s_begin + 64 * jf) >> 1) + 16 * g);
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(rq), fp4_operand(xb), acc, 4, 4, 0, (int)rs, 0, (int)xs);
  }

  // ---- combine the waves ------------------------------------------------------------
  // accumulator registers 4i..4i+3 of lane l hold channels 8i + 4*(l/32) + 0..3 of the block for token
  // l%32; only tokens < M are exchanged.  A wave parks its partials in its own region (dead as token
  // staging by now: its own LDS reads have completed) as [token][channel] rows of kRedPitch words.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  if (mv) {
    float* red = reinterpret_cast<float*>(my) + m * kRedPitch + 4 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<v4f*>(red + 8 * i) = (v4f){acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
  }
  __syncthreads();
  constexpr int NQ = 1024 / kThreads;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + q * kThreads;
    const int nl = id & 31, mt = id >> 5;
    if (mt >= hM) continue;
    float tot = 0.0f;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww)
      tot += *reinterpret_cast<const float*>(lds + (size_t)ww * p.region + 4 * (mt * kRedPitch + nl));
    if (ns > 1) {                                         // uniform over the workgroup
      uint32_t* slot0 = p.slots + ((size_t)nb * ns) * 1024 + id;
      const uint32_t prev = __hip_atomic_exchange(slot0 + (size_t)ks * 1024, __float_as_uint(tot), __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
      // the ticket is taken only after the exchange has returned, i.e. has been performed: the increment
      // is made to depend on the returned value (always zero: the slot was clean)
      uint32_t one = 1u;
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(one) : "v"(prev) : "memory");
      const uint32_t ticket = __hip_atomic_fetch_add(p.cnt + (size_t)nb * 1024 + id, one, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
      if (ticket != (uint32_t)(ns - 1)) continue;         // a later slice finishes this output
      // all the exchanges are issued before the first result is used: one round trip, not one per slice
      uint32_t part[kMaxSlices];
#pragma unroll
      for (int k = 0; k < kMaxSlices; ++k)
        part[k] = k < ns ? __hip_atomic_exchange(slot0 + (size_t)k * 1024, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                         : 0u;
      tot = 0.0f;
#pragma unroll
      for (int k = 0; k < kMaxSlices; ++k)
        if (k < ns) tot += __uint_as_float(part[k]);
      __hip_atomic_store(p.cnt + (size_t)nb * 1024 + id, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const size_t o = (size_t)mt * p.ldy + nb * 32 + nl;
    if (p.y_dtype == SERQ_F32) ((float*)p.Y)[o] = tot;
    else if (p.y_dtype == SERQ_BF16) ((uint16_t*)p.Y)[o] = f32_to_bf16_rne(tot);
    else ((uint16_t*)p.Y)[o] = f32_to_f16_rne(tot);
  }
}

}  // namespace

size_t skinny_mx_workspace_bytes(int N) {
  return (size_t)N / 32 * 1024 * 4 * (1 + kMaxSlices);   // tickets, then one slot per slice and output
}

int launch_skinny_mx(const MxLinearArgs& a, hipStream_t st) {
  const int ncu = device_cu_count();
  SkinnyMxParams p;
  p.Xq = a.Xq; p.xsc = a.xsc; p.Wq = a.Wq; p.wsc = a.wsc;
  p.Rq = a.r > 0 ? a.Rq : nullptr; p.rsc = a.rsc; p.s_begin = a.s_begin; p.r = a.Rq ? a.r : 0;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.Y = a.Y; p.y_dtype = a.y_dtype; p.ldy = a.ldy;
  const int KB = a.K / 64;
  const int T = (KB + 3) / 4;                            // scale tiles: the unit K is sliced in
  const int nblk = a.N / 32;
  const bool have_ws = a.workspace != nullptr && a.workspace_bytes >= skinny_mx_workspace_bytes(a.N);
  // K slices per block: as requested by the flags; else, when the blocks fill at most a quarter of
  // the CUs and a block is at least 128 fragments long (K >= 8192), as many as it takes to have about
  // one workgroup per CU with slices of at least 32 fragments.  The meeting costs two memory round
  // trips (about 0.7 us): measured on 16 .. 128 blocks, more blocks, shorter blocks or shorter slices
  // lose as much as they gain (16 blocks x K = 16384: 7.7 -> 4.6 us with 8 slices; 32 x 8192: 5.2 -> 4.5;
  // 64 x 8192: 5.4 -> 5.0; 128 x 11008: 7.3 -> 7.2 .. 7.7).  Needs the workspace; without it, none.
  int nsplit = 1;
  if (a.splitk > 1) {
    if (!have_ws) return SERQ_EWORKSPACE;                // an explicit request cannot be honoured
    nsplit = a.splitk;
  } else if (a.splitk == 0 && have_ws && 4 * nblk <= ncu && KB >= 128) {
    nsplit = ncu / nblk;
    const int smax = T / 8;
    if (nsplit > smax) nsplit = smax;
  }
  if (nsplit > kMaxSlices) nsplit = kMaxSlices;
  if (nsplit > T) nsplit = T;
  if (nsplit < 1) nsplit = 1;
  p.unit_per = T / nsplit;
  p.unit_rem = T % nsplit;
  p.cnt = (uint32_t*)a.workspace;
  p.slots = p.cnt ? p.cnt + (size_t)nblk * 1024 : nullptr;
  // Waves per workgroup: 8 once each of them gets a group of fragments of the longest slice, else 4;
  // groups of 8 fragments when every wave gets a full one.
  const int KBs = 4 * ((T + nsplit - 1) / nsplit);
  const int nw = KBs >= 32 ? 8 : 4;
  const int grp = KBs >= 8 * nw ? 8 : 4;
  // LDS per wave: the token rows of one group (a multiple of the rows one load covers), later its partial sums
  const int rowb = grp * 32;
  const int rpi = 1024 / rowb;
  const int rows = (a.M + rpi - 1) / rpi * rpi;
  int region = rows * rowb;
  const int red = a.M * kRedPitch * 4;
  if (red > region) region = red;
  region = (region + 15) & ~15;
  p.region = region;
  const size_t lds_bytes = (size_t)region * nw;
  dim3 grid((unsigned)nblk, (unsigned)nsplit), block((unsigned)nw * 64);
#define SERQ_SKINNY_MX_LAUNCH(NW, G) hipLaunchKernelGGL((serq_skinny_mx_kernel<NW, G>), grid, block, lds_bytes, st, p)
  if (nw == 4) { if (grp == 4) SERQ_SKINNY_MX_LAUNCH(4, 4); else SERQ_SKINNY_MX_LAUNCH(4, 8); }
  else { if (grp == 4) SERQ_SKINNY_MX_LAUNCH(8, 4); else SERQ_SKINNY_MX_LAUNCH(8, 8); }
#undef SERQ_SKINNY_MX_LAUNCH
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

}  // namespace serq
