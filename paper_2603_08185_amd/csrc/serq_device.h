// Device-side helpers shared by the SERQ kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/serq.h"

namespace serq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
// native vectors for anything staged in registers (aggregate vector structs
// would be kept in memory and moved around with memcpy)
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// Private packed layouts (all produced by the library itself).
//
// Weight blob Wq: [N/32][K/64] fragments of 1 KiB.  Fragment (nb,kb) holds the
// 32 output channels n = 32*nb + (lane & 31) and the 64 input channels
// 64*kb .. 64*kb+63.  Lane `lane` owns 16 bytes = 4 dwords; dword d covers the
// 8 channels k0 = 64*kb + 32*(lane>>5) + 8*d .. k0+7, and byte j of that dword
// holds channel k0+j in its low nibble and channel k0+4+j in its high nibble
// (two's complement).  One wave-wide 16-byte load therefore brings in exactly
// the A operands of two 32x32x32 int8 MFMAs, and
//      lo = (w << 4) & 0xF0F0F0F0,   hi = w & 0xF0F0F0F0
// are operand dwords holding 16*q for channels k0..k0+3 and k0+4..k0+7.
//
// Activations Xq, 8-bit: int8 [M][K], natural order.
// Activations Xq, 4-bit: [M][K/2] bytes; each dword covers 8 consecutive
// channels with the same nibble interleave as the weights.
//
// Low-rank blob Rp: [N/32][r/16] fragments of 1 KiB; lane owns 8 consecutive
// 16-bit elements R[16*jb + 8*(lane>>5) + p][32*nb + (lane & 31)], p = 0..7:
// the A operand of one 32x32x16 f16/bf16 MFMA.
// ---------------------------------------------------------------------------

constexpr uint32_t kNibMask = 0xF0F0F0F0u;

// 16x the signed nibbles of w, as two int8x4 operand dwords.
__device__ __forceinline__ void unpack16(uint32_t w, int& lo, int& hi) {
  lo = (int)((w << 4) & kNibMask);
  hi = (int)(w & kNibMask);
}

// One 16-byte packed fragment piece -> the operands of two K=32 MFMA steps.
__device__ __forceinline__ void unpack_frag(const u4& p, v4i& t0, v4i& t1) {
  int a, b;
  unpack16(p.x, a, b); t0.x = a; t0.y = b;
  unpack16(p.y, a, b); t0.z = a; t0.w = b;
  unpack16(p.z, a, b); t1.x = a; t1.y = b;
  unpack16(p.w, a, b); t1.z = a; t1.w = b;
}

__device__ __forceinline__ v4i as_v4i(const u4& p) { return __builtin_bit_cast(v4i, p); }

// storage-type helpers -------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ float f16_to_f32(uint16_t u) { return (float)__builtin_bit_cast(_Float16, u); }
// silu(g) * u in fp32 with the hardware's exp2 and reciprocal (an ulp each, so the product is good to
// a few ulps; the correctly rounded expf and an IEEE division made the fused quantisers VALU-bound);
// g -> -inf gives g * 0 = -0, g -> +inf gives g * 1
__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// ---- helpers shared by several kernels -------------------------------------------------------------
// LDS byte address of a pointer into shared memory
__device__ __forceinline__ uint32_t lds_addr(const void* ptr) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)ptr;
}
// Direct global -> LDS load, 16 bytes per lane, no staging registers: global (sbase + voff) lands at
// LDS (lds_base_uniform + 16 * lane).  Counted by hand with vmcnt by the callers.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base_uniform), "v"(voff), "s"(sbase) : "memory", "m0");
}
// 16 bytes of E2M1 codes as an operand of the block-scaled MFMA (its FP4 forms read the first 16 bytes only)
__device__ __forceinline__ v8i fp4_operand(const u4& v) {
  const v4i q = as_v4i(v);
  return __builtin_shufflevector(q, q, 0, 1, 2, 3, -1, -1, -1, -1);
}
// 8 consecutive channels (piece `chunk`) of a row stored as XDT, as fp32
template <int XDT>
__device__ __forceinline__ void load8(const void* row, int chunk, float v[8]) {
  if constexpr (XDT == SERQ_F32) {
    const float4* p = (const float4*)row + 2 * (size_t)chunk;
    float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
    uint4 u = ((const uint4*)row)[chunk];
    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (XDT == SERQ_BF16) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      } else {
        v[2 * i] = f16_to_f32((uint16_t)(w[i] & 0xffffu));
        v[2 * i + 1] = f16_to_f32((uint16_t)(w[i] >> 16));
      }
    }
  }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  v2f x = {f, 0.0f};
  v2bf y = __builtin_convertvector(x, v2bf);
  return (uint16_t)(__builtin_bit_cast(uint32_t, y) & 0xffffu);
}
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float a, float b) {
  v2f x = {a, b};
  v2bf y = __builtin_convertvector(x, v2bf);
  return __builtin_bit_cast(uint32_t, y);
}
__device__ __forceinline__ uint32_t f32x2_to_f16x2(float a, float b) {
  v2f x = {a, b};
  v2h y = __builtin_convertvector(x, v2h);
  return __builtin_bit_cast(uint32_t, y);
}
__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}

template <int DT> struct Elem;
template <> struct Elem<SERQ_F32> {
  typedef float T;
  static __device__ __forceinline__ float ld(const void* p, size_t i) { return ((const float*)p)[i]; }
};
template <> struct Elem<SERQ_F16> {
  typedef uint16_t T;
  static __device__ __forceinline__ float ld(const void* p, size_t i) { return f16_to_f32(((const uint16_t*)p)[i]); }
};
template <> struct Elem<SERQ_BF16> {
  typedef uint16_t T;
  static __device__ __forceinline__ float ld(const void* p, size_t i) { return bf16_to_f32(((const uint16_t*)p)[i]); }
};

__device__ __forceinline__ float ld_any(const void* p, int dt, size_t i) {
  if (dt == SERQ_F32) return ((const float*)p)[i];
  if (dt == SERQ_F16) return f16_to_f32(((const uint16_t*)p)[i]);
  return bf16_to_f32(((const uint16_t*)p)[i]);
}

// 8 signed codes -> 8 exact 16-bit floats (|code| <= 128 is exact in both formats).
// `lo`,`hi` hold the codes as bytes c0..c3 / c4..c7.
__device__ __forceinline__ u4 codes8_to_16bit(int c[8], bool bf16) {
  u4 o;
  if (bf16) {
    o.x = f32x2_to_bf16x2((float)c[0], (float)c[1]);
    o.y = f32x2_to_bf16x2((float)c[2], (float)c[3]);
    o.z = f32x2_to_bf16x2((float)c[4], (float)c[5]);
    o.w = f32x2_to_bf16x2((float)c[6], (float)c[7]);
  } else {
    o.x = f32x2_to_f16x2((float)c[0], (float)c[1]);
    o.y = f32x2_to_f16x2((float)c[2], (float)c[3]);
    o.z = f32x2_to_f16x2((float)c[4], (float)c[5]);
    o.w = f32x2_to_f16x2((float)c[6], (float)c[7]);
  }
  return o;
}

// the 8 codes of channels k0..k0+7 from an 8-bit row (two dwords) ...
__device__ __forceinline__ void codes_from_a8(uint32_t d0, uint32_t d1, int c[8]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    c[j] = __builtin_amdgcn_sbfe((int)d0, 8 * j, 8);
    c[4 + j] = __builtin_amdgcn_sbfe((int)d1, 8 * j, 8);
  }
}
// ... and from one interleaved 4-bit dword.
__device__ __forceinline__ void codes_from_a4(uint32_t d, int c[8]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    c[j] = __builtin_amdgcn_sbfe((int)d, 8 * j, 4);
    c[4 + j] = __builtin_amdgcn_sbfe((int)d, 8 * j + 4, 4);
  }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// Number of compute units of the current device, asked on every call (the library keeps no state);
// 256 if the runtime cannot say.
inline int device_cu_count() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  return n;
}

// ---------------------------------------------------------------------------
// host-side launchers implemented in the individual .hip files
// ---------------------------------------------------------------------------
struct LinearArgs {
  const uint8_t* Xq; const float* scale; int abits;
  const u4* Wq; const float* wscale;
  int s_begin; int r; const u4* Rp; int r_dtype;
  const float* rscale;                  // r_dtype == SERQ_I4: the per-channel scales inside the blob Rp
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int32_t* acc_out; int64_t ldacc;      // non-NULL: store raw accumulators instead of Y
  void* workspace; size_t workspace_bytes;
  int splitk; int groupm; int coltiles; int skinny_waves;
};

size_t skinny_workspace_bytes(int N);
int launch_skinny(const LinearArgs& a, hipStream_t st);
int launch_mfma(const LinearArgs& a, hipStream_t st);
size_t mfma_split_workspace_bytes(int M, int N, int K, int abits, int forced);
int launch_quantize_act(const void* X, const void* U, int x_dtype, const float* s_inv, int64_t M, int K, int64_t ldx,
                        int64_t ldu, int abits, void* Xq, float* scale, hipStream_t st);

int launch_mfma_peak(const void* operands, int iters, int workgroups, void* sink, hipStream_t st);
int launch_mfma_fp4_peak(const void* operands, int iters, int workgroups, int scale_a, int scale_b, void* sink,
                         hipStream_t st);
int launch_read_peak(const void* src, size_t bytes, int workgroups, void* sink, hipStream_t st);

// MXFP4 path (mx.hip, gemm_mx.hip)
struct MxLinearArgs {
  const uint8_t* Xq; const uint8_t* xsc;
  const u4* Wq; const uint8_t* wsc;
  int s_begin; int r; const u4* Rq; const uint8_t* rsc;
  int M, N, K;
  void* Y; int y_dtype; int64_t ldy;
  int coltiles;
  int splitk;                       // K slices: per channel block (decode kernel) or per tile (0 = choose, 1 = none)
  void* workspace; size_t workspace_bytes;
};
size_t mx_split_workspace_bytes(int M, int N, int K, int forced);
int launch_mx_quantize_act(const void* X, const void* U, int x_dtype, const float* s_inv, int64_t M, int K, int64_t ldx,
                           int64_t ldu, void* Xq, uint8_t* xsc, hipStream_t st);
int mx_pack_weights_impl(const void* W, int w_dtype, const float* s, const int32_t* perm, int N, int K, int r,
                         void* Wq, uint8_t* wsc, void* Rq, uint8_t* rsc, hipStream_t st);
int mx_unpack_weights_impl(const void* Wq, const uint8_t* wsc, int N, int K, uint8_t* codes, uint8_t* E, hipStream_t st);
int mx_unpack_act_impl(const void* Xq, const uint8_t* xsc, int64_t M, int K, uint8_t* codes, uint8_t* E, hipStream_t st);
int launch_mx_linear(const MxLinearArgs& a, hipStream_t st);
int launch_skinny_mx(const MxLinearArgs& a, hipStream_t st);
size_t skinny_mx_workspace_bytes(int N);

int pack_weights_impl(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int N, int K, int r,
                      void* Wq_out, float* wscale_out, int32_t* perm_out, float* s_inv_out, void* R_out,
                      int r_dtype, void* Rp_out, hipStream_t st);
int prepare_perm_impl(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int N, int K,
                      int32_t* perm_out, float* s_inv_out, hipStream_t st);
int pack_lowrank_impl(void* R, int N, int r, void* Rp, bool unpack, hipStream_t st);
size_t lowrank_q4_frag_bytes(int N, int r);
int pack_lowrank_q4_impl(const void* R, int r_dtype, int N, int r, void* Rq, hipStream_t st);
int unpack_lowrank_q4_impl(const void* Rq, int N, int r, int8_t* codes, float* rscale, hipStream_t st);
int unpack_weights_impl(const void* Wq, int N, int K, int8_t* out, hipStream_t st);
int unpack_act_impl(const void* Xq, int abits, int64_t M, int K, int8_t* out, hipStream_t st);

}  // namespace serq
