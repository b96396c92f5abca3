// C ABI of the library: argument checking and dispatch only (see include/serq.h).
#include "serq_device.h"
#include "../../include/serq_bench.h"

using namespace serq;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool dtype_ok(int dt) { return dt == SERQ_F32 || dt == SERQ_F16 || dt == SERQ_BF16; }
inline bool dtype16(int dt) { return dt == SERQ_F16 || dt == SERQ_BF16; }

int check_nk(int64_t N, int64_t K) {
  if (K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24)) return SERQ_ESHAPE;
  return SERQ_OK;
}

// plain fill kernel: safe to record into a HIP graph, unlike a memset node
__global__ __launch_bounds__(256) void zero_fill_kernel(uint32_t* p, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

int check_lowrank(int64_t K, int s_begin, int r) {
  if (r < 0 || (r % 16) != 0 || s_begin < 0 || (s_begin % 32) != 0) return SERQ_ESHAPE;
  if ((int64_t)s_begin + r > K) return SERQ_ESHAPE;
  return SERQ_OK;
}

}  // namespace

extern "C" {

int serq_version(void) { return 100; }

const char* serq_strerror(int code) {
  switch (code) {
    case SERQ_OK: return "ok";
    case SERQ_ENULL: return "required pointer is NULL";
    case SERQ_EDTYPE: return "unsupported dtype or activation bit-width";
    case SERQ_ESHAPE: return "size outside the supported limits";
    case SERQ_EALIGN: return "pointer or leading dimension misaligned";
    case SERQ_EWORKSPACE: return "workspace missing or too small";
    case SERQ_EHIP: return "HIP runtime error";
    case SERQ_EUNSUPPORTED: return "request not implemented";
    case SERQ_ELIMIT: return "size beyond the built-in scratch buffer of the allocation-free entry point";
    default: return "unknown error code";
  }
}

size_t serq_packed_act_bytes(int64_t M, int64_t K, int abits) {
  if (M < 0 || K <= 0 || (K % 64) != 0 || (abits != 4 && abits != 8)) return 0;
  return (size_t)M * (size_t)K * abits / 8;
}

size_t serq_packed_weight_bytes(int64_t N, int64_t K) {
  if (check_nk(N, K) != SERQ_OK) return 0;
  return (size_t)N * (size_t)K / 2;
}

size_t serq_packed_lowrank_bytes(int64_t N, int r) {
  if (N <= 0 || (N % 32) != 0 || r < 0 || (r % 16) != 0) return 0;
  return (size_t)N * (size_t)r * 2;
}

size_t serq_packed_lowrank_q4_bytes(int64_t N, int r) {
  if (N <= 0 || (N % 32) != 0 || N > (1 << 24) || r < 0 || (r % 16) != 0) return 0;
  return lowrank_q4_frag_bytes((int)N, r) + (size_t)N * 4;
}

size_t serq_workspace_bytes(int64_t M, int64_t N, int64_t K, int r, int abits) {
  (void)r;
  if (check_nk(N, K) != SERQ_OK || M < 0 || M > (1 << 30) || (abits != 4 && abits != 8)) return 0;
  // where the K slices of a channel block meet (decode path), then the parked INT32 tiles of the tiled
  // path's K slices (only layers with few tokens and a long K are sliced there)
  return skinny_workspace_bytes((int)N) + (M > 32 ? mfma_split_workspace_bytes((int)M, (int)N, (int)K, abits, 0) : 0);
}

int serq_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace_bytes == 0) return SERQ_OK;
  if (!workspace) return SERQ_ENULL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) || (workspace_bytes & 3u)) return SERQ_EALIGN;
  const size_t n = workspace_bytes / 4;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     (uint32_t*)workspace, n);
  return hipGetLastError() == hipSuccess ? SERQ_OK : SERQ_EHIP;
}

int serq_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in,
                      int64_t N, int64_t K, int r,
                      void* Wq_out, float* wscale_out, int32_t* perm_out, float* s_inv_out,
                      void* R_out, int r_dtype, void* Rp_out, void* stream) {
  if (!W || !Wq_out || !wscale_out || !perm_out || !s_inv_out) return SERQ_ENULL;
  if (!dtype_ok(w_dtype)) return SERQ_EDTYPE;
  int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  rc = check_lowrank(K, 0, r);
  if (rc != SERQ_OK) return rc;
  if (r > 0 && (R_out || Rp_out)) {
    if (!dtype_ok(r_dtype)) return SERQ_EDTYPE;
    if (Rp_out && !dtype16(r_dtype)) return SERQ_EDTYPE;
  }
  if (!aligned16(W) || !aligned16(Wq_out) || !aligned16(wscale_out) || !aligned16(perm_out) ||
      !aligned16(s_inv_out) || !aligned16(R_out) || !aligned16(Rp_out) || !aligned16(s) || !aligned16(perm_in))
    return SERQ_EALIGN;
  return pack_weights_impl(W, w_dtype, s, perm_in, (int)N, (int)K, r, Wq_out, wscale_out, perm_out, s_inv_out,
                           R_out, r_dtype, Rp_out, (hipStream_t)stream);
}

int serq_pack_lowrank(const void* R, int r_dtype, int64_t N, int r, void* Rp_out, void* stream) {
  if (!R || !Rp_out) return SERQ_ENULL;
  if (!dtype16(r_dtype)) return SERQ_EDTYPE;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || r < 0 || (r % 16) != 0) return SERQ_ESHAPE;
  if (!aligned16(R) || !aligned16(Rp_out)) return SERQ_EALIGN;
  return pack_lowrank_impl(const_cast<void*>(R), (int)N, r, Rp_out, false, (hipStream_t)stream);
}

int serq_unpack_lowrank(const void* Rp, int64_t N, int r, void* R_out, void* stream) {
  if (!Rp || !R_out) return SERQ_ENULL;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || r < 0 || (r % 16) != 0) return SERQ_ESHAPE;
  if (!aligned16(Rp) || !aligned16(R_out)) return SERQ_EALIGN;
  return pack_lowrank_impl(R_out, (int)N, r, const_cast<void*>(Rp), true, (hipStream_t)stream);
}

int serq_pack_lowrank_q4(const void* R, int r_dtype, int64_t N, int r, void* Rq_out, void* stream) {
  if (!R || !Rq_out) return SERQ_ENULL;
  if (!dtype_ok(r_dtype)) return SERQ_EDTYPE;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || r < 0 || (r % 16) != 0) return SERQ_ESHAPE;
  if (!aligned16(R) || !aligned16(Rq_out)) return SERQ_EALIGN;
  return pack_lowrank_q4_impl(R, r_dtype, (int)N, r, Rq_out, (hipStream_t)stream);
}

int serq_unpack_lowrank_q4(const void* Rq, int64_t N, int r, int8_t* codes_out, float* rscale_out, void* stream) {
  if (!Rq) return SERQ_ENULL;
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || r < 0 || (r % 16) != 0) return SERQ_ESHAPE;
  if (!aligned16(Rq) || (reinterpret_cast<uintptr_t>(rscale_out) & 3u)) return SERQ_EALIGN;
  return unpack_lowrank_q4_impl(Rq, (int)N, r, codes_out, rscale_out, (hipStream_t)stream);
}

int serq_unpack_weights(const void* Wq, int64_t N, int64_t K, int8_t* out, void* stream) {
  if (!Wq || !out) return SERQ_ENULL;
  const int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  if (!aligned16(Wq) || !aligned16(out)) return SERQ_EALIGN;
  return unpack_weights_impl(Wq, (int)N, (int)K, out, (hipStream_t)stream);
}

int serq_unpack_act(const void* Xq, int abits, int64_t M, int64_t K, int8_t* out, void* stream) {
  if (abits != 4 && abits != 8) return SERQ_EDTYPE;
  if (M < 0 || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!Xq || !out) return SERQ_ENULL;
  if (!aligned16(Xq) || !aligned16(out)) return SERQ_EALIGN;
  return unpack_act_impl(Xq, abits, M, (int)K, out, (hipStream_t)stream);
}

int serq_quantize_act(const void* X, int x_dtype, const float* s_inv,
                      int64_t M, int64_t K, int64_t ldx, int abits,
                      void* Xq_out, float* scale_out, void* stream) {
  if (abits != 4 && abits != 8) return SERQ_EDTYPE;
  if (!dtype_ok(x_dtype)) return SERQ_EDTYPE;
  if (M < 0 || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (ldx < K) return SERQ_ESHAPE;
  if ((ldx % 8) != 0) return SERQ_EALIGN;
  if (M == 0) return SERQ_OK;
  if (!X || !Xq_out || !scale_out) return SERQ_ENULL;
  if (!aligned16(X) || !aligned16(Xq_out) || !aligned16(s_inv) || (reinterpret_cast<uintptr_t>(scale_out) & 3u))
    return SERQ_EALIGN;
  return launch_quantize_act(X, nullptr, x_dtype, s_inv, M, (int)K, ldx, 0, abits, Xq_out, scale_out,
                             (hipStream_t)stream);
}

int serq_swiglu_quantize_act(const void* G, const void* U, int x_dtype, const float* s_inv,
                             int64_t M, int64_t K, int64_t ldg, int64_t ldu, int abits,
                             void* Xq_out, float* scale_out, void* stream) {
  if (abits != 4 && abits != 8) return SERQ_EDTYPE;
  if (!dtype_ok(x_dtype)) return SERQ_EDTYPE;
  if (M < 0 || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (ldg < K || ldu < K) return SERQ_ESHAPE;
  if ((ldg % 8) != 0 || (ldu % 8) != 0) return SERQ_EALIGN;
  if (M == 0) return SERQ_OK;
  if (!G || !U || !Xq_out || !scale_out) return SERQ_ENULL;
  if (!aligned16(G) || !aligned16(U) || !aligned16(Xq_out) || !aligned16(s_inv) ||
      (reinterpret_cast<uintptr_t>(scale_out) & 3u))
    return SERQ_EALIGN;
  return launch_quantize_act(G, U, x_dtype, s_inv, M, (int)K, ldg, ldu, abits, Xq_out, scale_out, (hipStream_t)stream);
}

static int linear_common(LinearArgs& a, int64_t M, int64_t N, int64_t K, int flags, void* stream) {
  if (a.abits != 4 && a.abits != 8) return SERQ_EDTYPE;
  int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  if (M < 0 || M > (1 << 30)) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!a.Xq || !a.Wq) return SERQ_ENULL;
  if (!aligned16(a.Xq) || !aligned16(a.Wq) || !aligned16(a.Rp) || !aligned16(a.wscale) || !aligned16(a.workspace))
    return SERQ_EALIGN;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.splitk = (flags >> 8) & 0xff;
  a.groupm = (flags >> 16) & 0xf;
  a.skinny_waves = a.groupm * 4;                     // the two paths share the field: 1, 2 -> 4, 8 waves
  a.coltiles = (flags >> 20) & 0x7ff;
  const int path = flags & 0xff;
  if (path != SERQ_PATH_AUTO && path != SERQ_PATH_SKINNY && path != SERQ_PATH_MFMA) return SERQ_EUNSUPPORTED;
  if (path == SERQ_PATH_SKINNY && M > 32) return SERQ_ESHAPE;
  const bool skinny = path == SERQ_PATH_SKINNY || (path == SERQ_PATH_AUTO && M <= 32);
  return skinny ? launch_skinny(a, (hipStream_t)stream) : launch_mfma(a, (hipStream_t)stream);
}

int serq_linear(const void* Xq, const float* scale, int abits,
                const void* Wq, const float* wscale,
                int s_begin, int r, const void* Rp, int r_dtype,
                int64_t M, int64_t N, int64_t K,
                void* Y, int y_dtype, int64_t ldy,
                void* workspace, size_t workspace_bytes, int flags, void* stream) {
  if (!dtype_ok(y_dtype)) return SERQ_EDTYPE;
  if (M > 0 && (!Y || !scale || !wscale)) return SERQ_ENULL;
  int rc = check_lowrank(K, s_begin, r);
  if (rc != SERQ_OK) return rc;
  if (r > 0 && Rp && !dtype16(r_dtype) && r_dtype != SERQ_I4) return SERQ_EDTYPE;
  if (r > 0 && Rp && r_dtype == SERQ_I4 && (int64_t)s_begin + 64 * ((r + 63) / 64) > K) return SERQ_ESHAPE;
  if (ldy < N) return SERQ_ESHAPE;
  if ((ldy % 8) != 0 || !aligned16(Y) || (reinterpret_cast<uintptr_t>(scale) & 3u)) return SERQ_EALIGN;
  LinearArgs a{};
  a.Xq = (const uint8_t*)Xq; a.scale = scale; a.abits = abits;
  a.Wq = (const u4*)Wq; a.wscale = wscale;
  a.s_begin = s_begin; a.r = (Rp ? r : 0); a.Rp = (r > 0 ? (const u4*)Rp : nullptr); a.r_dtype = r_dtype;
  a.rscale = (a.Rp && r_dtype == SERQ_I4) ? (const float*)((const char*)Rp + lowrank_q4_frag_bytes((int)N, r)) : nullptr;
  a.Y = Y; a.y_dtype = y_dtype; a.ldy = ldy;
  a.acc_out = nullptr; a.ldacc = 0;
  a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  return linear_common(a, M, N, K, flags, stream);
}

int serq_gemm_i32(const void* Xq, int abits, const void* Wq,
                  int64_t M, int64_t N, int64_t K,
                  int32_t* acc_out, int64_t ldacc,
                  void* workspace, size_t workspace_bytes, int flags, void* stream) {
  if (M > 0 && !acc_out) return SERQ_ENULL;
  if (ldacc < N) return SERQ_ESHAPE;
  if ((ldacc % 4) != 0 || !aligned16(acc_out)) return SERQ_EALIGN;
  LinearArgs a{};
  a.Xq = (const uint8_t*)Xq; a.scale = nullptr; a.abits = abits;
  a.Wq = (const u4*)Wq; a.wscale = nullptr;
  a.s_begin = 0; a.r = 0; a.Rp = nullptr; a.r_dtype = SERQ_BF16;
  a.Y = nullptr; a.y_dtype = SERQ_F32; a.ldy = 0;
  a.acc_out = acc_out; a.ldacc = ldacc;
  a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  return linear_common(a, M, N, K, flags, stream);
}

// ---- MXFP4 path -------------------------------------------------------------------------------------
size_t serq_mx_act_scale_bytes(int64_t M, int64_t K) {
  if (M < 0 || K < 64 || K > 131072 || (K % 64) != 0) return 0;
  return (size_t)((K + 255) / 256) * (size_t)((M + 1) & ~(int64_t)1) * 8;
}

size_t serq_mx_weight_scale_bytes(int64_t N, int64_t K) {
  if (N < 32 || (N % 32) != 0 || N > (1 << 24) || K < 64 || K > 131072 || (K % 64) != 0) return 0;
  return (size_t)(N / 32) * (size_t)((K + 255) / 256) * 256;
}

int serq_mx_quantize_act(const void* X, int x_dtype, const float* s_inv, int64_t M, int64_t K, int64_t ldx,
                         void* Xq_out, uint8_t* xscale_out, void* stream) {
  if (!dtype_ok(x_dtype)) return SERQ_EDTYPE;
  if (M < 0 || M > 0x7fffffff || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (ldx < K) return SERQ_ESHAPE;
  if ((ldx % 8) != 0) return SERQ_EALIGN;
  if (M == 0) return SERQ_OK;
  if (!X || !Xq_out || !xscale_out) return SERQ_ENULL;
  if (!aligned16(X) || !aligned16(Xq_out) || !aligned16(s_inv) || !aligned16(xscale_out)) return SERQ_EALIGN;
  return launch_mx_quantize_act(X, nullptr, x_dtype, s_inv, M, (int)K, ldx, 0, Xq_out, xscale_out, (hipStream_t)stream);
}

int serq_mx_swiglu_quantize_act(const void* G, const void* U, int x_dtype, const float* s_inv,
                                int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                void* Xq_out, uint8_t* xscale_out, void* stream) {
  if (!dtype_ok(x_dtype)) return SERQ_EDTYPE;
  if (M < 0 || M > 0x7fffffff || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (ldg < K || ldu < K) return SERQ_ESHAPE;
  if ((ldg % 8) != 0 || (ldu % 8) != 0) return SERQ_EALIGN;
  if (M == 0) return SERQ_OK;
  if (!G || !U || !Xq_out || !xscale_out) return SERQ_ENULL;
  if (!aligned16(G) || !aligned16(U) || !aligned16(Xq_out) || !aligned16(s_inv) || !aligned16(xscale_out))
    return SERQ_EALIGN;
  return launch_mx_quantize_act(G, U, x_dtype, s_inv, M, (int)K, ldg, ldu, Xq_out, xscale_out, (hipStream_t)stream);
}

int serq_mx_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in,
                         int64_t N, int64_t K, int r,
                         void* Wq_out, uint8_t* wscale_out, int32_t* perm_out, float* s_inv_out,
                         void* Rq_out, uint8_t* rscale_out, void* stream) {
  if (!W || !Wq_out || !wscale_out || !perm_out || !s_inv_out) return SERQ_ENULL;
  if (!dtype_ok(w_dtype)) return SERQ_EDTYPE;
  int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  if (r < 0 || (r % 32) != 0 || r > K) return SERQ_ESHAPE;
  if (r > 0 && (!Rq_out || !rscale_out)) return SERQ_ENULL;
  if (!aligned16(W) || !aligned16(Wq_out) || !aligned16(wscale_out) || !aligned16(perm_out) ||
      !aligned16(s_inv_out) || !aligned16(Rq_out) || !aligned16(rscale_out) || !aligned16(s) || !aligned16(perm_in))
    return SERQ_EALIGN;
  rc = prepare_perm_impl(W, w_dtype, s, perm_in, (int)N, (int)K, perm_out, s_inv_out, (hipStream_t)stream);
  if (rc != SERQ_OK) return rc;
  return mx_pack_weights_impl(W, w_dtype, s, perm_out, (int)N, (int)K, r, Wq_out, wscale_out, Rq_out, rscale_out,
                              (hipStream_t)stream);
}

int serq_mx_unpack_weights(const void* Wq, const uint8_t* wscale, int64_t N, int64_t K,
                           uint8_t* codes_out, uint8_t* exps_out, void* stream) {
  if (!Wq || !wscale || !codes_out || !exps_out) return SERQ_ENULL;
  const int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  if (!aligned16(Wq) || !aligned16(wscale)) return SERQ_EALIGN;
  return mx_unpack_weights_impl(Wq, wscale, (int)N, (int)K, codes_out, exps_out, (hipStream_t)stream);
}

int serq_mx_unpack_act(const void* Xq, const uint8_t* xscale, int64_t M, int64_t K,
                       uint8_t* codes_out, uint8_t* exps_out, void* stream) {
  if (M < 0 || M > 0x7fffffff || K < 64 || K > 131072 || (K % 64) != 0) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!Xq || !xscale || !codes_out || !exps_out) return SERQ_ENULL;
  if (!aligned16(Xq) || !aligned16(xscale)) return SERQ_EALIGN;
  return mx_unpack_act_impl(Xq, xscale, M, (int)K, codes_out, exps_out, (hipStream_t)stream);
}

size_t serq_mx_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (M < 0 || check_nk(N, K) != SERQ_OK) return 0;
  return skinny_mx_workspace_bytes((int)N) + (M > 32 ? mx_split_workspace_bytes((int)M, (int)N, (int)K, 0) : 0);
}

int serq_mx_linear(const void* Xq, const uint8_t* xscale, const void* Wq, const uint8_t* wscale,
                   int s_begin, int r, const void* Rq, const uint8_t* rscale,
                   int64_t M, int64_t N, int64_t K,
                   void* Y, int y_dtype, int64_t ldy,
                   void* workspace, size_t workspace_bytes, int flags, void* stream) {
  int rc = check_nk(N, K);
  if (rc != SERQ_OK) return rc;
  if (M < 0 || M > (1 << 24)) return SERQ_ESHAPE;
  if (!dtype_ok(y_dtype)) return SERQ_EDTYPE;
  if (r < 0 || (r % 32) != 0 || s_begin < 0 || (s_begin % 256) != 0) return SERQ_ESHAPE;
  if (r > 0 && Rq && (int64_t)s_begin + 64 * ((r + 63) / 64) > K) return SERQ_ESHAPE;
  if (ldy < N) return SERQ_ESHAPE;
  if (M == 0) return SERQ_OK;
  if (!Xq || !xscale || !Wq || !wscale || !Y) return SERQ_ENULL;
  if (r > 0 && Rq && !rscale) return SERQ_ENULL;
  if ((ldy % 8) != 0 || !aligned16(Y) || !aligned16(Xq) || !aligned16(xscale) || !aligned16(Wq) ||
      !aligned16(wscale) || !aligned16(Rq) || !aligned16(rscale) || !aligned16(workspace))
    return SERQ_EALIGN;
  MxLinearArgs a{};
  a.Xq = (const uint8_t*)Xq; a.xsc = xscale; a.Wq = (const u4*)Wq; a.wsc = wscale;
  a.s_begin = s_begin; a.r = (Rq ? r : 0); a.Rq = (r > 0 ? (const u4*)Rq : nullptr); a.rsc = rscale;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.Y = Y; a.y_dtype = y_dtype; a.ldy = ldy;
  a.coltiles = (flags >> 20) & 0x7ff;
  a.splitk = (flags >> 8) & 0xff;
  a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  const int path = flags & 0xff;
  if (path != SERQ_PATH_AUTO && path != SERQ_PATH_SKINNY && path != SERQ_PATH_MFMA) return SERQ_EUNSUPPORTED;
  if (path == SERQ_PATH_SKINNY && M > 32) return SERQ_ESHAPE;
  const bool skinny = path == SERQ_PATH_SKINNY || (path == SERQ_PATH_AUTO && M <= 32);
  return skinny ? launch_skinny_mx(a, (hipStream_t)stream) : launch_mx_linear(a, (hipStream_t)stream);
}

int serq_bench_mfma_peak(const void* operands, int iters, int workgroups, void* sink, void* stream) {
  if (!operands || !sink) return SERQ_ENULL;
  if (iters < 0 || workgroups <= 0 || workgroups > (1 << 20)) return SERQ_ESHAPE;
  if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return SERQ_EALIGN;
  return launch_mfma_peak(operands, iters, workgroups, sink, (hipStream_t)stream);
}

int serq_bench_mfma_fp4_peak(const void* operands, int iters, int workgroups, void* sink, void* stream) {
  if (!operands || !sink) return SERQ_ENULL;
  if (iters < 0 || workgroups <= 0 || workgroups > (1 << 20)) return SERQ_ESHAPE;
  if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return SERQ_EALIGN;
  return launch_mfma_fp4_peak(operands, iters, workgroups, 127, 127, sink, (hipStream_t)stream);
}

int serq_bench_read(const void* src, size_t bytes, int workgroups, void* sink, void* stream) {
  if (!src || !sink) return SERQ_ENULL;
  if ((bytes % 16) != 0 || workgroups <= 0 || workgroups > (1 << 20)) return SERQ_ESHAPE;
  if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return SERQ_EALIGN;
  if (bytes == 0) return SERQ_OK;
  return launch_read_peak(src, bytes, workgroups, sink, (hipStream_t)stream);
}

}  // extern "C"
