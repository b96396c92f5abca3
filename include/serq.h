/*
 * serq.h -- C ABI of the MI355X (gfx950) SERQ linear-layer library.
 *
 * The library implements the online hot path of SERQ (saliency-aware low-rank
 * error reconstruction): per-token activation quantisation, the INT4-weight
 * integer GEMM, and the single rank-r compensation fused into the
 * dequantising epilogue, plus the offline weight preparation.  Variants
 * declared further down: the compensation matrix on the INT4 grid
 * (serq_pack_lowrank_q4), the whole layer in MXFP4 (serq_mx_*), and the
 * quantisers fused into the producer of the down projection's input
 * (serq_swiglu_quantize_act, serq_mx_swiglu_quantize_act).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte
 *     aligned.  The library allocates nothing and keeps no state between
 *     calls (the number of compute units is asked of the runtime on every
 *     call); all work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and returns without waiting.
 *   - Matrices are row-major.  X is [M tokens, K input channels]; W is
 *     [N output channels, K input channels]; R is [r, N]; Y is [M, N].
 *     (The paper writes Y = X.W with W [d_in, d_out]: one of its "weight
 *     rows" -- an input channel -- is a column of our W.)
 *   - The activations handed to the online calls are ALREADY in the permuted
 *     channel order the packed weights use (the offline permutation of
 *     Sec. 3.2 guarantees this; there is no online gather).
 *   - Return value: SERQ_OK or a negative SERQ_E* code; nothing throws or
 *     aborts.  Non-finite inputs give undefined outputs, not an error.
 *   - Shape limits: K a multiple of 64, 64 <= K <= 131072; N a multiple of
 *     32; r a multiple of 16 with s_begin + r <= K, s_begin a multiple of 32.
 *   - Packed tensors (Xq, Wq, Rp) have library-private layouts; use the
 *     serq_unpack_* calls to read them back in canonical form.
 */
#ifndef SERQ_H_
#define SERQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define SERQ_OK            0
#define SERQ_ENULL        -1   /* a required pointer is NULL                    */
#define SERQ_EDTYPE       -2   /* unsupported dtype / activation bit-width      */
#define SERQ_ESHAPE       -3   /* a size violates the limits above              */
#define SERQ_EALIGN       -4   /* pointer or leading dimension misaligned       */
#define SERQ_EWORKSPACE   -5   /* workspace missing or too small                */
#define SERQ_EHIP         -6   /* the HIP runtime reported a launch error       */
#define SERQ_EUNSUPPORTED -7   /* valid request this build does not implement   */
#define SERQ_ELIMIT       -8   /* size beyond the built-in scratch of serq_linear_noalloc */

/* element types of caller-visible tensors */
#define SERQ_F32  0
#define SERQ_F16  1
#define SERQ_BF16 2
/* r_dtype of serq_linear only: the compensation matrix is the 4-bit blob of serq_pack_lowrank_q4 */
#define SERQ_I4   3

/* kernel selection for serq_linear / serq_gemm_i32 (low byte of `flags`) */
#define SERQ_PATH_AUTO   0     /* by M: skinny for M <= 32, tiled MFMA above    */
#define SERQ_PATH_SKINNY 1     /* weight-streaming split-K kernel (M <= 32)     */
#define SERQ_PATH_MFMA   2     /* LDS-tiled int8-MFMA kernel                    */
/* bits 8..15 of `flags`: number of K slices (0 = the library's choice; 1 = none; n > 1 = exactly n, which
 * needs the workspace) -- of the skinny path's channel blocks, or of the MFMA path's output tiles */
#define SERQ_FLAG_SPLITK(n) (((n) & 0xff) << 8)
/* bits 16..19 of `flags`: MFMA path: token-tile group height of the block order (0 = auto);
 * skinny path: waves per workgroup / 4 (1 or 2; anything else = auto) */
#define SERQ_FLAG_GROUPM(n) (((n) & 0xf) << 16)
/* bits 20..30 of `flags`: number of column tiles of the MFMA path (0 = auto; clamped to the valid range) */
#define SERQ_FLAG_COLTILES(n) (((n) & 0x7ff) << 20)

int         serq_version(void);
const char* serq_strerror(int code);

/* Sizes of the caller-allocated buffers, in bytes (0 on invalid arguments). */
size_t serq_packed_act_bytes(int64_t M, int64_t K, int abits);     /* Xq                    */
size_t serq_packed_weight_bytes(int64_t N, int64_t K);             /* Wq                    */
size_t serq_packed_lowrank_bytes(int64_t N, int r);                /* Rp (16-bit elements)  */
size_t serq_packed_lowrank_q4_bytes(int64_t N, int r);             /* Rq (4-bit codes + rscale) */
size_t serq_workspace_bytes(int64_t M, int64_t N, int64_t K, int r, int abits);

/* Zero a workspace before its first use.  serq_linear / serq_gemm_i32 leave the part
 * that must be zero (the decode path's meeting words, at its start) zeroed again when
 * they finish, so one call after allocation is enough; the rest (where the tiled path
 * parks the INT32 tiles of its K slices for layers with few tokens and a long K) is
 * scratch.  Two calls that share a workspace must not overlap in time. */
int serq_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Offline preparation of one layer (Sec. 3.2: Eq. 4 static flattening folded
 * into the weights, saliency order P and the permuted weights of Eq. 5/6,
 * per-output-channel symmetric INT4 quantisation per Eq. 1, and the
 * compensation matrix R = W~_s - Q(W~_s) of Eq. 5).
 *
 *   W        [N,K] fp16/bf16/fp32 (w_dtype), ORIGINAL channel order.
 *   s        [K] fp32 flattening vector (weights are multiplied by s, the
 *            activations by 1/s); NULL = all ones.
 *   perm_in  [K] int32, perm_in[kp] = original channel placed at permuted
 *            position kp; NULL = order by saliency: channel scale
 *            max_n |W[n,k]*s[k]|, descending, ties to the lower index.
 *            A caller-supplied perm_in is TRUSTED input: it must be a
 *            permutation of 0..K-1.  It is not checked: indices are clamped
 *            into 0..K-1 (nothing is read out of bounds), but a clamped or
 *            repeated index silently gives a wrong layer and the call still
 *            returns SERQ_OK (the same holds for serq_mx_pack_weights and
 *            serq_g128_pack_weights).
 *   Wq_out   serq_packed_weight_bytes(N,K) bytes.
 *   wscale_out [N] fp32: max_k |W~[n,k]| / 7 (1.0 for an all-zero row).
 *   perm_out [K] int32 (required; equals perm_in when that is given).
 *   s_inv_out [K] fp32 (required): 1/s in permuted order -- what
 *            serq_quantize_act multiplies by.
 *   R_out    [r,N] in r_dtype, the residual of the r leading (salient)
 *            channels, rounded to nearest even; may be NULL.
 *   Rp_out   the same residual in the packed layout serq_linear reads
 *            (serq_packed_lowrank_bytes(N,r)); may be NULL.  r_dtype must be
 *            SERQ_F16 or SERQ_BF16 when Rp_out is given.
 *   r may be 0 (then R_out / Rp_out are ignored).
 */
int serq_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in,
                      int64_t N, int64_t K, int r,
                      void* Wq_out, float* wscale_out, int32_t* perm_out, float* s_inv_out,
                      void* R_out, int r_dtype, void* Rp_out, void* stream);

/* Re-layout a caller-supplied compensation matrix R [r,N] (fp16/bf16) into the
 * packed form serq_linear reads (the single matrix of Eq. 5 / Eq. 7). */
int serq_pack_lowrank(const void* R, int r_dtype, int64_t N, int r, void* Rp_out, void* stream);

/*
 * The compensation matrix itself on the INT4 grid (Sec. 3.2, Eq. 7, second
 * line: "Q(R)").  R [r,N] fp16/bf16/fp32 (r_dtype) is quantised per output
 * channel as the weights are (Eq. 1 over each column):
 *   rscale[n] = max_j |R[j,n]| / 7 (1.0 for a zero column),
 *   Rq[j,n]   = clip(rne(R[j,n] / rscale[n]), -7, 7),
 * and laid out for serq_linear with r_dtype = SERQ_I4.  Rq_out takes
 * serq_packed_lowrank_q4_bytes(N,r) bytes (codes in 64-rank fragments, ranks past
 * r zero, followed by rscale [N] fp32).  r is a multiple of 16.
 */
int serq_pack_lowrank_q4(const void* R, int r_dtype, int64_t N, int r, void* Rq_out, void* stream);
/* Canonical view of that blob: codes int8 [r,N] and rscale fp32 [N] (either may be NULL). */
int serq_unpack_lowrank_q4(const void* Rq, int64_t N, int r, int8_t* codes_out, float* rscale_out, void* stream);

/* Canonical views of the packed tensors (parity checks). */
int serq_unpack_lowrank(const void* Rp, int64_t N, int r, void* R_out, void* stream);   /* 16-bit [r,N] */
int serq_unpack_weights(const void* Wq, int64_t N, int64_t K, int8_t* Wq_i8_out, void* stream); /* [N,K] */
int serq_unpack_act(const void* Xq, int abits, int64_t M, int64_t K, int8_t* Xq_i8_out, void* stream); /* [M,K] */

/*
 * Online step 1: static activation flattening (Eq. 4) + per-token symmetric
 * max-scaled quantisation (Eq. 1), round-half-to-even, codes in
 * [-(2^(abits-1)-1), +(2^(abits-1)-1)].
 *
 *   X      [M,K] fp16/bf16/fp32 (x_dtype), row stride ldx elements (multiple of 8).
 *   s_inv  [K] fp32 from serq_pack_weights, or NULL when X is already flattened.
 *   abits  4 or 8.
 *   Xq_out serq_packed_act_bytes(M,K,abits) bytes; scale_out [M] fp32:
 *          scale[m] = max_k |X[m,k]*s_inv[k]| / qmax in fp32 (1.0 for a zero token).
 * M may be 0 (nothing is done).
 */
int serq_quantize_act(const void* X, int x_dtype, const float* s_inv,
                      int64_t M, int64_t K, int64_t ldx, int abits,
                      void* Xq_out, float* scale_out, void* stream);

/*
 * The same step fused into the producer of the down projection's input (Sec. 3.2, "Offline Weight
 * Permutation" and the decoder-layer flow of Fig. 2(b): the gated product arrives in the permuted channel
 * order and the flattening is merged into the adjacent step): the row that is flattened and quantised is
 *   v[m,k] = silu(G[m,k]) * U[m,k],   silu(g) = g / (1 + exp(-g)),
 * formed in fp32 and never rounded to a 16-bit type.  G, U [M,K] in x_dtype with row strides ldg, ldu
 * (multiples of 8; the two may be halves of one [M,2K] buffer).  Everything else as serq_quantize_act.
 * The exponential makes the product good to a few ulps of fp32, not bit-defined: a code may differ from
 * the correctly rounded one where v / scale lies within that distance of a rounding boundary.
 */
int serq_swiglu_quantize_act(const void* G, const void* U, int x_dtype, const float* s_inv,
                             int64_t M, int64_t K, int64_t ldg, int64_t ldu, int abits,
                             void* Xq_out, float* scale_out, void* stream);

/*
 * Online step 2: the SERQ linear layer (Eq. 2 + Eq. 7, first line)
 *
 *   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k]*Wq[n,k]
 *                         + sum_{j<r} Xq[m, s_begin+j] * R[j,n] )
 *
 * with the integer sum exact in INT32 (int8 MFMA) and the rest in fp32; Y is
 * written once.  Rp is the packed compensation matrix (fp16 or bf16 per
 * r_dtype); r = 0 or Rp = NULL gives the plain W4A4 / W4A8 GEMM.
 * With r_dtype = SERQ_I4, Rp is the blob of serq_pack_lowrank_q4 and the layer is
 * the all-integer second line of Eq. 7,
 *   Y[m,n] = scale[m] * ( wscale[n] * sum_k Xq[m,k]*Wq[n,k]
 *                         + rscale[n] * sum_{j<r} Xq[m, s_begin+j] * Rq[j,n] ),
 * both sums exact in INT32; the 64-rank fragments make the kernel read the token
 * codes of channels s_begin .. s_begin + 64*ceil(r/64) - 1, which must exist
 * (s_begin + 64*ceil(r/64) <= K; the codes past r meet zero weights).
 *   Y [M,N] in y_dtype (fp32/fp16/bf16), row stride ldy elements (multiple of 8).
 *   workspace: serq_workspace_bytes(...) bytes prepared by serq_workspace_init
 * (both paths use it when they cut K into slices; pass NULL/0 to forbid that).  Sliced or
 * not, the INT32 sums are the same integers, so Y does not depend on it.
 *   flags: SERQ_PATH_* | SERQ_FLAG_*.
 */
int serq_linear(const void* Xq, const float* scale, int abits,
                const void* Wq, const float* wscale,
                int s_begin, int r, const void* Rp, int r_dtype,
                int64_t M, int64_t N, int64_t K,
                void* Y, int y_dtype, int64_t ldy,
                void* workspace, size_t workspace_bytes, int flags, void* stream);

/*
 * serq_linear for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, arithmetic and kernels as serq_linear, minus the
 * workspace: the words in which the K slices of the decode path meet live in a device array inside the
 * library (8 MiB per GPU, held until the process ends), so the call allocates nothing and asks the
 * caller for nothing.  Limit: N <= 32768; beyond it the call returns SERQ_ELIMIT and does nothing.
 * Results equal serq_linear's with a workspace, bit for bit.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (two
 * streams, two threads) race; calls on one stream, or otherwise ordered, are fine.  The kernels leave
 * the array zeroed when they finish, so successive calls of any size need no clearing in between.
 * The first call on a GPU also looks the array up and clears it once (a fill kernel on `stream`): make
 * that call before a capture begins, so that the graph records the layer's kernels only.
 */
int serq_linear_noalloc(const void* Xq, const float* scale, int abits,
                        const void* Wq, const float* wscale,
                        int s_begin, int r, const void* Rp, int r_dtype,
                        int64_t M, int64_t N, int64_t K,
                        void* Y, int y_dtype, int64_t ldy, int flags, void* stream);

/* Parity aid: the same main loops, storing the raw INT32 accumulators
 * acc[m,n] = sum_k Xq[m,k]*Wq[n,k] (first term of Eq. 7) to acc_out [M,N],
 * row stride ldacc elements (multiple of 4). */
int serq_gemm_i32(const void* Xq, int abits, const void* Wq,
                  int64_t M, int64_t N, int64_t K,
                  int32_t* acc_out, int64_t ldacc,
                  void* workspace, size_t workspace_bytes, int flags, void* stream);

/*
 * ---- MXFP4 variant of the layer ------------------------------------------------------------------
 * The paper's W4A4 latency runs use the 4-bit Microscaling format (Sec. 4.1 and the appendix on MXFP4
 * kernels); arithmetic per the OCP Microscaling specification: blocks of 32 consecutive (permuted)
 * input channels share one scale 2^(E-127), E = 127 + max(floor(log2(max|v|)) - 2, -127) (E = 127 for
 * an all-zero block), elements are E2M1 codes (bit 3 = sign, bits 0..2 index 0, 0.5, 1, 1.5, 2, 3, 4,
 * 6), round to nearest, ties to the code with an even mantissa bit, larger magnitudes saturate at 6.
 * Weights, activations and the compensation matrix (along its rank index) all take this form (Eq. 7,
 * second line, with Q = MXFP4), so the layer is
 *   Y[m,n] = sum_k X^[m,k] W^[n,k] + sum_{j<r} X^[m,s_begin+j] R^[n,j]
 * with no further scales.  It runs on the block-scaled FP4 matrix instructions, in a tiled kernel for
 * M > 32 and a weight-streaming kernel for M <= 32 (SERQ_PATH_* as for serq_linear).
 *
 * Buffers (device memory, 16-byte aligned; opaque except through the unpack calls):
 *   activation codes  serq_packed_act_bytes(M,K,4) bytes
 *   activation scales serq_mx_act_scale_bytes(M,K) bytes
 *   weight codes      serq_packed_weight_bytes(N,K) bytes
 *   weight scales     serq_mx_weight_scale_bytes(N,K) bytes
 *   compensation      codes serq_packed_weight_bytes(N, 64*ceil(r/64)), scales
 *                     serq_mx_weight_scale_bytes(N, 64*ceil(r/64)) (ranks past r are zero)
 */
size_t serq_mx_act_scale_bytes(int64_t M, int64_t K);
size_t serq_mx_weight_scale_bytes(int64_t N, int64_t K);

/* Online step 1 for the MXFP4 layer: flattening (Eq. 4; s_inv may be NULL) and MXFP4 quantisation of
 * each token in blocks of 32 channels.  X [M,K] fp16/bf16/fp32, row stride ldx (multiple of 8). */
int serq_mx_quantize_act(const void* X, int x_dtype, const float* s_inv, int64_t M, int64_t K, int64_t ldx,
                         void* Xq_out, uint8_t* xscale_out, void* stream);
/* serq_mx_quantize_act of the gated product silu(G) * U (see serq_swiglu_quantize_act). */
int serq_mx_swiglu_quantize_act(const void* G, const void* U, int x_dtype, const float* s_inv,
                                int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                void* Xq_out, uint8_t* xscale_out, void* stream);

/* Offline preparation for the MXFP4 layer (Sec. 3.2 with Q = MXFP4): W~ = (W * s)[:, perm] in fp32
 * (s, perm_in, perm_out, s_inv_out as in serq_pack_weights), MXFP4 per output channel in blocks of 32
 * input channels; R[n,j] = W~[n,j] - dequantised W~[n,j] for the r leading channels (one fp32
 * subtraction), itself in MXFP4 in blocks of 32 ranks.  r is a multiple of 32 (0: Rq_out / rscale_out
 * ignored). */
int serq_mx_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in,
                         int64_t N, int64_t K, int r,
                         void* Wq_out, uint8_t* wscale_out, int32_t* perm_out, float* s_inv_out,
                         void* Rq_out, uint8_t* rscale_out, void* stream);

/* Canonical views (parity checks): codes uint8 [rows,K] (0..15), exponent bytes uint8 [rows,K/32].
 * A packed compensation matrix is viewed with serq_mx_unpack_weights(Rq, rscale, N, 64*ceil(r/64)). */
int serq_mx_unpack_weights(const void* Wq, const uint8_t* wscale, int64_t N, int64_t K,
                           uint8_t* codes_out, uint8_t* exps_out, void* stream);
int serq_mx_unpack_act(const void* Xq, const uint8_t* xscale, int64_t M, int64_t K,
                       uint8_t* codes_out, uint8_t* exps_out, void* stream);

/* Bytes of workspace serq_mx_linear can use for this call.  Same rules as serq_workspace_bytes /
 * serq_workspace_init: zero it once after allocation; two calls that share a workspace must not overlap in
 * time.  The first part (the size this returns for M = 1) holds the words in which the decode kernel's K
 * slices meet, and the kernel leaves it zeroed; for M > 32 a second part behind it holds the fp32 tiles the
 * tiled kernel parks when it cuts K (few tokens, long K), which is scratch: written before it is read. */
size_t serq_mx_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* The MXFP4 layer.  Y [M,N] in y_dtype, row stride ldy (multiple of 8, >= N); fp32 accumulation over
 * k in the order of the hardware's 64-channel steps, the compensation sum added to the same
 * accumulators.  s_begin is a multiple of 256 with s_begin + 64*ceil(r/64) <= K; r a multiple of 32;
 * Rq may be NULL (no compensation).  workspace may be NULL: K is then never sliced; with it, layers that
 * would leave most compute units idle (decode: few blocks of 32 output channels; tiled kernel: few tokens)
 * and have a long K are cut into K slices whose partial sums are added in a fixed order, so results do not
 * vary from run to run, but they depend on the number of slices (fp32 addition).  SERQ_FLAG_SPLITK: 0 the
 * library's choice, 1 none, n > 1 exactly n (SERQ_EWORKSPACE if the workspace is missing or too small).
 * flags: SERQ_PATH_* | SERQ_FLAG_SPLITK | SERQ_FLAG_COLTILES.  M = 0 is a no-op. */
int serq_mx_linear(const void* Xq, const uint8_t* xscale, const void* Wq, const uint8_t* wscale,
                   int s_begin, int r, const void* Rq, const uint8_t* rscale,
                   int64_t M, int64_t N, int64_t K,
                   void* Y, int y_dtype, int64_t ldy,
                   void* workspace, size_t workspace_bytes, int flags, void* stream);

/*
 * ---- The accuracy-table setting: group-128 weight scales, asymmetric activations ---------------------
 * Sec. 4.1 (implementation details) runs the accuracy experiments with weights quantised in groups of
 * 128 input channels (round-to-nearest symmetric INT4) and activations quantised per token with
 * round-to-nearest ASYMMETRIC integers.  The paper gives no formulas; the arithmetic is the usual min-max
 * affine quantiser:
 *   token:   lo = min(0, min_k v), hi = max(0, max_k v), scale = (hi - lo) / (2^n - 1) (1.0 for a zero token),
 *            z = rne(-lo / scale), c = clip(rne(v / scale) + z, 0, 2^n - 1), value = scale (c - z); all fp32.
 *            Stored re-centred: Xq = c - 2^(n-1) in the containers of serq_quantize_act, zero = z - 2^(n-1).
 *   weights: gscale[n,g] = fp16(max_{k in group g} |W~[n,k]| / 7) kept within [2^-24, 65504] (1.0 for a zero
 *            group), Wq[n,k] = clip(rne(W~[n,k] / gscale[n, k/128]), -7, 7), value = gscale Wq.
 *   layer:   Y[m,n] = sum_k x^[m,k] w^[n,k] + sum_{j<r} x^[m,s_begin+j] R[j,n]            (Eq. 2 + Eq. 7)
 * with the integer sums of every group exact in INT32 and folded into fp32 group by group.
 * K is a multiple of 128 here.  Weight codes have the layout of serq_pack_weights (serq_unpack_weights reads
 * them back); the group scales take serq_g128_scale_bytes(N,K) bytes (opaque; serq_g128_unpack_scales gives
 * fp32 [N, K/128]); wsum [N] fp32 = sum_k gscale[n,k/128] Wq[n,k], what a token's zero point multiplies.
 */
size_t serq_g128_scale_bytes(int64_t N, int64_t K);
/* serq_quantize_act with the asymmetric grid above; zero_out [M] int32.  Everything else as serq_quantize_act. */
int serq_quantize_act_asym(const void* X, int x_dtype, const float* s_inv, int64_t M, int64_t K, int64_t ldx, int abits,
                           void* Xq_out, float* scale_out, int32_t* zero_out, void* stream);
/* serq_pack_weights with one scale per output channel and group of 128 (permuted) input channels; s, perm_in,
 * perm_out, s_inv_out, R_out, r_dtype, Rp_out as there (R = W~_s - gscale Wq over the r leading channels). */
int serq_g128_pack_weights(const void* W, int w_dtype, const float* s, const int32_t* perm_in, int64_t N, int64_t K, int r,
                           void* Wq_out, void* gscale_out, float* wsum_out, int32_t* perm_out, float* s_inv_out,
                           void* R_out, int r_dtype, void* Rp_out, void* stream);
int serq_g128_unpack_scales(const void* gscale, int64_t N, int64_t K, float* out, void* stream);
/* The layer.  zero may be NULL (symmetric codes of serq_quantize_act: the same layer without zero points).
 * Rp / r_dtype: the packed 16-bit compensation matrix as for serq_linear (r = 0 or NULL: none); s_begin a
 * multiple of 32.  Y [M,N] in y_dtype, row stride ldy (multiple of 8).  flags: SERQ_PATH_* only (M <= 32 takes
 * a weight-streaming kernel, larger M an LDS-tiled one).  fp32 sums are added in a fixed order: results do
 * not vary from run to run.  No workspace. */
int serq_g128_linear(const void* Xq, const float* scale, const int32_t* zero, int abits,
                     const void* Wq, const void* gscale, const float* wsum,
                     int s_begin, int r, const void* Rp, int r_dtype,
                     int64_t M, int64_t N, int64_t K, void* Y, int y_dtype, int64_t ldy, int flags, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SERQ_H_ */
