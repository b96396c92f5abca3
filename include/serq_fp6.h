/*
 * serq_fp6.h -- experiment exported by libserq.so: the exact INT32 sums of the W4A4 layer (Sec. 2.1, Eq. 2;
 * first term of Eq. 7 in Sec. 3.2) on the FP6 form of gfx950's block-scaled matrix instruction.  Every INT4
 * code -7..7 is exactly an E2M3 value, the products are exact and an fp32 sum of such integers is exact for
 * every supported K, so the route must reproduce the integer sums bit for bit.  (The paper notes only that
 * its hardware has no INT4 matrix kernels, Sec. 4.3; this route is this library's own idea, kept apart from
 * the layer's entry points until a measurement says it pays.)
 *
 * Device pointers, 16-byte aligned.  K a multiple of 128.  All calls only launch (asynchronous on `stream`)
 * and return SERQ_OK or a negative SERQ_E* code.
 */
#ifndef SERQ_FP6_H_
#define SERQ_FP6_H_

#include "serq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* bytes of the FP6 operand buffers (6 bits per code; 0 on invalid arguments) */
size_t serq_fp6_weight_bytes(int64_t N, int64_t K);
size_t serq_fp6_act_bytes(int64_t M, int64_t K);

/* Canonical INT4 codes (int8 [rows,K], values -7..7: what serq_unpack_weights / serq_unpack_act return) to
 * the FP6 operand layouts: weights in 32-channel x 64-channel fragments, activations row by row. */
int serq_fp6_pack_weights(const int8_t* codes, int64_t N, int64_t K, void* W6_out, void* stream);
int serq_fp6_pack_act(const int8_t* codes, int64_t M, int64_t K, void* X6_out, void* stream);

/* acc[m,n] = sum_k Xq[m,k] Wq[n,k] as INT32 [M,N] (row stride ldacc, a multiple of 4), from one plain
 * LDS-tiled kernel in two instantiations that differ only in the operand route:
 *   fp6 = 0: X, W are the 4-bit buffers of serq_quantize_act (abits = 4) / serq_pack_weights, widened in
 *            registers and multiplied on the int8 instruction;
 *   fp6 = 1: X, W are the buffers of serq_fp6_pack_act / serq_fp6_pack_weights, multiplied on the scaled
 *            instruction with both formats E2M3 and both scales 2^0, the fp32 sums converted to INT32. */
int serq_proto_gemm_i32(const void* X, const void* W, int fp6, int64_t M, int64_t N, int64_t K, int32_t* acc_out,
                        int64_t ldacc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SERQ_FP6_H_ */
