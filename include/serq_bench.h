/*
 * serq_bench.h -- measuring sticks exported by libserq.so for benchmarks.  No part of the layer: they
 * say what this part sustains with nothing in the way (matrix instructions only, reads only), so that a
 * kernel's rate can be put next to it.  Device pointers, 16-byte aligned unless noted; all only launch
 * (asynchronous on `stream`) and return SERQ_OK or a negative SERQ_E* code.
 */
#ifndef SERQ_BENCH_H_
#define SERQ_BENCH_H_

#include "serq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * serq_bench_mfma_peak: `workgroups` x 4 waves each run `iters` x 16 int8 MFMAs (32x32x32) on operands
 *   held in registers: 2 * 32*32*32 * 16 * iters * 4 * workgroups integer operations and nothing else.
 *   operands: 32 KiB (256 threads x 8 x 16 bytes: 4 A and 4 B operand registers per thread), device memory;
 *   the achieved rate depends on these bytes.  sink: 4 bytes of device memory (never written in practice).
 * serq_bench_mfma_fp4_peak: the same loop with the block-scaled FP4 MFMA (32x32x64, E2M1 codes, block
 *   exponent 127): 2 * 32*32*64 * 16 * iters * 4 * workgroups operations.  Each 16-byte operand slot holds
 *   the 32 codes of one lane.
 * serq_bench_read: reads [src, src + bytes) once with 16-byte loads from `workgroups` workgroups and
 *   does nothing else.  bytes a multiple of 16.
 */
int serq_bench_mfma_peak(const void* operands, int iters, int workgroups, void* sink, void* stream);
int serq_bench_mfma_fp4_peak(const void* operands, int iters, int workgroups, void* sink, void* stream);
int serq_bench_read(const void* src, size_t bytes, int workgroups, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SERQ_BENCH_H_ */
