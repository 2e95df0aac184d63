/*
 * dpclip_probes -- measurement probes that ship with libdpclip.so.
 *
 * They are not part of the method: each launches one small kernel that
 * exercises a single unit of the MI355X the way the library's kernels use it,
 * so that a benchmark can quote the library's kernels against what this very
 * part sustains (next to the published peaks).  The caller times the launch
 * (HIP events on `hip_stream`); the amount of work of one launch is returned.
 * Conventions as in dpclip.h: device pointers, asynchronous on `hip_stream`,
 * dp_status errors, nothing allocated.
 */
#ifndef DPCLIP_PROBES_H
#define DPCLIP_PROBES_H

#include "dpclip.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Floats that `sink` of the probes below must hold (every thread writes one
 * value, so that the compiler keeps the probe's work). */
#define DP_PROBE_SINK_FLOATS (1024 * 256)

/* Matrix units with operands in registers and no memory traffic at all: 1024
 * workgroups of 4 waves (two per SIMD when resident), each wave issuing `iters`
 * times 8 independent 32x32 MFMAs of `dtype`'s instruction (DP_BF16:
 * 32x32x16 bf16, DP_F16: 32x32x16 f16, DP_F8_*: 32x32x64 f8f6f4 with the
 * type's formats).  random_operands != 0: four operand pairs of pseudo-random
 * bits (finite values of magnitude about one) taken in turn, as streaming data
 * looks to the multipliers; 0: one operand pair, every value 1.0, which is
 * what reaches the published peak.  *flops receives the floating-point
 * operations of the launch.  DP_F32 and other types: DP_ERR_UNSUPPORTED. */
dp_status dp_probe_mfma(dp_dtype dtype, int random_operands, int64_t iters,
                        float* sink, double* flops, void* hip_stream);

/* Plain streaming read of `bytes` bytes (a multiple of 16) at `src`, 16 bytes
 * per lane and sixteen loads in flight per lane, every workgroup on a
 * contiguous range of its own: what a kernel that only reads
 * can get from HBM (src larger than the 256 MB last-level cache) or from that
 * cache (src smaller, second pass). */
dp_status dp_probe_read(const void* src, size_t bytes, float* sink, void* hip_stream);

/* LDS read rate of a compute unit: 1024 workgroups of 4 waves (two per compute
 * unit when resident: 8 waves as in the library's kernels), each wave issuing
 * `iters` times 8 reads of kind
 *   0: ds_read_b128, lanes reading consecutive 16-byte pieces
 *   1: ds_read_b64_tr_b16 (the transposing read of the clipped-sum kernels),
 *      4 rows x 64 bytes per 32 lanes, rows of 512 bytes with the kernels'
 *      chunk swizzle
 * *bytes receives the bytes that all lanes of the launch receive. */
dp_status dp_probe_lds_read(int kind, int64_t iters, float* sink, double* bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DPCLIP_PROBES_H */
