/*
 * rf_diag.h - measurement aids and the fusion-level study, exported by the same library as
 * rf.h but not part of the cascaded-reduction path.  Nothing in rf.h depends on them; they
 * exist so that the benchmark can report measured ceilings (a plain copy, a read-only sweep,
 * an MFMA-only loop) next to the published peaks, scale hardware traffic counters,
 * repeat the paper's fusion-level comparison of the safe-softmax cascade (Section 5.3) and
 * compare two tilings of the attention cascade.
 * Conventions (device pointers owned by the caller, asynchronous on `stream`, status codes)
 * are those of rf.h.
 */
#ifndef RF_DIAG_H_
#define RF_DIAG_H_

#include "rf.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Fusion-level study of the safe-softmax cascade (Section 5.3 of the paper: the same cascade
 * fused at different levels of the reduction tree).  Same result as rf_safe_softmax on
 * x, y : [rows, n] bf16, n % 8 == 0, n <= 8192, rows 16-byte aligned; what differs is where
 * the two reductions are fused:
 *   level 0  not fused: three kernels (max, sum of exponentials, normalise), three reads of x;
 *            ml_buf: device memory for 2 * rows floats (the row maxima and sums)
 *   level 1  fused per lane: every lane runs the incremental form over its own elements,
 *            lane states merged with the level-k expression
 *   level 2  fused per wavefront: what rf_safe_softmax runs for rows of up to 4096 values
 *   level 3  fused per workgroup: lane states merged across four wavefronts through LDS
 *   level 4  fused across workgroups (the paper's inter-block level): a row is cut into four
 *            segments handled by wavefronts of different workgroups; the first kernel stores
 *            each segment's state (m, l), the second merges them with the level-k expression
 *            and normalises; two reads of x.  ml_buf: device memory for 8 * rows floats
 * ml_buf is ignored for levels 1..3.
 */
RF_API rf_status rf_diag_softmax_level(const rf_tensor* x, rf_tensor* y, int level, float* ml_buf,
                                       rf_stream stream);

/*
 * Tiling study of the fused attention cascade (Section 4.3 single-segment strategy, Appendix
 * A.4): the same result as rf_cascade_attention with causal == 0, computed by a kernel that
 * gives every wavefront 64 query rows and a SIMD to itself (the entry point in rf.h gives it
 * 32 rows and shares the SIMD between two wavefronts).  Kept to measure the two tilings side
 * by side.  q, k, v, o as for rf_cascade_attention, bf16 only, head dimension 128, at least
 * 64 keys, row pitches of k and v below 2^24 elements; other shapes: RF_ERR_UNSUPPORTED.
 */
RF_API rf_status rf_diag_attention_wide(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                                        rf_tensor* o, float scale, rf_stream stream);

/*
 * Measurement aids, not part of the cascaded-reduction path.  They provide the two
 * measured ceilings that roofline fractions are reported next to (a plain copy kernel for
 * HBM, an MFMA-only loop for the matrix pipe) and the reference dispatch that scales the
 * FETCH_SIZE / WRITE_SIZE hardware counters.
 *   rf_diag_copy : dst[0..bytes) = src[0..bytes); device pointers, 16-byte aligned,
 *                  bytes a multiple of 16, buffers must not overlap.
 *   rf_diag_read : reads src[0..bytes) once with non-temporal 128-bit loads and writes one
 *                  32-bit word per wavefront into `sink`, a device buffer of at least
 *                  RF_DIAG_READ_SINK_BYTES bytes (content: the XOR of what the wavefront read; the rest of the buffer is left as it was).
 *                  The ceiling for kernels that only read HBM.
 *   rf_diag_mfma : `workgroups` workgroups of 4 wavefronts each issue iters*32 dense bf16
 *                  32x32x16 MFMAs (32768 flop each) on constant (random_operands == 0) or
 *                  pseudo-random operands; `sink` is a device buffer of workgroups*256 floats
 *                  that receives the accumulator sums.
 */
RF_API rf_status rf_diag_copy(const void* src, void* dst, int64_t bytes, rf_stream stream);
#define RF_DIAG_READ_SINK_BYTES (8192 * 4 * 4)
RF_API rf_status rf_diag_read(const void* src, int64_t bytes, void* sink, rf_stream stream);
RF_API rf_status rf_diag_mfma(float* sink, int workgroups, int iters, int random_operands,
                              rf_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* RF_DIAG_H_ */
