/*
 * ta_probe.h -- C ABI of the measurement aids that go with the paged-KV attention
 * library (libta_probe.so, a library of its own: nothing of the hot path depends on
 * it and no hot-path entry point lives here).  No passage of the paper stands behind
 * these calls: they measure, they compute nothing.  The benchmark uses them to state,
 * in the same run as its kernel timings, what the matrix cores sustain on operands of
 * a given kind and what a plain streaming read delivers.
 *
 * All pointers are DEVICE pointers; work is enqueued on hip_stream (hipStream_t as
 * void*, NULL = default stream) and not awaited; nothing is allocated.  Return value:
 * 0, -1 for an invalid argument, -3 when a HIP call failed.
 */
#ifndef TA_PROBE_H
#define TA_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TA_PROBE_API __attribute__((visibility("default")))

/*
 * Measurement aid (no paper passage: it measures, it computes nothing useful).
 * Runs iters x 16 independent v_mfma_f32_32x32x16_bf16 per wave, one wave per
 * SIMD on 256 workgroups, on the caller's operand values, so that the caller
 * can time the rate the matrix cores sustain on data of that kind: the shader
 * clock under such a load is set by power management and depends on how many
 * operand bits toggle.  Floating-point operations enqueued:
 *   TA_PROBE_FLOP_PER_ITER * iters.
 *
 *   operands  DEVICE, 8192 bytes, 16-byte aligned: eight operand registers
 *             (A0, B0, A1, B1, ...) x 64 lanes x 8 bf16, any finite values
 *   iters     >= 1
 *   sink      DEVICE, TA_PROBE_SINK_BYTES, written (keeps the work alive)
 *   hip_stream  hipStream_t as void*, may be NULL
 *
 * Returns -1 for NULL or misaligned pointers or iters < 1.
 * Nothing is allocated; the work is enqueued, not awaited.
 */
#define TA_PROBE_FLOP_PER_ITER (256.0 * 4.0 * 16.0 * 2.0 * 32.0 * 32.0 * 16.0)
#define TA_PROBE_SINK_BYTES (256 * 256 * 4)
TA_PROBE_API int ta_matrix_core_probe(const void *operands, int32_t iters, void *sink, void *hip_stream);

/*
 * Measurement aid (no paper passage).  Reads the buffer once with the load shape
 * of the decode kernel (16 bytes per lane, non-temporal, four loads in flight)
 * and no arithmetic, so that the caller can time the read bandwidth the memory
 * system delivers to such a kernel.
 *
 *   src     DEVICE, `bytes` bytes, 16-byte aligned, only read
 *   bytes   a positive multiple of 16
 *   sink    DEVICE, TA_STREAM_SINK_BYTES, written
 *
 * Returns -1 for NULL or misaligned pointers or a bad size.
 */
#define TA_STREAM_SINK_BYTES (8192 * 256 * 4)
TA_PROBE_API int ta_stream_read_probe(const void *src, size_t bytes, void *sink, void *hip_stream);

/*
 * Measurement aid (no paper passage).  Two waves per SIMD on every CU; per iteration every wave
 * issues matrix_per_iter independent v_mfma_f32_32x32x16_bf16 and vector_per_iter independent
 * fp32 FMAs, interleaved.  Timing (8, 0), (0, 80) and (8, 80) shows whether the two kinds of
 * work overlap on a SIMD: if a matrix instruction left the vector issue port alone, (8, 80) would
 * take as long as the longer of the other two.
 *
 *   matrix_per_iter  0 or 8;  vector_per_iter  0, 40 or 80 (not both 0)
 *   iters            >= 1
 *   sink             DEVICE, TA_ISSUE_SINK_BYTES, written
 *
 * Returns -1 for a combination that is not built, a NULL sink or iters < 1.
 */
#define TA_ISSUE_SINK_BYTES (256 * 512 * 4)
TA_PROBE_API int ta_issue_port_probe(int32_t matrix_per_iter, int32_t vector_per_iter, int32_t iters, void *sink,
                                     void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TA_PROBE_H */
