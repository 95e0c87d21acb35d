/*
 * ltri_bench.h — measurement helpers exported by libltri.so for bench.py. They are not part of the
 * product boundary (ltri.h): no step of the path calls them. They give the ceilings of the GPU at hand,
 * to be read next to the published peaks: the attention of Sec. 3.4's third step is a dense bf16
 * contraction (priced against the matrix-core rate), the gather that precedes it is a pure copy and the
 * one-token step a pure read (priced against the memory rate).
 *
 * Each call launches a small kernel on hip_stream (hipStream_t, NULL = default stream), times it with
 * events on that stream and synchronises; no context is needed. Device pointers are the caller's.
 * Errors: LTRI_EINVAL (NULL pointers, sizes), LTRI_EHIP.
 */
#ifndef LTRI_BENCH_H
#define LTRI_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Rate of back-to-back v_mfma_f32_32x32x16_bf16 on every SIMD, in TFLOP/s. sink: device buffer of at
 * least 512 KiB that the kernel may overwrite. random_operands: 0 = all operands 1.0, 1 = pseudo-random
 * operands; the clock the chip sustains depends on the operand data, real inputs behave like the
 * random case. */
int32_t ltri_measure_mfma_peak(void* sink, size_t sink_bytes, int32_t random_operands, void* hip_stream,
                               double* tflops);
/* Read + write rate, in GB/s, of a streaming copy of `bytes` bytes (a multiple of 16384, at least 1 MiB)
 * from src to dst (device, disjoint): every lane keeps four independent 16-byte loads in flight. Use
 * buffers well beyond the last-level cache (256 MiB) for a memory figure. */
int32_t ltri_measure_copy_peak(void* dst, const void* src, size_t bytes, void* hip_stream, double* gbps);
/* Read rate, in GB/s, of a streaming read of `bytes` bytes (a multiple of 16384, at least 1 MiB) from src
 * (device), same access pattern; sink: device buffer of at least 512 KiB that the kernel may overwrite. */
int32_t ltri_measure_read_peak(const void* src, size_t bytes, void* sink, size_t sink_bytes, void* hip_stream,
                               double* gbps);

#ifdef __cplusplus
}
#endif
#endif /* LTRI_BENCH_H */
