/*
 * abq_probe.h — measurement aids built as a library of their own (libabq_probe.so); no part of the
 * quantized-matmul method and not linked into libabq.so.  The benchmark uses them to price achieved figures
 * against what the machine delivers for the same kind of work, beside its published peaks, and to push the
 * timed weight buffers out of the last-level cache.  Conventions as in abq.h: plain C, int status (0 = ok,
 * negative = the ABQ_ERR_* value of the same meaning), device pointers 16-byte aligned, work enqueued on the
 * caller's stream, nothing allocated.  Each call enqueues ONE kernel; the caller times it.
 */
#ifndef ABQ_PROBE_H
#define ABQ_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streaming read of `bytes` bytes (a multiple of 16) at `buf` with 128-bit non-temporal loads, the access
 * the decode kernel uses for its weights; nothing is written (`sink`: >= 2 KiB of device memory that
 * stays untouched in practice). */
int abq_probe_stream_read(const void* buf, size_t bytes, void* sink, void* stream);

/* Reads that hit in L2: 8 regions of `region_bytes` (a multiple of 32 KiB, at most 64 MiB) lie back to back at `buf`;
 * every compute unit runs `wgs_per_cu` (1..8) workgroups of 256 threads, and a workgroup reads the whole region of its
 * XCD `passes` times with 128-bit loads, eight in flight per lane.  With regions of one or two MiB the data stays in
 * each XCD's L2 after the first pass.  `buf` holds 8 * region_bytes (the caller's to guarantee).  Status as the other
 * probes (null pointer, argument out of range, misaligned pointer).  abq_probe_l2_read_bytes: the bytes one such
 * launch requests. */
int abq_probe_l2_read(const void* buf, size_t region_bytes, int passes, int wgs_per_cu, void* sink, void* stream);
double abq_probe_l2_read_bytes(size_t region_bytes, int passes, int wgs_per_cu);

/* Dense int8 MFMA issue loop on every CU: `iters` rounds of eight independent 16x16x64 MFMAs per wave,
 * 32 waves per CU.  pattern 0: three of four operand bytes zero; pattern 1: every operand byte non-zero
 * and varying from lane to lane (the sustained rate depends on the data: the chip lowers its clock on
 * the latter).  abq_probe_mfma_i8_ops(iters) is the
 * number of integer operations (2 per MAC) one such launch performs on the current device (0 for
 * iters < 1). */
int abq_probe_mfma_i8(int iters, int pattern, void* sink, void* stream);
double abq_probe_mfma_i8_ops(int iters);

/* The same issue loop on gfx950's 4-bit floating-point MFMA (16x16x128, E2M1 operands, binary32 accumulate, block
 * scales of one; the codes of a 1- or 2-bit operand are E2M1 values and their product sums stay exact): the rate a
 * very-low-bit prefill kernel could price itself against.  Arguments, patterns and errors as abq_probe_mfma_i8;
 * abq_probe_mfma_f4_ops(iters) counts 2 operations per multiply-accumulate. */
int abq_probe_mfma_f4(int iters, int pattern, void* sink, void* stream);
double abq_probe_mfma_f4_ops(int iters);

#ifdef __cplusplus
}
#endif
#endif /* ABQ_PROBE_H */
