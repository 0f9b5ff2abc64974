/*
 * ge_probes -- measured ceilings of the device, for the measurement report only.
 *
 * They are not part of the operator and live in a library of their own (libge_probes.so).  The paper times its kernels against a
 * reference implementation on the same GPU ("Experiments", evaluation setup:
 * warm-up, then repeated timed runs); here the reference points are what the
 * GPU itself sustains: a register-resident bf16 MFMA loop under the power cap,
 * a plain streaming fp32 store, and a stream whose mix of reads and writes is
 * that of the workload being reported (a store-only stream, a copy and a
 * read-only stream reach different rates on this memory system).  bench.py
 * reports them next to the datasheet peaks.
 *
 * All pointers are DEVICE pointers owned by the caller.  The calls enqueue one
 * kernel on `stream` (hipStream_t as void*, NULL = default stream) and return
 * without synchronising; the caller times them.  On a status other than GE_OK
 * nothing was enqueued.
 */
#ifndef GE_PROBES_H
#define GE_PROBES_H

#include <stddef.h>
#include "gemm_epilogue.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Dense v_mfma_f32_16x16x32_bf16 loop with operands held in registers.
 *   operands  at least 65536 bytes of bf16 values, 16-byte aligned, only read (their
 *             statistics set the switching power, hence the sustained clock);
 *   sink      blocks*512 floats, written once at the end (keeps the loop alive);
 *   blocks    workgroups of 512 threads (8 wavefronts), 1 .. 65536;
 *   iters     loop trips, 1 .. 1<<24; each wavefront issues 16 MFMAs per trip.
 * FLOP per launch = blocks * 8 * iters * 16 * (2*16*16*32).
 * Errors: GE_ERR_NULL, GE_ERR_ALIGN, GE_ERR_SHAPE (blocks or iters out of range), GE_ERR_LAUNCH. */
ge_status_t ge_probe_mfma_bf16(const void *operands, float *sink, int blocks, int iters, void *stream);

/* Streaming store: dst[i] = value for i < count, 16 bytes per lane, consecutive lanes on
 * consecutive addresses.  dst must be 16-byte aligned and count a multiple of 4.
 * Errors: GE_ERR_NULL, GE_ERR_ALIGN, GE_ERR_SHAPE (count == 0 or not a multiple of 4), GE_ERR_LAUNCH. */
ge_status_t ge_probe_store_f32(float *dst, size_t count, float value, void *stream);

/* Stream with a chosen mix: `trips` steps, each reading `reads` and writing `writes` pieces
 * of 16 bytes, consecutive lanes on consecutive pieces (src holds reads*trips*16 bytes, dst
 * writes*trips*16 bytes, at least 16; with writes == 0 dst is a sink that is not written).
 * (reads, writes) is one of (1,0) (2,0) (1,1) (1,2) (1,4) (1,8) (0,1); src may be NULL when
 * reads == 0.  Bytes moved per launch = (reads + writes) * trips * 16.
 * Errors: GE_ERR_NULL, GE_ERR_ALIGN (16 bytes), GE_ERR_SHAPE (trips), GE_ERR_CONFIG (mix), GE_ERR_LAUNCH. */
ge_status_t ge_probe_stream_mix(const void *src, void *dst, size_t trips, int reads, int writes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
