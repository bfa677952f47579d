/*
 * kvcapsule_dev.h -- developer and measurement aids of libkvcapsule.so.
 *
 * Nothing here is part of the KVCapsule method or needed by a caller of kvcapsule.h: these symbols
 * exist so that the two device code paths can be checked against each other, so that the benchmark
 * can set the library's rates beside what the chip reaches on a plain read, and so that tuning
 * choices can be swept from a script.  Same conventions as kvcapsule.h.
 */
#ifndef KVCAPSULE_DEV_H
#define KVCAPSULE_DEV_H

#include "kvcapsule.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The same operation and contract as kvc_reconstruct_attend_decode, forced onto
 * the shape-agnostic scalar kernels (any n, m, d <= 256, either dtype).  The
 * main entry point uses these for shapes its matrix-core kernels do not cover;
 * this symbol exists so both code paths can be checked against each other. */
kvc_status kvc_reconstruct_attend_decode_generic(const kvc_shape *shape, const kvc_params *params,
                                                 const void *q, const void *Kc, const void *Vc,
                                                 void *K_text, void *V_text,
                                                 int32_t text_len, int32_t text_cap,
                                                 const void *k_new, const void *v_new,
                                                 float softmax_scale,
                                                 void *out, float *lse_out,
                                                 void *workspace, size_t workspace_bytes,
                                                 void *stream);

/* Same contract as kvc_compress, forced onto the scalar kernels. */
kvc_status kvc_compress_generic(const kvc_shape *shape, const kvc_params *params,
                                const void *K, const void *V,
                                int64_t stride_b, int64_t stride_h, int64_t stride_s,
                                int32_t vis_start, int32_t seq_len,
                                void *Kc, void *Vc,
                                void *workspace, size_t workspace_bytes, void *stream);

/* Measurement aid (no part of the method): a plain streaming read of `bytes` bytes of device
   memory at `buf` (16-byte aligned, bytes a multiple of 16), 16 bytes per lane, grid-stride, every
   value folded into a checksum that is written to `sink` (device, at least 4 bytes) only if it
   equals a fixed pattern.  Timing it over a buffer much larger than the caches gives the
   streaming-read rate this chip reaches, to set beside the published HBM peak.  Asynchronous on
   `stream`.  Errors: KVC_ERR_NULL, KVC_ERR_ALIGN, KVC_ERR_HIP. */
kvc_status kvc_probe_read(const void *buf, size_t bytes, void *sink, void *stream);

/* Full-cache decode: steps of 128 cache rows per split (0 restores the built-in rule).  Process-wide,
 * not thread-safe; for sweeps only. */
void kvc_dev_full_decode_chunk_steps(int32_t steps);

/* Knobs of the matrix-core decode kernels, for tests and sweeps; a negative value leaves a knob as it is.
 * Process-wide, not thread-safe.
 *  row_tiles : 16-row tiles of query rows per workgroup of the third kernel (1, 2, or 4 -- 4 only for
 *              n = 256); 0 restores the built-in rule.
 *  separate  : 1 runs the first two kernels (compressed scores; probabilities) as separate launches even
 *              where they could run as one; 0 restores the rule (one launch when all its workgroups can
 *              be resident at once).
 *  wait_ticks: in the one-launch form, how long a workgroup waits for the other workgroups of its group
 *              to deliver their compressed scores before it computes them itself, in units of 10 ns
 *              (default 2000 = 20 us; 0: it never waits, which tests use to run that path). */
void kvc_dev_decode_knobs(int32_t row_tiles, int32_t separate, int32_t wait_ticks);

/* Which decode kernels serve a call that comes with kvc_params.theta_packed (process-wide):
 *  -1 the built-in rule (the one-pass kernel for calls of fewer than two workgroups per compute unit whose
 *     shape has an instance), 0 never the one-pass kernel, 1 the one-pass kernel wherever an instance exists. */
void kvc_dev_stream_decode(int32_t mode);

/* Decode calls the one-pass kernel has served since the library was loaded (host-side count). */
int64_t kvc_dev_stream_calls(void);

/* Workgroups that gave up waiting and computed alone since the library was loaded (current device;
 * synchronises with the device), or -1. */
int64_t kvc_dev_decode_fallbacks(void);

/* Developer switches of the matrix-core compress kernel (process-wide; negative leaves a setting
 * unchanged).
 *  waves: 4 or 8 wavefronts per workgroup; 0 restores the built-in rule (8 when a workgroup owns more
 *         than 4 tiles of 16 rows of U).
 *  jt   : workgroups per image block (clamped to what the kernel supports); 0 restores the cost model. */
void kvc_dev_compress_knobs(int32_t waves, int32_t jt);

#ifdef __cplusplus
}
#endif
#endif /* KVCAPSULE_DEV_H */
