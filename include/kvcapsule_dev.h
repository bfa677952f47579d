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
                                int32_t vis_start,
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

#ifdef __cplusplus
}
#endif
#endif /* KVCAPSULE_DEV_H */
