/*
 * mux_probes.h - measurement probes shipped inside libmux.so, NOT part of the product boundary
 * declared in mux.h: what the GPU at hand sustains for a plain streaming read and for
 * back-to-back matrix instructions.  Reports (bench.py) put the attention kernels' figures next
 * to these ceilings.  Both calls only enqueue on `stream`; the caller times them.
 */
#ifndef MUX_PROBES_H
#define MUX_PROBES_H

#include "mux.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------------
 * mux_probe_stream_read: `workgroups` x 4 waves read the whole 8 KiB chunks of `bytes`
 *   (>= 8192) of DEVICE memory at `buf` (16-byte aligned) once, 16 bytes per lane per load;
 *   `sink` = 4 bytes of DEVICE memory (never written in practice).
 * mux_probe_mfma: `workgroups` x 4 waves each issue iters x 16 (8 independent chains)
 *   v_mfma_f32_16x16x32_bf16; *flops (HOST, may be NULL) = floating-point operations of
 *   the launch; `sink` = 4 bytes of DEVICE memory.
 * ------------------------------------------------------------------------------- */
MUX_API int mux_probe_stream_read(const void *buf, size_t bytes, void *sink, int32_t workgroups, void *stream);
MUX_API int mux_probe_mfma(void *sink, int32_t workgroups, int32_t iters, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MUX_PROBES_H */
