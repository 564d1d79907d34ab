/*
 * ckpt_probe.h - measurement probes of the MI355X (gfx950) checkpoint-selection
 * library: small kernels of known work that measure what the part delivers, so
 * that the roofline fractions of the solver kernels can be quoted against
 * measured rates next to the data-sheet ones (8 TB/s HBM; 256 compute units x
 * 64 lanes x 2.4 GHz = 39.32e12 32-bit integer lane-operations per second).
 * They compute nothing of the method.  Every pointer is a DEVICE pointer owned
 * by the caller; each call enqueues one kernel on `hip_stream` (a hipStream_t
 * as void*) and returns a ckpt_status; the caller times it with HIP events.
 */
#ifndef CKPT_PROBE_H
#define CKPT_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streams `bytes` (a multiple of 16) from src and writes 8 bytes to sink: the
 * read rate of a kernel that does nothing else. */
int ckpt_probe_hbm_read(const void *src, size_t bytes, void *sink, void *hip_stream);

/* Copies `bytes` (a multiple of 16) from src to dst (no overlap): one read and
 * one write per byte. */
int ckpt_probe_hbm_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Vector-integer issue rate: `waves` wavefronts (a multiple of 4) each execute
 * iters x 256 independent instructions of one kind on all 64 lanes.
 * which: 0 v_add_u32, 1 v_min_i32, 2 v_max_u32, 3 v_cndmask_b32.
 * Lane-operations per launch = waves x 64 x iters x 256.  sink: 4 bytes. */
int ckpt_probe_valu(int which, int64_t waves, int32_t iters, void *sink, void *hip_stream);

/* LDS instruction rate: `waves` one-wave workgroups each execute iters x 16
 * LDS instructions of one kind, every lane on a word of its own (no bank
 * conflicts), 16 rows of 256 bytes.
 * which: 0 ds_read_b32, 1 ds_write_b32, 2 ds_max_u32 (no return value).
 * LDS lane-accesses per launch = waves x 64 x iters x 16.  sink: 4 bytes. */
int ckpt_probe_lds(int which, int64_t waves, int32_t iters, void *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CKPT_PROBE_H */
