/*
 * libmorphkv -- diagnostics.  NOT part of the product interface (include/morphkv.h): these calls exist for the
 * parity tests (the fused scores a decision was taken on), for profiling (phase time stamps of the decode
 * kernel, in a separate build of it) and as yardsticks for hardware counters and bandwidth (a plain copy and
 * a plain read of known size).  Same conventions as morphkv.h: return codes, device pointers, the caller's stream.
 */
#ifndef MORPHKV_DIAG_H
#define MORPHKV_DIAG_H
#include "morphkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Optional capture of the fused scores each decode step takes its decision on:
 * F device [U][n_pad] fp32, n_pad = Cs + R rounded up to a multiple of 32 (Cs as for morphkv_export_positions): the
 * score of every eviction candidate -- a token older than the window that includes the new token -- at the slot
 * morphkv_export_positions reported for it before the step; other elements are left as they are.  NULL to stop.
 * Costs 4 bytes written per older token per step while enabled. */
int morphkv_capture_scores(morphkv_handle *h, float *F);

/* clocks device [U][8] int64, or NULL to stop.  bf16 configurations with head_dim 128 only (MORPHKV_EINVAL at the
 * next decode step otherwise).  While set, every decode step runs a separate build of the kernel that stores the
 * constant-rate device clock (100 MHz) per unit at: 0 kernel start, 1 end of the K pass, 2 end of
 * softmax/record, 3 end of the V pass, 4 end of the step, 5 / 6 last / first wave reaches the first
 * barrier, 7 first barrier passed. */
int morphkv_capture_phase_clocks(morphkv_handle *h, long long *clocks);

/* A plain device-to-device copy of `bytes` (multiple of 16) with a grid-stride kernel,
 * enqueued on the stream.  It moves a known number of bytes each way and serves as the yardstick the
 * profiler's HBM counters are scaled by. */
int morphkv_calib_copy(void *dst, const void *src, size_t bytes, void *stream);

/* A plain read of `bytes` (multiple of 16) of device memory; every 16-byte piece is loaded once and
 * folded into sink[256] (device, uint32, xor-accumulated: zero it first if the value matters).  Times what the
 * device sustains when a kernel only streams: the practical ceiling next to the 8 TB/s of the data sheet.  Buffers
 * of more than 208 MiB are read with non-temporal loads, as the decode kernels read what they do not keep in the
 * memory-side cache. */
int morphkv_calib_read(uint32_t *sink, const void *src, size_t bytes, void *stream);

/* How a decode launch over n_units units (all of the handle's, or one layer's) is laid out: 1 workgroup per unit
 * = the fused kernel; more = the split kernel, each workgroup on blocks_per_workgroup blocks of 32 slots.  For a
 * handle whose layers all keep every token: the workgroups per unit of the kernel made for those layers (1 or more)
 * and the blocks each takes when the layer is full. */
int morphkv_decode_plan(morphkv_handle *h, int32_t n_units, int32_t *workgroups_per_unit, int32_t *blocks_per_workgroup);

#ifdef __cplusplus
}
#endif
#endif
