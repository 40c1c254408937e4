/*
 * zqfp_probe.h -- measurement probes exported by libzqfp next to its C ABI
 * (zqfp.h).  They are tooling for the benchmark, no part of the W4A8 path: two
 * kernels that show what the device itself sustains, so that roofline
 * fractions can be quoted against measured ceilings as well as published peaks.
 */
#ifndef ZQFP_PROBE_H
#define ZQFP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Both only enqueue work on `stream` (a hipStream_t as void*); the caller times it.
 * Error codes are those of zqfp.h.
 *
 * zqfp_probe_stream_read -- a plain streaming read of `bytes` bytes at `src`
 *   (device, 16-byte aligned; the last bytes % (workgroups * 32 KB) are not
 *   read).  sink: device, >= 4 * workgroups bytes, written at most once per
 *   workgroup with a value that means nothing.
 * zqfp_probe_mfma -- `iters` rounds of 32 independent
 *   v_mfma_scale_f32_16x16x128_f8f6f4 instructions (FP8 x FP4) per wave, 8 waves
 *   per workgroup, operands held in registers: 2 * 16*16*128 * 32 * 8 * iters *
 *   workgroups floating-point operations in total.  operands: device, 4096
 *   bytes of anything; sink: device, >= 2048 * workgroups bytes.
 *
 * Return ZQFP_OK, ZQFP_E_NULL, ZQFP_E_SHAPE (non-positive sizes), ZQFP_E_ALIGN
 * or ZQFP_E_HIP.
 */
int zqfp_probe_stream_read(const void *src, int64_t bytes, void *sink,
                           int workgroups, void *stream);
int zqfp_probe_mfma(const void *operands, void *sink, int iters,
                    int workgroups, void *stream);

/*
 * zqfp_probe_force_tile_plan -- tuning hook for sweeps and tests: every following
 * zqfp_w4a8_gemm* call with more than 16 tokens (and zqfp_gemm_workspace_bytes,
 * which must agree with it) uses bm x bn output tiles, `kg` wave groups per
 * workgroup and `ksplit` slices of K (1 = none) instead of planning them from
 * the problem size.  Tile shapes: 64x128, 64x192, 64x256, 128x128, 128x192,
 * 128x256, 256x256; kg 1, or 2 with 64-row tiles (it then needs an even number
 * of 128-wide k-tiles per slice, else one group runs); ksplit 1..64 (capped at
 * the number of k-tiles).  (0, 0, 0, 0) returns to automatic planning.
 * Process-wide, not meant for concurrent use with GEMM calls of other threads.
 * Returns ZQFP_OK or ZQFP_E_SHAPE.
 */
int zqfp_probe_force_tile_plan(int bm, int bn, int ksplit, int kg);

/*
 * zqfp_probe_force_decode_waves -- tuning hook: 8 (default) or 16 waves per
 * workgroup of the decode GEMM (at most 16 tokens) where K <= 4096.
 * Process-wide.  Returns ZQFP_OK or ZQFP_E_SHAPE.
 */
int zqfp_probe_force_decode_waves(int nw);

#ifdef __cplusplus
}
#endif
#endif /* ZQFP_PROBE_H */
