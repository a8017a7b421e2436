/*
 * sdp_measure.h -- measurement aids of libsdp_hip.so.  Nothing here is a step of the method: per-kernel
 * event timing for the benchmark, and a probe of the rate the matrix cores sustain on given operand values.
 * The method's own entry points are in sdp.h.
 */
#ifndef SDP_MEASURE_H
#define SDP_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------------------------
 * Per-kernel timing.  With profiling on, every kernel launch is bracketed by HIP events on its
 * stream.  sdp_profile_read synchronises those events and returns, for up to `cap` distinct
 * kernel names, the launch count and total milliseconds since the last reset.
 *   names  host array of cap pointers, set to static strings owned by the library
 *   calls, ms host arrays of cap entries.   Returns the number of entries filled, or < 0.
 * sdp_profile_filter(name) restricts the bracketing to launches of that one kernel name (NULL or ""
 * = all): events between back-to-back kernels keep them from overlapping their launch and drain
 * phases, so timing every kernel slows a step by about a tenth; timing one kernel does not.
 * ------------------------------------------------------------------------------------------- */
int sdp_profile_enable(int on);
int sdp_profile_filter(const char* name);
int sdp_profile_reset(void);
int sdp_profile_read(int cap, const char** names, int64_t* calls, double* ms);

/* Tile shape and workgroup -> tile order of the last MFMA contraction launched under `name` (e.g. "mlp_dw")
 * while timing was on: what a recorded counter figure for that kernel has to be matched against.
 *   tile_m, tile_n: outputs per workgroup;  group_m: tile-rows walked together;  stacked: 1 if the problems of a
 *   batched launch that share an operand were walked as one matrix.  All host out.
 * INVALID_ARG when a pointer is null or no such launch has been seen. */
int sdp_profile_launch_shape(const char* name, int* tile_m, int* tile_n, int* group_m, int* stacked);

/* ---------------------------------------------------------------------------------------------
 * Measurement aid (not a step of the method): the rate at which this GPU's matrix cores sustain the
 * bf16 MFMA instruction the contractions use, on operand values supplied by the caller and with no
 * memory traffic inside the loop.  The clock the chip holds under MFMA load depends on the operand
 * values (power), so this is the practical ceiling that the contractions' rates can be read against.
 *   operands  device, sdp_probe_mfma_operand_bytes() bytes of bf16 values, 16-byte aligned
 *   shape     16: v_mfma_f32_16x16x32_bf16 (the instruction the contractions use; sdp_probe_mfma_tflops measures
 *             this one), 32: v_mfma_f32_32x32x16_bf16 (the same flops draw more power on random operands)
 *   blocks    workgroups of 512 lanes to launch (a few per CU), iters: 1,048,576 flops per wave each
 *   sink      device scratch, sdp_probe_mfma_sink_bytes(blocks) bytes (written, never read)
 *   tflops    host out.  The call launches the loop twice, times the second launch with HIP events
 *             and synchronises `stream`.
 * ------------------------------------------------------------------------------------------- */
size_t sdp_probe_mfma_operand_bytes(void);
size_t sdp_probe_mfma_sink_bytes(int blocks);
int sdp_probe_mfma_tflops(const void* operands, int blocks, int iters, void* sink, double* tflops, void* stream);
int sdp_probe_mfma_shape_tflops(int shape, const void* operands, int blocks, int iters, void* sink, double* tflops,
                                void* stream);

/* ---------------------------------------------------------------------------------------------
 * Measurement aid (not a step of the method): the rate at which a plain streaming kernel moves data through
 * HBM on this GPU, with the 16-byte non-temporal accesses the average kernels use.  The published 8 TB/s is
 * a pin rate; reads alone and a mix of reads and writes sustain different fractions of it, and the
 * HBM-bound kernels' rates can be read against these.
 *   copy      0: read `bytes` from src (dst: at least 4 bytes, written only if the data hits one magic value);
 *             1: copy `bytes` from src to dst
 *   src, dst  device, 16-byte aligned, `bytes` each (dst: see above); bytes is rounded down to whole 16 KiB chunks
 *             and should exceed the 256 MB of last-level cache many times
 *   launches  timed launches (after one untimed)
 *   gbs       host out: bytes moved (read + written) per second / 1e9.  Synchronises `stream`.
 * Returns SDP_ERR_INVALID_ARG for null or misaligned pointers, launches < 1 or bytes below one chunk.
 * ------------------------------------------------------------------------------------------- */
int sdp_probe_hbm_gbs(int copy, const void* src, void* dst, size_t bytes, int launches, double* gbs, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SDP_MEASURE_H */
