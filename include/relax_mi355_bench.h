/*
 * relax_mi355_bench.h -- measurement and test aids of librelax_mi355.so.
 *
 * Nothing here is part of the product interface (include/relax_mi355.h): these calls exist for bench.py and for A/B
 * tests.  They never change a result.  The switches are process-wide (atomic; a call that races with a change sees
 * the old or the new value), the event hook is per host thread.
 */
#ifndef RELAX_MI355_BENCH_H
#define RELAX_MI355_BENCH_H

#include "relax_mi355.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test switches.
 * "fuse_finish" (default 1): in the few-row path (2 <= n <= 128: batched decode, short prefills) the finishing pass of a
 * split-K matmul also does the light step that follows it (rotary embedding + KV append after QKV, the RMSNorm after
 * the output projection, and in relax_model_step the first RMSNorm of the next layer after the down projection:
 * Sec. 4.2 operator fusion); 0 runs them as launches of their own.  Results are identical bit for bit either way.
 * "gemm_waves_per_simd" (default 2): the 256 x 256 tile of the tiled GEMM runs as eight wavefronts (two per SIMD) or, with 1,
 * as four (one per SIMD); identical results.
 * "layer_matvec_rows" (default 4, 1 .. 64): relax_decoder_layer and relax_model_step keep a call of up to this many rows on
 * the matrix-vector kernels (two or four rows of x share one pass over the weights): two rows on every model, more when
 * every matrix of the layer is at most "layer_matvec_mb" MB of packed codes (default 96, 0 .. 4096) -- a model that mostly
 * stays in the last-level cache; above it the few-row matrix path takes the call.  1: matrix path from two rows on.
 * "half_matmul_gemm_rows" (default 0): relax_half_matmul takes the tiled GEMM from this many rows on; 0: by estimate.
 * Unknown name: RELAX_ERR_UNSUPPORTED.                                                                           */
relax_status relax_set_option(const char *name, int32_t value);

/* Measurement aids for the roofline figures: what the device at hand reaches on a plain
 * streaming read and on a bare loop of fp16 matrix-core instructions (the published
 * peaks, 8 TB/s and 2.5 PFLOP/s, are upper bounds of these).  Time them with events.
 * relax_probe_stream_read: every byte of buf (16-byte aligned, bytes >= 16) is loaded
 * once with 16-byte loads; sink: one device word.
 * relax_probe_mfma: one workgroup of four wavefronts per CU, each issuing 16 independent
 * 32x32x16 fp16 MFMAs per iteration on register operands (random_data != 0: operands
 * drawn from a hash, which costs clock under the power limit; 0: near-constant
 * operands); sink: device fp32 [CUs * 256]; *flops receives the operation count of the
 * launch.                                                                               */
relax_status relax_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, relax_stream stream);
relax_status relax_probe_mfma(float *sink, int32_t iters, int32_t random_data, int64_t *flops, relax_stream stream);

/* Measurement aid: the next relax_decoder_layer call on this host thread records `start`
 * before and `stop` after the launch of one of its steps (0 QKV matvec/GEMM, 1 attention,
 * 2 output projection, 3 gate/up, 4 down projection) on the call's stream; the setting is
 * consumed by that one call.  start/stop are hipEvent_t handles owned by the caller;
 * step < 0 or NULL events clear the setting.  Lets a benchmark time one kernel of the
 * layer with HIP events on the stream the kernel really runs on.                        */
void relax_profile_step_events(void *start, void *stop, int32_t step);

/* Measurement aid: while q_alt / s_alt (device pointers to another packed matrix and its scales, of the shape of
 * the layer's gate/up matrix) are set, every relax_decoder_layer call with n == 1 launches its gate/up matvec
 * once more, on those weights, ahead of the real launch (whose result then overwrites it).  Inside a captured
 * schedule the kernels run back to back, so the duration of that launch there is the difference between the
 * schedule timed with and without the extra launch -- on weights that are cold like the real ones.  NULL, NULL
 * switches it off (default).  The caller owns the memory and keeps it alive while set.                         */
void relax_profile_alt_gate_up(const void *q_alt, const void *s_alt);

#ifdef __cplusplus
}
#endif
#endif
