/*
 * adloco_internal.h -- measurement aids of libadloco.  NOT part of the library's interface: these
 * two calls exist for the repository's own benchmark and tests (kernel variants, per-kernel
 * timing); nothing a caller of the library needs depends on them, and they may change or go
 * without notice.
 */
#ifndef ADLOCO_INTERNAL_H
#define ADLOCO_INTERNAL_H

#include "adloco.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning knob for benchmarking kernel variants ("gram_variant", "wgrad_variant",
 * "stream_blocks_per_cu", "ip_group", "stats_variant", "overlap_aux", ...).  Unknown names give
 * ADLOCO_EINVAL.  Results never depend on a knob beyond floating-point summation order. */
int adloco_set_tuning(adloco_ctx* ctx, const char* name, int value);

/* Measurement aid.  After adloco_set_tuning(ctx, "profile", 1) every launch of the named
 * kernel ("gram", "wgrad", "finalize", "sqnorm", "outer_step", "merge", "vector_table",
 * "inner_step", "inner_products", "tile_stats") is bracketed by HIP
 * events on the call's stream.  adloco_profile_read waits for the recorded events of that
 * kernel, returns their summed duration in milliseconds and their count, and forgets them. */
int adloco_profile_read(adloco_ctx* ctx, const char* kernel, double* total_ms, int* launches);

/* The rate at which the chip's MFMA units run when their bf16 operands come from LDS and nothing
 * else happens (no global loads, no barriers): the practical ceiling of the Gram and gradient-sum
 * kernels.  variant 0: 64 x 64 wave tiles, 1: 128 x 64 wave tiles; one 8-wave workgroup per CU,
 * `ksteps` k-steps of 16.  Runs on the null stream and waits for it.  ms: kernel time, flops: MFMA
 * flops executed in it. */
int adloco_probe_mfma_lds(adloco_ctx* ctx, int variant, int ksteps, double* ms, double* flops);

/* Number of times the context has built its shape-dependent tables (tile, job and descriptor
 * tables): it moves on the first call with a new list of shapes and stays put while only the
 * addresses in a, delta and grad_sum change from call to call. */
int adloco_table_builds(const adloco_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* ADLOCO_INTERNAL_H */
