/*
 * wisv_diag.h - diagnostics and measurement helpers of libwisv.
 *
 * Not part of the verification round itself (wisv.h): copies of intermediate buffers for parity tests, the duration
 * of the last round, per-kernel timing for the benchmark's roofline line, and a copy kernel of known traffic for
 * calibrating hardware memory counters.  Same conventions as wisv.h (status codes, one host thread per ctx).
 */
#ifndef WISV_DIAG_H
#define WISV_DIAG_H

#include "wisv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WISV_DBG_HIDDEN = 0, /* float [batch*k, d_model]: h^T of the last round */
    WISV_DBG_LOGITS = 1  /* float [batch*k, vocab]: logits of the last round run with WISV_FLAG_KEEP_LOGITS */
} wisv_debug_what;

/* Copies a diagnostic buffer of the last round to host memory (synchronises). */
int wisv_debug_copy(wisv_ctx *ctx, int32_t what, void *host_dst, size_t bytes);

/* Duration in milliseconds of the GPU work of the last wisv_verify_round, measured with HIP events
 * recorded on the ctx's stream around the round's kernels (waits for the round to finish). */
int wisv_last_round_ms(wisv_ctx *ctx, float *ms);

/* Per-kernel timing.  While enabled, every kernel launch of a round is bracketed by a HIP event pair
 * on the ctx's stream.  wisv_profile_collect() waits for the stream and adds the elapsed times of the
 * launches since the last collect to per-class totals; wisv_profile_read() returns one class's name
 * (static string), accumulated milliseconds and launch count.  Enabling or disabling resets the totals.
 * The class "event_pair_overhead" times one empty event pair per round: what the bracketing itself adds.
 * kclass runs from 0 until wisv_profile_read() returns WISV_EINVAL. */
int wisv_profile_enable(wisv_ctx *ctx, int32_t on);
int wisv_profile_collect(wisv_ctx *ctx);
int wisv_profile_read(wisv_ctx *ctx, int32_t kclass, const char **name, double *total_ms, int64_t *launches);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned
 * device memory) on the ctx's stream: a kernel of known traffic, used to calibrate hardware memory counters
 * when profiling the round. */
int wisv_calibration_copy(wisv_ctx *ctx, void *dst, const void *src, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* WISV_DIAG_H */
