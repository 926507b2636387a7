/*
 * wisv.h - C ABI of the edge-side verification round of WISV
 * (Wireless-Informed Semantic Verification for distributed speculative decoding).
 *
 * One call to wisv_verify_round() is one pass of Algorithm 1's edge-side body for a batch
 * of independent device streams:
 *
 *   Verify    the target decoder forwards each stream's block of K drafted tokens against
 *             that stream's KV cache, giving greedy target tokens and final hidden states
 *             h^T (Sec. III-A step 2; Alg. 1 "Verify");
 *   Localize  mismatch set S = { j : draft_j != target greedy token for position j }
 *             (Sec. III-A step 2, Sec. V-C; Alg. 1 "Localize");
 *   Head      the CSI-aware decision head scores positions from z = [h^D ; h^T ; c]:
 *             s = w2 . act(W1 z + b1) + b2, p_rej = sigmoid(s) (Sec. V-A, eqs. feature_concat,
 *             head_forward, mlp_form), with drafter hidden states h^D uploaded for every
 *             position (full-hidden, FH) or only for S (selective-hidden, SH) (Sec. III-B);
 *   Decide    thresholding (eq. threshold), earliest rejected position, accepted prefix and
 *             the correction token, or the bonus token on full acceptance
 *             (Sec. III-A step 4; Alg. 1 last block).
 *
 * Polarity.  The paper's head emits a rejection probability p_rej and rejects when
 * p_rej >= tau_paper.  This interface reports p_accept = 1 - p_rej and ACCEPTS a gated
 * position when p_accept >= tau, i.e. tau = 1 - tau_paper: tau <= 0 accepts every block in
 * full, tau > 1 rejects every gated position (plain greedy verification, Sec. II-A).
 *
 * The target is a Llama-style decoder (RMSNorm, rotary embedding with rotate-half pairing,
 * grouped-query attention, SwiGLU, no biases).  Everything runs on one GPU (gfx950); the
 * library needs the HIP runtime and a device and has no CPU fallback.
 *
 * General rules
 *   - every function returns a wisv_status (0 = success, negative = error); nothing throws,
 *     aborts or prints.  After an error the outputs are untouched and wisv_last_error()
 *     describes it.  Per-stream soft conditions are reported in wisv_round_out.status.
 *   - "device pointer" = memory of the ctx's GPU; "host pointer" = ordinary process memory.
 *   - a ctx is used by one host thread at a time; the library keeps no global state.
 *   - identical inputs give identical bits (no floating-point atomics anywhere).
 */
#ifndef WISV_H
#define WISV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wisv_ctx wisv_ctx; /* opaque */

typedef enum {
    WISV_OK = 0,
    WISV_EINVAL = -1,      /* bad argument or configuration */
    WISV_ENOMEM = -2,      /* host or device allocation failed */
    WISV_EHIP = -3,        /* a HIP runtime call failed */
    WISV_ESTATE = -4,      /* stream state does not allow the call (e.g. cache full) */
    WISV_EUNSUPPORTED = -5 /* valid request this build cannot serve */
} wisv_status;

typedef enum { WISV_F32 = 0, WISV_BF16 = 1 } wisv_dtype;
typedef enum { WISV_PROTO_FH = 0, WISV_PROTO_SH = 1 } wisv_proto; /* Sec. III-B */
typedef enum { WISV_ACT_SILU = 0, WISV_ACT_RELU = 1 /* eq. mlp_form */ } wisv_act;

/* wisv_round_in.flags */
#define WISV_FLAG_GATE_ALL 1u    /* the head gates every position, not only S (needs h^D everywhere) */
#define WISV_FLAG_NO_COMMIT 2u   /* leave kv_len / pred_next of the streams unchanged */
#define WISV_FLAG_DEVICE_IO 4u   /* all round_in / round_out pointers are device pointers; enqueue only.  The host
                                    cannot see which slots such a round uses or how much it accepted: after a committing
                                    device-I/O round it assumes every slot grew by k, and refuses further rounds with
                                    WISV_ESTATE once that bound reaches max_ctx.  wisv_get_state(slot) reads the true
                                    length back and resets the bound of that slot. */
#define WISV_FLAG_KEEP_LOGITS 8u /* also materialise fp32 logits for wisv_debug_copy (debug, slow) */
/* The selective-hidden protocol in two calls (Alg. 1: Verify, Localize, RequestHidden(S), then the head on the
 * uploaded rows; Sec. III-B).  VERIFY_ONLY runs the target forward and the localisation: target_argmax and
 * mismatch_mask (the request message) are final, nothing is committed, and accepted_len / correction_token are
 * those of plain greedy verification (no hidden state has been uploaded yet).  DECIDE_ONLY, given next for the
 * same streams, k and draft tokens, skips the forward: it runs the decision head on the rows uploaded now, the
 * first-reject scan and the commit.  Both together, or DECIDE_ONLY without a matching VERIFY_ONLY before it, are
 * errors (WISV_EINVAL / WISV_ESTATE).  The pending round lives in the ctx's scratch: any other round, a
 * wisv_prefill, wisv_set_state or wisv_kv_import on this ctx between the two calls drops it, and the DECIDE_ONLY
 * call then fails with WISV_ESTATE (run VERIFY_ONLY again).  wisv_get_state and wisv_kv_export leave it alone. */
#define WISV_FLAG_VERIFY_ONLY 16u
#define WISV_FLAG_DECIDE_ONLY 32u

/* wisv_round_out.status bits */
#define WISV_STATUS_MISSING_HIDDEN 1u /* a gated position had no h^D row: it was rejected */

#define WISV_MAX_K 16 /* largest draft block per stream */

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;   /* wisv_dtype: storage type of every weight, of the KV cache and of h^D.
                        Arithmetic: WISV_F32 all float.  WISV_BF16: weights and cached k, v are bf16 values;
                        activations stay float (residual stream, norms, softmax, decision head) and enter
                        the matrix cores as two bf16 terms x = hi + lo (|x - hi - lo| <= 2^-17 |x|), one
                        MFMA each, accumulated in float.  Rounds of more than 16 rows: see
                        WISV_OPT_ONE_TERM_CLASSES. */
    int32_t d_draft; /* width of a drafter hidden state h^D */
    int32_t d_csi;   /* number of CSI features (1..16) */
    int32_t d_head_hidden; /* d_J, hidden width of the decision head */
    int32_t head_act;      /* wisv_act */
    int32_t max_batch;     /* number of stream slots (each owns a KV cache of max_ctx positions) */
    int32_t max_ctx;       /* KV positions per slot, drafted block included */
    int32_t max_k;         /* largest k of a round, <= WISV_MAX_K */
    int32_t device_id;
    void *hip_stream; /* hipStream_t all work is enqueued on (borrowed).  NULL: the ctx creates a stream of its own
                         (an ordinary blocking stream: it orders itself against the null stream both ways) */
    void *kv_cache;   /* device pointer to borrowed cache memory, or NULL: the ctx allocates.
                         Layout [n_layers][max_batch][2 (K,V)][n_kv_heads] planes of ctx_pad * head_dim elements,
                         ctx_pad = max_ctx rounded up to a multiple of 32, dtype as above.
                         K plane: [ctx_pad][head_dim] (position-major).
                         V plane: blocks of 32 positions, [ctx_pad / 32][head_dim][32]: element (pos, dim) sits at
                         ((pos / 32) * head_dim + dim) * 32 + pos % 32, so that the attention kernel reads 32 cached
                         values of one feature contiguously.  wisv_kv_import / wisv_kv_export convert from / to
                         plain [n_kv_heads][len][head_dim] host arrays. */
    size_t kv_bytes;  /* size of kv_cache when borrowed (must cover the layout) */
} wisv_config;

/* Model parameters: device pointers, canonical [out_features, in_features] row-major tensors of
 * config.dtype, borrowed for the duration of wisv_ctx_create only (the ctx keeps private,
 * re-tiled copies).  Per-layer members are host arrays of n_layers device pointers. */
typedef struct {
    const void *embed;      /* [vocab, d_model] */
    const void *lm_head;    /* [vocab, d_model] */
    const void *final_norm; /* [d_model] */
    const void *const *attn_norm; /* [d_model] */
    const void *const *wq;        /* [n_heads*head_dim, d_model] */
    const void *const *wk;        /* [n_kv_heads*head_dim, d_model] */
    const void *const *wv;        /* [n_kv_heads*head_dim, d_model] */
    const void *const *wo;        /* [d_model, n_heads*head_dim] */
    const void *const *ffn_norm;  /* [d_model] */
    const void *const *w_gate;    /* [d_ff, d_model] */
    const void *const *w_up;      /* [d_ff, d_model] */
    const void *const *w_down;    /* [d_model, d_ff] */
    const void *head_w1; /* [d_J, d_draft + d_model + d_csi], columns ordered [h^D ; h^T ; c] (eq. feature_concat) */
    const void *head_b1; /* [d_J] */
    const void *head_w2; /* [d_J] */
    const void *head_b2; /* [1] */
} wisv_weights;

/* One round for `batch` streams, k drafted tokens each.  Host pointers unless WISV_FLAG_DEVICE_IO. */
typedef struct {
    int32_t batch; /* 1..max_batch */
    int32_t k;     /* 1..max_k */
    const int32_t *stream_ids;   /* [batch] distinct slot indices in [0, max_batch) */
    const int32_t *draft_tokens; /* [batch*k] drafted token ids */
    const int32_t *proto;        /* [batch] wisv_proto of each stream */
    const void *hd;         /* uploaded drafter hidden states [n_hd, d_draft] of config.dtype (may be NULL if n_hd == 0) */
    const int32_t *hd_row;  /* [batch*k] row of hd holding position (b, j), or -1 = not uploaded;
                               NULL = identity map (row b*k + j; needs n_hd == batch*k) */
    int32_t n_hd;
    const float *csi; /* [batch, d_csi] CSI feature vector c^r of each stream, float */
    const float *tau; /* [batch] accept threshold of each stream */
    uint32_t flags;
} wisv_round_in;

/* Caller-owned, caller-sized outputs.  The first three are required. */
typedef struct {
    int32_t *accepted_len;     /* [batch] A in [0, k]: drafts before the earliest rejected position */
    int32_t *correction_token; /* [batch] target greedy token for position A (the bonus token when A == k) */
    float *p_accept;           /* [batch*k] 1 - sigmoid(s) where the head was evaluated (FH: every position with
                                  an h^D row; SH: mismatch positions with an h^D row), 1.0 elsewhere */
    int32_t *target_argmax;    /* [batch*(k+1)] target greedy tokens for positions 0..k, or NULL */
    uint32_t *mismatch_mask;   /* [batch] bit j set <=> position j is in S (the SH request), or NULL */
    uint32_t *status;          /* [batch] WISV_STATUS_* bits, or NULL */
} wisv_round_out;

/* Builds a context: validates the configuration (before any GPU call), allocates the KV cache
 * (unless borrowed), scratch and rotary tables on config.device_id, and copies the weights into
 * private layouts.  On failure *out is NULL and, when `err` is non-NULL, a message of at most
 * err_len bytes (NUL included) is written there. */
int wisv_ctx_create(const wisv_config *config, const wisv_weights *weights, wisv_ctx **out,
                    char *err, size_t err_len);

/* One verification round (see the top of this file).  Host-pointer mode copies the inputs in,
 * runs the round and returns after the results are in the caller's buffers.  With
 * WISV_FLAG_DEVICE_IO the round is only enqueued on the ctx's stream.
 * Unless WISV_FLAG_NO_COMMIT: the K/V rows of the k drafted tokens stay in the cache, each
 * stream's length grows by A (rows beyond are dead and overwritten by the next round) and its
 * pred_next becomes the correction token (Sec. IV-B: the state recursion of the committed prefix).
 * The target's greedy token for draft position 0 is the stream's pred_next state. */
int wisv_verify_round(wisv_ctx *ctx, const wisv_round_in *in, wisv_round_out *out);

/* --- speculative-sampling verification ----------------------------------------------------------
 * The stochastic verifier of Sec. II-A on the same target forward: position j of a block is accepted with
 * probability alpha_j = min{1, p_T(y_j) / p_D(y_j)} (eq. ss_accept_prob), positions are taken in order until the
 * first rejection, and the token emitted there is drawn from the residual distribution proportional to
 * p_T - alpha p_D = max(0, p_T - p_D) (eq. ss_residual); when all k are accepted the emitted token is drawn from
 * the target distribution after the block.  p_T is the softmax of the target's logits (temperature 1).
 *
 * The random numbers are inputs: position j is accepted iff u_accept < alpha_j, and the emitted token is the
 * smallest token id whose cumulative weight exceeds u_sample times the total weight.
 * Position 0 of a block is the stream's pending token (pred_next: the token the previous round emitted, whose
 * K/V row this forward appends): its target distribution is the point mass there, so alpha_0 is 1 if
 * draft_tokens[0] is that token and 0 otherwise, and a rejection at position 0 emits the pending token again.
 * The drafter's distribution of position 0 is not read.  A drafted token with p_D = 0 is accepted.
 * Arithmetic: float exponentials, double normalisers and cumulative sums in a fixed order (equal inputs give
 * equal outputs); a decision that a rounding error of about 1e-7 relative could turn may differ from an exact
 * evaluation. */
typedef struct {
    int32_t batch; /* 1..max_batch */
    int32_t k;     /* 1..max_k */
    const int32_t *stream_ids;   /* [batch] distinct slot indices */
    const int32_t *draft_tokens; /* [batch*k] */
    const float *draft_probs;    /* [batch*k, vocab]: row b*k + j is the drafter's distribution token j was drawn from
                                    (nonnegative; rows with j = 0 are not read) */
    const float *u_accept;       /* [batch*k] uniform numbers in [0, 1) */
    const float *u_sample;       /* [batch] uniform numbers in [0, 1) */
    uint32_t flags;              /* WISV_FLAG_NO_COMMIT, WISV_FLAG_DEVICE_IO */
} wisv_ss_in;

typedef struct {                 /* caller-owned; all required */
    int32_t *accepted_len;     /* [batch] A in [0, k] */
    int32_t *correction_token; /* [batch] the emitted token */
    float *alpha;              /* [batch*k] acceptance probability of every position (also those after A) */
} wisv_ss_out;

/* One speculative-sampling round: the target forward of wisv_verify_round with all logits kept, then the rule
 * above.  Host pointers, or device pointers with WISV_FLAG_DEVICE_IO (enqueue only).  Commit as in
 * wisv_verify_round: each stream's length grows by A and its pending token becomes the emitted one.  In host
 * mode the first call allocates a device staging buffer of max_batch * max_k * vocab floats for draft_probs. */
int wisv_ss_verify_round(wisv_ctx *ctx, const wisv_ss_in *in, wisv_ss_out *out);

/* The rule alone on logits the caller holds: all pointers are device pointers (16-byte aligned rows make the
 * kernels use vector loads), nothing of the ctx's stream state is read or written, the work is enqueued on the
 * ctx's stream.  logits [batch*k, vocab]: row b*k + j is the target's output after token j of stream b;
 * pending_tokens [batch]; vocab at most the ctx's.  Outputs as in wisv_ss_out. */
int wisv_ss_decide(wisv_ctx *ctx, int32_t batch, int32_t k, int32_t vocab, const float *logits,
                   const int32_t *pending_tokens, const int32_t *draft_tokens, const float *draft_probs,
                   const float *u_accept, const float *u_sample, int32_t *accepted_len, int32_t *emitted_token,
                   float *alpha);

/* wisv_ss_decide for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results; the kernels' scratch (chunk
 * statistics, normalisers, chunk weights: about 2 MiB) is a static array inside the library instead of memory of
 * the ctx, so the sizes are bounded by that array and not by the ctx: batch * k <= 1024, k <= WISV_MAX_K,
 * vocab <= 262144 (WISV_EUNSUPPORTED beyond).  The call allocates and frees nothing, on the device or through any
 * library; each GPU holds its copy of the array from library load to process end, and wisv_ctx_create looks its
 * address up for the ctx's device.  All calls on one GPU share that array, whatever their ctx: calls that overlap
 * in time on one GPU (two streams, two threads) race on it and must be serialised by the caller.  Nothing in it
 * needs clearing between calls (every kernel writes what the next reads). */
int wisv_ss_decide_static(wisv_ctx *ctx, int32_t batch, int32_t k, int32_t vocab, const float *logits,
                          const int32_t *pending_tokens, const int32_t *draft_tokens, const float *draft_probs,
                          const float *u_accept, const float *u_sample, int32_t *accepted_len, int32_t *emitted_token,
                          float *alpha);

/* Frees everything the ctx owns (not the borrowed stream / cache).  NULL is a no-op. */
int wisv_destroy(wisv_ctx *ctx);

/* --- options ------------------------------------------------------------------------------------ */

/* WISV_OPT_ONE_TERM_CLASSES: which matrix products of the target take their activations as ONE half-precision
 * term when a round has more than 16 rows (the regime bound by the matrix cores, Sec. IV-B's f_T with many streams).
 * There the default for a WISV_BF16 ctx is gate/up, down and the LM head (nine tenths of the matrix work; the QKV
 * and O products keep two terms, their rounding costs the most accuracy): each activation is rounded to an IEEE half (11
 * significant bits; magnitudes beyond 65504 saturate) and meets the weights converted to halves (exact for
 * |w| >= 2^-14, absolute error <= 2^-25 below; a ctx whose weights exceed the half range keeps the two-term form and
 * refuses this option), one MFMA per operand pair instead of the two of the two-term bf16 form.  A cleared bit keeps
 * that class on two bf16 terms (error 2^-17 per activation instead of 2^-12, twice the matrix-core work).  Rounds of
 * at most 16 rows are bound by memory and always use two terms.  value: OR of the WISV_TERM_* bits. */
#define WISV_OPT_ONE_TERM_CLASSES 1
#define WISV_TERM_QKV 1
#define WISV_TERM_O 2
#define WISV_TERM_GATE_UP 4
#define WISV_TERM_DOWN 8
#define WISV_TERM_LM_HEAD 16
int wisv_set_option(wisv_ctx *ctx, int32_t option, int64_t value);
int wisv_get_option(wisv_ctx *ctx, int32_t option, int64_t *value);

/* --- state helpers --------------------------------------------------------------------------- */

/* Runs the target over n prompt tokens (host pointer) of an empty or partly filled slot with the
 * round's own kernels, appends their K/V, and sets pred_next to the greedy token after the last. */
int wisv_prefill(wisv_ctx *ctx, int32_t stream_id, const int32_t *tokens, int32_t n);

/* Sets a slot's cached length and pred_next directly (cache contents: wisv_kv_import). */
int wisv_set_state(wisv_ctx *ctx, int32_t stream_id, int32_t kv_len, int32_t pred_next);

/* Reads a slot's cached length and pred_next (synchronises the stream). */
int wisv_get_state(wisv_ctx *ctx, int32_t stream_id, int32_t *kv_len, int32_t *pred_next);

/* Copies positions [0, len) of one (slot, layer) between the cache and host buffers laid out
 * [n_kv_heads][len][head_dim] in config.dtype.  K is stored rotated (rotary embedding applied). */
int wisv_kv_import(wisv_ctx *ctx, int32_t stream_id, int32_t layer, const void *host_k,
                   const void *host_v, int32_t len);
int wisv_kv_export(wisv_ctx *ctx, int32_t stream_id, int32_t layer, void *host_k, void *host_v,
                   int32_t len);

/* Diagnostics and measurement helpers (debug copies, per-kernel timing, the counter-calibration copy) are declared
 * in wisv_diag.h. */

/* Message of the last error on this ctx ("" if none).  Never NULL. */
const char *wisv_last_error(const wisv_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* WISV_H */
