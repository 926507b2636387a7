/*
 * CPU oracle for the edge-side verification round of WISV.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path is
 * checked against; the product never links, loads or calls it.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * What it computes (one stream at a time), in the paper's order:
 *   Verify    one forward pass of the target decoder over the K drafted tokens
 *             against the stream's KV cache -> logits and final hidden states
 *             (Sec. III-A step 2; Alg. 1 "Verify")
 *   Localize  mismatch set S = { j : draft_j != target argmax for position j }
 *             (Sec. III-A step 2; Sec. V-C; Alg. 1 "Localize")
 *   Head      z = [h^D ; h^T ; c], s = w2 . act(W1 z + b1) + b2, p = sigmoid(s)
 *             (Sec. V-A, eqs. feature_concat, head_forward, mlp_form)
 *   Decide    threshold the head at tau, first rejected position, accepted prefix,
 *             correction / bonus token (eq. threshold; Alg. 1 last block; Sec. III-A step 4)
 *
 * The decoder is Llama-style (RMSNorm, rotary embedding with rotate-half pairing,
 * grouped-query attention, SwiGLU FFN, no biases) - the family of the paper's target
 * models (Sec. VI "Experiment Settings").
 *
 * Arithmetic: activations are float; every dot product, norm and softmax accumulates
 * in double and rounds once.  Weights are float arrays or bf16 bit patterns widened
 * exactly.  round_bf16 selects what else a bf16 target stores in bf16 (nearest-even):
 *   bit 0  the KV cache: rotated k and v are rounded when written to the cache;
 *   bit 1  every operand handed to a matrix product - normalised activations, rotated
 *          q, k, v, attention output, SwiGLU output, LM-head input - is rounded where
 *          it is produced (implies bit 0).
 * The residual stream, softmax and the decision head stay float in every mode.
 *
 * Pinned by tests/test_oracle_*.py: a cache-free fp64 forward composed from PyTorch CPU
 * library routines, closed forms of RMSNorm / RoPE / attention / head, exhaustive
 * enumeration of the decision rule, and the invariants the paper states.
 * Parity unpinned: none of the functions below lacks such a pin; absolute values on the
 * 8B-shaped workloads have no printed example in the paper to compare with.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff, vocab;
    float   rms_eps, rope_theta;
    int32_t storage;      /* 0: weights are float; 1: weights are bf16 bit patterns (uint16) */
    int32_t round_bf16;   /* bit 0: KV cache stored in bf16; bit 1: every matrix-product operand rounded */
    int32_t d_draft, d_csi, d_j, head_act;   /* head_act 0: SiLU, 1: ReLU */
} orc_model;

typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void **attn_norm, **wq, **wk, **wv, **wo, **ffn_norm, **w_gate, **w_up, **w_down;
    const void *head_w1, *head_b1, *head_w2, *head_b2;
} orc_weights;

/* ------------------------------------------------------------------ scalar helpers */

static inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even to bf16, returned as float */
float orc_round_bf16(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x;          /* NaN stays NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static inline float wget(const void *w, int storage, size_t i) {
    return storage ? bf16_bits_to_float(((const uint16_t *)w)[i]) : ((const float *)w)[i];
}

static inline float maybe_round(const orc_model *m, float x) {      /* matrix-product operands */
    return (m->round_bf16 & 2) ? orc_round_bf16(x) : x;
}
static inline float cache_round(const orc_model *m, float x) {      /* what goes into the KV cache */
    return (m->round_bf16 & 3) ? orc_round_bf16(x) : x;
}

/* ------------------------------------------------------------------ building blocks */

/* out_i = x_i / sqrt(mean(x^2) + eps) * g_i */
void orc_rmsnorm(const float *x, const void *g, int storage, int n, float eps, float *out) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += (double)x[i] * (double)x[i];
    double inv = 1.0 / sqrt(ss / n + (double)eps);
    for (int i = 0; i < n; ++i) out[i] = (float)((double)x[i] * inv * (double)wget(g, storage, i));
}

/* y[r][o] = sum_i x[r][i] * W[o][i]   (W is [n_out, n_in] row-major, no bias) */
void orc_linear(const float *x, const void *W, int storage, int rows, int n_in, int n_out, float *y) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o) {
        for (int r = 0; r < rows; ++r) {
            const float *xr = x + (size_t)r * n_in;
            double acc = 0.0;
            if (storage) {
                const uint16_t *wr = (const uint16_t *)W + (size_t)o * n_in;
#pragma omp simd reduction(+ : acc)
                for (int i = 0; i < n_in; ++i) acc += (double)xr[i] * (double)bf16_bits_to_float(wr[i]);
            } else {
                const float *wr = (const float *)W + (size_t)o * n_in;
#pragma omp simd reduction(+ : acc)
                for (int i = 0; i < n_in; ++i) acc += (double)xr[i] * (double)wr[i];
            }
            y[(size_t)r * n_out + o] = (float)acc;
        }
    }
}

/* rotary embedding of one head vector at absolute position pos:
 * pairs (i, i + hd/2), angle pos * theta^(-2i/hd) */
void orc_rope(float *v, int head_dim, int pos, float theta) {
    int half = head_dim / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)head_dim);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = (float)(a * c - b * s);
        v[i + half] = (float)(b * c + a * s);
    }
}

/* one query vector against keys/values 0..n_vis-1 of one KV head:
 * out = sum_s softmax_s(q.k_s / sqrt(hd)) v_s ; kc, vc are [*, hd] row-major */
void orc_attend(const float *q, const float *kc, const float *vc, int n_vis, int hd, float *out,
                double *score_buf) {
    double scale = 1.0 / sqrt((double)hd), mx = -INFINITY;
    for (int s = 0; s < n_vis; ++s) {
        double acc = 0.0;
        const float *k = kc + (size_t)s * hd;
        for (int i = 0; i < hd; ++i) acc += (double)q[i] * (double)k[i];
        score_buf[s] = acc * scale;
        if (score_buf[s] > mx) mx = score_buf[s];
    }
    double den = 0.0;
    for (int s = 0; s < n_vis; ++s) {
        score_buf[s] = exp(score_buf[s] - mx);
        den += score_buf[s];
    }
    for (int i = 0; i < hd; ++i) {
        double acc = 0.0;
        for (int s = 0; s < n_vis; ++s) acc += score_buf[s] * (double)vc[(size_t)s * hd + i];
        out[i] = (float)(acc / den);
    }
}

/* index of the largest entry (lowest index among equals), its lead over the runner-up, its value */
void orc_argmax(const float *z, int n, int32_t *idx, float *gap, float *top) {
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (z[i] > z[best]) best = i;
    float second = -INFINITY;
    for (int i = 0; i < n; ++i)
        if (i != best && z[i] > second) second = z[i];
    *idx = best;
    *gap = (n > 1) ? z[best] - second : INFINITY;
    if (top) *top = z[best];
}

static inline double silu(double x) { return x / (1.0 + exp(-x)); }

/* ------------------------------------------------------------------ Verify: target forward */

/*
 * Forward K tokens of one stream at positions L .. L+K-1 against its cache.
 *   cache   float [n_layers][2][n_kv_heads][l_max][head_dim]; rows L..L+K-1 are written
 *   h_t     [K][d_model]  post-final-norm hidden state of each row (float, never rounded)
 *   logits  [K][vocab] or NULL
 *   amax    [K] argmax of each row's logits;  gap [K] top1 - top2;  top1 [K] the largest logit (or NULL)
 * Row j's logits predict the token after draft j.
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int orc_forward_block(const orc_model *m, const orc_weights *w, float *cache, int l_max, int L,
                      const int32_t *tokens, int K, float *h_t, float *logits, int32_t *amax,
                      float *gap, float *top1) {
    const int d = m->d_model, H = m->n_heads, G = m->n_kv_heads, hd = m->head_dim, F = m->d_ff;
    const int st = m->storage, dq = H * hd, dkv = G * hd, rep = H / G;
    if (K <= 0 || L < 0 || L + K > l_max || H % G) return -1;
    for (int j = 0; j < K; ++j)
        if (tokens[j] < 0 || tokens[j] >= m->vocab) return -1;

    float *x = malloc(sizeof(float) * K * d), *a = malloc(sizeof(float) * K * d);
    float *q = malloc(sizeof(float) * K * dq), *kk = malloc(sizeof(float) * K * dkv);
    float *vv = malloc(sizeof(float) * K * dkv), *o = malloc(sizeof(float) * K * dq);
    float *upd = malloc(sizeof(float) * K * d), *g = malloc(sizeof(float) * K * F);
    float *u = malloc(sizeof(float) * K * F);
    float *zrow = malloc(sizeof(float) * (size_t)K * m->vocab);
    if (!x || !a || !q || !kk || !vv || !o || !upd || !g || !u || !zrow) return -1;

    for (int j = 0; j < K; ++j)
        for (int i = 0; i < d; ++i) x[j * d + i] = wget(w->embed, st, (size_t)tokens[j] * d + i);

    const size_t head_stride = (size_t)l_max * hd, kv_stride = (size_t)G * head_stride;
    for (int l = 0; l < m->n_layers; ++l) {
        float *kc = cache + (size_t)l * 2 * kv_stride, *vc = kc + kv_stride;

        for (int j = 0; j < K; ++j) {
            orc_rmsnorm(x + j * d, w->attn_norm[l], st, d, m->rms_eps, a + j * d);
            for (int i = 0; i < d; ++i) a[j * d + i] = maybe_round(m, a[j * d + i]);
        }
        orc_linear(a, w->wq[l], st, K, d, dq, q);
        orc_linear(a, w->wk[l], st, K, d, dkv, kk);
        orc_linear(a, w->wv[l], st, K, d, dkv, vv);
        for (int j = 0; j < K; ++j) {
            int pos = L + j;
            for (int h = 0; h < H; ++h) {
                float *qh = q + (size_t)j * dq + h * hd;
                orc_rope(qh, hd, pos, m->rope_theta);
                for (int i = 0; i < hd; ++i) qh[i] = maybe_round(m, qh[i]);
            }
            for (int c = 0; c < G; ++c) {
                float *kh = kk + (size_t)j * dkv + c * hd, *vh = vv + (size_t)j * dkv + c * hd;
                orc_rope(kh, hd, pos, m->rope_theta);
                for (int i = 0; i < hd; ++i) {
                    kc[c * head_stride + (size_t)pos * hd + i] = cache_round(m, kh[i]);
                    vc[c * head_stride + (size_t)pos * hd + i] = cache_round(m, vh[i]);
                }
            }
        }
#pragma omp parallel
        {
            double *sbuf = malloc(sizeof(double) * (L + K));
#pragma omp for collapse(2) schedule(static)
            for (int j = 0; j < K; ++j)
                for (int h = 0; h < H; ++h) {
                    int c = h / rep;
                    float *oh = o + (size_t)j * dq + h * hd;
                    orc_attend(q + (size_t)j * dq + h * hd, kc + c * head_stride, vc + c * head_stride,
                               L + j + 1, hd, oh, sbuf);
                    for (int i = 0; i < hd; ++i) oh[i] = maybe_round(m, oh[i]);
                }
            free(sbuf);
        }
        orc_linear(o, w->wo[l], st, K, dq, d, upd);
        for (int i = 0; i < K * d; ++i) x[i] += upd[i];

        for (int j = 0; j < K; ++j) {
            orc_rmsnorm(x + j * d, w->ffn_norm[l], st, d, m->rms_eps, a + j * d);
            for (int i = 0; i < d; ++i) a[j * d + i] = maybe_round(m, a[j * d + i]);
        }
        orc_linear(a, w->w_gate[l], st, K, d, F, g);
        orc_linear(a, w->w_up[l], st, K, d, F, u);
        for (int i = 0; i < K * F; ++i) g[i] = maybe_round(m, (float)(silu((double)g[i]) * (double)u[i]));
        orc_linear(g, w->w_down[l], st, K, F, d, upd);
        for (int i = 0; i < K * d; ++i) x[i] += upd[i];
    }

    for (int j = 0; j < K; ++j) {
        orc_rmsnorm(x + j * d, w->final_norm, st, d, m->rms_eps, h_t + j * d);
        for (int i = 0; i < d; ++i) a[j * d + i] = maybe_round(m, h_t[j * d + i]);
    }
    orc_linear(a, w->lm_head, st, K, d, m->vocab, zrow);
    for (int j = 0; j < K; ++j) orc_argmax(zrow + (size_t)j * m->vocab, m->vocab, &amax[j], &gap[j], top1 ? &top1[j] : NULL);
    if (logits) memcpy(logits, zrow, sizeof(float) * (size_t)K * m->vocab);

    free(x); free(a); free(q); free(kk); free(vv); free(o); free(upd); free(g); free(u); free(zrow);
    return 0;
}

/* ------------------------------------------------------------------ decision head */

/*
 * One position: z = [h_d ; h_t ; c] (never materialised: W1 is walked in that column order).
 * h_d is [d_draft] float (already holding the uploaded precision), h_t [d_model], c [d_csi].
 * Outputs the logit s, the paper's rejection probability sigmoid(s), and 1 - it computed
 * as 1/(1+e^s).
 */
void orc_head(const orc_model *m, const orc_weights *w, const float *h_d, const float *h_t,
              const float *c, float *s_out, float *p_rej, float *p_acc) {
    const int st = m->storage, dD = m->d_draft, dT = m->d_model, dC = m->d_csi, din = dD + dT + dC;
    double s = (double)wget(w->head_b2, st, 0);
    for (int r = 0; r < m->d_j; ++r) {
        size_t row = (size_t)r * din;
        double acc = (double)wget(w->head_b1, st, r);
        for (int i = 0; i < dD; ++i) acc += (double)wget(w->head_w1, st, row + i) * (double)h_d[i];
        for (int i = 0; i < dT; ++i) acc += (double)wget(w->head_w1, st, row + dD + i) * (double)h_t[i];
        for (int i = 0; i < dC; ++i) acc += (double)wget(w->head_w1, st, row + dD + dT + i) * (double)c[i];
        double act = m->head_act == 1 ? (acc > 0.0 ? acc : 0.0) : silu(acc);
        s += (double)wget(w->head_w2, st, r) * act;
    }
    *s_out = (float)s;
    *p_rej = (float)(1.0 / (1.0 + exp(-s)));
    *p_acc = (float)(1.0 / (1.0 + exp(s)));
}

/* number of threads the parallel loops above run on */
int orc_num_threads(void) {
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
    return n;
}

/* FLOPs of one head evaluation as the paper counts them: 2 d_in d_J + d_J + 2 d_J + 1 */
int64_t orc_head_flops(int d_in, int d_j) {
    return 2ll * d_in * d_j + d_j + 2ll * d_j + 1;
}

/* ------------------------------------------------------------------ localize + decide */

/*
 * t[0..K]    target greedy tokens: t[j] is the prediction for draft position j, t[K] the bonus
 * draft[K]   drafted tokens
 * scored[K]  1 where the head was evaluated (a drafter hidden state was available)
 * p_acc[K]   1 - rejection probability where scored
 * gate_all   0: the head gates only mismatch positions (the paper's rule);
 *            1: every position must pass the head
 * A position is rejected when it is gated and its accept probability is below tau, or when it
 * is gated and has no score.  Outputs the accepted length A (first rejected position minus one,
 * K if none), the token for position A (correction, or bonus when A == K), the mismatch mask
 * (bit j <=> draft_j != t_j) and a status word (bit 0: a gated position had no score).
 */
void orc_decide(int K, const int32_t *draft, const int32_t *t, const int32_t *scored,
                const float *p_acc, float tau, int gate_all, int32_t *A, int32_t *y_star,
                uint32_t *mask, uint32_t *status) {
    uint32_t mm = 0, stt = 0;
    int first = K;
    for (int j = 0; j < K; ++j)
        if (draft[j] != t[j]) mm |= 1u << j;
    for (int j = K - 1; j >= 0; --j) {
        int gated = gate_all || ((mm >> j) & 1u);
        if (!gated) continue;
        int reject;
        if (!scored[j]) { reject = 1; stt |= 1u; }
        else reject = !(p_acc[j] >= tau);
        if (reject) first = j;
    }
    *A = first;
    *y_star = t[first];
    *mask = mm;
    *status = stt;
}

/* ------------------------------------------------------------------ one whole round, one stream */

/*
 * Verify -> Localize -> Head -> Decide for one stream.
 *   pred_next  target argmax for the first draft position (state left by the previous forward)
 *   hd         [n_hd][d_draft] float; hd_row[K] row of hd per position or -1 (not uploaded)
 *   proto      0 full-hidden, 1 selective-hidden: under SH only mismatch positions are scored
 * Outputs: A, y_star, p_acc[K] (1.0 where not scored), t[K+1], gap[K] / top1[K] (lead and value of the
 *          largest logit of rows 0..K-1),
 *          mask, status, h_t[K][d_model], p_rej[K] (0.0 where not scored).
 */
int orc_verify_round(const orc_model *m, const orc_weights *w, float *cache, int l_max, int L,
                     int32_t pred_next, const int32_t *draft, int K, int proto, const float *hd,
                     const int32_t *hd_row, const float *csi, float tau, int gate_all,
                     int32_t *A, int32_t *y_star, float *p_acc, float *p_rej, int32_t *t,
                     float *gap, float *top1, uint32_t *mask, uint32_t *status, float *h_t,
                     float *logits) {
    if (K > 31) return -1;
    int32_t *amax = malloc(sizeof(int32_t) * K);
    int32_t *scored = malloc(sizeof(int32_t) * K);
    if (!amax || !scored) return -1;
    int rc = orc_forward_block(m, w, cache, l_max, L, draft, K, h_t, logits, amax, gap, top1);
    if (rc) { free(amax); free(scored); return rc; }
    t[0] = pred_next;
    for (int j = 0; j < K; ++j) t[j + 1] = amax[j];
    for (int j = 0; j < K; ++j) {
        int mismatch = draft[j] != t[j];
        int want = (proto == 0) ? 1 : mismatch;
        scored[j] = want && hd_row[j] >= 0;
        p_acc[j] = 1.0f;
        p_rej[j] = 0.0f;
        if (scored[j]) {
            float s;
            orc_head(m, w, hd + (size_t)hd_row[j] * m->d_draft, h_t + (size_t)j * m->d_model, csi,
                     &s, &p_rej[j], &p_acc[j]);
        }
    }
    orc_decide(K, draft, t, scored, p_acc, tau, gate_all, A, y_star, mask, status);
    free(amax); free(scored);
    return 0;
}
