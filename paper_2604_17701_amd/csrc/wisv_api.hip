// C ABI of the WISV verify round: context management, argument checking and the order in which
// the kernels of one round are enqueued (Alg. 1: Verify -> Localize -> head -> first reject).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "wisv_internal.h"

using namespace wisv;

struct wisv_ctx : public wisv::Ctx {};

namespace wisv {

void *kv_ptr(const Ctx *c, int layer, int slot, int which) {
    const wisv_config &g = c->cfg;
    const size_t half = (size_t)g.n_kv_heads * c->ctx_pad * g.head_dim;
    const size_t off = (((size_t)layer * g.max_batch + slot) * 2 + which) * half;
    return (char *)c->kv + off * c->esz;
}

ProfScope::ProfScope(Ctx *c_, int kclass) : c(c_), idx(-1) {
    if (!c->profiling) return;
    if (c->ev_used + 2 > c->ev_pool.size()) {
        for (int i = 0; i < 2; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->ev_pool.push_back(e);
        }
    }
    idx = (int)c->ev_used;
    c->ev_used += 2;
    c->ev_class.resize(c->ev_used / 2);
    c->ev_class[idx / 2] = kclass;
    (void)hipEventRecord(c->ev_pool[idx], c->stream);
}
ProfScope::~ProfScope() {
    if (idx >= 0) (void)hipEventRecord(c->ev_pool[idx + 1], c->stream);
}

}  // namespace wisv

// ------------------------------------------------------------------------------------------ helpers

static int fail(Ctx *c, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, call)                                                                                   \
    do {                                                                                                   \
        hipError_t e_ = (call);                                                                            \
        if (e_ != hipSuccess) return fail((c), WISV_EHIP, "%s: %s", #call, hipGetErrorString(e_));         \
    } while (0)

static const char *check_config(const wisv_config *g) {
    if (!g) return "config is NULL";
    if (g->n_layers < 1 || g->n_layers > 1024) return "n_layers out of range";
    if (g->d_model < 8 || g->d_model % 8) return "d_model must be a positive multiple of 8";
    if (g->n_heads < 1 || g->n_kv_heads < 1 || g->n_heads % g->n_kv_heads) return "n_heads must be a multiple of n_kv_heads";
    if (g->head_dim != 32 && g->head_dim != 64 && g->head_dim != 128 && g->head_dim != 256)
        return "head_dim must be 32, 64, 128 or 256";
    if (g->d_ff < 8 || g->d_ff % 8) return "d_ff must be a positive multiple of 8";
    if (g->vocab < 2) return "vocab must be at least 2";
    if (!(g->rms_eps > 0.f) || !(g->rope_theta > 1.f)) return "rms_eps must be > 0 and rope_theta > 1";
    if (g->dtype != WISV_F32 && g->dtype != WISV_BF16) return "dtype must be WISV_F32 or WISV_BF16";
    if (g->d_draft < 1 || g->d_csi < 1 || g->d_csi > 16 || g->d_head_hidden < 1) return "decision-head sizes out of range";
    if (g->head_act != WISV_ACT_SILU && g->head_act != WISV_ACT_RELU) return "head_act must be SiLU or ReLU";
    if (g->max_batch < 1 || g->max_batch > 4096) return "max_batch out of range";
    if (g->max_k < 1 || g->max_k > WISV_MAX_K) return "max_k out of range";
    if (g->max_ctx <= g->max_k || g->max_ctx > (1 << 20)) return "max_ctx must exceed max_k (and be at most 2^20)";
    if (g->device_id < 0) return "device_id is negative";
    const size_t esz = g->dtype == WISV_BF16 ? 2 : 4;
    const size_t ctx_pad = ((size_t)g->max_ctx + 31) / 32 * 32;
    const size_t need = (size_t)g->n_layers * g->max_batch * 2 * g->n_kv_heads * ctx_pad * g->head_dim * esz;
    if (g->kv_cache && g->kv_bytes < need) return "borrowed kv_cache is smaller than the cache layout";
    return nullptr;
}

static const char *check_weights(const wisv_config *g, const wisv_weights *w) {
    if (!w) return "weights is NULL";
    if (!w->embed || !w->lm_head || !w->final_norm || !w->head_w1 || !w->head_b1 || !w->head_w2 || !w->head_b2)
        return "a weight pointer is NULL";
    if (!w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        return "a per-layer pointer array is NULL";
    for (int l = 0; l < g->n_layers; ++l)
        if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] ||
            !w->w_up[l] || !w->w_down[l])
            return "a per-layer weight pointer is NULL";
    return nullptr;
}

template <typename T> static hipError_t dalloc(Ctx *c, T **p, size_t count) {
    void *q = nullptr;
    hipError_t e = hipMalloc(&q, std::max<size_t>(count, 1) * sizeof(T));
    if (e == hipSuccess) c->owned.push_back(q);
    *p = (T *)q;
    return e;
}

static void destroy_ctx(Ctx *c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device_id);
    (void)hipStreamSynchronize(c->stream);
    if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
    for (void *p : c->owned) (void)hipFree(p);
    if (c->stream_owned) (void)hipStreamDestroy(c->stream);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    if (c->ev_round[0]) (void)hipEventDestroy(c->ev_round[0]);
    if (c->ev_round[1]) (void)hipEventDestroy(c->ev_round[1]);
    delete static_cast<wisv_ctx *>(c);
}

// ------------------------------------------------------------------------------------------ create / destroy

extern "C" int wisv_ctx_create(const wisv_config *config, const wisv_weights *weights, wisv_ctx **out, char *err,
                               size_t err_len) {
    auto report = [&](int code, const std::string &msg) {
        if (err && err_len) snprintf(err, err_len, "%s", msg.c_str());
        if (out) *out = nullptr;
        return code;
    };
    if (!out) return report(WISV_EINVAL, "out is NULL");
    *out = nullptr;
    if (const char *m = check_config(config)) return report(WISV_EINVAL, m);
    if (const char *m = check_weights(config, weights)) return report(WISV_EINVAL, m);

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1)
        return report(WISV_EHIP, "no HIP device available: this library has no CPU fallback");
    if (config->device_id >= ndev) return report(WISV_EINVAL, "device_id exceeds the device count");

    wisv_ctx *c = new (std::nothrow) wisv_ctx();
    if (!c) return report(WISV_ENOMEM, "host allocation failed");
    c->cfg = *config;
    c->stream = (hipStream_t)config->hip_stream;
    c->ctx_pad = (config->max_ctx + 31) / 32 * 32;
    c->stream_owned = false;
    c->graph_exec = nullptr;
    c->graph_len_ub = -1;
    memset(&c->graph_in, 0, sizeof c->graph_in);
    memset(&c->graph_out, 0, sizeof c->graph_out);
    c->bf16 = config->dtype == WISV_BF16;
    c->esz = c->bf16 ? 2 : 4;
    c->d_q = config->n_heads * config->head_dim;
    c->d_kv = config->n_kv_heads * config->head_dim;
    c->d_qkv = c->d_q + 2 * c->d_kv;
    c->rows_max = config->max_batch * config->max_k;
    c->profiling = false;
    c->ev_used = 0;
    c->ev_round[0] = c->ev_round[1] = nullptr;
    c->logits = nullptr;
    c->logits_rows = 0;
    c->ss_ws = nullptr;
    c->d_ss_q = c->d_ss_u = c->d_ss_v = nullptr;
    c->last_rows = 0;
    c->launch_failed = false;
    memset(c->prof_ms, 0, sizeof c->prof_ms);
    memset(c->prof_n, 0, sizeof c->prof_n);
    c->h_len_ub.assign(config->max_batch, 0);

    auto bail = [&](int code, const std::string &msg) {
        destroy_ctx(c);
        return report(code, msg);
    };
#define CREATE_TRY(call)                                                                        \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return bail(e_ == hipErrorOutOfMemory ? WISV_ENOMEM : WISV_EHIP,                    \
                        std::string(#call) + ": " + hipGetErrorString(e_));                     \
    } while (0)

    const wisv_config &g = c->cfg;
    const size_t esz = c->esz;
    const int d = g.d_model, F = g.d_ff, V = g.vocab, R = c->rows_max;
    CREATE_TRY(hipSetDevice(g.device_id));
    if (!c->stream) {
        CREATE_TRY(hipStreamCreate(&c->stream));
        c->stream_owned = true;
    }
    CREATE_TRY(hipEventCreate(&c->ev_round[0]));
    CREATE_TRY(hipEventCreate(&c->ev_round[1]));
    CREATE_TRY(ss_static_init(g.device_id));   // address of the static scratch on this device (wisv_ss_decide_static)

    // ---- parameters: private copies; q/k/v and gate/up are stacked so that one product serves each group
    auto copy_in = [&](void **dst, const void *src, size_t elems) -> hipError_t {
        char *p;
        hipError_t e = dalloc(c, &p, elems * esz);
        if (e != hipSuccess) return e;
        *dst = p;
        return hipMemcpyAsync(p, src, elems * esz, hipMemcpyDeviceToDevice, c->stream);
    };
    CREATE_TRY(copy_in(&c->embed, weights->embed, (size_t)V * d));
    CREATE_TRY(copy_in(&c->lm_head, weights->lm_head, (size_t)V * d));
    CREATE_TRY(copy_in(&c->final_norm, weights->final_norm, d));
    CREATE_TRY(copy_in(&c->head_w1, weights->head_w1, (size_t)g.d_head_hidden * (g.d_draft + d + g.d_csi)));
    CREATE_TRY(copy_in(&c->head_b1, weights->head_b1, g.d_head_hidden));
    CREATE_TRY(copy_in(&c->head_w2, weights->head_w2, g.d_head_hidden));
    CREATE_TRY(copy_in(&c->head_b2, weights->head_b2, 1));
    c->layers.resize(g.n_layers);
    for (int l = 0; l < g.n_layers; ++l) {
        LayerW &L = c->layers[l];
        CREATE_TRY(copy_in(&L.attn_norm, weights->attn_norm[l], d));
        CREATE_TRY(copy_in(&L.ffn_norm, weights->ffn_norm[l], d));
        CREATE_TRY(copy_in(&L.wo, weights->wo[l], (size_t)d * c->d_q));
        CREATE_TRY(copy_in(&L.wdown, weights->w_down[l], (size_t)d * F));
        char *p;
        CREATE_TRY(dalloc(c, &p, (size_t)c->d_qkv * d * esz));
        L.wqkv = p;
        CREATE_TRY(hipMemcpyAsync(p, weights->wq[l], (size_t)c->d_q * d * esz, hipMemcpyDeviceToDevice, c->stream));
        CREATE_TRY(hipMemcpyAsync(p + (size_t)c->d_q * d * esz, weights->wk[l], (size_t)c->d_kv * d * esz,
                                  hipMemcpyDeviceToDevice, c->stream));
        CREATE_TRY(hipMemcpyAsync(p + (size_t)(c->d_q + c->d_kv) * d * esz, weights->wv[l], (size_t)c->d_kv * d * esz,
                                  hipMemcpyDeviceToDevice, c->stream));
        CREATE_TRY(dalloc(c, &p, (size_t)2 * F * d * esz));
        L.wgu = p;
        CREATE_TRY(hipMemcpyAsync(p, weights->w_gate[l], (size_t)F * d * esz, hipMemcpyDeviceToDevice, c->stream));
        CREATE_TRY(hipMemcpyAsync(p + (size_t)F * d * esz, weights->w_up[l], (size_t)F * d * esz,
                                  hipMemcpyDeviceToDevice, c->stream));
    }

    // ---- decision head: W1 zero-padded to a multiple of 32 columns (the gathered z is padded alike)
    {
        const int din = g.d_draft + d + g.d_csi;
        c->din_pad = (din + 31) / 32 * 32;
        char *p;
        CREATE_TRY(dalloc(c, &p, (size_t)g.d_head_hidden * c->din_pad * esz));
        c->head_w1_pad = p;
        launch_pad_cols(c, c->head_w1, p, g.d_head_hidden, din, c->din_pad);
        CREATE_TRY(hipGetLastError());
        c->head_w1_t = nullptr;
    }

    // ---- re-tiled copies for the weight-streaming MFMA GEMM (bf16, every reduction length a multiple of 32)
    c->ws_ok = c->bf16 && d % 32 == 0 && c->d_q % 32 == 0 && F % 32 == 0;
    c->lm_head_t = c->lm_head_h = nullptr;
    c->half_ok = false;
    c->one_term_mask = 0;
    if (c->ws_ok) {
        auto retile = [&](void **dst, const void *src, int n_rows, int kd, int pair_rows) -> hipError_t {
            const int nrb = pair_rows > 0 ? ws_padded_pair_blocks(pair_rows) : ws_padded_row_blocks(n_rows);
            char *p;
            hipError_t e = dalloc(c, &p, (size_t)nrb * 16 * kd * 2);
            if (e != hipSuccess) return e;
            *dst = p;
            launch_retile(c, src, n_rows, kd, pair_rows, p, nrb);
            return hipGetLastError();
        };
        // the same tiles as IEEE halves when rounds of more than 16 rows can occur: there the products are bound by
        // the matrix cores and take their activations as one half-precision term instead of two bf16 terms
        const bool want_half = R > 16;
        int32_t *d_overflow = nullptr;
        if (want_half) {
            CREATE_TRY(dalloc(c, &d_overflow, 1));
            CREATE_TRY(hipMemsetAsync(d_overflow, 0, 4, c->stream));
        }
        auto retile_h = [&](void **dst, const void *src, int n_rows, int kd, int pair_rows) -> hipError_t {
            *dst = nullptr;
            if (!want_half) return hipSuccess;
            const int nrb = pair_rows > 0 ? ws_padded_pair_blocks(pair_rows) : ws_padded_row_blocks(n_rows);
            char *p;
            hipError_t e = dalloc(c, &p, (size_t)nrb * 16 * kd * 2);
            if (e != hipSuccess) return e;
            *dst = p;
            launch_retile(c, src, n_rows, kd, pair_rows, p, nrb, d_overflow);
            return hipGetLastError();
        };
        CREATE_TRY(retile_h(&c->lm_head_h, c->lm_head, V, d, 0));
        for (int l = 0; l < g.n_layers; ++l) {
            LayerW &L = c->layers[l];
            CREATE_TRY(retile_h(&L.wqkv_h, L.wqkv, c->d_qkv, d, 0));
            CREATE_TRY(retile_h(&L.wo_h, L.wo, d, c->d_q, 0));
            CREATE_TRY(retile_h(&L.wgu_h, L.wgu, 2 * F, d, F));
            CREATE_TRY(retile_h(&L.wdown_h, L.wdown, d, F, 0));
        }
        if (want_half) {
            int32_t overflow = 0;
            CREATE_TRY(hipMemcpyAsync(&overflow, d_overflow, 4, hipMemcpyDeviceToHost, c->stream));
            CREATE_TRY(hipStreamSynchronize(c->stream));
            c->half_ok = overflow == 0;   // a weight beyond the half range: stay with two bf16 terms everywhere
        }
        // default: the feed-forward products and the LM head (9/10 of the matrix work).  The QKV and O products keep
        // two terms: their rounding passes through the softmax and costs the most accuracy per unit of work saved.
        c->one_term_mask = c->half_ok ? (TERM_GATE_UP | TERM_DOWN | TERM_LM_HEAD) : 0;
        CREATE_TRY(retile(&c->lm_head_t, c->lm_head, V, d, 0));
        CREATE_TRY(retile(&c->head_w1_t, c->head_w1_pad, g.d_head_hidden, c->din_pad, 0));
        for (int l = 0; l < g.n_layers; ++l) {
            LayerW &L = c->layers[l];
            CREATE_TRY(retile(&L.wqkv_t, L.wqkv, c->d_qkv, d, 0));
            CREATE_TRY(retile(&L.wo_t, L.wo, d, c->d_q, 0));
            CREATE_TRY(retile(&L.wgu_t, L.wgu, 2 * F, d, F));
            CREATE_TRY(retile(&L.wdown_t, L.wdown, d, F, 0));
        }
    }

    // ---- rotary tables, computed in double: angle(pos, i) = pos * theta^(-2i/hd)
    {
        const int half = g.head_dim / 2;
        std::vector<float> hc((size_t)g.max_ctx * half), hs((size_t)g.max_ctx * half);
        for (int i = 0; i < half; ++i) {
            const double inv = pow((double)g.rope_theta, -2.0 * i / g.head_dim);
            for (int p = 0; p < g.max_ctx; ++p) {
                hc[(size_t)p * half + i] = (float)cos(p * inv);
                hs[(size_t)p * half + i] = (float)sin(p * inv);
            }
        }
        CREATE_TRY(dalloc(c, &c->rope_cos, hc.size()));
        CREATE_TRY(dalloc(c, &c->rope_sin, hs.size()));
        CREATE_TRY(hipMemcpy(c->rope_cos, hc.data(), hc.size() * 4, hipMemcpyHostToDevice));
        CREATE_TRY(hipMemcpy(c->rope_sin, hs.data(), hs.size() * 4, hipMemcpyHostToDevice));
    }

    // ---- KV cache and stream state
    const size_t kv_elems = (size_t)g.n_layers * g.max_batch * 2 * g.n_kv_heads * c->ctx_pad * g.head_dim;
    if (g.kv_cache) {
        c->kv = g.kv_cache;
        c->kv_owned = false;
    } else {
        char *p;
        CREATE_TRY(dalloc(c, &p, kv_elems * esz));
        c->kv = p;
        c->kv_owned = true;
        CREATE_TRY(hipMemsetAsync(p, 0, kv_elems * esz, c->stream));
    }
    CREATE_TRY(dalloc(c, &c->d_kv_len, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_pred_next, g.max_batch));
    CREATE_TRY(hipMemsetAsync(c->d_kv_len, 0, g.max_batch * 4, c->stream));
    CREATE_TRY(hipMemsetAsync(c->d_pred_next, 0, g.max_batch * 4, c->stream));

    // ---- staging of a round's inputs / outputs, scratch of the forward
    CREATE_TRY(dalloc(c, &c->d_stream_ids, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_tokens, R));
    CREATE_TRY(dalloc(c, &c->d_proto, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_hd_row, R));
    {
        char *p;
        CREATE_TRY(dalloc(c, &p, (size_t)R * g.d_draft * esz));
        c->d_hd = p;
    }
    CREATE_TRY(dalloc(c, &c->d_csi, (size_t)g.max_batch * g.d_csi));
    CREATE_TRY(dalloc(c, &c->d_tau, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_alen, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_ytok, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_targ, (size_t)g.max_batch * (g.max_k + 1)));
    CREATE_TRY(dalloc(c, &c->d_pacc, R));
    CREATE_TRY(dalloc(c, &c->d_mask, g.max_batch));
    CREATE_TRY(dalloc(c, &c->d_status, g.max_batch));
    CREATE_TRY(dalloc(c, &c->row_slot, R));
    CREATE_TRY(dalloc(c, &c->row_pos, R));
    CREATE_TRY(dalloc(c, &c->amax, R));
    CREATE_TRY(dalloc(c, &c->scored, R));
    CREATE_TRY(dalloc(c, &c->x, (size_t)R * d));
    CREATE_TRY(dalloc(c, &c->x_alt, (size_t)R * d));
    CREATE_TRY(dalloc(c, &c->ss, (size_t)MAX_SPLITS * R));
    CREATE_TRY(dalloc(c, &c->ss2, (size_t)((d + 15) / 16) * std::min(R, 16)));
    c->graph_refused = false;
    CREATE_TRY(dalloc(c, &c->y, (size_t)MAX_SPLITS * R * d));
    CREATE_TRY(dalloc(c, &c->qkv, (size_t)MAX_SPLITS * R * c->d_qkv));
    {
        const size_t n_cand = ws_padded_row_blocks(V);
        CREATE_TRY(dalloc(c, &c->cand_val, (size_t)R * n_cand));
        CREATE_TRY(dalloc(c, &c->cand_idx, (size_t)R * n_cand));
    }
    CREATE_TRY(dalloc(c, &c->gu, (size_t)R * 2 * F));
    CREATE_TRY(dalloc(c, &c->h_t, (size_t)R * d));
    CREATE_TRY(dalloc(c, &c->hu, (size_t)((g.d_head_hidden + 15) / 16) * R));   // the head's partial sums [row-block][row]
    auto act_alloc = [&](ActBuf *a, size_t n, bool half) -> hipError_t {
        hipError_t e = dalloc(c, &a->f, n);
        if (e == hipSuccess) e = dalloc(c, &a->hi, n);
        if (e == hipSuccess) e = dalloc(c, &a->lo, n);
        a->h16 = nullptr;
        if (e == hipSuccess && half) e = dalloc(c, &a->h16, n);
        return e;
    };
    CREATE_TRY(act_alloc(&c->a, (size_t)R * d, c->half_ok));
    CREATE_TRY(act_alloc(&c->o, (size_t)R * c->d_q, c->half_ok));
    CREATE_TRY(act_alloc(&c->h, (size_t)R * F, c->half_ok));
    CREATE_TRY(dalloc(c, &c->q, (size_t)R * c->d_q));
    {
        // split-KV attention partials: as many splits as fit 64 MiB, at most 64
        const size_t per_split = (size_t)R * c->d_q;
        c->att_max_splits = (int)std::max<size_t>(1, std::min<size_t>(64, ((size_t)16 << 20) / per_split));
        CREATE_TRY(dalloc(c, &c->att_o, per_split * c->att_max_splits));
        CREATE_TRY(dalloc(c, &c->att_m, (size_t)R * g.n_heads * c->att_max_splits));
        CREATE_TRY(dalloc(c, &c->att_l, (size_t)R * g.n_heads * c->att_max_splits));
    }
    CREATE_TRY(dalloc(c, &c->logits, (size_t)R * V));
    c->logits_rows = R;
    {
        char *p;
        CREATE_TRY(dalloc(c, &p, ss_workspace_bytes(R, V, g.max_batch)));
        c->ss_ws = p;
    }
    CREATE_TRY(dalloc(c, &c->d_ss_u, R));
    CREATE_TRY(dalloc(c, &c->d_ss_v, g.max_batch));
    c->d_ss_q = nullptr;
    CREATE_TRY(hipStreamSynchronize(c->stream));
#undef CREATE_TRY
    *out = c;
    if (err && err_len) err[0] = 0;
    return WISV_OK;
}

extern "C" int wisv_destroy(wisv_ctx *ctx) {
    destroy_ctx(ctx);
    return WISV_OK;
}

extern "C" const char *wisv_last_error(const wisv_ctx *ctx) { return ctx ? ctx->err.c_str() : ""; }

// ------------------------------------------------------------------------------------------ the target forward

// Enqueues the decoder over f.rows rows (Alg. 1 "Verify"): leaves h^T in c->h_t and the greedy token of
// every row in c->amax.
// The folded RMSNorms make every workgroup of the consuming product sum the slices (or stage the whole attention row)
// itself, work that grows with the rows while the launch it saves does not.  At the 8B shape, one stream over 512
// cached tokens: 4 rows 3.43 -> 3.38 ms per round with the folds; 8 rows 3.52 -> 3.72 ms, 16 rows 3.84 -> 4.14 ms.
constexpr int FOLD_MAX_ROWS = 4;

static void enqueue_forward(Ctx *c, const Fwd &f) {
    const wisv_config &g = c->cfg;
    const int d = g.d_model, F = g.d_ff;
    launch_prep_rows(c, f);
    launch_embed(c, f);
    c->o_planes = ACT_ALL;
    if (c->ws_ok) {
        // bf16 weight-streaming path: every product leaves k-split partial slices that the next
        // kernel sums in a fixed order; gate/up and the LM head fuse SwiGLU / argmax instead
        const size_t ys = (size_t)c->rows_max * d, qs = (size_t)c->rows_max * c->d_qkv;
        // a product whose shape the streaming kernel cannot serve falls back to the generic kernel (one slice)
        // wh: the half-precision tiles when this product class runs with one term (more than 16 rows only)
        auto half = [&](const void *wh, uint32_t cls) { return f.rows > 16 && (c->one_term_mask & cls) ? wh : nullptr; };
        // have_f: the float plane of X is current (the generic kernel reads that one)
        auto product = [&](const void *wt, const void *w, const void *wh, const ActBuf &X, float *Yp, size_t stride, int n, int kd, int kclass,
                           bool have_f = true) {
            int ns = launch_gemm_ws_partial(c, wt, X, Yp, stride, MAX_SPLITS, f.rows, n, kd, kclass, nullptr, wh);
            if (!ns) {
                if (!have_f) {
                    c->launch_failed = true;
                    c->launch_err = "a product fell back to the generic kernel after its input was written without the float plane";
                    return 1;
                }
                launch_gemm_ref(c, X.f, w, Yp, f.rows, n, kd, kclass);
                ns = 1;
            }
            return ns;
        };
        // Beyond 16 rows an activation buffer is written in the one representation its consumer reads: the half
        // plane when that product class runs with one term, else the two bf16 planes; never the float plane
        auto planes_for = [&](const void *wh) { return f.rows <= 16 ? ACT_ALL : wh && c->a.h16 ? ACT_HALF : ACT_TWO_TERM; };
        const bool full = f.rows <= 16;   // every representation is written
        if (g.n_layers) c->o_planes = planes_for(half(c->layers[0].wo_h, TERM_O));
        bool h_has_f = true;
        auto gate_up = [&](const LayerW &L, int n_ss) {
            h_has_f = full;
            if (!launch_gemm_ws_swiglu(c, L.wgu_t, c->a, c->h, f.rows, F, d, KC_GEMM_GATEUP, half(L.wgu_h, TERM_GATE_UP), c->ss2, n_ss,
                                       planes_for(half(L.wdown_h, TERM_DOWN)))) {
                if (!full) {   // c->a came without its float plane
                    c->launch_failed = true;
                    c->launch_err = "gate/up fell back to the generic kernel after its input was written without the float plane";
                    return;
                }
                h_has_f = true;
                if (n_ss > 0) {   // only the streaming kernel applies the deferred 1 / rms
                    c->launch_failed = true;
                    c->launch_err = "gate/up: the streaming kernel does not serve this shape after a folded RMSNorm";
                    return;
                }
                launch_gemm_ref(c, c->a.f, L.wgu, c->gu, f.rows, 2 * F, d, KC_GEMM_GATEUP);
                launch_swiglu(c, f.rows);
            }
        };
        int ny = 0;
        const bool fuse_rope = attn_mfma_fuses_rope(c, f);
        for (int l = 0; l < g.n_layers; ++l) {
            const LayerW &L = c->layers[l];
            // Few rows, attention with the fused prologue: the attention norm is folded into the QKV product
            // (it sums the previous slices into the residual stream itself and is fed x * gain) and the attention
            // prologue, which sums the QKV slices anyway, applies 1 / rms.  One launch less per layer.
            int nq = 0, n_ss = 0;
            if (fuse_rope && f.rows <= FOLD_MAX_ROWS) {
                nq = n_ss = launch_gemm_ws_normfold(c, L.wqkv_t, c->x, c->x_alt, ny, L.attn_norm, c->qkv, qs, MAX_SPLITS, f.rows,
                                                    c->d_qkv, d, c->ss, KC_GEMM_QKV);
                if (nq) std::swap(c->x, c->x_alt);
            }
            if (!nq) {
                launch_rmsnorm(c, f.rows, ny, L.attn_norm, act_planes(c->a, planes_for(half(L.wqkv_h, TERM_QKV))), nullptr);
                nq = product(L.wqkv_t, L.wqkv, half(L.wqkv_h, TERM_QKV), c->a, c->qkv, qs, c->d_qkv, d, KC_GEMM_QKV, full);
            }
            // with few k-splits and few rows the O projection combines the attention partials while it stages them
            const bool defer = fuse_rope && f.rows <= 16 && g.head_dim == 128;
            int att_splits = 1;
            if (!(fuse_rope && launch_attn_mfma(c, f, l, nq, !defer, &att_splits, n_ss))) {
                att_splits = 1;
                launch_rope_append(c, f, l, nq, n_ss);
                if (!launch_attn_mfma(c, f, l, 0)) launch_attn_ref(c, f, l);
            }
            ny = 0;
            // Few rows: the O projection keeps its k-split inside the workgroup, adds the residual stream itself
            // and hands x * gain and the rows' sums of squares to gate/up, which applies 1 / rms: the FFN norm's launch
            // goes too.  It takes the attention's k-split partials as they are when there are few of them.
            int n_ss2 = 0;
            if (f.rows <= FOLD_MAX_ROWS) {
                const AttnPartials ap{c->att_o, c->att_m, c->att_l, att_splits, f.rows, g.n_heads};
                const bool partials = defer && att_splits > 1;
                if (!partials || att_splits <= WS_PRO_SPLITS)
                    n_ss2 = launch_gemm_ws_resid(c, L.wo_t, c->o, partials ? &ap : nullptr, c->x, L.ffn_norm, c->a, c->ss2, f.rows, d,
                                                 c->d_q, KC_GEMM_O);
            }
            if (!n_ss2) {
                if (defer && att_splits > 1) {
                    if (att_splits <= WS_PRO_SPLITS) {
                        const AttnPartials ap{c->att_o, c->att_m, c->att_l, att_splits, f.rows, g.n_heads};
                        ny = launch_gemm_ws_partial(c, L.wo_t, c->o, c->y, ys, MAX_SPLITS, f.rows, d, c->d_q, KC_GEMM_O, &ap);
                    }
                    if (!ny) launch_attn_combine(c, f, att_splits);   // more splits than the projection takes: a kernel of its own
                }
                if (!ny) ny = product(L.wo_t, L.wo, half(L.wo_h, TERM_O), c->o, c->y, ys, d, c->d_q, KC_GEMM_O, full);
                launch_rmsnorm(c, f.rows, ny, L.ffn_norm, act_planes(c->a, planes_for(half(L.wgu_h, TERM_GATE_UP))), nullptr);
            }
            gate_up(L, n_ss2);
            ny = product(L.wdown_t, L.wdown, half(L.wdown_h, TERM_DOWN), c->h, c->y, ys, d, F, KC_GEMM_DOWN, h_has_f);
        }
        launch_rmsnorm(c, f.rows, ny, c->final_norm, act_planes(c->a, planes_for(half(c->lm_head_h, TERM_LM_HEAD))), c->h_t);
        if (!launch_gemm_ws_argmax(c, c->lm_head_t, c->a, f.keep_logits ? c->logits : nullptr, f.rows, g.vocab, d,
                                   KC_LMHEAD, half(c->lm_head_h, TERM_LM_HEAD))) {
            if (!full) {
                c->launch_failed = true;
                c->launch_err = "the LM head fell back to the generic kernel after its input was written without the float plane";
                return;
            }
            launch_gemm_ref(c, c->a.f, c->lm_head, c->logits, f.rows, g.vocab, d, KC_LMHEAD);
            launch_argmax(c, f.rows);
        }
        return;
    }
    for (int l = 0; l < g.n_layers; ++l) {
        const LayerW &L = c->layers[l];
        launch_rmsnorm(c, f.rows, l == 0 ? 0 : 1, L.attn_norm, c->a, nullptr);     // + previous FFN update
        launch_gemm_ref(c, c->a.f, L.wqkv, c->qkv, f.rows, c->d_qkv, d, KC_GEMM_QKV);
        launch_rope_append(c, f, l, 1);
        launch_attn_ref(c, f, l);
        launch_gemm_ref(c, c->o.f, L.wo, c->y, f.rows, d, c->d_q, KC_GEMM_O);
        launch_rmsnorm(c, f.rows, 1, L.ffn_norm, c->a, nullptr);                   // + attention update
        launch_gemm_ref(c, c->a.f, L.wgu, c->gu, f.rows, 2 * F, d, KC_GEMM_GATEUP);
        launch_swiglu(c, f.rows);
        launch_gemm_ref(c, c->h.f, L.wdown, c->y, f.rows, d, F, KC_GEMM_DOWN);
    }
    launch_rmsnorm(c, f.rows, 1, c->final_norm, c->a, c->h_t);
    launch_gemm_ref(c, c->a.f, c->lm_head, c->logits, f.rows, g.vocab, d, KC_LMHEAD);
    launch_argmax(c, f.rows);
}

// ------------------------------------------------------------------------------------------ verify round

static int check_round(Ctx *c, const wisv_round_in *in, const wisv_round_out *out) {
    if (!in || !out) return fail(c, WISV_EINVAL, "round_in / round_out is NULL");
    const wisv_config &g = c->cfg;
    if (in->batch < 1 || in->batch > g.max_batch) return fail(c, WISV_EINVAL, "batch %d outside [1, %d]", in->batch, g.max_batch);
    if (in->k < 1 || in->k > g.max_k) return fail(c, WISV_EINVAL, "k %d outside [1, max_k = %d]", in->k, g.max_k);
    if (!in->stream_ids || !in->draft_tokens || !in->proto || !in->csi || !in->tau)
        return fail(c, WISV_EINVAL, "a required round_in pointer is NULL");
    if (in->n_hd < 0 || in->n_hd > in->batch * in->k) return fail(c, WISV_EINVAL, "n_hd %d outside [0, batch*k]", in->n_hd);
    if (in->n_hd > 0 && !in->hd) return fail(c, WISV_EINVAL, "hd is NULL but n_hd > 0");
    if (!in->hd_row && in->n_hd != in->batch * in->k)
        return fail(c, WISV_EINVAL, "hd_row is NULL (identity map) but n_hd != batch*k");
    if (!out->accepted_len || !out->correction_token || !out->p_accept)
        return fail(c, WISV_EINVAL, "a required round_out pointer is NULL");
    if (in->flags & ~(WISV_FLAG_GATE_ALL | WISV_FLAG_NO_COMMIT | WISV_FLAG_DEVICE_IO | WISV_FLAG_KEEP_LOGITS |
                      WISV_FLAG_VERIFY_ONLY | WISV_FLAG_DECIDE_ONLY))
        return fail(c, WISV_EINVAL, "unknown flag bits 0x%x", in->flags);
    if ((in->flags & WISV_FLAG_VERIFY_ONLY) && (in->flags & WISV_FLAG_DECIDE_ONLY))
        return fail(c, WISV_EINVAL, "WISV_FLAG_VERIFY_ONLY and WISV_FLAG_DECIDE_ONLY exclude each other");
    if ((in->flags & (WISV_FLAG_VERIFY_ONLY | WISV_FLAG_DECIDE_ONLY)) && (in->flags & WISV_FLAG_DEVICE_IO))
        return fail(c, WISV_EUNSUPPORTED, "the two-call protocol takes host buffers (it checks that both calls name the same round)");
    return WISV_OK;
}

extern "C" int wisv_verify_round(wisv_ctx *ctx, const wisv_round_in *in, wisv_round_out *out) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    int rc = check_round(c, in, out);
    if (rc) return rc;
    const wisv_config &g = c->cfg;
    const int B = in->batch, K = in->k, R = B * K;
    const bool verify_only = in->flags & WISV_FLAG_VERIFY_ONLY, decide_only = in->flags & WISV_FLAG_DECIDE_ONLY;
    const bool dev_io = in->flags & WISV_FLAG_DEVICE_IO, commit = !(in->flags & WISV_FLAG_NO_COMMIT) && !verify_only;

    int len_ub = 0;
    if (!dev_io) {
        // host-visible arguments: check their values before anything is enqueued
        std::vector<char> seen(g.max_batch, 0);
        for (int b = 0; b < B; ++b) {
            const int s = in->stream_ids[b];
            if (s < 0 || s >= g.max_batch) return fail(c, WISV_EINVAL, "stream_ids[%d] = %d outside [0, %d)", b, s, g.max_batch);
            if (seen[s]) return fail(c, WISV_EINVAL, "stream id %d appears twice", s);
            seen[s] = 1;
            if (in->proto[b] != WISV_PROTO_FH && in->proto[b] != WISV_PROTO_SH)
                return fail(c, WISV_EINVAL, "proto[%d] = %d is neither FH nor SH", b, in->proto[b]);
            if ((in->flags & WISV_FLAG_GATE_ALL) && in->proto[b] != WISV_PROTO_FH)
                return fail(c, WISV_EINVAL, "WISV_FLAG_GATE_ALL needs full-hidden upload on every stream");
            if (c->h_len_ub[s] + K > g.max_ctx)
                return fail(c, WISV_ESTATE, "stream %d: cached length %d + k %d exceeds max_ctx %d", s, c->h_len_ub[s], K, g.max_ctx);
            len_ub = std::max(len_ub, c->h_len_ub[s] + K);
        }
        for (int m = 0; m < R; ++m) {
            if (in->draft_tokens[m] < 0 || in->draft_tokens[m] >= g.vocab)
                return fail(c, WISV_EINVAL, "draft_tokens[%d] = %d outside the vocabulary", m, in->draft_tokens[m]);
            if (in->hd_row && (in->hd_row[m] < -1 || in->hd_row[m] >= in->n_hd))
                return fail(c, WISV_EINVAL, "hd_row[%d] = %d outside [-1, n_hd)", m, in->hd_row[m]);
        }
    } else {
        // device-resident arguments cannot be inspected here; kernels clamp ids, tokens and rows
        for (int s = 0; s < g.max_batch; ++s) len_ub = std::max(len_ub, c->h_len_ub[s] + K);
        if (len_ub > g.max_ctx)
            return fail(c, WISV_ESTATE, "a stream may exceed max_ctx; resynchronise with wisv_get_state");
    }

    // the two-call protocol: the second call must name the round the first one ran
    if (decide_only) {
        bool same = c->pending_valid && c->pending_batch == B && c->pending_k == K;
        for (int b = 0; same && b < B; ++b) same = c->pending_ids[b] == in->stream_ids[b];
        for (int m = 0; same && m < R; ++m) same = c->pending_tokens[m] == in->draft_tokens[m];
        if (!same) return fail(c, WISV_ESTATE, "WISV_FLAG_DECIDE_ONLY without a WISV_FLAG_VERIFY_ONLY call for the same round before it");
    }
    c->pending_valid = false;   // any round overwrites what a VERIFY_ONLY call left behind

    HIP_TRY(c, hipSetDevice(g.device_id));
    wisv_round_in din = *in;
    wisv_round_out dout = *out;
    if (!dev_io) {
        HIP_TRY(c, hipMemcpyAsync(c->d_stream_ids, in->stream_ids, B * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_tokens, in->draft_tokens, R * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_proto, in->proto, B * 4, hipMemcpyHostToDevice, c->stream));
        if (in->hd_row) HIP_TRY(c, hipMemcpyAsync(c->d_hd_row, in->hd_row, R * 4, hipMemcpyHostToDevice, c->stream));
        if (in->n_hd)
            HIP_TRY(c, hipMemcpyAsync(c->d_hd, in->hd, (size_t)in->n_hd * g.d_draft * c->esz, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_csi, in->csi, (size_t)B * g.d_csi * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_tau, in->tau, B * 4, hipMemcpyHostToDevice, c->stream));
        din.stream_ids = c->d_stream_ids;
        din.draft_tokens = c->d_tokens;
        din.proto = c->d_proto;
        din.hd_row = in->hd_row ? c->d_hd_row : nullptr;
        din.hd = c->d_hd;
        din.csi = c->d_csi;
        din.tau = c->d_tau;
        dout.accepted_len = c->d_alen;
        dout.correction_token = c->d_ytok;
        dout.p_accept = c->d_pacc;
        dout.target_argmax = c->d_targ;
        dout.mismatch_mask = c->d_mask;
        dout.status = c->d_status;
    }

    Fwd f;
    f.rows = R;
    f.batch = B;
    f.k = K;
    f.stream_ids = din.stream_ids;
    f.tokens = din.draft_tokens;
    f.keep_logits = in->flags & WISV_FLAG_KEEP_LOGITS;
    f.max_len_ub = len_ub;

    // A device-I/O round repeated with identical arguments (a serving loop re-using its buffers) is captured
    // into a HIP graph the second time it is seen and replayed from then on: one submission instead of a
    // few hundred launches.  Positions are read from device state, so a replay stays valid while the upper
    // bound of the cached lengths (which sizes the attention launch) is unchanged.
    const bool graphable = dev_io && !c->profiling;
    auto same_in = [](const wisv_round_in &x, const wisv_round_in &y) {
        return x.batch == y.batch && x.k == y.k && x.stream_ids == y.stream_ids && x.draft_tokens == y.draft_tokens &&
               x.proto == y.proto && x.hd == y.hd && x.hd_row == y.hd_row && x.n_hd == y.n_hd && x.csi == y.csi &&
               x.tau == y.tau && x.flags == y.flags;
    };
    auto same_out = [](const wisv_round_out &x, const wisv_round_out &y) {
        return x.accepted_len == y.accepted_len && x.correction_token == y.correction_token && x.p_accept == y.p_accept &&
               x.target_argmax == y.target_argmax && x.mismatch_mask == y.mismatch_mask && x.status == y.status;
    };
    const bool same_call = graphable && c->graph_len_ub == len_ub && same_in(c->graph_in, *in) && same_out(c->graph_out, *out);
    HIP_TRY(c, hipEventRecord(c->ev_round[0], c->stream));
    c->launch_failed = false;
    auto enqueue_round = [&]() -> hipError_t {
        { ProfScope empty(c, KC_EMPTY); }   // an event pair with nothing in between: what the bracketing itself costs
        if (!decide_only) enqueue_forward(c, f);   // else: h^T, the greedy tokens and the appended K/V are still there
        if (c->launch_failed) return hipSuccess;   // a step was not served: nothing may be decided or committed from the rest
        if (verify_only) {
            // localisation only: no hidden state counts as uploaded, nothing is committed
            din.n_hd = 0;
            din.hd_row = c->d_hd_row;
            hipError_t e = hipMemsetAsync(c->d_hd_row, 0xff, (size_t)R * 4, c->stream);   // every row: -1, not uploaded
            if (e != hipSuccess) return e;
            din.flags |= WISV_FLAG_NO_COMMIT;
        }
        launch_head_decide(c, f, din, dout);
        return hipSuccess;
    };
    if (same_call && c->graph_exec) {
        HIP_TRY(c, hipGraphLaunch(c->graph_exec, c->stream));
    } else {
        // calls that cannot be replayed (host I/O, profiling) run eagerly and leave the cached graph alone
        if (graphable && c->graph_exec) {
            (void)hipGraphExecDestroy(c->graph_exec);
            c->graph_exec = nullptr;
        }
        bool captured = false;
        if (same_call && !c->graph_refused) {   // the first call of a kind always runs eagerly (one-time kernel attribute set-up)
            // Capture, instantiate, launch.  Whatever fails, the capture is ended and its graph dropped, and the round
            // is enqueued eagerly instead: a failed capture must not leave the (possibly borrowed) stream capturing.
            if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal) == hipSuccess) {
                const hipError_t e_enq = enqueue_round();
                hipGraph_t graph = nullptr;
                const hipError_t e_end = hipStreamEndCapture(c->stream, &graph);
                hipGraphExec_t exec = nullptr;
                if (e_enq == hipSuccess && e_end == hipSuccess && graph && !c->launch_failed &&
                    hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess) {
                    if (hipGraphLaunch(exec, c->stream) == hipSuccess) {
                        c->graph_exec = exec;
                        captured = true;
                    } else {
                        (void)hipGraphExecDestroy(exec);
                    }
                }
                if (graph) (void)hipGraphDestroy(graph);
                (void)hipGetLastError();   // a capture error is not this round's error: the eager path decides
                if (!captured) c->graph_refused = true;   // e.g. a launch the capture does not take: do not try every round
            }
        }
        if (!captured && !c->launch_failed) HIP_TRY(c, enqueue_round());
        if (graphable) {
            c->graph_in = *in;        // compared member by member (struct padding is not part of the key)
            c->graph_out = *out;
            c->graph_len_ub = len_ub;
        }
    }
    if (c->launch_failed) {
        c->graph_len_ub = -1;
        return fail(c, WISV_EUNSUPPORTED, "%s", c->launch_err.c_str());
    }
    HIP_TRY(c, hipEventRecord(c->ev_round[1], c->stream));
    HIP_TRY(c, hipGetLastError());
    c->last_rows = R;

    if (!dev_io) {
        std::vector<int32_t> alen(B);
        HIP_TRY(c, hipMemcpyAsync(alen.data(), c->d_alen, B * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipMemcpyAsync(out->correction_token, c->d_ytok, B * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipMemcpyAsync(out->p_accept, c->d_pacc, R * 4, hipMemcpyDeviceToHost, c->stream));
        if (out->target_argmax)
            HIP_TRY(c, hipMemcpyAsync(out->target_argmax, c->d_targ, (size_t)B * (K + 1) * 4, hipMemcpyDeviceToHost, c->stream));
        if (out->mismatch_mask) HIP_TRY(c, hipMemcpyAsync(out->mismatch_mask, c->d_mask, B * 4, hipMemcpyDeviceToHost, c->stream));
        if (out->status) HIP_TRY(c, hipMemcpyAsync(out->status, c->d_status, B * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        for (int b = 0; b < B; ++b) {
            out->accepted_len[b] = alen[b];
            if (commit) c->h_len_ub[in->stream_ids[b]] += alen[b];
        }
        if (verify_only) {
            c->pending_valid = true;
            c->pending_batch = B;
            c->pending_k = K;
            c->pending_ids.assign(in->stream_ids, in->stream_ids + B);
            c->pending_tokens.assign(in->draft_tokens, in->draft_tokens + R);
        }
    } else if (commit) {
        for (int s = 0; s < g.max_batch; ++s) c->h_len_ub[s] = std::min(c->h_len_ub[s] + K, g.max_ctx);
    }
    return WISV_OK;
}

// ------------------------------------------------------------------------------------------ speculative sampling

extern "C" int wisv_ss_verify_round(wisv_ctx *ctx, const wisv_ss_in *in, wisv_ss_out *out) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (!in || !out) return fail(c, WISV_EINVAL, "ss_in / ss_out is NULL");
    const wisv_config &g = c->cfg;
    if (in->batch < 1 || in->batch > g.max_batch) return fail(c, WISV_EINVAL, "batch %d outside [1, %d]", in->batch, g.max_batch);
    if (in->k < 1 || in->k > g.max_k) return fail(c, WISV_EINVAL, "k %d outside [1, max_k = %d]", in->k, g.max_k);
    if (!in->stream_ids || !in->draft_tokens || !in->draft_probs || !in->u_accept || !in->u_sample)
        return fail(c, WISV_EINVAL, "a required ss_in pointer is NULL");
    if (!out->accepted_len || !out->correction_token || !out->alpha) return fail(c, WISV_EINVAL, "a required ss_out pointer is NULL");
    if (in->flags & ~(WISV_FLAG_NO_COMMIT | WISV_FLAG_DEVICE_IO)) return fail(c, WISV_EINVAL, "unknown flag bits 0x%x", in->flags);
    const int B = in->batch, K = in->k, R = B * K, V = g.vocab;
    if (V > SS_MAX_VOCAB) return fail(c, WISV_EUNSUPPORTED, "vocabulary %d beyond what the sampling kernel serves (%d)", V, SS_MAX_VOCAB);
    const bool dev_io = in->flags & WISV_FLAG_DEVICE_IO, commit = !(in->flags & WISV_FLAG_NO_COMMIT);

    int len_ub = 0;
    if (!dev_io) {
        std::vector<char> seen(g.max_batch, 0);
        for (int b = 0; b < B; ++b) {
            const int s = in->stream_ids[b];
            if (s < 0 || s >= g.max_batch) return fail(c, WISV_EINVAL, "stream_ids[%d] = %d outside [0, %d)", b, s, g.max_batch);
            if (seen[s]) return fail(c, WISV_EINVAL, "stream id %d appears twice", s);
            seen[s] = 1;
            if (c->h_len_ub[s] + K > g.max_ctx)
                return fail(c, WISV_ESTATE, "stream %d: cached length %d + k %d exceeds max_ctx %d", s, c->h_len_ub[s], K, g.max_ctx);
            len_ub = std::max(len_ub, c->h_len_ub[s] + K);
            if (!(in->u_sample[b] >= 0.f && in->u_sample[b] < 1.f)) return fail(c, WISV_EINVAL, "u_sample[%d] outside [0, 1)", b);
        }
        for (int m = 0; m < R; ++m) {
            if (in->draft_tokens[m] < 0 || in->draft_tokens[m] >= V)
                return fail(c, WISV_EINVAL, "draft_tokens[%d] = %d outside the vocabulary", m, in->draft_tokens[m]);
            if (!(in->u_accept[m] >= 0.f && in->u_accept[m] < 1.f)) return fail(c, WISV_EINVAL, "u_accept[%d] outside [0, 1)", m);
        }
    } else {
        for (int s = 0; s < g.max_batch; ++s) len_ub = std::max(len_ub, c->h_len_ub[s] + K);
        if (len_ub > g.max_ctx) return fail(c, WISV_ESTATE, "a stream may exceed max_ctx; resynchronise with wisv_get_state");
    }
    c->pending_valid = false;

    HIP_TRY(c, hipSetDevice(g.device_id));
    SsArgs a;
    a.batch = B;
    a.k = K;
    a.vocab = V;
    a.logits = c->logits;
    a.pending_tokens = nullptr;
    a.commit = commit;
    if (!dev_io) {
        if (!c->d_ss_q) HIP_TRY(c, dalloc(c, &c->d_ss_q, (size_t)c->rows_max * V));
        HIP_TRY(c, hipMemcpyAsync(c->d_stream_ids, in->stream_ids, B * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_tokens, in->draft_tokens, R * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_ss_q, in->draft_probs, (size_t)R * V * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_ss_u, in->u_accept, R * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_ss_v, in->u_sample, B * 4, hipMemcpyHostToDevice, c->stream));
        a.stream_ids = c->d_stream_ids;
        a.tokens = c->d_tokens;
        a.draft_probs = c->d_ss_q;
        a.u_accept = c->d_ss_u;
        a.u_sample = c->d_ss_v;
        a.accepted_len = c->d_alen;
        a.emitted_token = c->d_ytok;
        a.alpha = c->d_pacc;
    } else {
        a.stream_ids = in->stream_ids;
        a.tokens = in->draft_tokens;
        a.draft_probs = in->draft_probs;
        a.u_accept = in->u_accept;
        a.u_sample = in->u_sample;
        a.accepted_len = out->accepted_len;
        a.emitted_token = out->correction_token;
        a.alpha = out->alpha;
    }
    Fwd f;
    f.rows = R;
    f.batch = B;
    f.k = K;
    f.stream_ids = a.stream_ids;
    f.tokens = a.tokens;
    f.keep_logits = true;
    f.max_len_ub = len_ub;

    HIP_TRY(c, hipEventRecord(c->ev_round[0], c->stream));
    { ProfScope empty(c, KC_EMPTY); }
    c->launch_failed = false;
    enqueue_forward(c, f);
    if (c->launch_failed) return fail(c, WISV_EUNSUPPORTED, "%s", c->launch_err.c_str());
    launch_ss(c, a);
    HIP_TRY(c, hipEventRecord(c->ev_round[1], c->stream));
    HIP_TRY(c, hipGetLastError());
    c->last_rows = R;

    if (!dev_io) {
        HIP_TRY(c, hipMemcpyAsync(out->accepted_len, c->d_alen, B * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipMemcpyAsync(out->correction_token, c->d_ytok, B * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipMemcpyAsync(out->alpha, c->d_pacc, R * 4, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        if (commit)
            for (int b = 0; b < B; ++b) c->h_len_ub[in->stream_ids[b]] += out->accepted_len[b];
    } else if (commit) {
        for (int s = 0; s < g.max_batch; ++s) c->h_len_ub[s] = std::min(c->h_len_ub[s] + K, g.max_ctx);
    }
    return WISV_OK;
}

static int ss_decide_common(wisv_ctx *ctx, bool static_scratch, int32_t batch, int32_t k, int32_t vocab, const float *logits,
                            const int32_t *pending_tokens, const int32_t *draft_tokens, const float *draft_probs,
                            const float *u_accept, const float *u_sample, int32_t *accepted_len, int32_t *emitted_token,
                            float *alpha) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    const wisv_config &g = c->cfg;
    if (static_scratch) {
        // sized by the library's static scratch, not by the ctx
        if (batch < 1 || k < 1 || k > WISV_MAX_K) return fail(c, WISV_EINVAL, "batch %d / k %d outside [1, ..] / [1, %d]", batch, k, WISV_MAX_K);
        if (vocab < 1) return fail(c, WISV_EINVAL, "vocab %d is not positive", vocab);
    } else {
        if (batch < 1 || batch > g.max_batch) return fail(c, WISV_EINVAL, "batch %d outside [1, %d]", batch, g.max_batch);
        if (k < 1 || k > g.max_k) return fail(c, WISV_EINVAL, "k %d outside [1, max_k = %d]", k, g.max_k);
        if (vocab < 1 || vocab > g.vocab) return fail(c, WISV_EINVAL, "vocab %d outside [1, %d] (the scratch is sized for the ctx's vocabulary)", vocab, g.vocab);
    }
    if (vocab > SS_MAX_VOCAB) return fail(c, WISV_EUNSUPPORTED, "vocabulary %d beyond what the sampling kernel serves (%d)", vocab, SS_MAX_VOCAB);
    if (!logits || !pending_tokens || !draft_tokens || !draft_probs || !u_accept || !u_sample || !accepted_len ||
        !emitted_token || !alpha)
        return fail(c, WISV_EINVAL, "a pointer argument is NULL");
    HIP_TRY(c, hipSetDevice(g.device_id));
    SsArgs a;
    a.batch = batch;
    a.k = k;
    a.vocab = vocab;
    a.logits = logits;
    a.stream_ids = nullptr;
    a.pending_tokens = pending_tokens;
    a.tokens = draft_tokens;
    a.draft_probs = draft_probs;
    a.u_accept = u_accept;
    a.u_sample = u_sample;
    a.accepted_len = accepted_len;
    a.emitted_token = emitted_token;
    a.alpha = alpha;
    a.commit = false;
    if (static_scratch) {
        if (const char *why = launch_ss_static(c, a)) return fail(c, WISV_EUNSUPPORTED, "wisv_ss_decide_static: %s", why);
    } else {
        launch_ss(c, a);
    }
    HIP_TRY(c, hipGetLastError());
    return WISV_OK;
}

extern "C" int wisv_ss_decide(wisv_ctx *ctx, int32_t batch, int32_t k, int32_t vocab, const float *logits,
                              const int32_t *pending_tokens, const int32_t *draft_tokens, const float *draft_probs,
                              const float *u_accept, const float *u_sample, int32_t *accepted_len, int32_t *emitted_token,
                              float *alpha) {
    return ss_decide_common(ctx, false, batch, k, vocab, logits, pending_tokens, draft_tokens, draft_probs, u_accept, u_sample,
                            accepted_len, emitted_token, alpha);
}

extern "C" int wisv_ss_decide_static(wisv_ctx *ctx, int32_t batch, int32_t k, int32_t vocab, const float *logits,
                                     const int32_t *pending_tokens, const int32_t *draft_tokens, const float *draft_probs,
                                     const float *u_accept, const float *u_sample, int32_t *accepted_len,
                                     int32_t *emitted_token, float *alpha) {
    return ss_decide_common(ctx, true, batch, k, vocab, logits, pending_tokens, draft_tokens, draft_probs, u_accept, u_sample,
                            accepted_len, emitted_token, alpha);
}

// ------------------------------------------------------------------------------------------ options

extern "C" int wisv_set_option(wisv_ctx *ctx, int32_t option, int64_t value) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (option != WISV_OPT_ONE_TERM_CLASSES) return fail(c, WISV_EINVAL, "unknown option %d", option);
    if (value < 0 || value > TERM_ALL) return fail(c, WISV_EINVAL, "class mask 0x%llx outside [0, 0x%x]", (long long)value, (int)TERM_ALL);
    if (value && !c->half_ok)
        return fail(c, WISV_EUNSUPPORTED, "this ctx has no half-precision weight tiles (fp32 target, at most 16 rows per round, "
                                          "or a weight beyond the half range)");
    c->one_term_mask = (uint32_t)value;
    if (c->graph_exec) {   // a captured round holds the launches of the old setting
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        (void)hipGraphExecDestroy(c->graph_exec);
        c->graph_exec = nullptr;
    }
    c->graph_len_ub = -1;
    return WISV_OK;
}

extern "C" int wisv_get_option(wisv_ctx *ctx, int32_t option, int64_t *value) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (option != WISV_OPT_ONE_TERM_CLASSES) return fail(c, WISV_EINVAL, "unknown option %d", option);
    if (!value) return fail(c, WISV_EINVAL, "value is NULL");
    *value = c->one_term_mask;
    return WISV_OK;
}

// ------------------------------------------------------------------------------------------ state helpers

static int check_slot(Ctx *c, int32_t s) {
    if (s < 0 || s >= c->cfg.max_batch) return fail(c, WISV_EINVAL, "stream_id %d outside [0, %d)", s, c->cfg.max_batch);
    return WISV_OK;
}

extern "C" int wisv_set_state(wisv_ctx *ctx, int32_t stream_id, int32_t kv_len, int32_t pred_next) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (int rc = check_slot(c, stream_id)) return rc;
    if (kv_len < 0 || kv_len > c->cfg.max_ctx) return fail(c, WISV_EINVAL, "kv_len %d outside [0, max_ctx]", kv_len);
    if (pred_next < 0 || pred_next >= c->cfg.vocab) return fail(c, WISV_EINVAL, "pred_next %d outside the vocabulary", pred_next);
    HIP_TRY(c, hipSetDevice(c->cfg.device_id));
    HIP_TRY(c, hipMemcpyAsync(c->d_kv_len + stream_id, &kv_len, 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_pred_next + stream_id, &pred_next, 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->h_len_ub[stream_id] = kv_len;
    c->pending_valid = false;   // a VERIFY_ONLY round decided after a state change would commit against another state
    return WISV_OK;
}

extern "C" int wisv_get_state(wisv_ctx *ctx, int32_t stream_id, int32_t *kv_len, int32_t *pred_next) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (int rc = check_slot(c, stream_id)) return rc;
    HIP_TRY(c, hipSetDevice(c->cfg.device_id));
    int32_t l = 0, p = 0;
    HIP_TRY(c, hipMemcpyAsync(&l, c->d_kv_len + stream_id, 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(&p, c->d_pred_next + stream_id, 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->h_len_ub[stream_id] = l;
    if (kv_len) *kv_len = l;
    if (pred_next) *pred_next = p;
    return WISV_OK;
}

extern "C" int wisv_prefill(wisv_ctx *ctx, int32_t stream_id, const int32_t *tokens, int32_t n) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (int rc = check_slot(c, stream_id)) return rc;
    if (!tokens || n < 1) return fail(c, WISV_EINVAL, "tokens is NULL or n < 1");
    const wisv_config &g = c->cfg;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= g.vocab) return fail(c, WISV_EINVAL, "tokens[%d] outside the vocabulary", i);
    int32_t len = 0;
    if (int rc = wisv_get_state(ctx, stream_id, &len, nullptr)) return rc;
    if (len + n > g.max_ctx) return fail(c, WISV_ESTATE, "prefill of %d tokens at length %d exceeds max_ctx %d", n, len, g.max_ctx);
    c->pending_valid = false;   // the forward below overwrites h^T, the greedy tokens and the row map a VERIFY_ONLY call left
    HIP_TRY(c, hipMemcpyAsync(c->d_stream_ids, &stream_id, 4, hipMemcpyHostToDevice, c->stream));
    const int chunk = c->rows_max;
    for (int c0 = 0; c0 < n; c0 += chunk) {
        const int rows = std::min(chunk, n - c0);
        HIP_TRY(c, hipMemcpyAsync(c->d_tokens, tokens + c0, rows * 4, hipMemcpyHostToDevice, c->stream));
        Fwd f;
        f.rows = rows;
        f.batch = 1;
        f.k = rows;
        f.stream_ids = c->d_stream_ids;
        f.tokens = c->d_tokens;
        f.keep_logits = false;
        f.max_len_ub = len + c0 + rows;
        c->launch_failed = false;
        enqueue_forward(c, f);
        // the slot's state moves only past chunks whose every kernel was launched
        if (c->launch_failed) return fail(c, WISV_EUNSUPPORTED, "%s", c->launch_err.c_str());
        HIP_TRY(c, hipGetLastError());
        launch_set_pred_next(c, stream_id, rows - 1, len + c0 + rows);
        HIP_TRY(c, hipStreamSynchronize(c->stream));   // d_tokens is reused by the next chunk
        c->h_len_ub[stream_id] = len + c0 + rows;
    }
    HIP_TRY(c, hipGetLastError());
    c->h_len_ub[stream_id] = len + n;
    return WISV_OK;
}

static int kv_copy(Ctx *c, int32_t stream_id, int32_t layer, void *host_k, void *host_v, int32_t len, bool to_device) {
    if (int rc = check_slot(c, stream_id)) return rc;
    const wisv_config &g = c->cfg;
    if (layer < 0 || layer >= g.n_layers) return fail(c, WISV_EINVAL, "layer %d outside [0, %d)", layer, g.n_layers);
    if (len < 0 || len > g.max_ctx) return fail(c, WISV_EINVAL, "len %d outside [0, max_ctx]", len);
    if (!host_k || !host_v) return fail(c, WISV_EINVAL, "host buffer is NULL");
    if (len == 0) return WISV_OK;
    if (to_device) c->pending_valid = false;   // the cache a pending VERIFY_ONLY round ran against is being replaced
    HIP_TRY(c, hipSetDevice(g.device_id));
    const size_t row = (size_t)g.head_dim * c->esz;
    // K: device pitch ctx_pad rows per head, host pitch len rows per head
    char *dev_k = (char *)kv_ptr(c, layer, stream_id, 0);
    if (to_device)
        HIP_TRY(c, hipMemcpy2DAsync(dev_k, (size_t)c->ctx_pad * row, host_k, (size_t)len * row, (size_t)len * row,
                                    g.n_kv_heads, hipMemcpyHostToDevice, c->stream));
    else
        HIP_TRY(c, hipMemcpy2DAsync(host_k, (size_t)len * row, dev_k, (size_t)c->ctx_pad * row, (size_t)len * row,
                                    g.n_kv_heads, hipMemcpyDeviceToHost, c->stream));
    // V: through a row-major staging buffer on the device, re-blocked by a kernel
    const size_t v_bytes = (size_t)g.n_kv_heads * len * row;
    void *stage = nullptr;
    HIP_TRY(c, hipMalloc(&stage, v_bytes));
    hipError_t e = hipSuccess;
    if (to_device) {
        e = hipMemcpyAsync(stage, host_v, v_bytes, hipMemcpyHostToDevice, c->stream);
        if (e == hipSuccess) launch_v_reblock(c, stage, kv_ptr(c, layer, stream_id, 1), len, true);
    } else {
        launch_v_reblock(c, stage, kv_ptr(c, layer, stream_id, 1), len, false);
        e = hipMemcpyAsync(host_v, stage, v_bytes, hipMemcpyDeviceToHost, c->stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    (void)hipFree(stage);
    HIP_TRY(c, e);
    return WISV_OK;
}

extern "C" int wisv_kv_import(wisv_ctx *ctx, int32_t stream_id, int32_t layer, const void *host_k, const void *host_v,
                              int32_t len) {
    if (!ctx) return WISV_EINVAL;
    return kv_copy(ctx, stream_id, layer, (void *)host_k, (void *)host_v, len, true);
}

extern "C" int wisv_kv_export(wisv_ctx *ctx, int32_t stream_id, int32_t layer, void *host_k, void *host_v, int32_t len) {
    if (!ctx) return WISV_EINVAL;
    return kv_copy(ctx, stream_id, layer, host_k, host_v, len, false);
}

// ------------------------------------------------------------------------------------------ diagnostics

extern "C" int wisv_debug_copy(wisv_ctx *ctx, int32_t what, void *host_dst, size_t bytes) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (!host_dst) return fail(c, WISV_EINVAL, "host_dst is NULL");
    const void *src = nullptr;
    size_t have = 0;
    if (what == WISV_DBG_HIDDEN) {
        src = c->h_t;
        have = (size_t)c->last_rows * c->cfg.d_model * 4;
    } else if (what == WISV_DBG_LOGITS) {
        src = c->logits;
        have = (size_t)c->last_rows * c->cfg.vocab * 4;
    } else
        return fail(c, WISV_EINVAL, "unknown debug buffer %d", what);
    if (bytes > have) return fail(c, WISV_EINVAL, "asked for %zu bytes, the last round left %zu", bytes, have);
    HIP_TRY(c, hipSetDevice(c->cfg.device_id));
    HIP_TRY(c, hipMemcpyAsync(host_dst, src, bytes, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return WISV_OK;
}

extern "C" int wisv_last_round_ms(wisv_ctx *ctx, float *ms) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (!ms) return fail(c, WISV_EINVAL, "ms is NULL");
    HIP_TRY(c, hipEventSynchronize(c->ev_round[1]));
    HIP_TRY(c, hipEventElapsedTime(ms, c->ev_round[0], c->ev_round[1]));
    return WISV_OK;
}

__global__ void k_calibration_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

extern "C" int wisv_calibration_copy(wisv_ctx *ctx, void *dst, const void *src, size_t bytes) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (!dst || !src || bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16)
        return fail(c, WISV_EINVAL, "calibration copy needs 16-byte aligned pointers and a multiple of 16 bytes");
    HIP_TRY(c, hipSetDevice(c->cfg.device_id));
    hipLaunchKernelGGL(k_calibration_copy, dim3(8192), dim3(256), 0, c->stream, (const uint4 *)src, (uint4 *)dst, bytes / 16);
    HIP_TRY(c, hipGetLastError());
    return WISV_OK;
}

static const char *kClassNames[KC_COUNT] = {"prep_rows", "embed", "rmsnorm", "gemm_qkv", "gemm_gate_up", "rope_append", "attention", "attention_combine",
                                            "swiglu", "lm_head", "argmax", "head", "decide", "spec_sampling", "event_pair_overhead",
                                            "gemm_o", "gemm_down"};

extern "C" int wisv_profile_enable(wisv_ctx *ctx, int32_t on) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->profiling = on != 0;
    c->ev_used = 0;
    memset(c->prof_ms, 0, sizeof c->prof_ms);
    memset(c->prof_n, 0, sizeof c->prof_n);
    return WISV_OK;
}

extern "C" int wisv_profile_collect(wisv_ctx *ctx) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, c->ev_pool[i], c->ev_pool[i + 1]));
        c->prof_ms[c->ev_class[i / 2]] += ms;
        c->prof_n[c->ev_class[i / 2]] += 1;
    }
    c->ev_used = 0;
    return WISV_OK;
}

extern "C" int wisv_profile_read(wisv_ctx *ctx, int32_t kclass, const char **name, double *total_ms, int64_t *launches) {
    if (!ctx) return WISV_EINVAL;
    Ctx *c = ctx;
    if (kclass < 0 || kclass >= KC_COUNT) return fail(c, WISV_EINVAL, "kernel class %d outside [0, %d)", kclass, (int)KC_COUNT);
    if (name) *name = kClassNames[kclass];
    if (total_ms) *total_ms = c->prof_ms[kclass];
    if (launches) *launches = c->prof_n[kclass];
    return WISV_OK;
}
