// Decision head, mismatch localisation and the first-reject scan (Sec. V-A eqs. feature_concat /
// head_forward / mlp_form; eq. threshold; Alg. 1 last block).
//
//   1. concat   z = [h^D ; h^T ; c] is gathered for every position that is to be scored (FH: positions with an
//               uploaded h^D row; SH: mismatch positions with one), zero-padded to the padded width of W1
//   2. product  u = W1 z: the weight-streaming MFMA GEMM (bf16 path) or the generic GEMM
//   3. finish   s = w2 . act(u + b1) + b2, p_accept = 1 / (1 + e^s)
//   4. decide   per stream: mismatch mask, earliest rejected position, accepted length, correction token,
//               and the commit of the stream state
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

// dst[r][0..cols_pad) = src[r][0..cols) followed by zeros
template <typename WT>
__global__ void k_pad_cols(const WT *__restrict__ src, WT *__restrict__ dst, int cols, int cols_pad) {
    const int r = blockIdx.x;
    for (int i = threadIdx.x; i < cols_pad; i += blockDim.x)
        dst[(size_t)r * cols_pad + i] = i < cols ? src[(size_t)r * cols + i] : (WT)0;
}

void launch_pad_cols(Ctx *c, const void *src, void *dst, int rows, int cols, int cols_pad) {
    if (c->bf16)
        hipLaunchKernelGGL(k_pad_cols<bf16_t>, dim3(rows), dim3(256), 0, c->stream, (const bf16_t *)src, (bf16_t *)dst, cols, cols_pad);
    else
        hipLaunchKernelGGL(k_pad_cols<float>, dim3(rows), dim3(256), 0, c->stream, (const float *)src, (float *)dst, cols, cols_pad);
}

// one block per drafted position m = (stream b, position j)
template <typename WT>
__global__ void k_head_concat(int dD, int dT, int dC, int din_pad, const WT *__restrict__ hd,
                              const int32_t *__restrict__ hd_row, int n_hd, const float *__restrict__ h_t,
                              const float *__restrict__ csi, const int32_t *__restrict__ stream_ids,
                              const int32_t *__restrict__ proto, const int32_t *__restrict__ tokens,
                              const int32_t *__restrict__ amax, const int32_t *__restrict__ pred_next, int k,
                              int max_batch, int gate_all, ActBuf z, int32_t *scored) {
    const int m = blockIdx.x, b = m / k, j = m - b * k, tid = threadIdx.x;
    const int slot = min(max(stream_ids[b], 0), max_batch - 1);
    const int t_pred = j == 0 ? pred_next[slot] : amax[m - 1];   // the target's greedy token for position j
    const bool mismatch = tokens[m] != t_pred;
    int hr = hd_row ? hd_row[m] : m;
    if (hr >= n_hd) hr = -1;
    const bool want = gate_all || proto[b] == WISV_PROTO_FH || mismatch;
    const bool sc = want && hr >= 0;
    if (tid == 0) scored[m] = sc ? 1 : 0;
    const size_t z0 = (size_t)m * din_pad;
    if (!sc) {
        for (int i = tid; i < din_pad; i += blockDim.x) act_store(z, z0 + i, 0.f);
        return;
    }
    const WT *hdr = hd + (size_t)hr * dD;
    for (int i = tid; i < dD; i += blockDim.x) act_store(z, z0 + i, Elem<WT>::load(hdr + i));
    for (int i = tid; i < dT; i += blockDim.x) act_store(z, z0 + dD + i, h_t[(size_t)m * dT + i]);
    for (int i = tid; i < din_pad - dD - dT; i += blockDim.x)
        act_store(z, z0 + dD + dT + i, i < dC ? csi[(size_t)b * dC + i] : 0.f);
}

// one block per position: u = sum of the product's slices (fixed order), then the second layer
template <typename WT>
__global__ void k_head_finish(const float *__restrict__ u, int n_partial, size_t partial_stride, int dJ, int act,
                              const WT *__restrict__ b1, const WT *__restrict__ w2, const WT *__restrict__ b2,
                              const int32_t *__restrict__ scored, float *p_acc) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    if (!scored[m]) {
        if (tid == 0) p_acc[m] = 1.0f;
        return;
    }
    float part = 0.f;
    for (int r = tid; r < dJ; r += 256) {
        float v = Elem<WT>::load(b1 + r);
        for (int p = 0; p < n_partial; ++p) v += u[p * partial_stride + (size_t)m * dJ + r];
        const float a = act == WISV_ACT_RELU ? fmaxf(v, 0.f) : v / (1.0f + expf(-v));
        part = fmaf(Elem<WT>::load(w2 + r), a, part);
    }
    part = wave_sum(part);
    if ((tid & 63) == 0) red[tid >> 6] = part;
    __syncthreads();
    if (tid == 0) {
        const float s = ((red[0] + red[1]) + (red[2] + red[3])) + Elem<WT>::load(b2);
        p_acc[m] = 1.0f / (1.0f + expf(s));
    }
}

// one thread per stream
__global__ void k_decide(int batch, int k, int max_batch, const int32_t *__restrict__ stream_ids,
                         const int32_t *__restrict__ tokens, const int32_t *__restrict__ amax,
                         const float *__restrict__ p_acc, const int32_t *__restrict__ scored,
                         const float *__restrict__ tau, int gate_all, int commit, int32_t *kv_len, int32_t *pred_next,
                         int32_t *alen, int32_t *ytok, int32_t *targ, uint32_t *mask_out, uint32_t *status_out) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int slot = min(max(stream_ids[b], 0), max_batch - 1);
    const int pn = pred_next[slot];
    uint32_t mask = 0, status = 0;
    int first = k;
    for (int j = k - 1; j >= 0; --j) {
        const int m = b * k + j;
        const int t = j == 0 ? pn : amax[m - 1];
        const bool mismatch = tokens[m] != t;
        if (mismatch) mask |= 1u << j;
        if (gate_all || mismatch) {
            bool reject;
            if (!scored[m]) { reject = true; status |= WISV_STATUS_MISSING_HIDDEN; }
            else reject = !(p_acc[m] >= tau[b]);
            if (reject) first = j;
        }
    }
    const int y = first == 0 ? pn : amax[b * k + first - 1];
    alen[b] = first;
    ytok[b] = y;
    if (targ) {
        targ[b * (k + 1)] = pn;
        for (int j = 0; j < k; ++j) targ[b * (k + 1) + j + 1] = amax[b * k + j];
    }
    if (mask_out) mask_out[b] = mask;
    if (status_out) status_out[b] = status;
    if (commit) {
        kv_len[slot] += first;
        pred_next[slot] = y;
    }
}

void launch_head_decide(Ctx *c, const Fwd &f, const wisv_round_in &in, const wisv_round_out &out) {
    const wisv_config &g = c->cfg;
    const int gate_all = (in.flags & WISV_FLAG_GATE_ALL) ? 1 : 0, commit = (in.flags & WISV_FLAG_NO_COMMIT) ? 0 : 1;
    const int dJ = g.d_head_hidden, din_pad = c->din_pad;
    const size_t ustride = (size_t)c->rows_max * dJ;
    int n_partial = 1;
    {
        ProfScope ps(c, KC_HEAD);
        if (c->bf16)
            hipLaunchKernelGGL(k_head_concat<bf16_t>, dim3(f.rows), dim3(256), 0, c->stream, g.d_draft, g.d_model, g.d_csi,
                               din_pad, (const bf16_t *)in.hd, in.hd_row, in.n_hd, c->h_t, in.csi, in.stream_ids, in.proto,
                               in.draft_tokens, c->amax, c->d_pred_next, f.k, g.max_batch, gate_all, c->z, c->scored);
        else
            hipLaunchKernelGGL(k_head_concat<float>, dim3(f.rows), dim3(256), 0, c->stream, g.d_draft, g.d_model, g.d_csi,
                               din_pad, (const float *)in.hd, in.hd_row, in.n_hd, c->h_t, in.csi, in.stream_ids, in.proto,
                               in.draft_tokens, c->amax, c->d_pred_next, f.k, g.max_batch, gate_all, c->z, c->scored);
    }
    // u = W1 z
    bool streamed = c->head_w1_t != nullptr;
    if (streamed) {
        n_partial = launch_gemm_ws_partial(c, c->head_w1_t, c->z, c->hu, ustride, MAX_SPLITS, f.rows, dJ, din_pad, KC_HEAD);
        streamed = n_partial > 0;
    }
    if (!streamed) {
        n_partial = 1;
        launch_gemm_ref(c, c->z.f, c->head_w1_pad, c->hu, f.rows, dJ, din_pad, KC_HEAD);
    }
    {
        ProfScope ps(c, KC_HEAD);
        if (c->bf16)
            hipLaunchKernelGGL(k_head_finish<bf16_t>, dim3(f.rows), dim3(256), 0, c->stream, c->hu, n_partial, ustride, dJ,
                               g.head_act, (const bf16_t *)c->head_b1, (const bf16_t *)c->head_w2,
                               (const bf16_t *)c->head_b2, c->scored, out.p_accept);
        else
            hipLaunchKernelGGL(k_head_finish<float>, dim3(f.rows), dim3(256), 0, c->stream, c->hu, n_partial, ustride, dJ,
                               g.head_act, (const float *)c->head_b1, (const float *)c->head_w2, (const float *)c->head_b2,
                               c->scored, out.p_accept);
    }
    {
        ProfScope ps(c, KC_DECIDE);
        hipLaunchKernelGGL(k_decide, dim3((f.batch + 63) / 64), dim3(64), 0, c->stream, f.batch, f.k, g.max_batch,
                           in.stream_ids, in.draft_tokens, c->amax, out.p_accept, c->scored, in.tau, gate_all, commit,
                           c->d_kv_len, c->d_pred_next, out.accepted_len, out.correction_token, out.target_argmax,
                           out.mismatch_mask, out.status);
    }
}

}  // namespace wisv
