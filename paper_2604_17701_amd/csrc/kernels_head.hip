// Decision head, mismatch localisation and the first-reject scan (Sec. V-A eqs. feature_concat /
// head_forward / mlp_form; eq. threshold; Alg. 1 last block).
//
//   1. head     one kernel: gather of [h^D ; h^T ; c] for the scored positions (FH: positions with an uploaded h^D
//               row; SH: mismatch positions with one), first layer, activation, second-layer partial sums
//   2. decide   per stream: accept probabilities from the partial sums, mismatch mask, earliest rejected position,
//               accepted length, correction token, and the commit of the stream state
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

// ------------------------------------------------------------------------------------------ the fused head
// u = W1 [h^D ; h^T ; c] + b1, t = w2 . act(u) for every scored position, in one kernel and without ever writing the
// concatenated vector: the three column slices of W1 meet h^D (read through hd_row from what the device uploaded),
// h^T (the target's final hidden state) and c (the stream's CSI vector) where they lie.
//
// bf16 weights: W1 is held re-tiled for the 16x16x32 MFMA (kernels_gemm.hip), one workgroup = (row-block of 16
// hidden units, tile of 16 positions), its WK waves split the columns among them and each wave builds its own B
// operands (16 positions x 32 columns, two bf16 terms) straight from global memory - no two waves of a workgroup
// need the same columns, so nothing is staged in LDS.  The waves' accumulators are added through LDS in wave order;
// wave 0 adds b1, applies the activation, multiplies by w2 and adds up its 16 hidden units: one partial sum per
// (row-block, position), which k_decide adds up in row-block order.  Positions that are not scored (not uploaded,
// or matching drafts of a selective-hidden stream) are never loaded; a tile without a scored position exits.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct HeadArgs {
    const u32x4 *w1t;          // re-tiled W1 [nrb][nkt][64] (bf16 path)
    const void *w1;            // W1 [dJ][din] row-major (generic path)
    int nkt, nrb, dJ, dD, dT, dC, din;
    const void *hd;            // uploaded drafter hidden states [n_hd][dD], weight dtype
    const int32_t *hd_row;     // [rows] or null (identity)
    int n_hd;
    const float *h_t, *csi;    // [rows][dT], [batch][dC]
    const int32_t *stream_ids, *proto, *tokens, *amax, *pred_next;
    int k, rows, max_batch, gate_all, act;
    const void *b1, *w2;
    float *sp;                 // [parts][rows] partial second-layer sums
    int32_t *scored;           // [rows]
};

// is position m scored, and from which row of hd: Alg. 1's localisation (mismatch against the target's greedy token)
// and the upload protocol (Sec. III-B: full-hidden streams are scored everywhere, selective-hidden ones at mismatches)
__device__ __forceinline__ bool head_scored(const HeadArgs &a, int m, int *hr_out) {
    const int b = m / a.k, j = m - b * a.k;
    const int slot = min(max(a.stream_ids[b], 0), a.max_batch - 1);
    const int t_pred = j == 0 ? a.pred_next[slot] : a.amax[m - 1];
    const bool mismatch = a.tokens[m] != t_pred;
    int hr = a.hd_row ? a.hd_row[m] : m;
    if (hr >= a.n_hd) hr = -1;
    *hr_out = hr;
    return (a.gate_all || a.proto[b] == WISV_PROTO_FH || mismatch) && hr >= 0;
}

// element c of z = [h^D ; h^T ; c ; 0...] of position m
template <typename WT> __device__ __forceinline__ float head_z(const HeadArgs &a, int m, int hr, int c) {
    if (c < a.dD) return Elem<WT>::load((const WT *)a.hd + (size_t)hr * a.dD + c);
    if (c < a.dD + a.dT) return a.h_t[(size_t)m * a.dT + c - a.dD];
    if (c < a.din) return a.csi[(size_t)(m / a.k) * a.dC + c - a.dD - a.dT];
    return 0.f;
}

__device__ __forceinline__ float head_act(int act, float v) { return act == WISV_ACT_RELU ? fmaxf(v, 0.f) : v / (1.0f + expf(-v)); }

// WK waves split the columns; a wave multiplies RB row-blocks of hidden units with NT tiles of 16 positions (every A
// operand meets NT B operands and every B operand RB A operands) and requests TB k-tiles at a time
template <int WK, int RB, int NT, int TB>
__global__ __launch_bounds__(64 * WK) void k_head_fused(HeadArgs a) {
    __shared__ floatx4 red[WK][RB * NT][64];
    __shared__ int any_scored;
    const int rb0 = blockIdx.x * RB, tile0 = blockIdx.y * NT;
    const int tid = threadIdx.x, lane = tid & 63, wk = tid >> 6, bj = lane & 15, bg = lane >> 4;
    int m[NT], hr[NT];
    bool sc[NT];
    const bf16_t *hd_row[NT];
    const float *ht_row[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m[t] = (tile0 + t) * 16 + bj;
        hr[t] = -1;
        sc[t] = m[t] < a.rows && head_scored(a, m[t], &hr[t]);
        hd_row[t] = (const bf16_t *)a.hd + (size_t)max(hr[t], 0) * a.dD;
        ht_row[t] = a.h_t + (size_t)min(m[t], a.rows - 1) * a.dT;
    }
    if (tid == 0) any_scored = 0;
    __syncthreads();
    if (wk == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (blockIdx.x == 0 && bg == 0 && m[t] < a.rows) a.scored[m[t]] = sc[t] ? 1 : 0;
            if (sc[t]) any_scored = 1;      // every writer stores the same value
        }
    }
    __syncthreads();
    if (!any_scored) return;         // the whole workgroup leaves together

    const int sub = (a.nkt + WK - 1) / WK, k_begin = wk * sub, k_end = min(a.nkt, k_begin + sub);
    floatx4 acc[RB][NT];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    // one B operand (two bf16 terms) of position tile t against the RB A operands
    auto mma = [&](const u32x4 (&av)[RB], int t, u32x4 bh, u32x4 bl, bool two) {
        if (!sc[t]) { bh = u32x4{0u, 0u, 0u, 0u}; bl = bh; }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            u32x4 a_ = av[r];
            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&a_), *reinterpret_cast<bf16x8 *>(&bh), acc[r][t], 0, 0, 0);
            if (two) acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&a_), *reinterpret_cast<bf16x8 *>(&bl), acc[r][t], 0, 0, 0);
        }
    };
    auto split8 = [&](const float (&z)[8], u32x4 &bh, u32x4 &bl) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            bf16_t h0, l0, h1, l1;
            split2(z[2 * e], h0, l0);
            split2(z[2 * e + 1], h1, l1);
            bh[e] = h0 | ((uint32_t)h1 << 16);
            bl[e] = l0 | ((uint32_t)l1 << 16);
        }
    };
    // A wave's k-tiles fall into three runs (uniform per wave): tiles inside h^D, tiles inside h^T, and the rest (a tile
    // that straddles two sources, the CSI features, the padding).  Each run is a loop without branches around its
    // loads: TB tiles are requested at once (tiles past the run re-read its last one and are not used).  The launcher
    // sends only widths that are multiples of 8 here, so a lane's eight columns never straddle two sources inside a run.
    const int d_end = a.dD / 32, t_begin = (a.dD + 31) / 32, t_end = (a.dD + a.dT) / 32;   // [0, d_end) in h^D; [t_begin, t_end) in h^T
    const u32x4 *wt[RB];   // row-blocks past the last re-read it; their results are not written
#pragma unroll
    for (int r = 0; r < RB; ++r) wt[r] = a.w1t + (size_t)min(rb0 + r, a.nrb - 1) * a.nkt * 64 + lane;
    {   // ---- h^D: bf16 values are their own high term, there is no low term
        const int r0 = k_begin, r1 = min(k_end, d_end);
        for (int k0 = r0; k0 < r1; k0 += TB) {
            u32x4 av[TB][RB], hv[TB][NT];
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                const int kt = min(k0 + u, r1 - 1);
#pragma unroll
                for (int r = 0; r < RB; ++r) av[u][r] = wt[r][(size_t)kt * 64];
#pragma unroll
                for (int t = 0; t < NT; ++t) hv[u][t] = *reinterpret_cast<const u32x4 *>(hd_row[t] + kt * 32 + bg * 8);
            }
#pragma unroll
            for (int u = 0; u < TB; ++u)
                if (k0 + u < r1) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) mma(av[u], t, hv[u][t], u32x4{0u, 0u, 0u, 0u}, false);
                }
        }
    }
    {   // ---- h^T: float, split into two bf16 terms
        const int r0 = max(k_begin, t_begin), r1 = min(k_end, t_end);
        for (int k0 = r0; k0 < r1; k0 += TB) {
            u32x4 av[TB][RB];
            floatx4 f0[TB][NT], f1[TB][NT];
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                const int kt = min(k0 + u, r1 - 1);
#pragma unroll
                for (int r = 0; r < RB; ++r) av[u][r] = wt[r][(size_t)kt * 64];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    f0[u][t] = *reinterpret_cast<const floatx4 *>(ht_row[t] + kt * 32 + bg * 8 - a.dD);
                    f1[u][t] = *reinterpret_cast<const floatx4 *>(ht_row[t] + kt * 32 + bg * 8 - a.dD + 4);
                }
            }
#pragma unroll
            for (int u = 0; u < TB; ++u)
                if (k0 + u < r1) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const float z[8] = {f0[u][t][0], f0[u][t][1], f0[u][t][2], f0[u][t][3], f1[u][t][0], f1[u][t][1], f1[u][t][2], f1[u][t][3]};
                        u32x4 bh, bl;
                        split8(z, bh, bl);
                        mma(av[u], t, bh, bl, true);
                    }
                }
        }
    }
    for (int kt = k_begin; kt < k_end; ++kt) {   // ---- the rest, element by element (a handful of tiles)
        if (kt < d_end || (kt >= t_begin && kt < t_end)) continue;
        u32x4 av[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) av[r] = wt[r][(size_t)kt * 64];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float z[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = sc[t] ? head_z<bf16_t>(a, m[t], hr[t], kt * 32 + bg * 8 + e) : 0.f;
            u32x4 bh, bl;
            split8(z, bh, bl);
            mma(av, t, bh, bl, true);
        }
    }
    // ---- the waves' column slices, added in wave order
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[wk][r * NT + t][lane] = acc[r][t];
    __syncthreads();
    if (wk != 0) return;
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            floatx4 u = acc[r][t];
            for (int w = 1; w < WK; ++w) u += red[w][r * NT + t][lane];
            // lane (bj, bg) holds u[hidden 16 (rb0 + r) + 4 bg + e][position bj of tile t]
            float s2 = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = (rb0 + r) * 16 + bg * 4 + e;
                if (j < a.dJ)
                    s2 = fmaf(bf16_to_f32(((const bf16_t *)a.w2)[j]), head_act(a.act, u[e] + bf16_to_f32(((const bf16_t *)a.b1)[j])), s2);
            }
            s2 += __shfl_xor(s2, 16, 64);
            s2 += __shfl_xor(s2, 32, 64);
            if (bg == 0 && sc[t] && rb0 + r < a.nrb) a.sp[(size_t)(rb0 + r) * a.rows + m[t]] = s2;
        }
}

// Generic form (float weights, or shapes the re-tiled form does not serve): one workgroup per position, its waves
// take the hidden units in turn; one partial sum per position.
template <typename WT>
__global__ __launch_bounds__(256) void k_head_ref(HeadArgs a) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int hr;
    const bool sc = head_scored(a, m, &hr);
    if (tid == 0) a.scored[m] = sc ? 1 : 0;
    if (!sc) return;
    float t = 0.f;
    for (int j = wave; j < a.dJ; j += 4) {
        const WT *wr = (const WT *)a.w1 + (size_t)j * a.din;
        float dot = 0.f;
        for (int c = lane; c < a.din; c += 64) dot = fmaf(Elem<WT>::load(wr + c), head_z<WT>(a, m, hr, c), dot);
        dot = wave_sum(dot);
        t = fmaf(Elem<WT>::load((const WT *)a.w2 + j), head_act(a.act, dot + Elem<WT>::load((const WT *)a.b1 + j)), t);
    }
    if (lane == 0) red[wave] = t;
    __syncthreads();
    if (tid == 0) a.sp[m] = (red[0] + red[1]) + (red[2] + red[3]);
}

// one wave per stream: accept probabilities from the head's partial sums (lane q adds parts q, q + 64, ..; then a
// fixed shuffle tree), threshold, earliest rejected position, correction token, commit
__global__ __launch_bounds__(64) void k_decide(int batch, int k, int max_batch, const int32_t *__restrict__ stream_ids,
                         const int32_t *__restrict__ tokens, const int32_t *__restrict__ amax,
                         const float *__restrict__ sp, int parts, int rows, const void *__restrict__ b2, int b2_bf16,
                         const int32_t *__restrict__ scored, const float *__restrict__ tau, int gate_all, int commit,
                         int32_t *kv_len, int32_t *pred_next, float *p_acc, int32_t *alen, int32_t *ytok, int32_t *targ,
                         uint32_t *mask_out, uint32_t *status_out) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int slot = min(max(stream_ids[b], 0), max_batch - 1);
    const int pn = pred_next[slot];
    const float bias = b2_bf16 ? bf16_to_f32(*(const bf16_t *)b2) : *(const float *)b2;
    // second-layer sums of the block's positions: every load first (positions past k re-read the last one)
    float part[WISV_MAX_K];
#pragma unroll
    for (int j = 0; j < WISV_MAX_K; ++j) {
        const int m = b * k + min(j, k - 1);
        float v = 0.f;
        for (int q = lane; q < parts; q += 64) v += sp[(size_t)q * rows + m];
        part[j] = v;
    }
    float s_j[WISV_MAX_K];
#pragma unroll
    for (int j = 0; j < WISV_MAX_K; ++j) s_j[j] = wave_sum(part[j]);
    if (lane != 0) return;
    uint32_t mask = 0, status = 0;
    int first = k;
#pragma unroll
    for (int j = WISV_MAX_K - 1; j >= 0; --j) {
        if (j >= k) continue;
        const int m = b * k + j;
        const int t = j == 0 ? pn : amax[m - 1];
        const bool mismatch = tokens[m] != t;
        if (mismatch) mask |= 1u << j;
        const bool sc = scored[m] != 0;
        const float p = sc ? 1.0f / (1.0f + expf(s_j[j] + bias)) : 1.0f;   // p_accept = 1 - sigmoid(s); 1 where not evaluated
        p_acc[m] = p;
        if (gate_all || mismatch) {
            bool reject;
            if (!sc) { reject = true; status |= WISV_STATUS_MISSING_HIDDEN; }
            else reject = !(p >= tau[b]);
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
    HeadArgs a{};
    a.w1t = (const u32x4 *)c->head_w1_t; a.w1 = c->head_w1;
    a.dJ = g.d_head_hidden; a.dD = g.d_draft; a.dT = g.d_model; a.dC = g.d_csi; a.din = g.d_draft + g.d_model + g.d_csi;
    a.nkt = c->din_pad / 32; a.nrb = (g.d_head_hidden + 15) / 16;
    // no uploaded rows: the kernels still form addresses inside hd (and never use what they read there)
    a.hd = in.n_hd > 0 && in.hd ? in.hd : c->d_hd;
    a.hd_row = in.hd_row; a.n_hd = in.n_hd;
    a.h_t = c->h_t; a.csi = in.csi;
    a.stream_ids = in.stream_ids; a.proto = in.proto; a.tokens = in.draft_tokens; a.amax = c->amax; a.pred_next = c->d_pred_next;
    a.k = f.k; a.rows = f.rows; a.max_batch = g.max_batch; a.gate_all = gate_all; a.act = g.head_act;
    a.b1 = c->head_b1; a.w2 = c->head_w2;
    a.sp = c->hu; a.scored = c->scored;
    int parts;
    {
        ProfScope ps(c, KC_HEAD);
        if (c->head_w1_t && g.d_draft % 8 == 0 && g.d_draft >= 8) {
            // sixteen waves split the columns when few positions leave the chip empty otherwise, four when there are many
            parts = a.nrb;
            if (f.rows <= 64)
                hipLaunchKernelGGL((k_head_fused<16, 1, 1, 8>), dim3(a.nrb, (f.rows + 15) / 16), dim3(1024), 0, c->stream, a);
            else   // many positions: 2 x 2 operand tiles per wave halve what every workgroup reads
                hipLaunchKernelGGL((k_head_fused<8, 2, 2, 4>), dim3((a.nrb + 1) / 2, (f.rows + 31) / 32), dim3(512), 0, c->stream, a);
        } else {
            parts = 1;
            if (c->bf16) hipLaunchKernelGGL(k_head_ref<bf16_t>, dim3(f.rows), dim3(256), 0, c->stream, a);
            else hipLaunchKernelGGL(k_head_ref<float>, dim3(f.rows), dim3(256), 0, c->stream, a);
        }
    }
    {
        ProfScope ps(c, KC_DECIDE);
        hipLaunchKernelGGL(k_decide, dim3(f.batch), dim3(64), 0, c->stream, f.batch, f.k, g.max_batch,
                           in.stream_ids, in.draft_tokens, c->amax, c->hu, parts, f.rows, c->head_b2, c->bf16 ? 1 : 0,
                           c->scored, in.tau, gate_all, commit, c->d_kv_len, c->d_pred_next, out.p_accept,
                           out.accepted_len, out.correction_token, out.target_argmax, out.mismatch_mask, out.status);
    }
}

}  // namespace wisv
