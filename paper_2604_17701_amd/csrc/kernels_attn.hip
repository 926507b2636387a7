// Grouped-query attention of the drafted block over the KV cache (bf16 cache, head_dim 128):
// the K query rows of a stream x the query heads that share one KV head form one tile of up to 64 rows, so
// every cached key/value byte is read once per (stream, KV head) and meets all of them.
//
// One workgroup = (k-split, KV head, stream); its waves take steps of 32 keys round-robin and never meet before
// the end: nothing is staged in LDS.  K rows go straight from the cache into the A operand of S^T = K Q^T
// (16x16x32 MFMA, two tiles of 16 keys per step, queries as two bf16 terms in the B operand).  The keys of a
// step are dealt to the two tiles so that lane group g ends up holding the scores of the eight consecutive keys
// 8 g .. 8 g + 7 of every query: after the float online softmax these eight probabilities are, as they stand,
// the B operand of O^T += V^T P^T on the 16x16x32 MFMA (two bf16 terms again, so P.V is exact to 2^-17), whose A
// operand - 16 features x 32 keys of V^T - is one 16-byte load per lane from the cache's V plane, which keeps
// 32 positions of a feature contiguous for exactly this reason.  Waves are merged through LDS at the end with
// the usual (max, sum, unnormalised output) rule in wave order; k-splits, when there are several, by a small
// kernel, otherwise the workgroup writes the attention output itself.
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int HD = 128, STEP = 32;

struct AttnArgs {
    const float *q;           // rotated queries [rows][H * 128]
    const bf16_t *kv_layer;   // this layer's cache: [slot][K|V][G] planes of ctx_pad * 128
    size_t slot_stride;       // elements per slot
    int H, G, rep, K, max_ctx, ctx_pad, n_splits, rows;
    const int32_t *row_slot, *row_pos;
    float *po, *pm, *pl;      // partials [split][rows][H][128], [split][rows][H]  (n_splits > 1); pm in units of ln 2
    ActBuf o;                 // attention output [rows][H][128]                    (n_splits == 1)
    // FUSE: the kernel sums the k-split slices of the QKV product itself, rotates q and k, appends k and v
    const float *qkv;         // [n_partial][partial_stride] slices of [rows][H*128 + 2 G*128]
    int n_partial;
    size_t partial_stride;
    const float *cs, *sn;     // rotary tables [max_ctx][64]
    // FUSE, n_ss > 0: the slices are products of x * gain; row m is scaled by 1 / sqrt(sum_p ss[p][m] / d_model + eps)
    const float *ss;          // [n_ss][rows] (always a readable address)
    int n_ss, d_model;
    float eps;
    bf16_t *kv_write;         // == kv_layer
};

// NQ: 16-row query tiles; NW: waves per workgroup; FUSE: RoPE and the cache append happen here: every workgroup
// rotates the queries it needs from the slices of the QKV product, and the workgroup of a (stream, KV head) whose
// k-split ends the sequence writes the new k, v rows before any of its waves reads them (no other split reads them)
template <int NQ, int NW, bool FUSE>
__global__ __launch_bounds__(64 * NW) void k_attn_mfma(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, bj = lane & 15, bg = lane >> 4;
    const int m0 = b * a.K;
    const int L = a.row_pos[m0], slot = a.row_slot[m0];
    const int n_keys = min(L + a.K, a.max_ctx), R = a.rep * a.K;
    const bf16_t *kc = a.kv_layer + (size_t)slot * a.slot_stride + (size_t)g * a.ctx_pad * HD;
    const bf16_t *vc = kc + (size_t)a.G * a.ctx_pad * HD;
    const int n_steps = (n_keys + STEP - 1) / STEP, sps = (n_steps + a.n_splits - 1) / a.n_splits;
    int s_begin = split * sps, s_end = min(n_steps, s_begin + sps);
    // FUSE with several k-splits: the last split appends the block's k, v rows, so it owns every step from the one
    // that holds position L on (at most two steps more than its share); the others stop there
    const bool appends = FUSE && split == a.n_splits - 1;
    if (FUSE && a.n_splits > 1) {
        const int tail = L / STEP;
        if (appends) {
            s_begin = min(s_begin, tail);
            s_end = n_steps;
        } else {
            s_end = min(s_end, tail);
            s_begin = min(s_begin, s_end);
        }
    }

    // ---- the first step's loads go out before anything else.  Lane (bj, bg): tile A row bj is key
    //      8 (bj / 4) + bj % 4 of the step, tile B row bj the key four further; V^T row bj of feature tile dt.
    u32x4 ka[4], kb[4], va[8];
    const int krow = 8 * (bj >> 2) + (bj & 3);
#define WISV_ATTN_LOAD_K(s_)                                                                              \
    {                                                                                                     \
        const bf16_t *pa_ = kc + (size_t)min((s_) * STEP + krow, n_keys - 1) * HD + 8 * bg;               \
        const bf16_t *pb_ = kc + (size_t)min((s_) * STEP + krow + 4, n_keys - 1) * HD + 8 * bg;           \
        _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                                   \
            ka[t] = *reinterpret_cast<const u32x4 *>(pa_ + 32 * t);                                       \
            kb[t] = *reinterpret_cast<const u32x4 *>(pb_ + 32 * t);                                       \
        }                                                                                                 \
    }
#define WISV_ATTN_LOAD_V(s_)                                                                              \
    {                                                                                                     \
        const bf16_t *pv_ = vc + ((size_t)(s_) * HD + bj) * STEP + 8 * bg;                                \
        _Pragma("unroll") for (int dt = 0; dt < 8; ++dt) va[dt] = *reinterpret_cast<const u32x4 *>(pv_ + (size_t)dt * 16 * STEP); \
    }
    constexpr bool Q_IN_LDS = NQ > 1 || FUSE;
    constexpr int QREG = NQ > 1 ? 1 : NQ;
    u32x4 qhi[QREG][4], qlo[QREG][4];
    u32x4 *qs = reinterpret_cast<u32x4 *>(lds);   // [NQ][4][2][64] query operands; the merge at the end re-uses the space
    int s = s_begin + wave;
    if (FUSE) {
        // this wave's first step is requested now; if it holds appended rows it is requested again below
        const int s0 = min(s, n_steps - 1);
        WISV_ATTN_LOAD_K(s0)
        WISV_ATTN_LOAD_V(s0)
    }
    if (FUSE) {
        // ---- RoPE + append.  Work item = (row, pair of features i, i + 64): q rows rho < R of this KV head's query
        //      heads go, rotated and split into two bf16 terms, straight into the operand layout in LDS; the K new
        //      rows of k (rotated) and v go to the cache.  Slices are added in slice order.
        const int d_q = a.H * HD, d_kv = a.G * HD, d_all = d_q + 2 * d_kv;
        bf16_t *kw = a.kv_write + (size_t)slot * a.slot_stride + (size_t)g * a.ctx_pad * HD;
        bf16_t *vw = kw + (size_t)a.G * a.ctx_pad * HD;
        bf16_t *q16 = reinterpret_cast<bf16_t *>(qs);
        for (int it = tid; it < (16 * NQ + (appends ? 2 * a.K : 0)) * 16; it += 64 * NW) {
            const int row = it >> 4, i = (it & 15) * 4;   // features i .. i + 3 and their partners i + 64 .. i + 67
            int j, col;                      // token of the block, first column of the head in a qkv row
            if (row < 16 * NQ) {
                const int rho = min(row, R - 1);
                j = rho / a.rep;
                col = (g * a.rep + rho % a.rep) * HD;
            } else if (row < 16 * NQ + a.K) {
                j = row - 16 * NQ;
                col = d_q + g * HD;
            } else {
                j = row - 16 * NQ - a.K;
                col = d_q + d_kv + g * HD;
            }
            const float *src = a.qkv + (size_t)(m0 + j) * d_all + col + i;
            // every slice is requested before the first is used (slices past the last re-read it and count as 0)
            floatx4 xs[MAX_SPLITS], ys[MAX_SPLITS];
#pragma unroll
            for (int p = 0; p < MAX_SPLITS; ++p) {
                const size_t off = (size_t)min(p, a.n_partial - 1) * a.partial_stride;
                xs[p] = *reinterpret_cast<const floatx4 *>(src + off);
                ys[p] = *reinterpret_cast<const floatx4 *>(src + off + 64);
            }
            float ssp[MAX_SPLITS];
#pragma unroll
            for (int p = 0; p < MAX_SPLITS; ++p) ssp[p] = a.ss[(size_t)min(p, max(a.n_ss, 1) - 1) * a.rows + m0 + j];
            const int pos = min(L + j, a.max_ctx - 1);
            const floatx4 co = *reinterpret_cast<const floatx4 *>(a.cs + (size_t)pos * 64 + i);
            const floatx4 si = *reinterpret_cast<const floatx4 *>(a.sn + (size_t)pos * 64 + i);
            floatx4 x = xs[0], y = ys[0];
#pragma unroll
            for (int p = 1; p < MAX_SPLITS; ++p) {
                const bool on = p < a.n_partial;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    x[c] += on ? xs[p][c] : 0.f;
                    y[c] += on ? ys[p][c] : 0.f;
                }
            }
            if (a.n_ss > 0) {   // the deferred 1 / rms of the folded RMSNorm (sums of squares in slice order)
                float t = 0.f;
#pragma unroll
                for (int p = 0; p < MAX_SPLITS; ++p) t += p < a.n_ss ? ssp[p] : 0.f;
                const float inv = 1.0f / sqrtf(t / (float)a.d_model + a.eps);
#pragma unroll
                for (int c = 0; c < 4; ++c) { x[c] *= inv; y[c] *= inv; }
            }
            float r0[4], r1[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                r0[c] = x[c] * co[c] - y[c] * si[c];
                r1[c] = y[c] * co[c] + x[c] * si[c];
            }
            if (row < 16 * NQ) {
                // element (rho, dim) of operand (nq, t = dim / 32, plane): lane 16 ((dim % 32) / 8) + rho % 16, slot dim % 8
                const int nq = row >> 4, bjq = row & 15;
                const int e = i & 7, ln = 16 * ((i & 31) >> 3) + bjq, t0 = i >> 5;
                bf16_t h0[4], l0[4], h1[4], l1[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    split2(row < R ? r0[c] : 0.f, h0[c], l0[c]);
                    split2(row < R ? r1[c] : 0.f, h1[c], l1[c]);
                }
                auto pack = [](const bf16_t (&v)[4]) { return make_uint2(v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16)); };
                *reinterpret_cast<uint2 *>(q16 + ((((nq * 4 + t0) * 2 + 0) * 64 + ln) << 3) + e) = pack(h0);
                *reinterpret_cast<uint2 *>(q16 + ((((nq * 4 + t0) * 2 + 1) * 64 + ln) << 3) + e) = pack(l0);
                *reinterpret_cast<uint2 *>(q16 + ((((nq * 4 + t0 + 2) * 2 + 0) * 64 + ln) << 3) + e) = pack(h1);
                *reinterpret_cast<uint2 *>(q16 + ((((nq * 4 + t0 + 2) * 2 + 1) * 64 + ln) << 3) + e) = pack(l1);
            } else if (row < 16 * NQ + a.K) {
                bf16_t k0[4], k1[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) { k0[c] = f32_to_bf16(r0[c]); k1[c] = f32_to_bf16(r1[c]); }
                *reinterpret_cast<uint2 *>(kw + (size_t)pos * HD + i) = make_uint2(k0[0] | ((unsigned)k0[1] << 16), k0[2] | ((unsigned)k0[3] << 16));
                *reinterpret_cast<uint2 *>(kw + (size_t)pos * HD + i + 64) = make_uint2(k1[0] | ((unsigned)k1[1] << 16), k1[2] | ((unsigned)k1[3] << 16));
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    vw[v_plane_index(pos, i + c, HD)] = f32_to_bf16(x[c]);
                    vw[v_plane_index(pos, i + c + 64, HD)] = f32_to_bf16(y[c]);
                }
            }
        }
        __syncthreads();   // the appended rows and the query operands are visible to the whole workgroup
    }
    // (no load below is conditional - a branch around a load makes the compiler wait for it on the spot: a wave
    // without a further step re-reads a step that exists and ignores it)
    {
        const int s0 = min(s, n_steps - 1);
        if (!FUSE || (s0 + 1) * STEP > L) {
            WISV_ATTN_LOAD_K(s0)
            WISV_ATTN_LOAD_V(s0)
        }
    }

    // ---- queries as MFMA B operands (two bf16 terms): lane (bj, bg) holds Q[rho = 16 nq + bj][32 t + 8 bg ..].
    //      One query tile lives in registers; more would crowd out the accumulators, so they are parked in LDS
    //      (built once, shared by the waves) and re-read at each use.
    if (!FUSE) {
        if (NQ > 1) {
            // the NQ x 4 operand pairs are dealt to the waves; rows past R load row 0 (no branch around the loads)
            // and become zero
            for (int item = wave; item < NQ * 4; item += NW) {
                const int nq = item >> 2, t = item & 3, rho = nq * 16 + bj;
                const bool valid = rho < R;
                const float *qp = a.q + ((size_t)(m0 + (valid ? rho / a.rep : 0)) * a.H + (size_t)g * a.rep + (valid ? rho % a.rep : 0)) * HD;
                const float4 x0 = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg);
                const float4 x1 = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg + 4);
                const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                uint32_t h[4], l[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bf16_t h0, l0, h1, l1;
                    split2(valid ? xs[2 * e] : 0.f, h0, l0);
                    split2(valid ? xs[2 * e + 1] : 0.f, h1, l1);
                    h[e] = h0 | ((uint32_t)h1 << 16);
                    l[e] = l0 | ((uint32_t)l1 << 16);
                }
                qs[(item * 2 + 0) * 64 + lane] = u32x4{h[0], h[1], h[2], h[3]};
                qs[(item * 2 + 1) * 64 + lane] = u32x4{l[0], l[1], l[2], l[3]};
            }
            __syncthreads();
        } else {
            const bool valid = bj < R;
            const float *qp = a.q + ((size_t)(m0 + (valid ? bj / a.rep : 0)) * a.H + (size_t)g * a.rep + (valid ? bj % a.rep : 0)) * HD;
            // all eight loads first, then the arithmetic
            float4 xq[4][2];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                xq[t][0] = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg);
                xq[t][1] = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg + 4);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t h[4], l[4];
                const float4 x0 = xq[t][0], x1 = xq[t][1];
                const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bf16_t h0, l0, h1, l1;
                    split2(valid ? xs[2 * e] : 0.f, h0, l0);
                    split2(valid ? xs[2 * e + 1] : 0.f, h1, l1);
                    h[e] = h0 | ((uint32_t)h1 << 16);
                    l[e] = l0 | ((uint32_t)l1 << 16);
                }
                qhi[0][t] = u32x4{h[0], h[1], h[2], h[3]};
                qlo[0][t] = u32x4{l[0], l[1], l[2], l[3]};
            }
        }
    } else if (NQ == 1) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            qhi[0][t] = qs[(t * 2 + 0) * 64 + lane];
            qlo[0][t] = qs[(t * 2 + 1) * 64 + lane];
        }
    }

    float m_run[NQ], l_run[NQ];
    floatx4 oacc[NQ][8];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) oacc[nq][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const float scale = 0.08838834764831845f * 1.4426950408889634f;   // log2(e) / sqrt(128): scores in units of ln 2
    for (; s < s_end; s += NW) {
        const int kbase = s * STEP + 8 * bg;     // this lane's eight keys: kbase .. kbase + 7
        const int s_next = min(s + NW, n_steps - 1);
        u32x4 phi[NQ], plo[NQ];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            floatx4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                u32x4 qh, ql;
                if (NQ > 1) {
                    qh = qs[((nq * 4 + t) * 2 + 0) * 64 + lane];
                    ql = qs[((nq * 4 + t) * 2 + 1) * 64 + lane];
                } else {
                    qh = qhi[nq][t];
                    ql = qlo[nq][t];
                }
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&ka[t]), *reinterpret_cast<bf16x8 *>(&qh), sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&kb[t]), *reinterpret_cast<bf16x8 *>(&qh), sb, 0, 0, 0);
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&ka[t]), *reinterpret_cast<bf16x8 *>(&ql), sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&kb[t]), *reinterpret_cast<bf16x8 *>(&ql), sb, 0, 0, 0);
            }
            // lane holds keys kbase + e (e = 0..3 from tile A, 4..7 from tile B) of query rho = 16 nq + bj
            const int rho = nq * 16 + bj;
            const int qpos = L + rho / a.rep;
            float sv[8], mx = -INFINITY;
            if (s * STEP + STEP - 1 <= L) {
                // every query of the block sees every key of this step (wave-uniform): no mask.  Rows past R hold
                // zero queries; their scores are finite and never stored.
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    sv[e] = (e < 4 ? sa[e] : sb[e - 4]) * scale;
                    mx = fmaxf(mx, sv[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int kp = kbase + e;
                    const float x = e < 4 ? sa[e] : sb[e - 4];
                    sv[e] = (rho < R && kp <= qpos && kp < n_keys) ? x * scale : -INFINITY;
                    mx = fmaxf(mx, sv[e]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            // Scores are in units of ln 2, so the exponentials are single v_exp_f32 instructions; exp2(-inf) = 0 covers
            // masked keys and a row's first step, and a row that has seen no key at all subtracts 0 instead of -inf.
            const float m_new = fmaxf(m_run[nq], mx);
            const float m_sub = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[nq] - m_sub);
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(sv[e] - m_sub);
            l_run[nq] = l_run[nq] * alpha + (((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7])));
            m_run[nq] = m_new;
            // the running maximum rarely moves after a row's first steps: scaling by exactly 1 is skipped (wave-uniform)
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) oacc[nq][dt] *= alpha;
            }
            uint32_t h[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                bf16_t h0, l0, h1, l1;
                split2(p[2 * e], h0, l0);
                split2(p[2 * e + 1], h1, l1);
                h[e] = h0 | ((uint32_t)h1 << 16);
                l[e] = l0 | ((uint32_t)l1 << 16);
            }
            phi[nq] = u32x4{h[0], h[1], h[2], h[3]};
            plo[nq] = u32x4{l[0], l[1], l[2], l[3]};
            __builtin_amdgcn_sched_barrier(0);   // one query tile at a time: their temporaries must not pile up
        }
        // the K registers are free: request the next step's keys
        WISV_ATTN_LOAD_K(s_next)
        // positions past the end of the sequence may hold anything (0 x NaN would poison the sum): clear them
        if (s * STEP + STEP > n_keys) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t keep = (kbase + 2 * e < n_keys ? 0xffffu : 0u) | (kbase + 2 * e + 1 < n_keys ? 0xffff0000u : 0u);
                    va[dt][e] &= keep;
                }
        }
        // O^T tiles: rows = 16 features (A operand = V^T), columns = 16 queries, k = this lane group's 8 keys
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                oacc[nq][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&va[dt]),
                                                                      *reinterpret_cast<bf16x8 *>(&phi[nq]), oacc[nq][dt], 0, 0, 0);
                oacc[nq][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&va[dt]),
                                                                      *reinterpret_cast<bf16x8 *>(&plo[nq]), oacc[nq][dt], 0, 0, 0);
            }
        }
        WISV_ATTN_LOAD_V(s_next)
    }
#undef WISV_ATTN_LOAD_K
#undef WISV_ATTN_LOAD_V

    // ---- sums over the four lane groups (each held eight keys of every step), fixed order
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l1 = l_run[nq] + __shfl_xor(l_run[nq], 16, 64);
        l_run[nq] = l1 + __shfl_xor(l1, 32, 64);
    }

    // ---- merge the waves.  Every wave publishes (m, l) of its queries, rescales its output to the common
    //      maximum and publishes that too; wave w then adds up feature tiles w, w + NW, .. of all waves in
    //      wave order.  LDS: sm, sl [NW][NQ][16] floats, then so [NW][NQ][8][64] floatx4.
    float *sm = reinterpret_cast<float *>(lds), *sl = sm + NW * NQ * 16;
    floatx4 *so = reinterpret_cast<floatx4 *>(sl + NW * NQ * 16);
    __syncthreads();   // every wave is done with the query operands that live in the same LDS
    if (bg == 0) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            sm[(wave * NQ + nq) * 16 + bj] = m_run[nq];
            sl[(wave * NQ + nq) * 16 + bj] = l_run[nq];
        }
    }
    __syncthreads();
    float m_all[NQ], l_all[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        float mx = -INFINITY;
        for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm[(w * NQ + nq) * 16 + bj]);
        float ls = 0.f;
        for (int w = 0; w < NW; ++w) {
            const float mw = sm[(w * NQ + nq) * 16 + bj];
            if (mw != -INFINITY) ls += sl[(w * NQ + nq) * 16 + bj] * exp2f(mw - mx);
        }
        m_all[nq] = mx;
        l_all[nq] = ls;
        const float mine = m_run[nq] == -INFINITY ? 0.f : exp2f(m_run[nq] - mx);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) so[((wave * NQ + nq) * 8 + dt) * 64 + lane] = oacc[nq][dt] * mine;
    }
    __syncthreads();
    for (int dt = wave; dt < 8; dt += NW) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            const int rho = nq * 16 + bj;
            floatx4 acc = so[((0 * NQ + nq) * 8 + dt) * 64 + lane];
            for (int w = 1; w < NW; ++w) acc += so[((w * NQ + nq) * 8 + dt) * 64 + lane];
            if (rho >= R) continue;
            // lane holds features 16 dt + 4 bg + r of query rho
            const int m = m0 + rho / a.rep, h = g * a.rep + rho % a.rep;
            if (a.n_splits == 1) {
                const float inv = 1.0f / l_all[nq];
                act_store4(a.o, ((size_t)m * a.H + h) * HD + 16 * dt + 4 * bg, acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
            } else {
                const size_t row = ((size_t)split * a.rows + m) * a.H + h;
                *reinterpret_cast<floatx4 *>(a.po + row * HD + 16 * dt + 4 * bg) = acc;
                if (dt == 0 && bg == 0) {
                    a.pm[row] = m_all[nq];
                    a.pl[row] = l_all[nq];
                }
            }
        }
    }
}

// o[m][h][:] = sum_s 2^(m_s - m*) O_s / sum_s 2^(m_s - m*) l_s (the maxima are kept in units of ln 2), splits in index
// order; one block per (row, head).
// Splits are taken BATCH at a time, all loads of a batch issued before the first is used (slots past the last
// split re-read it and weigh zero), batches chained with the same rescaling rule.
template <int BATCH>
__global__ void k_attn_combine(const float *__restrict__ po, const float *__restrict__ pm, const float *__restrict__ pl,
                               int n_splits, int rows, int H, ActBuf o) {
    const int m = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
    float mx = -INFINITY, num = 0.f, den = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += BATCH) {
        float ms[BATCH], ls[BATCH], os[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const size_t row = ((size_t)min(s0 + i, n_splits - 1) * rows + m) * H + h;
            ms[i] = pm[row];
            ls[i] = pl[row];
            os[i] = po[row * HD + d];
        }
        float bmx = mx;
#pragma unroll
        for (int i = 0; i < BATCH; ++i) bmx = fmaxf(bmx, s0 + i < n_splits ? ms[i] : -INFINITY);
        if (bmx == -INFINITY) continue;
        const float keep = mx == -INFINITY ? 0.f : exp2f(mx - bmx);
        num *= keep;
        den *= keep;
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const bool on = s0 + i < n_splits && ms[i] != -INFINITY;
            const float w = on ? exp2f(ms[i] - bmx) : 0.f;
            den = fmaf(w, on ? ls[i] : 0.f, den);
            num = fmaf(w, on ? os[i] : 0.f, num);
        }
        mx = bmx;
    }
    act_store(o, ((size_t)m * H + h) * HD + d, num / den);
}

template <int NQ, int NW, bool FUSE> static bool launch_nq(Ctx *c, const AttnArgs &a, dim3 grid) {
    // the merge area at the end of the kernel, which also holds the parked query operands before that
    const size_t lds = std::max((size_t)NW * NQ * (2 * 16 * 4 + 8 * 64 * 16), (size_t)NQ * 8 * 1024);
    static bool allowed[MAX_DEVICES];
    if (lds > 64 * 1024 && !allow_big_lds(c, reinterpret_cast<const void *>(&k_attn_mfma<NQ, NW, FUSE>), allowed)) return false;
    hipLaunchKernelGGL((k_attn_mfma<NQ, NW, FUSE>), grid, dim3(64 * NW), lds, c->stream, a);
    return true;
}

// One workgroup per (stream, KV head) when that fills the chip (then the workgroup writes the output itself);
// otherwise k-splits of at least one 32-key step per wave, never more workgroups than CUs (a second round of
// workgroups costs more than the splits gain: 12 streams x 8 KV heads over 2048 cached tokens, 3 splits = 288
// workgroups 44.7 us, 2 splits 29.1 us; 24 streams over 4096: 2 splits 112.8 us, 1 split 98.7 us) and 16 in all
// (one stream over 512: the round takes 3.51 ms with 3 splits and their combine kernel, 3.55 ms with one).
// 0: the shape is not served.
static int attn_splits(const Ctx *c, const Fwd &f) {
    const wisv_config &g = c->cfg;
    const int rep = g.n_heads / g.n_kv_heads, R = rep * f.k;
    if (!c->bf16 || g.head_dim != HD || R > 64 || f.rows != f.batch * f.k) return 0;
    const int nw = R <= 32 ? 8 : 4;
    const int n_steps = (f.max_len_ub + STEP - 1) / STEP, wgs = f.batch * g.n_kv_heads;
    const int want = std::max(1, std::min(256 / wgs, (n_steps + nw - 1) / nw));
    return std::max(1, std::min(std::min(want, 16), c->att_max_splits));   // 16: one batch of the combine kernel
}

// With several k-splits every split repeats the query part of the prologue (it sums the QKV slices of its queries
// and rotates them; the split that ends the sequence also appends).  That always beat or equalled a kernel of its own
// for RoPE and the append: 8 rows over 4096 cached tokens 4.04 -> 3.92 ms per round; 96 rows, 2 splits 6.34 -> 6.15;
// 72 rows, 3 splits 6.25 -> 6.09; 32 rows over 4096 tokens, 8 splits 4.98 -> 4.86; 24 rows over 8192 tokens, 16
// splits 4.88 -> 4.89.  k_rope_append serves the shapes this kernel does not take.
bool attn_mfma_fuses_rope(const Ctx *c, const Fwd &f) { return attn_splits(c, f) >= 1; }

// c->o from the k-split partials in c->att_o / att_m / att_l
void launch_attn_combine(Ctx *c, const Fwd &f, int n_splits) {
    const wisv_config &g = c->cfg;
    ProfScope ps(c, KC_ATTN_COMBINE);
    if (n_splits <= 4)
        hipLaunchKernelGGL(k_attn_combine<4>, dim3(f.rows, g.n_heads), dim3(HD), 0, c->stream, c->att_o, c->att_m, c->att_l,
                           n_splits, f.rows, g.n_heads, act_planes(c->o, c->o_planes));
    else
        hipLaunchKernelGGL(k_attn_combine<16>, dim3(f.rows, g.n_heads), dim3(HD), 0, c->stream, c->att_o, c->att_m, c->att_l,
                           n_splits, f.rows, g.n_heads, act_planes(c->o, c->o_planes));
}

// n_partial > 0: the k-split slices of the QKV product are in c->qkv and the kernel does RoPE and the append
// itself; n_partial == 0: launch_rope_append has run
bool launch_attn_mfma(Ctx *c, const Fwd &f, int layer, int n_partial, bool with_combine, int *n_splits, int n_ss) {
    const wisv_config &g = c->cfg;
    const int rep = g.n_heads / g.n_kv_heads, R = rep * f.k;
    AttnArgs a;
    a.n_splits = attn_splits(c, f);
    if (!a.n_splits || (n_partial > 0 && !attn_mfma_fuses_rope(c, f))) return false;
    a.q = c->q;
    a.kv_layer = (const bf16_t *)kv_ptr(c, layer, 0, 0);
    a.kv_write = (bf16_t *)kv_ptr(c, layer, 0, 0);
    a.slot_stride = (size_t)2 * g.n_kv_heads * c->ctx_pad * g.head_dim;
    a.H = g.n_heads; a.G = g.n_kv_heads; a.rep = rep; a.K = f.k; a.max_ctx = g.max_ctx; a.ctx_pad = c->ctx_pad; a.rows = f.rows;
    a.row_slot = c->row_slot; a.row_pos = c->row_pos;
    a.po = c->att_o; a.pm = c->att_m; a.pl = c->att_l;
    a.o = act_planes(c->o, c->o_planes);
    a.qkv = c->qkv; a.n_partial = n_partial; a.partial_stride = (size_t)c->rows_max * c->d_qkv;
    a.cs = c->rope_cos; a.sn = c->rope_sin;
    a.ss = c->ss; a.n_ss = n_ss; a.d_model = g.d_model; a.eps = g.rms_eps;
    if (n_ss > 0 && n_partial == 0) return false;   // only the fused prologue applies the scale
    dim3 grid(a.n_splits, g.n_kv_heads, f.batch);
    {
        ProfScope ps(c, KC_ATTN);
        bool ok;
        const bool fuse = n_partial > 0;
        switch ((R + 15) / 16) {
            case 1: ok = fuse ? launch_nq<1, 8, true>(c, a, grid) : launch_nq<1, 8, false>(c, a, grid); break;
            case 2: ok = fuse ? launch_nq<2, 8, true>(c, a, grid) : launch_nq<2, 8, false>(c, a, grid); break;
            case 3: ok = fuse ? launch_nq<3, 4, true>(c, a, grid) : launch_nq<3, 4, false>(c, a, grid); break;
            default: ok = fuse ? launch_nq<4, 4, true>(c, a, grid) : launch_nq<4, 4, false>(c, a, grid); break;
        }
        if (!ok) return false;
    }
    if (n_splits) *n_splits = a.n_splits;
    if (a.n_splits > 1 && with_combine) launch_attn_combine(c, f, a.n_splits);
    return true;
}

}  // namespace wisv
