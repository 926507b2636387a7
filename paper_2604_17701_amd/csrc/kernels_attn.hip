// Grouped-query attention of the drafted block over the KV cache (bf16 cache, head_dim 128):
// the K query rows of a stream x the query heads that share one KV head form one tile of up to 64 rows, so
// every cached key/value byte is read once per (stream, KV head) and meets all of them.
//
// One workgroup = (k-split, KV head, stream).  Per 64-key chunk the four waves stage K and V through LDS
// (coalesced 16-byte loads, rows padded against bank conflicts, next chunk prefetched into registers),
// each wave takes 16 keys:  S^T = K Q^T on the 16x16x32 MFMA (queries fed as two bf16 terms), float online
// softmax with wavefront reductions over the key dimension, then O^T += V^T P^T on the 16x16x16 MFMA
// (probabilities fed as two bf16 terms, so P.V is exact to 2^-17).  Waves and k-splits are merged with the
// usual (max, sum, unnormalised output) rule in a fixed order; a small kernel normalises.
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int HD = 128, CHUNK = 64, PITCH = 272;            // bytes per staged row: 256 + 16
constexpr int BUF_BYTES = 2 * CHUNK * PITCH;                // K rows then V rows of one chunk

struct AttnArgs {
    const float *q;           // rotated queries [rows][H * 128]
    const bf16_t *kv_layer;   // this layer's cache: [slot][K|V][G][max_ctx][128]
    size_t slot_stride;       // elements per slot
    int H, G, rep, K, max_ctx, n_splits, rows;
    const int32_t *row_slot, *row_pos;
    float *po, *pm, *pl;      // partials [split][rows][H][128], [split][rows][H]
};

template <int NQ>
__global__ __launch_bounds__(256) void k_attn_mfma(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, bj = lane & 15, bg = lane >> 4;
    const int m0 = b * a.K;
    const int L = a.row_pos[m0], slot = a.row_slot[m0];
    const int n_keys = min(L + a.K, a.max_ctx), R = a.rep * a.K;
    const bf16_t *kc = a.kv_layer + (size_t)slot * a.slot_stride + (size_t)g * a.max_ctx * HD;
    const bf16_t *vc = kc + (size_t)a.G * a.max_ctx * HD;
    const int n_chunks = (n_keys + CHUNK - 1) / CHUNK, cps = (n_chunks + a.n_splits - 1) / a.n_splits;
    const int c_begin = split * cps, c_end = min(n_chunks, c_begin + cps);

    // ---- queries as MFMA B operands (two bf16 terms): lane (bj, bg) holds Q[rho = 16 nq + bj][32 t + 8 bg ..]
    uint4 qhi[NQ][4], qlo[NQ][4];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int rho = nq * 16 + bj;
        const bool valid = rho < R;
        const float *qp = a.q + ((size_t)(m0 + (valid ? rho / a.rep : 0)) * a.H + (size_t)g * a.rep + (valid ? rho % a.rep : 0)) * HD;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t h[4] = {0, 0, 0, 0}, l[4] = {0, 0, 0, 0};
            if (valid) {
                const float4 x0 = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg);
                const float4 x1 = *reinterpret_cast<const float4 *>(qp + 32 * t + 8 * bg + 4);
                const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bf16_t h0, l0, h1, l1;
                    split2(xs[2 * e], h0, l0);
                    split2(xs[2 * e + 1], h1, l1);
                    h[e] = h0 | ((uint32_t)h1 << 16);
                    l[e] = l0 | ((uint32_t)l1 << 16);
                }
            }
            qhi[nq][t] = make_uint4(h[0], h[1], h[2], h[3]);
            qlo[nq][t] = make_uint4(l[0], l[1], l[2], l[3]);
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

    // ---- chunk loop.  Thread tid moves 16-byte segment `seg` of staged rows krow, krow + 16, krow + 32, krow + 48
    //      of the chunk's K and V.
    // (named registers rather than arrays: the prefetched chunk must stay in VGPRs across the loop)
    uint4 k0, k1, k2, k3, v0, v1, v2, v3;
    const int seg = tid & 15, krow = tid >> 4;               // segment i covers staged row krow + 16 i
#define WISV_ATTN_LOAD(c_, i_, kr_, vr_)                                                      \
    {                                                                                         \
        const int key_ = min((c_) * CHUNK + krow + 16 * (i_), n_keys - 1);                    \
        kr_ = *reinterpret_cast<const uint4 *>(kc + (size_t)key_ * HD + seg * 8);             \
        vr_ = *reinterpret_cast<const uint4 *>(vc + (size_t)key_ * HD + seg * 8);             \
    }
#define WISV_ATTN_FETCH(c_)          \
    WISV_ATTN_LOAD(c_, 0, k0, v0)    \
    WISV_ATTN_LOAD(c_, 1, k1, v1)    \
    WISV_ATTN_LOAD(c_, 2, k2, v2)    \
    WISV_ATTN_LOAD(c_, 3, k3, v3)
#define WISV_ATTN_PUT(i_, kr_, vr_)                                                                        \
    *reinterpret_cast<uint4 *>(buf + (krow + 16 * (i_)) * PITCH + seg * 16) = kr_;                         \
    *reinterpret_cast<uint4 *>(buf + CHUNK * PITCH + (krow + 16 * (i_)) * PITCH + seg * 16) = vr_;
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    if (c_begin < c_end) { WISV_ATTN_FETCH(c_begin) }
    for (int c = c_begin; c < c_end; ++c) {
        unsigned char *buf = lds + (size_t)((c - c_begin) & 1) * BUF_BYTES;
        WISV_ATTN_PUT(0, k0, v0)
        WISV_ATTN_PUT(1, k1, v1)
        WISV_ATTN_PUT(2, k2, v2)
        WISV_ATTN_PUT(3, k3, v3)
        __syncthreads();   // chunk c staged; the other buffer is free (everyone finished chunk c - 1)
        if (c + 1 < c_end) { WISV_ATTN_FETCH(c + 1) }
        const unsigned char *kb = buf + (16 * wave) * PITCH, *vb = buf + CHUNK * PITCH + (16 * wave) * PITCH;
        const int kbase = c * CHUNK + 16 * wave;
        if (kbase >= n_keys) continue;

        // S^T tile: rows = 16 keys (A operand from LDS), columns = 16 queries
        uint4 ka[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) ka[t] = *reinterpret_cast<const uint4 *>(kb + bj * PITCH + (32 * t + 8 * bg) * 2);
        uint2 phi[NQ], plo[NQ];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            floatx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&ka[t]),
                                                            *reinterpret_cast<bf16x8 *>(&qhi[nq][t]), s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&ka[t]),
                                                            *reinterpret_cast<bf16x8 *>(&qlo[nq][t]), s, 0, 0, 0);
            }
            // lane holds keys kbase + 4 bg + r (r = 0..3) of query rho = 16 nq + bj
            const int rho = nq * 16 + bj;
            const int qpos = L + rho / a.rep;
            float sv[4], mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int kp = kbase + 4 * bg + r;
                sv[r] = (rho < R && kp <= qpos && kp < n_keys) ? s[r] * scale : -INFINITY;
                mx = fmaxf(mx, sv[r]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[nq], mx);
            float alpha = 1.f, p[4] = {0.f, 0.f, 0.f, 0.f};
            if (m_new != -INFINITY) {
                alpha = m_run[nq] == -INFINITY ? 0.f : expf(m_run[nq] - m_new);
#pragma unroll
                for (int r = 0; r < 4; ++r) p[r] = sv[r] == -INFINITY ? 0.f : expf(sv[r] - m_new);
            }
            l_run[nq] = l_run[nq] * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
            m_run[nq] = m_new;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) oacc[nq][dt] *= alpha;
            bf16_t h[4], l[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) split2(p[r], h[r], l[r]);
            phi[nq] = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
            plo[nq] = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
        }
        // O^T tiles: rows = 16 features (A operand = V^T gathered from LDS), columns = 16 queries, k = 16 keys
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            uint16_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const uint16_t *>(vb + (4 * bg + e) * PITCH + (16 * dt + bj) * 2);
            uint2 va = make_uint2(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16));
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                oacc[nq][dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*reinterpret_cast<s16x4 *>(&va),
                                                                        *reinterpret_cast<s16x4 *>(&phi[nq]), oacc[nq][dt], 0, 0, 0);
                oacc[nq][dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*reinterpret_cast<s16x4 *>(&va),
                                                                        *reinterpret_cast<s16x4 *>(&plo[nq]), oacc[nq][dt], 0, 0, 0);
            }
        }
    }

#undef WISV_ATTN_FETCH
#undef WISV_ATTN_LOAD
#undef WISV_ATTN_PUT

    // ---- sums over the four lane groups (each held the keys 4 bg + r of every tile), fixed order
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l1 = l_run[nq] + __shfl_xor(l_run[nq], 16, 64);
        l_run[nq] = l1 + __shfl_xor(l1, 32, 64);
    }

    // ---- merge waves 1..3 into wave 0 through LDS, one at a time.  Layout of one wave's state:
    //      [nq][dt][lane] floatx4, then m[nq][lane], l[nq][lane]
    floatx4 *so = reinterpret_cast<floatx4 *>(lds);
    float *sm = reinterpret_cast<float *>(lds) + NQ * 8 * 64 * 4, *sl = sm + NQ * 64;
    for (int w = 1; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) so[(nq * 8 + dt) * 64 + lane] = oacc[nq][dt];
                sm[nq * 64 + lane] = m_run[nq];
                sl[nq * 64 + lane] = l_run[nq];
            }
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                const float mw = sm[nq * 64 + lane], lw = sl[nq * 64 + lane];
                const float m_new = fmaxf(m_run[nq], mw);
                float a0 = 1.f, aw = 0.f;
                if (m_new != -INFINITY) {
                    a0 = m_run[nq] == -INFINITY ? 0.f : expf(m_run[nq] - m_new);
                    aw = mw == -INFINITY ? 0.f : expf(mw - m_new);
                }
                l_run[nq] = l_run[nq] * a0 + lw * aw;
                m_run[nq] = m_new;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) oacc[nq][dt] = oacc[nq][dt] * a0 + so[(nq * 8 + dt) * 64 + lane] * aw;
            }
        }
    }
    if (wave != 0) return;

    // ---- this split's partial: lane holds features 16 dt + 4 bg + r of query rho = 16 nq + bj
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int rho = nq * 16 + bj;
        if (rho >= R) continue;
        const size_t row = ((size_t)split * a.rows + m0 + rho / a.rep) * a.H + (size_t)g * a.rep + rho % a.rep;
        if (bg == 0) {
            a.pm[row] = m_run[nq];
            a.pl[row] = l_run[nq];
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<floatx4 *>(a.po + row * HD + 16 * dt + 4 * bg) = oacc[nq][dt];
    }
}

// o[m][h][:] = sum_s e^(m_s - m*) O_s / sum_s e^(m_s - m*) l_s, splits in index order; one block per (row, head)
__global__ void k_attn_combine(const float *__restrict__ po, const float *__restrict__ pm, const float *__restrict__ pl,
                               int n_splits, int rows, int H, ActBuf o) {
    const int m = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
    float mx = -INFINITY;
    for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, pm[((size_t)s * rows + m) * H + h]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const size_t row = ((size_t)s * rows + m) * H + h;
        const float ms = pm[row];
        if (ms == -INFINITY) continue;
        const float w = expf(ms - mx);
        den = fmaf(w, pl[row], den);
        num = fmaf(w, po[row * HD + d], num);
    }
    act_store(o, ((size_t)m * H + h) * HD + d, num / den);
}

template <int NQ> static bool launch_nq(Ctx *c, const AttnArgs &a, dim3 grid) {
    static bool opted_in = false;
    if (!opted_in) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_mfma<NQ>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return false;
        opted_in = true;
    }
    const size_t merge = (size_t)NQ * (8 * 64 * 16 + 2 * 64 * 4);
    hipLaunchKernelGGL(k_attn_mfma<NQ>, grid, dim3(256), std::max<size_t>(2 * BUF_BYTES, merge), c->stream, a);
    return true;
}

bool launch_attn_mfma(Ctx *c, const Fwd &f, int layer) {
    const wisv_config &g = c->cfg;
    const int rep = g.n_heads / g.n_kv_heads, R = rep * f.k;
    if (!c->bf16 || g.head_dim != HD || R > 64 || f.rows != f.batch * f.k) return false;
    AttnArgs a;
    a.q = c->q;
    a.kv_layer = (const bf16_t *)kv_ptr(c, layer, 0, 0);
    a.slot_stride = (size_t)2 * g.n_kv_heads * g.max_ctx * g.head_dim;
    a.H = g.n_heads; a.G = g.n_kv_heads; a.rep = rep; a.K = f.k; a.max_ctx = g.max_ctx; a.rows = f.rows;
    a.row_slot = c->row_slot; a.row_pos = c->row_pos;
    a.po = c->att_o; a.pm = c->att_m; a.pl = c->att_l;
    // enough workgroups to cover the chip twice, at least two 64-key chunks per split
    const int n_chunks = (f.max_len_ub + CHUNK - 1) / CHUNK;
    const int want = (512 + f.batch * g.n_kv_heads - 1) / (f.batch * g.n_kv_heads);
    a.n_splits = std::max(1, std::min(std::min(want, (n_chunks + 1) / 2), c->att_max_splits));
    dim3 grid(a.n_splits, g.n_kv_heads, f.batch);
    {
        ProfScope ps(c, KC_ATTN);
        bool ok;
        switch ((R + 15) / 16) {
            case 1: ok = launch_nq<1>(c, a, grid); break;
            case 2: ok = launch_nq<2>(c, a, grid); break;
            case 3: ok = launch_nq<3>(c, a, grid); break;
            default: ok = launch_nq<4>(c, a, grid); break;
        }
        if (!ok) return false;
    }
    {
        ProfScope ps(c, KC_ATTN_COMBINE);
        hipLaunchKernelGGL(k_attn_combine, dim3(f.rows, g.n_heads), dim3(HD), 0, c->stream, c->att_o, c->att_m, c->att_l,
                           a.n_splits, f.rows, g.n_heads, c->o);
    }
    return true;
}

}  // namespace wisv
