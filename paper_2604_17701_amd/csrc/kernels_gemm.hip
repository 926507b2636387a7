// Weight-streaming bf16 GEMM for a small number of activation rows (the memory-bound regime of the
// verify round: every weight byte is read once per round and meets at most a few hundred rows).
//
// Y[m, n] = sum_k X[m, k] W[n, k] is computed "swapped": the 16x16x32 MFMA takes a 16-row block of W as
// its A operand and 16 activation rows as its B operand, so the output-feature dimension fills the
// matrix core however few rows there are.  W is stored re-tiled: tile (rb, kt) holds W[16rb..+16][32kt..+32]
// as 64 lanes x 8 bf16 in exactly the order the MFMA wants, so that one wave-wide 16-byte load fetches a
// contiguous KiB and a wave walking along k reads one contiguous stream.  Activations arrive as two bf16
// planes (x = hi + lo, written by whichever kernel produced them), one MFMA each: the products are then
// exact to about 2^-17 while the weights stay bf16; the second MFMA costs issue slots this memory-bound
// kernel has to spare.
//
// A workgroup is WR x WK waves: WR groups of RB row-blocks share the activation chunk in LDS, and WK slices
// of the workgroup's k-range whose accumulators are added through LDS in slice order.  The grid's y
// dimension splits k into partial outputs, its z dimension walks tiles of 16 NT rows.
// The weight stream is software-pipelined through a ring of U register slots: the steady-state loop has no
// branches, and every slot is refilled right after the MFMAs that read it (scheduling barriers keep that
// order), so that the compiler's wait counts let U loads stay in flight.
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------ re-tiling
// out[((rb * nkt + kt) * 64 + lane) * 8 + e] = W[row(rb, lane % 16)][32 kt + 8 (lane / 16) + e]
// pair_rows > 0: W stacks two matrices of pair_rows rows each (gate over up); row-block rb then holds
// gate rows 8rb..8rb+7 in its rows 0..7 and up rows 8rb..8rb+7 in its rows 8..15, so that one MFMA tile
// carries both halves of SwiGLU for 8 features.
// overflow != null: every element is converted to an IEEE half (nearest-even; magnitudes below 2^-14 keep what a
// subnormal half holds, an absolute error of at most 2^-25); *overflow is set when one does not fit the half range
__global__ void k_retile(const bf16_t *__restrict__ W, int n_rows, int kd, int nrb, int nkt, int pair_rows,
                         uint4 *__restrict__ out, int32_t *overflow) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)nrb * nkt * 64) return;
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int kt = tile % nkt, rb = tile / nkt, i = lane & 15;
    int row;
    bool valid;
    if (pair_rows > 0) {
        const int f = rb * 8 + (i & 7);
        row = (i >> 3) * pair_rows + f;
        valid = f < pair_rows;
    } else {
        row = rb * 16 + i;
        valid = row < n_rows;
    }
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid) v = *reinterpret_cast<const uint4 *>(W + (size_t)row * kd + 32 * kt + 8 * (lane >> 4));
    if (overflow) {
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
        bool bad = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = __uint_as_float(w[e] << 16), b = __uint_as_float(w[e] & 0xffff0000u);
            bad = bad || !(fabsf(a) <= 65504.0f) || !(fabsf(b) <= 65504.0f);
            w[e] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)a) | ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)b) << 16);
        }
        if (bad) atomicOr(overflow, 1);
        v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    out[idx] = v;
}

void launch_retile(Ctx *c, const void *W, int n_rows, int kd, int pair_rows, void *out, int nrb, int32_t *overflow) {
    const int nkt = kd / 32;
    const size_t total = (size_t)nrb * nkt * 64;
    hipLaunchKernelGGL(k_retile, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, (const bf16_t *)W,
                       n_rows, kd, nrb, nkt, pair_rows, (uint4 *)out, overflow);
}

// row-blocks are padded to a multiple of 16 so that a workgroup may own up to 16 of them
int ws_padded_row_blocks(int n_rows) { return ((n_rows + 15) / 16 + 15) / 16 * 16; }
// gate/up pairs: 8 features per row-block
int ws_padded_pair_blocks(int features) { return ((features + 7) / 8 + 15) / 16 * 16; }

// ------------------------------------------------------------------------------------------ the GEMM
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2, EPI_RESID = 3 };

struct GemmArgs {
    const u32x4 *Wt;           // re-tiled weights [nrb][nkt][64]
    const bf16_t *Xhi, *Xlo;   // activation planes [M][kd]
    const uint16_t *X16;       // the activations as one half each (k_gemm_mm with ONE term; Wt then holds halves too)
    int M, N, kd, nrb, nkt, kt_per_split;
    int kcw;                   // k-tiles per wave staged in LDS at a time (a multiple of the prefetch depth)
    float *Yp;                 // EPI_PARTIAL: [S][split_stride];  EPI_ARGMAX with logits != null: [M][N]
    size_t split_stride;
    ActBuf H;                  // EPI_SWIGLU: [M][N] float + planes (N = features)
    float *cand_val;           // EPI_ARGMAX: [M][n_cand]
    int32_t *cand_idx;
    int n_cand;
    int gx, gz, gs;            // k_gemm_mm: row-block groups, row tiles and k-splits the 1-D grid decodes into
    // PRO: the activations are the attention output, still in k-split partials (up to WS_PRO_SPLITS of them):
    // o [split][rows][heads][128], running maximum m (in units of ln 2) and sum l [split][rows][heads]
    const float *att_o, *att_m, *att_l;
    int att_splits, att_rows, att_H;
    // PRO_NORM: the activations are the residual stream, still to be updated: v = xin + the n_partial slices of the
    // previous product (ys), a = v * gain (the RMSNorm gain; its 1 / rms factor is applied by whoever sums this
    // product's slices).  Workgroups with blockIdx.x == 0 also write v to xout and the sum of v^2 over their k-range
    // to ss_out[split][row].
    const float *xin, *ys;
    float *xout, *ss_out;
    const bf16_t *gain;
    int n_partial;
    size_t ys_stride;
    // EPI_RESID (a product whose k-split stays inside the workgroup: complete sums): v = xin + Y is written to xout,
    // v * gain to H (float and two-term planes: the next block's RMSNorm without its 1 / rms), and the sum of v^2 over
    // the workgroup's 16 RB features of every row to ss_out[row-block group][row]; xin may be xout.
    // EPI_SWIGLU with ss_in: the activations came that way; both halves are scaled by
    // 1 / sqrt(sum of the n_ss_in partial sums of the row / kd + rms_eps) before the SiLU.
    const float *ss_in;
    int n_ss_in;
    float rms_eps;
};
enum { PRO_NONE = 0, PRO_ATTN = 1, PRO_NORM = 2 };

// ------------------------------------------------------------------------------------------ epilogues
// acc[r][t][e] = Y[m = m_base + 16 t + lane % 16][row 4 (lane / 16) + e of row-block rb0 + r]; `split` is the
// partial-output slice, `slot` the wave's candidate slot (one per group of RB row-blocks)
template <int NT, int RB, int EPI>
__device__ __forceinline__ void ws_epilogue(const GemmArgs &g, floatx4 (&acc)[RB][NT], int m_base, int rb0, int split,
                                            int slot, int lane, const float *s_inv, const floatx4 (&res_x)[RB][NT],
                                            const uint2 (&res_g)[RB]) {
    const int bj = lane & 15, bg = lane >> 4;
    if (EPI == EPI_PARTIAL) {
        float *out = g.Yp + (size_t)split * g.split_stride;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + t * 16 + bj;
            if (m >= g.M) continue;
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int n = (rb0 + r) * 16 + bg * 4;
                if (n + 3 < g.N && (g.N & 3) == 0) *reinterpret_cast<floatx4 *>(out + (size_t)m * g.N + n) = acc[r][t];
                else
                    for (int e = 0; e < 4; ++e)
                        if (n + e < g.N) out[(size_t)m * g.N + n + e] = acc[r][t][e];
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        // rows 0..7 of a block are gate, rows 8..15 up, of features 8 (rb0 + r) ..: lanes 32..63 hold the up
        // values that lanes 0..31 need
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + t * 16 + bj;
            if (g.ss_in) {   // the deferred 1 / rms of a folded RMSNorm, computed by the kernel's prologue
                const float inv = s_inv[min(t * 16 + bj, 16 * NT - 1)];
#pragma unroll
                for (int r = 0; r < RB; ++r)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][t][e] *= inv;
            }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                floatx4 up;
#pragma unroll
                for (int e = 0; e < 4; ++e) up[e] = __shfl_xor(acc[r][t][e], 32, 64);
                if (bg < 2 && m < g.M) {
                    const int f = (rb0 + r) * 8 + bg * 4;
                    float hv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gt = acc[r][t][e];
                        hv[e] = gt / (1.0f + expf(-gt)) * up[e];
                    }
                    if (f + 3 < g.N && (g.N & 3) == 0) act_store4(g.H, (size_t)m * g.N + f, hv[0], hv[1], hv[2], hv[3]);
                    else
                        for (int e = 0; e < 4; ++e)
                            if (f + e < g.N) act_store(g.H, (size_t)m * g.N + f + e, hv[e]);
                }
            }
        }
    } else if (EPI == EPI_RESID) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + t * 16 + bj;
            float q2 = 0.f;
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int n = (rb0 + r) * 16 + bg * 4;     // N is a multiple of 16 here (checked by the launcher)
                if ((rb0 + r) * 16 >= g.N) continue;       // a padding row-block (uniform over the wave)
                const floatx4 xv = res_x[r][t];            // requested when the kernel started
                const uint2 gw = res_g[r];
                const floatx4 v = {xv[0] + acc[r][t][0], xv[1] + acc[r][t][1], xv[2] + acc[r][t][2], xv[3] + acc[r][t][3]};
                if (m < g.M) {
                    *reinterpret_cast<floatx4 *>(g.xout + (size_t)m * g.N + n) = v;
                    act_store4(g.H, (size_t)m * g.N + n, v[0] * __uint_as_float(gw.x << 16), v[1] * __uint_as_float(gw.x & 0xffff0000u),
                               v[2] * __uint_as_float(gw.y << 16), v[3] * __uint_as_float(gw.y & 0xffff0000u));
                }
                q2 += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
            }
            q2 += __shfl_xor(q2, 16, 64);
            q2 += __shfl_xor(q2, 32, 64);
            if (bg == 0 && m < g.M && rb0 * 16 < g.N) g.ss_out[(size_t)slot * g.M + m] = q2;
        }
    } else {   // EPI_ARGMAX: best (value, lowest index) of this wave's 16*RB features for every row
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + t * 16 + bj;
            float best = -INFINITY;
            int idx = 0x7fffffff;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int n = (rb0 + r) * 16 + bg * 4 + e;
                    const float v = acc[r][t][e];
                    if (n < g.N) {
                        if (g.Yp && m < g.M) g.Yp[(size_t)m * g.N + n] = v;
                        if (v > best || (v == best && n < idx)) { best = v; idx = n; }
                    }
                }
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                const float ov = __shfl_xor(best, o, 64);
                const int oi = __shfl_xor(idx, o, 64);
                if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
            }
            if (bg == 0 && m < g.M) {
                g.cand_val[(size_t)m * g.n_cand + slot] = best;
                g.cand_idx[(size_t)m * g.n_cand + slot] = idx;
            }
        }
    }
}

// NT: 16-row activation tiles per wave; RB: row-blocks per wave; WR x WK waves per workgroup; U: prefetch depth;
// PRO_ATTN: the activations are combined from the attention kernel's k-split partials while they are staged (the rule
// of k_attn_combine: weights e^(m_s - max m), splits in index order), so that no kernel of its own has to do it.
// PRO_NORM: the activations are the residual stream plus the previous product's slices, times the norm gain (see
// GemmArgs); WK == 1 and a single activation chunk
template <int NT, int RB, int WR, int WK, int U, int PRO, int EPI>
__global__ __launch_bounds__(64 * WR * WK, PRO == PRO_NORM ? 6 : 1) void k_gemm_ws(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NTH = 64 * WR * WK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wr = wave / WK, wk = wave % WK;
    const int kt0 = blockIdx.y * g.kt_per_split;
    const int ntile = min(g.kt_per_split, g.nkt - kt0);
    const int sub = (ntile + WK - 1) / WK;                         // k-tiles per wave
    const int my0 = wk * sub, myn = max(0, min(sub, ntile - my0));
    const int rb0 = (blockIdx.x * WR + wr) * RB;
    const bool active = rb0 < g.nrb;                               // RB * WR divides nrb (padded)
    const int m_base = blockIdx.z * (16 * NT), Mt = min(16 * NT, g.M - m_base);   // this workgroup's rows

    // ---- start the weight stream before anything else: it does not depend on the activations
    const u32x4 *wp[RB];
    u32x4 abuf[U][RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) wp[r] = g.Wt + ((size_t)(active ? rb0 + r : 0) * g.nkt + kt0 + my0) * 64 + lane;
    if (active) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (u < myn) abuf[u][r] = __builtin_nontemporal_load(wp[r] + (size_t)u * 64);
    }

    floatx4 acc[RB][NT];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // EPI_RESID: the residual stream and the gain of this wave's outputs are requested now, by the waves that will
    // run the epilogue (lane (bj, bg): row m_base + 16 t + bj, features 16 (rb0 + r) + 4 bg ..)
    floatx4 res_x[RB][NT];
    uint2 res_g[RB];
    if (EPI == EPI_RESID && wk == 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int n = min((rb0 + r) * 16, g.N - 16) + (lane >> 4) * 4;
            res_g[r] = *reinterpret_cast<const uint2 *>(g.gain + n);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                res_x[r][t] = *reinterpret_cast<const floatx4 *>(g.xin + (size_t)min(m_base + t * 16 + (lane & 15), g.M - 1) * g.N + n);
        }
    }

    // ---- activations: chunk ch holds, for every k-slice w, its tiles [ch kcw, (ch+1) kcw) as
    //      lds[ch & 1][plane][w][m][kcw * 64 + 16 bytes]; the 16 spreads rows over the banks
    const int kcw = g.kcw, pitch = kcw * 64 + 16, wk_bytes = Mt * pitch, plane_bytes = WK * wk_bytes,
              buf_bytes = 2 * plane_bytes;
    const int nchunk = (sub + kcw - 1) / kcw;
    auto stage = [&](int ch) {
        unsigned char *dst = lds + (size_t)(ch & 1) * buf_bytes;
        const int vec_per_row = kcw * 4, per_wk = Mt * vec_per_row;
        if (PRO == PRO_NORM) {
            // An item is four consecutive features of one row; the four lane groups of a wave share 16 items and take
            // four slices each (every load is unconditional: slices past the last re-read it and count as zero), then
            // add their sums in a fixed order: ((x + s0..s3) + (s4..s7)) + ((s8..s11) + (s12..s15)).
            float *ssq = reinterpret_cast<float *>(lds + 2 * buf_bytes);   // per item: sum of v^2
            const int grp = lane >> 4, np = max(g.n_partial, 1);
            const int item_per_row = kcw * 8, n_item = Mt * item_per_row;
            for (int base = wave * 16; base < n_item; base += (NTH / 64) * 16) {
                const int raw = base + (lane & 15), it = min(raw, n_item - 1);
                const int m = it / item_per_row, v = it - m * item_per_row, lt = v >> 3;
                const bool live = raw < n_item && lt < sub && lt < ntile;
                const int col = (kt0 + min(lt, ntile - 1)) * 32 + (v & 7) * 4;
                const size_t off = (size_t)(m_base + m) * g.kd + col;
                const floatx4 xa = *reinterpret_cast<const floatx4 *>(g.xin + off);
                floatx4 sa[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    sa[q] = *reinterpret_cast<const floatx4 *>(g.ys + (size_t)min(grp * 4 + q, np - 1) * g.ys_stride + off);
                const uint2 gw = *reinterpret_cast<const uint2 *>(g.gain + col);
                floatx4 t = grp == 0 ? xa : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool on = grp * 4 + q < g.n_partial;   // a select: the unused re-read may hold anything
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] += on ? sa[q][e] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    t[e] += __shfl_xor(t[e], 16, 64);
                    t[e] += __shfl_xor(t[e], 32, 64);
                }
                bf16_t h[4], l[4];
                split2(t[0] * __uint_as_float(gw.x << 16), h[0], l[0]);
                split2(t[1] * __uint_as_float(gw.x & 0xffff0000u), h[1], l[1]);
                split2(t[2] * __uint_as_float(gw.y << 16), h[2], l[2]);
                split2(t[3] * __uint_as_float(gw.y & 0xffff0000u), h[3], l[3]);
                if (live) {
                    unsigned char *d = dst + (size_t)m * pitch + v * 8;
                    if (grp == 0) *reinterpret_cast<uint2 *>(d) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                    if (grp == 1) *reinterpret_cast<uint2 *>(d + plane_bytes) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
                    if (grp == 2 && blockIdx.x == 0) *reinterpret_cast<floatx4 *>(g.xout + off) = t;
                }
                if (grp == 3 && raw < n_item) ssq[raw] = live ? (t[0] * t[0] + t[1] * t[1]) + (t[2] * t[2] + t[3] * t[3]) : 0.f;
            }
            return;
        }
        for (int i = tid; i < WK * per_wk; i += NTH) {
            const int w = i / per_wk, rem = i - w * per_wk, m = rem / vec_per_row, v = rem - m * vec_per_row;
            const int lt = ch * kcw + (v >> 2), kt = w * sub + lt;          // tile within the slice / the workgroup range
            if (lt < sub && kt < ntile) {
                unsigned char *d = dst + (size_t)w * wk_bytes + (size_t)m * pitch + v * 16;
                if (PRO == PRO_ATTN) {
                    // eight consecutive features of one head (head_dim 128) of row m_base + m
                    const int col = (kt0 + kt) * 32 + (v & 3) * 8, head = col >> 7, dd = col & 127;
                    float ms[WS_PRO_SPLITS], ls[WS_PRO_SPLITS];
                    floatx4 oa[WS_PRO_SPLITS], ob[WS_PRO_SPLITS];
#pragma unroll
                    for (int sp = 0; sp < WS_PRO_SPLITS; ++sp) {   // splits past the last re-read it and weigh zero
                        const size_t row = ((size_t)min(sp, g.att_splits - 1) * g.att_rows + m_base + m) * g.att_H + head;
                        ms[sp] = g.att_m[row];
                        ls[sp] = g.att_l[row];
                        oa[sp] = *reinterpret_cast<const floatx4 *>(g.att_o + row * 128 + dd);
                        ob[sp] = *reinterpret_cast<const floatx4 *>(g.att_o + row * 128 + dd + 4);
                    }
                    float mx = -INFINITY;
#pragma unroll
                    for (int sp = 0; sp < WS_PRO_SPLITS; ++sp) mx = fmaxf(mx, sp < g.att_splits ? ms[sp] : -INFINITY);
                    float den = 0.f, num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int sp = 0; sp < WS_PRO_SPLITS; ++sp) {
                        const bool on = sp < g.att_splits && ms[sp] != -INFINITY;
                        const float wgt = on ? exp2f(ms[sp] - mx) : 0.f;   // the maxima are in units of ln 2
                        den = fmaf(wgt, on ? ls[sp] : 0.f, den);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            num[e] = fmaf(wgt, on ? oa[sp][e] : 0.f, num[e]);
                            num[4 + e] = fmaf(wgt, on ? ob[sp][e] : 0.f, num[4 + e]);
                        }
                    }
                    uint32_t hw[4], lw[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        bf16_t h0, l0, h1, l1;
                        split2(num[2 * e] / den, h0, l0);
                        split2(num[2 * e + 1] / den, h1, l1);
                        hw[e] = h0 | ((uint32_t)h1 << 16);
                        lw[e] = l0 | ((uint32_t)l1 << 16);
                    }
                    *reinterpret_cast<uint4 *>(d) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                    *reinterpret_cast<uint4 *>(d + plane_bytes) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                } else {
                    const size_t off = (size_t)(m_base + m) * g.kd + (size_t)(kt0 + kt) * 32 + (v & 3) * 8;
                    *reinterpret_cast<uint4 *>(d) = *reinterpret_cast<const uint4 *>(g.Xhi + off);
                    *reinterpret_cast<uint4 *>(d + plane_bytes) = *reinterpret_cast<const uint4 *>(g.Xlo + off);
                }
            }
        }
    };
    const int bj = lane & 15, bg = lane >> 4;
    // B operands of one k-tile: lanes whose row does not exist read row Mt - 1 and are zeroed (no branch)
    auto mfma_tile = [&](const unsigned char *buf, int lt, const u32x4 *a) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = t * 16 + bj;
            const unsigned char *p = buf + (size_t)min(m, Mt - 1) * pitch + (lt * 32 + bg * 8) * 2;
            uint4 bh = *reinterpret_cast<const uint4 *>(p);
            uint4 bl = *reinterpret_cast<const uint4 *>(p + plane_bytes);
            if (m >= Mt) { bh = make_uint4(0, 0, 0, 0); bl = bh; }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                u32x4 av = a[r];
                acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&av),
                                                                   *reinterpret_cast<bf16x8 *>(&bh), acc[r][t], 0, 0, 0);
                acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<bf16x8 *>(&av),
                                                                   *reinterpret_cast<bf16x8 *>(&bl), acc[r][t], 0, 0, 0);
            }
        }
    };
    // EPI_SWIGLU after a folded RMSNorm: 1 / rms of every row from the partial sums of squares the producer left.
    // Wave w takes rows w, w + waves, ..; its loads go out before the staging loads and are reduced after them
    // (lane-strided sums in index order, then a fixed shuffle tree).
    __shared__ float s_inv[16 * NT];
    float ssv[4] = {0.f, 0.f, 0.f, 0.f};
    const bool scale_rows = EPI == EPI_SWIGLU && g.ss_in != nullptr;
    if (scale_rows && wave < Mt) {
#pragma unroll
        for (int q = 0; q < 4; ++q) ssv[q] = g.ss_in[(size_t)min(lane + 64 * q, g.n_ss_in - 1) * g.M + m_base + wave];
    }
    stage(0);
    if (scale_rows) {
        for (int r = wave; r < Mt; r += NTH / 64) {
            float v = 0.f;
            if (r == wave) {   // the first row's partial sums are already here
#pragma unroll
                for (int q = 0; q < 4; ++q) v += lane + 64 * q < g.n_ss_in ? ssv[q] : 0.f;
                for (int p = lane + 256; p < g.n_ss_in; p += 64) v += g.ss_in[(size_t)p * g.M + m_base + r];
            } else {
                for (int p = lane; p < g.n_ss_in; p += 64) v += g.ss_in[(size_t)p * g.M + m_base + r];
            }
            v = wave_sum(v);
            if (lane == 0) s_inv[r] = 1.0f / sqrtf(v / (float)g.kd + g.rms_eps);
        }
    }
    for (int ch = 0; ch < nchunk; ++ch) {
        __syncthreads();   // chunk ch is staged; everyone is done with the buffer chunk ch + 1 goes to
        if (PRO == PRO_NORM && blockIdx.x == 0 && wave == 0) {
            // sum of v^2 of every row over this k-range: the items of a row in index order, lanes then a fixed tree
            const float *ssq = reinterpret_cast<const float *>(lds + 2 * buf_bytes);
            const int item_per_row = kcw * 8;
            for (int m = 0; m < Mt; ++m) {
                float q2 = 0.f;
                for (int i = lane; i < item_per_row; i += 64) q2 += ssq[m * item_per_row + i];
                q2 = wave_sum(q2);
                if (lane == 0) g.ss_out[(size_t)blockIdx.y * g.M + m_base + m] = q2;
            }
        }
        if (ch + 1 < nchunk) stage(ch + 1);
        if (!active) continue;
        const unsigned char *buf = lds + (size_t)(ch & 1) * buf_bytes + (size_t)wk * wk_bytes;
        const int kend = min(myn, (ch + 1) * kcw);
        int kt = ch * kcw;
        // steady state: U tiles consumed and U refills issued per pass, no conditionals in between
        for (; kt + U <= kend && kt + 2 * U <= myn; kt += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                mfma_tile(buf, kt + u - ch * kcw, abuf[u]);
                // the slot is free once its MFMAs have issued: refill it, and keep this order
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < RB; ++r) abuf[u][r] = __builtin_nontemporal_load(wp[r] + (size_t)(kt + u + U) * 64);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the last tiles of the slice (and slices shorter than 2 U): guarded
        for (; kt < kend; kt += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kt + u < kend) {
                    u32x4 a[RB];
#pragma unroll
                    for (int r = 0; r < RB; ++r) {
                        a[r] = abuf[u][r];
                        if (kt + u + U < myn) abuf[u][r] = __builtin_nontemporal_load(wp[r] + (size_t)(kt + u + U) * 64);
                    }
                    mfma_tile(buf, kt + u - ch * kcw, a);
                }
            }
        }
    }

    // ---- add the WK k-slices of each row-block group through LDS, in slice order
    if (WK > 1) {
        __syncthreads();
        floatx4 *red = reinterpret_cast<floatx4 *>(lds);
        if (wk > 0 && active) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    red[(((size_t)(wr * (WK - 1) + wk - 1) * RB + r) * NT + t) * 64 + lane] = acc[r][t];
        }
        __syncthreads();
        if (wk > 0 || !active) return;
        for (int s = 1; s < WK; ++s)
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[r][t] += red[(((size_t)(wr * (WK - 1) + s - 1) * RB + r) * NT + t) * 64 + lane];
    } else if (!active) {
        return;
    }

    ws_epilogue<NT, RB, EPI>(g, acc, m_base, rb0, blockIdx.y, blockIdx.x * WR + wr, lane, s_inv, res_x, res_g);
}

// ------------------------------------------------------------------------------------------ many rows
// The compute-bound regime (tens to hundreds of rows) uses the 32x32x16 MFMA, which sustains about 1.5 times
// the rate of the 16x16x32 one and needs half the B-operand bytes per flop.  Its A operand wants lane l to
// hold row l % 32 and the 8 k-values of slot l / 32.  Two vertically adjacent re-tiled row-blocks (lane l:
// row l % 16, k-group l / 16 of a 32-wide k-tile) hold two such operands - 32 weight rows with k-groups (0, 2)
// and (1, 3) - each lane of which is a 16-byte piece of one of the two tiles, so they are loaded directly in
// that order.  The activations are staged in LDS already split the same way: operand `op` of k-tile kt and
// 32-row tile t holds, at lane l, X[32 t + l % 32][32 kt + 8 op + 16 (l / 32) ..+8] - a wave stores and later
// reads a contiguous KiB.
//
// Eight waves, two per SIMD (a lone wave issues in order and leaves the matrix pipe idle while it issues
// anything else): WN x WM of them, a wave owns RP pairs of row-blocks of W, streamed straight into a ring of U
// register slots as above, and meets 32 NT rows of the workgroup's row tile.  Staging is double-buffered in chunks of KC k-tiles: the loads of chunk ch + 1 are
// issued before the MFMAs of chunk ch and written to LDS after them.  The 1-D grid is decoded so that the row
// tiles sharing a slice of W run on the same XCD at the same time (workgroup ids are dealt round-robin to the
// 8 XCDs): W then comes from HBM once and from that L2 afterwards.
typedef float floatx16 __attribute__((ext_vector_type(16)));
// acc[p][t][e] = Y[m = m_base + 32 t + lane % 32][row 8 (e / 4) + 4 (lane / 32) + e % 4 of the 32 rows that
// row-blocks rb0 + 2 p and rb0 + 2 p + 1 make]
template <int NT, int RP, int EPI>
__device__ __forceinline__ void mm_epilogue(const GemmArgs &g, floatx16 (&acc)[RP][NT], int m_base, int rb0, int split,
                                            int slot, int lane) {
    const int mj = lane & 31, h = lane >> 5;
    if (EPI == EPI_PARTIAL) {
        float *out = g.Yp + (size_t)split * g.split_stride;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + 32 * t + mj;
            if (m >= g.M) continue;
#pragma unroll
            for (int p = 0; p < RP; ++p)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int n = (rb0 + 2 * p) * 16 + 8 * v + 4 * h;
                    const floatx4 val = {acc[p][t][4 * v], acc[p][t][4 * v + 1], acc[p][t][4 * v + 2], acc[p][t][4 * v + 3]};
                    if (n + 3 < g.N && (g.N & 3) == 0) *reinterpret_cast<floatx4 *>(out + (size_t)m * g.N + n) = val;
                    else
                        for (int e = 0; e < 4; ++e)
                            if (n + e < g.N) out[(size_t)m * g.N + n + e] = val[e];
                }
        }
    } else if (EPI == EPI_SWIGLU) {
        // a row-block holds 8 gate rows over 8 up rows of the same features: this lane's registers 8 b + c and
        // 8 b + 4 + c are gate and up of feature 8 (rb0 + 2 p + b) + 4 h + c
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + 32 * t + mj;
            if (m >= g.M) continue;
#pragma unroll
            for (int p = 0; p < RP; ++p)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int f = (rb0 + 2 * p + b) * 8 + 4 * h;
                    float hv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gt = acc[p][t][8 * b + e], up = acc[p][t][8 * b + 4 + e];
                        hv[e] = gt / (1.0f + expf(-gt)) * up;
                    }
                    if (f + 3 < g.N && (g.N & 3) == 0) act_store4(g.H, (size_t)m * g.N + f, hv[0], hv[1], hv[2], hv[3]);
                    else
                        for (int e = 0; e < 4; ++e)
                            if (f + e < g.N) act_store(g.H, (size_t)m * g.N + f + e, hv[e]);
                }
        }
    } else {   // EPI_ARGMAX: best (value, lowest index) of this wave's 32 RP features for every row
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = m_base + 32 * t + mj;
            float best = -INFINITY;
            int idx = 0x7fffffff;
#pragma unroll
            for (int p = 0; p < RP; ++p)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int n = (rb0 + 2 * p) * 16 + 8 * (e / 4) + 4 * h + (e % 4);
                    const float v = acc[p][t][e];
                    if (n < g.N) {
                        if (g.Yp && m < g.M) g.Yp[(size_t)m * g.N + n] = v;
                        if (v > best || (v == best && n < idx)) { best = v; idx = n; }
                    }
                }
            const float ov = __shfl_xor(best, 32, 64);
            const int oi = __shfl_xor(idx, 32, 64);
            if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
            if (h == 0 && m < g.M) {
                g.cand_val[(size_t)m * g.n_cand + slot] = best;
                g.cand_idx[(size_t)m * g.n_cand + slot] = idx;
            }
        }
    }
}

// NT: 32-row tiles per wave; NW waves: WM along the rows, WK along k (each takes KC / WK of a chunk's k-tiles and
// the WK partial results are added through LDS at the end, in order), NW / (WM WK) along the row-blocks; RP: pairs
// of row-blocks per wave; KC: k-tiles per LDS chunk; U: register slots of a wave's weight stream
// NPL: 2 = activations as two bf16 terms (planes hi and lo, two MFMAs per operand pair); 1 = one half-precision term
// (plane X16 against half-precision weight tiles, one MFMA per pair: half the matrix-core work and half the staging)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
template <int NPL> __device__ __forceinline__ floatx16 mm_mfma(const u32x4 &a, const u32x4 &b, const floatx16 &c) {
    if (NPL == 2) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(&a), *reinterpret_cast<const bf16x8 *>(&b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const f16x8 *>(&a), *reinterpret_cast<const f16x8 *>(&b), c, 0, 0, 0);
}
template <int NT, int WM, int NW, int WK, int RP, int KC, int U, int EPI, int NPL, bool DEEP = false, bool WEAVE = false>
__global__ __launch_bounds__(64 * NW) void k_gemm_mm(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char lds[];
    static_assert(KC % WK == 0, "every k-slice takes the same number of k-tiles of a chunk");
    constexpr int KW = KC / WK;                           // k-tiles of a chunk one wave multiplies
    static_assert(U % KW == 0, "a turn of the ring is a whole number of chunks");
    constexpr int WN = NW / (WM * WK), RB = 2 * RP;
    constexpr int NTW = NT * WM;                          // 32-row tiles of the workgroup
    constexpr int OPS = KC * NTW * 2;                     // B operands of one plane in a chunk
    constexpr int PER_WAVE = (NPL * OPS + NW - 1) / NW;   // operand loads a wave issues per chunk (all planes)
    constexpr int BUF = NPL * OPS * 1024;                 // bytes of one chunk buffer
    constexpr int G = 2 * NPL;                            // operand groups (op, plane) of a k-tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wn = wave / (WM * WK), wm = wave % WM;
    const int wk = WK == 1 ? 0 : __builtin_amdgcn_readfirstlane((wave / WM) % WK);
    // ---- which (row-block group bx, k-split by, row tile z)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int z = slot % g.gz, q = (slot / g.gz) * 8 + xcd;
    if (q >= g.gx * g.gs) return;                         // the whole workgroup leaves: no barrier is reached
    const int bx = q % g.gx, by = q / g.gx;
    const int kt0 = by * g.kt_per_split;
    const int ntile = min(g.kt_per_split, g.nkt - kt0);
    const int rb0 = (bx * WN + wn) * RB;
    const bool active = rb0 < g.nrb;                      // RB divides the padded number of row-blocks
    const int m_base = z * (32 * NTW);

    // A operands straight from the re-tiled W: lane l of operand `op` of pair p wants row l % 32 of the pair and
    // k-group 2 (l / 32) + op, which row-block rb0 + 2 p + (l % 32) / 16 keeps at lane 16 (2 (l / 32) + op) + l % 16.
    // A wave-wide load then reads four contiguous 256-byte runs, and the two operands of a pair together read
    // both of its tiles exactly once.  Waves that differ only in wm stream the same row-blocks: the second one
    // finds them in the vector L1.
    const u32x4 *wp = g.Wt + ((size_t)((active ? rb0 : 0) + ((lane & 31) >> 4)) * g.nkt + kt0) * 64 + 32 * (lane >> 5) + (lane & 15);
    const size_t wstep = (size_t)2 * g.nkt * 64;          // from one pair of row-blocks to the next
    u32x4 abuf[U][RP][2];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int p = 0; p < RP; ++p)
#pragma unroll
            for (int op = 0; op < 2; ++op)   // a slot past the last k-tile re-reads that tile and is never used
                abuf[u][p][op] = wp[p * wstep + (size_t)min((u / KW) * KC + wk * KW + u % KW, ntile - 1) * 64 + 16 * op];

    floatx16 acc[RP][NT];
#pragma unroll
    for (int p = 0; p < RP; ++p)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[p][t][e] = 0.f;

    // ---- staging: operand id i in [0, 2 OPS): plane i / OPS, then (k-tile, row tile, op) = ((i % OPS) / (2 NTW),
    //      ((i % OPS) / 2) % NTW, i % 2); wave w takes ids w, w + NW, ...  No load is conditional (a branch would
    //      make the compiler wait for each one at once): rows past M re-read row M - 1, k-tiles past the end
    //      re-read the last one; neither is ever used.
    static_assert((NPL * OPS) % NW == 0, "every wave stages the same number of operands");
    const int srow = m_base + (lane & 31);
    const int scol = (lane >> 5) * 16;
    constexpr int TURN = U / KW;   // chunks per turn of the ring
    constexpr int SD = DEEP ? TURN : 1;   // chunks of activations in flight
    u32x4 sreg[SD][PER_WAVE];
#define WISV_MM_STAGE_LOAD(ch, S)                                                                                   \
    _Pragma("unroll") for (int j = 0; j < PER_WAVE; ++j) {                                                         \
        const int i = wave + NW * j, pl = i / OPS, rem = i % OPS, lt = rem / (2 * NTW), t = (rem / 2) % NTW, op = rem & 1; \
        const int kt = min((ch) * KC + lt, ntile - 1);                                                             \
        const int row = min(srow + 32 * t, g.M - 1);                                                               \
        sreg[S][j] = *reinterpret_cast<const u32x4 *>((NPL == 1 ? g.X16 : pl ? g.Xlo : g.Xhi) + (size_t)row * g.kd +  \
                                                   (size_t)(kt0 + kt) * 32 + 8 * op + scol);                       \
    }
#define WISV_MM_STAGE_STORE(ch, S)                                                                                  \
    _Pragma("unroll") for (int j = 0; j < PER_WAVE; ++j)                                                           \
        *reinterpret_cast<u32x4 *>(lds + (size_t)((ch) & 1) * BUF + (size_t)(wave + NW * j) * 1024 + lane * 16) = sreg[S][j];
    // A k-tile is G groups (op, plane) of NT B operands, each feeding NT RP independent MFMAs.  The B
    // operands of group gi + 1 are read from LDS before the MFMAs of group gi issue (scheduling barriers keep
    // that order): the LDS latency hides behind matrix work, the other wave of the SIMD fills what is left.
    // WEAVE asks the scheduler to place those reads between the MFMAs instead (one read after every RP of them),
    // and reads the first group of the chunk's next k-tile the same way: the matrix pipe does not drain while
    // eight reads issue.  Measured gain only for the widest products without k-splits (512 rows: gate/up
    // 142 -> 135 us; the down projection and 96-row gate/up lose 3 %).
    // group og of k-tile lt: plane og % NPL, operand og / NPL
#define WISV_MM_READ_B(lt, og, DST)                                                                                \
    _Pragma("unroll") for (int t = 0; t < NT; ++t)                                                                 \
        DST[t] = *reinterpret_cast<const u32x4 *>(buf + ((((og) % NPL) * OPS) + (((lt) * NTW + t) * 2 + (og) / NPL)) * 1024);
#define WISV_MM_GROUP(og, A, SRC)                                                                                  \
    _Pragma("unroll") for (int t = 0; t < NT; ++t) _Pragma("unroll") for (int p = 0; p < RP; ++p)                  \
        acc[p][t] = mm_mfma<NPL>(A[p][(og) / NPL], SRC[t], acc[p][t]);
    u32x4 bv[2][NT];

    // One chunk: CC (a compile-time number) places it in a turn of the weight ring, which spans U / KC chunks.
    // The next chunk's activations are requested before this chunk's MFMAs and written to LDS after them; the
    // write must wait for exactly these loads while the weight refills issued after them stay in flight, and
    // the compiler can count those only if every path through the chunk issues the same number of loads.
    // Loads complete in order, so that wait also ends every weight refill issued before them, which caps the ring
    // at about one chunk whatever U is.  DEEP keeps as many chunks of activations in flight as the ring has
    // (requested right after the previous occupant of their registers went to LDS, a whole turn before they are
    // written): the wait then ends only refills that are due in the same chunk anyway.
#define WISV_MM_CHUNK(ch, CC)                                                                                      \
    {                                                                                                              \
        __syncthreads(); /* chunk ch is in LDS; nobody still reads the buffer chunk ch + 1 goes to */             \
        /* this wave's row tiles start at tile wm NT of the workgroup's */                                        \
        const unsigned char *buf = lds + (size_t)((ch) & 1) * BUF + (size_t)(wm * NT) * 2048 + lane * 16;          \
        const int kbase = (ch) * KC;                                                                               \
        if (!DEEP) { WISV_MM_STAGE_LOAD((ch) + 1, 0) }                                                             \
        _Pragma("unroll") for (int lw = 0; lw < KW; ++lw) {                                                        \
            const int lt = wk * KW + lw; /* this wave's k-tile of the chunk */                                    \
            if (kbase + lt < ntile) { /* uniform per wave; no load inside, so the load counts hold on every path */ \
                if (!WEAVE || lw == 0) {                                                                           \
                    WISV_MM_READ_B(lt, 0, bv[0])                                                                   \
                    if (WEAVE) __builtin_amdgcn_sched_barrier(0);                                                  \
                }                                                                                                  \
                _Pragma("unroll") for (int og = 0; og < G; ++og) {                                                 \
                    if (og < G - 1) { WISV_MM_READ_B(lt, og + 1, bv[(og + 1) & 1]) }                               \
                    else if (WEAVE && lw + 1 < KW) { WISV_MM_READ_B(lt + 1, 0, bv[0]) }                            \
                    if (!WEAVE) __builtin_amdgcn_sched_barrier(0);                                                 \
                    WISV_MM_GROUP(og, abuf[(CC) * KW + lw], bv[og & 1])                                            \
                    if (WEAVE && (og < G - 1 || lw + 1 < KW)) {                                                    \
                        /* one LDS read of the next group after every RP matrix instructions of this one */       \
                        _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                           \
                            __builtin_amdgcn_sched_group_barrier(0x008, RP, 0);                                    \
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                     \
                        }                                                                                          \
                    }                                                                                              \
                    __builtin_amdgcn_sched_barrier(0);                                                             \
                }                                                                                                  \
            }                                                                                                      \
            /* refill the slot right after its use; past the end the last tile is re-read into a slot nobody uses */ \
            _Pragma("unroll") for (int p = 0; p < RP; ++p) _Pragma("unroll") for (int op = 0; op < 2; ++op)        \
                abuf[(CC) * KW + lw][p][op] = wp[p * wstep + (size_t)min(kbase + lt + TURN * KC, ntile - 1) * 64 + 16 * op]; \
            __builtin_amdgcn_sched_barrier(0);                                                                     \
        }                                                                                                          \
        WISV_MM_STAGE_STORE((ch) + 1, DEEP ? ((CC) + 1) % TURN : 0)                                                \
        if (DEEP) { WISV_MM_STAGE_LOAD((ch) + 1 + TURN, ((CC) + 1) % TURN) }                                       \
    }

    const int nchunk = (ntile + KC - 1) / KC;
    if (DEEP) {
#pragma unroll
        for (int cc = 0; cc < TURN; ++cc) { WISV_MM_STAGE_LOAD(cc, cc) }
        WISV_MM_STAGE_STORE(0, 0)
        WISV_MM_STAGE_LOAD(TURN, 0)
    } else {
        WISV_MM_STAGE_LOAD(0, 0)
        WISV_MM_STAGE_STORE(0, 0)
    }
    int ch = 0;
    for (; ch + TURN <= nchunk; ch += TURN) {   // whole turns: no branch around any load
#pragma unroll
        for (int cc = 0; cc < TURN; ++cc) WISV_MM_CHUNK(ch + cc, cc)
    }
#pragma unroll
    for (int cc = 0; cc < TURN - 1; ++cc)       // the last, partial turn
        if (ch + cc < nchunk) WISV_MM_CHUNK(ch + cc, cc)
#undef WISV_MM_CHUNK
#undef WISV_MM_STAGE_LOAD
#undef WISV_MM_STAGE_STORE
#undef WISV_MM_READ_B
#undef WISV_MM_GROUP
    if (WK > 1) {
        // the k-slices of a tile are added in slice order through LDS (the staging buffers are free after a barrier)
        floatx4 *red = reinterpret_cast<floatx4 *>(lds);   // [WN WM][RP][NT][4][64]
        const int grp = wn * WM + wm;
        for (int sl = 1; sl < WK; ++sl) {
            __syncthreads();
            if (wk == sl) {
#pragma unroll
                for (int p = 0; p < RP; ++p)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            red[((((size_t)grp * RP + p) * NT + t) * 4 + e) * 64 + lane] =
                                floatx4{acc[p][t][4 * e], acc[p][t][4 * e + 1], acc[p][t][4 * e + 2], acc[p][t][4 * e + 3]};
            }
            __syncthreads();
            if (wk == 0) {
#pragma unroll
                for (int p = 0; p < RP; ++p)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const floatx4 v = red[((((size_t)grp * RP + p) * NT + t) * 4 + e) * 64 + lane];
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[p][t][4 * e + c] += v[c];
                        }
            }
        }
        if (wk != 0) return;
    }
    if (!active) return;
    mm_epilogue<NT, RP, EPI>(g, acc, m_base + wm * (32 * NT), rb0, by, bx * WN + wn, lane);
}

// final argmax over the per-group candidates of every row
__global__ __launch_bounds__(1024) void k_argmax_cand(const float *__restrict__ val, const int32_t *__restrict__ idxs, int n_cand,
                                                     int stride, int32_t *amax) {
    __shared__ float bv[16];
    __shared__ int bi[16];
    const int m = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    // four candidates per pass, all loads first (slots past the end re-read the last one: same value, same index)
    for (int i0 = tid; i0 < n_cand; i0 += 4096) {
        float v[4];
        int n[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + 1024 * u, n_cand - 1);
            v[u] = val[(size_t)m * stride + i];
            n[u] = idxs[(size_t)m * stride + i];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (v[u] > best || (v[u] == best && n[u] < idx)) { best = v[u]; idx = n[u]; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    if ((tid & 63) == 0) { bv[tid >> 6] = best; bi[tid >> 6] = idx; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        amax[m] = idx == 0x7fffffff ? 0 : idx;
    }
}

// ------------------------------------------------------------------------------------------ launch
// LDS bytes: activation chunk (two planes, WK slices; two buffers when a slice needs several chunks),
// or the slice-reduction scratch if that is larger
static size_t ws_lds(int Mt, int kcw, int sub, int NT, int RB, int WR, int WK) {
    const size_t x = (size_t)(sub > kcw ? 2 : 1) * 2 * WK * Mt * (kcw * 64 + 16);
    const size_t red = (size_t)WR * (WK - 1) * RB * NT * 1024;
    return std::max(x, red);
}

template <int NT, int RB, int WR, int WK, int U, int EPI, int PRO = PRO_NONE>
static bool launch_ws_t(Ctx *c, GemmArgs &g, int splits, size_t soft_budget) {
    const int sub = (g.kt_per_split + WK - 1) / WK, Mt = std::min(g.M, 16 * NT);
    // largest chunk (a multiple of U) within the soft budget, else within what a CU has
    int kcw = (sub + U - 1) / U * U;
    for (size_t budget : {soft_budget, (size_t)150 * 1024}) {
        kcw = (sub + U - 1) / U * U;
        while (kcw > U && ws_lds(Mt, kcw, sub, NT, RB, WR, WK) > budget) kcw = (kcw / 2 + U - 1) / U * U;
        if (ws_lds(Mt, kcw, sub, NT, RB, WR, WK) <= budget) break;
    }
    size_t lds = ws_lds(Mt, kcw, sub, NT, RB, WR, WK);
    if (PRO == PRO_NORM) {
        // one chunk only (the row sums of squares are taken once), and room for one float per staged item behind
        // the two chunk buffers
        if (sub > kcw || WK != 1) return false;
        lds = (size_t)2 * 2 * Mt * (kcw * 64 + 16) + (size_t)Mt * kcw * 8 * 4;
    }
    if (lds > 150 * 1024) return false;
    g.kcw = kcw;
    static bool allowed[MAX_DEVICES];     // per instantiation
    if (lds > 64 * 1024 && !allow_big_lds(c, reinterpret_cast<const void *>(&k_gemm_ws<NT, RB, WR, WK, U, PRO, EPI>), allowed))
        return false;
    dim3 grid((g.nrb / RB + WR - 1) / WR, splits, (g.M + 16 * NT - 1) / (16 * NT));
    hipLaunchKernelGGL((k_gemm_ws<NT, RB, WR, WK, U, PRO, EPI>), grid, dim3(64 * WR * WK), lds, c->stream, g);
    return true;
}

constexpr int MM_RP = 2;            // pairs of row-blocks per wave of k_gemm_mm
constexpr int MM_RB = 2 * MM_RP;

template <int NT, int WM, int NW, int WK, int KC, int U, int EPI, int NPL, bool DEEP = false, bool WEAVE = false>
static bool launch_mm_t(Ctx *c, GemmArgs &g, int splits) {
    constexpr int WN = NW / (WM * WK), NTW = NT * WM;
    g.gx = (g.nrb + WN * MM_RB - 1) / (WN * MM_RB);
    g.gz = (g.M + 32 * NTW - 1) / (32 * NTW);
    g.gs = splits;
    // two buffers, two planes, 2 operands per (k-tile, row tile); or the k-slice reduction: one accumulator set per tile group
    const size_t lds = std::max((size_t)2 * NPL * KC * NTW * 2 * 1024, WK > 1 ? (size_t)WN * WM * MM_RP * NT * 4096 : (size_t)0);
    static bool allowed[MAX_DEVICES];     // per instantiation
    if (lds > 64 * 1024 &&
        !allow_big_lds(c, reinterpret_cast<const void *>(&k_gemm_mm<NT, WM, NW, WK, MM_RP, KC, U, EPI, NPL, DEEP, WEAVE>), allowed))
        return false;
    const unsigned grid = (unsigned)((g.gx * g.gs + 7) / 8 * 8 * g.gz);
    hipLaunchKernelGGL((k_gemm_mm<NT, WM, NW, WK, MM_RP, KC, U, EPI, NPL, DEEP, WEAVE>), dim3(grid), dim3(64 * NW), lds, c->stream, g);
    return true;
}

// Workgroup shapes of k_gemm_mm.  Up to 64 rows: one row tile met by all eight waves (each 64 weight rows).
// Beyond: tiles of 128 rows, met by 4 x 2 waves (256 weight rows per workgroup, every weight tile loaded by two
// waves), or - "wide" - by 8 x 1 waves with four row tiles each (512 weight rows, half the L2 traffic per flop,
// but half as many workgroups), or - "narrow" - by 2 x 2 waves (128 weight rows; two workgroups share a CU).
// With k-splits wide pays when it still fills the chip (>= 200 workgroups) and a split keeps >= 24 k-tiles; without
// them the shape with the fewest rounds of workgroups, weighted by what a round of that shape costs, is taken.
// A product without k-splits over at most 64 rows and few row-blocks (gate/up) would fill a quarter of the chip
// that way: "k-slice" workgroups cover 128 weight rows only and their waves split each chunk's k-tiles among them
// (98.9 -> 50.5 us at 32 rows, 116.9 -> 76.8 us at 64).  Beyond 64 rows workgroups that narrow re-read the
// activations so often that the L2 fabric binds, and the shape gains nothing.
enum { MM_NARROW = 0, MM_NORMAL = 1, MM_WIDE = 2, MM_KSLICE = 3 };   // 2 x 2, 4 x 2, 8 x 1 waves for more than 64 rows
static int mm_layout(int rows, int nrb, int nkt, bool can_split, int max_splits) {
    if (!can_split && rows <= 64 && (nrb + 8 * MM_RB - 1) / (8 * MM_RB) < 200) return MM_KSLICE;
    // Products with k-splits over at most 128 rows: every slice costs rows x n floats to write and to read back, so
    // narrow workgroups that need fewer splits to fill the chip win: k-slice workgroups up to 64 rows (32 rows at
    // the 8B shape: round 5.07 -> 4.63 ms, 64 rows: 5.89 -> 5.59), 2 x 2 waves beyond (96 rows: 7.10 -> 6.63 ms).
    if (can_split && rows <= 64) return MM_KSLICE;
    if (can_split && rows <= 128) return MM_NARROW;
    if (rows <= 64) return MM_NORMAL;
    const int tiles = (rows + 127) / 128;
    const int base8 = ((nrb + 8 * MM_RB - 1) / (8 * MM_RB)) * tiles, base4 = ((nrb + 4 * MM_RB - 1) / (4 * MM_RB)) * tiles;
    if (!can_split) {
        // A workgroup takes about the same time however many of them run, so the cost is rounds of 256 workgroups
        // times the time of one round, measured on gate/up at the 8B shape: wide 118 us (512 rows), 4 x 2 waves
        // 88 us (256 rows), narrow 67 us (128 rows).  384 rows: 336 workgroups of 4 x 2 waves took 154 us where 168
        // wide ones take one round.
        const int base2 = ((nrb + 2 * MM_RB - 1) / (2 * MM_RB)) * tiles;
        const double c8 = (base8 + 255) / 256 * 1.34, c4 = (base4 + 255) / 256 * 1.0, c2 = (base2 + 255) / 256 * 0.76;
        return c8 <= c4 && c8 <= c2 ? MM_WIDE : c4 <= c2 ? MM_NORMAL : MM_NARROW;
    }
    const int s = std::max(1, std::min(256 / std::max(1, base8), max_splits));
    return base8 * s >= 200 && nkt / s >= 24 ? MM_WIDE : MM_NORMAL;
}

// returns the number of row tiles and of row-blocks a workgroup covers
static int mm_shape(int rows, int layout, int *rb_per_wg) {
    if (layout == MM_KSLICE) {
        *rb_per_wg = 2 * MM_RB;
        return 1;
    }
    *rb_per_wg = (rows <= 64 || layout == MM_WIDE ? 8 : layout == MM_NORMAL ? 4 : 2) * MM_RB;
    return rows <= 64 ? 1 : (rows + 127) / 128;
}

// More than 16 rows: k_gemm_mm
template <int EPI, int NPL> static bool launch_ws_many_t(Ctx *c, GemmArgs &g, int splits, int layout) {
    if (layout == MM_KSLICE) {   // 2 row-block groups x 4 k-slices
        if (g.M <= 32) return launch_mm_t<1, 1, 8, 4, 4, 4, EPI, NPL>(c, g, splits);
        if (g.M <= 64) return launch_mm_t<2, 1, 8, 4, 4, 4, EPI, NPL>(c, g, splits);
        if (g.M <= 96) return launch_mm_t<3, 1, 8, 4, 4, 4, EPI, NPL>(c, g, splits);
        return launch_mm_t<4, 1, 8, 4, 4, 4, EPI, NPL>(c, g, splits);
    }
    if (g.M <= 32) {   // one row tile, one plane: chunks of four k-tiles give every wave an operand to stage
        if (NPL == 1) return launch_mm_t<1, 1, 8, 1, 4, 4, EPI, NPL>(c, g, splits);
        return launch_mm_t<1, 1, 8, 1, 2, 2, EPI, 2>(c, g, splits);
    }
    if (g.M <= 64) return launch_mm_t<2, 1, 8, 1, 2, 2, EPI, NPL>(c, g, splits);
    if (layout == MM_WIDE) {
        if (EPI != EPI_PARTIAL) return launch_mm_t<4, 1, 8, 1, 2, 2, EPI, NPL, false, true>(c, g, splits);
        return launch_mm_t<4, 1, 8, 1, 2, 2, EPI, NPL>(c, g, splits);
    }
    if (layout == MM_NARROW) {
        // gate/up (no k-split, 65 to 128 rows) streams the most weights per workgroup: a ring of two chunks with the
        // activations staged as deep (96 rows: 72.8 -> 65.8 us; the split products measured no gain from it)
        if (EPI == EPI_SWIGLU) return launch_mm_t<2, 2, 4, 1, 2, 4, EPI, NPL, true>(c, g, splits);
        return launch_mm_t<2, 2, 4, 1, 2, 2, EPI, NPL>(c, g, splits);
    }
    return launch_mm_t<2, 2, 8, 1, 2, 2, EPI, NPL>(c, g, splits);
}
// Wh: the half-precision tiles, or null for the two-term product on the bf16 tiles already in g.Wt
template <int EPI> static bool launch_ws_many(Ctx *c, GemmArgs &g, int splits, int layout, const void *Wh) {
    if (Wh && g.X16) {
        g.Wt = (const u32x4 *)Wh;
        return launch_ws_many_t<EPI, 1>(c, g, splits, layout);
    }
    return launch_ws_many_t<EPI, 2>(c, g, splits, layout);
}

bool ws_supported(const Ctx *c, int rows, int kd) {
    return c->bf16 && kd % 32 == 0 && rows >= 1;
}

static void fill_args(GemmArgs &g, const void *Wt, const ActBuf &X, int rows, int n, int kd) {
    g.Wt = (const u32x4 *)Wt;
    g.Xhi = X.hi; g.Xlo = X.lo; g.X16 = X.h16;
    g.M = rows; g.N = n; g.kd = kd;
    g.nrb = ws_padded_row_blocks(n); g.nkt = kd / 32;
}

// Y partial slices: returns the number of slices written to `Yp` ([S][split_stride]), 0 if the shape cannot
// be served (nothing was launched)
int launch_gemm_ws_partial(Ctx *c, const void *Wt, const ActBuf &X, float *Yp, size_t split_stride, int max_splits,
                           int rows, int n, int kd, int kclass, const AttnPartials *ap, const void *Wh) {
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, X, rows, n, kd);
    g.Yp = Yp; g.split_stride = split_stride;
    int s;
    int layout = MM_NORMAL;
    if (rows <= 16) {
        // one row-block per wave: split k until about 6144 waves stream (three workgroups per CU), a wave keeps
        // at least 8 k-tiles
        s = (6144 + g.nrb - 1) / g.nrb;
        s = std::max(1, std::min(s, std::min(max_splits, std::max(1, g.nkt / 8))));
    } else {
        // about one workgroup per CU over (row-block groups) x (row tiles) x splits; a split keeps >= 8 k-tiles
        int rb_per_wg;
        layout = mm_layout(rows, g.nrb, g.nkt, true, std::min(max_splits, std::max(1, g.nkt / 8)));
        const int tiles = mm_shape(rows, layout, &rb_per_wg);
        const int base = ((g.nrb + rb_per_wg - 1) / rb_per_wg) * tiles;
        s = std::max(1, std::min(256 / std::max(1, base), std::min(max_splits, std::max(1, g.nkt / 8))));
    }
    g.kt_per_split = (g.nkt + s - 1) / s;
    const int splits = (g.nkt + g.kt_per_split - 1) / g.kt_per_split;
    if (ap) {   // the activations are the attention output, still in k-split partials
        if (rows > 16 || ap->splits < 1 || ap->splits > WS_PRO_SPLITS || kd != ap->heads * 128) return 0;
        g.att_o = ap->o; g.att_m = ap->m; g.att_l = ap->l;
        g.att_splits = ap->splits; g.att_rows = ap->rows; g.att_H = ap->heads;
        return launch_ws_t<1, 1, 8, 1, 4, EPI_PARTIAL, PRO_ATTN>(c, g, splits, 40 * 1024) ? splits : 0;
    }
    const bool ok = rows <= 16 ? launch_ws_t<1, 1, 8, 1, 4, EPI_PARTIAL>(c, g, splits, 40 * 1024)
                               : launch_ws_many<EPI_PARTIAL>(c, g, splits, layout, Wh);
    return ok ? splits : 0;
}

// The product that opens a block, with the block's RMSNorm folded in (at most 16 rows): the kernel adds the previous
// product's n_partial slices (c->y) to the residual stream x_in while it stages it, writes the sum to x_out, feeds
// x * gain to the matrix cores and leaves the sum of squares of every row in ss[split][row]; whoever adds this
// product's slices multiplies by 1 / sqrt(sum ss / kd + eps).  Returns the number of slices, 0 if the shape is not
// served (nothing was launched).
int launch_gemm_ws_normfold(Ctx *c, const void *Wt, const float *x_in, float *x_out, int n_partial, const void *gain,
                            float *Yp, size_t split_stride, int max_splits, int rows, int n, int kd, float *ss, int kclass) {
    if (rows > 16 || n_partial > MAX_SPLITS) return 0;
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, ActBuf{}, rows, n, kd);
    g.Yp = Yp; g.split_stride = split_stride;
    int s = (6144 + g.nrb - 1) / g.nrb;
    s = std::max(1, std::min(s, std::min(max_splits, std::max(1, g.nkt / 8))));
    g.kt_per_split = (g.nkt + s - 1) / s;
    const int splits = (g.nkt + g.kt_per_split - 1) / g.kt_per_split;
    g.xin = x_in; g.xout = x_out; g.ys = c->y; g.ys_stride = (size_t)c->rows_max * kd; g.n_partial = n_partial;
    g.gain = (const bf16_t *)gain; g.ss_out = ss;
    return launch_ws_t<1, 1, 8, 1, 4, EPI_PARTIAL, PRO_NORM>(c, g, splits, 40 * 1024) ? splits : 0;
}

// A product that closes a residual branch, complete inside one kernel (at most 16 rows): one row-block per
// workgroup, 16 waves split k among them and add their results through LDS, and the epilogue adds the residual
// stream, writes it back, writes x * gain as the next block's activations and the rows' partial sums of squares to
// ss[row-block][row] (see EPI_RESID).  `ap`: the activations are still the attention kernel's k-split partials.
// Returns the number of partial sums per row, 0 if the shape is not served (nothing was launched).
int launch_gemm_ws_resid(Ctx *c, const void *Wt, const ActBuf &X, const AttnPartials *ap, float *x, const void *gain,
                         const ActBuf &A_out, float *ss, int rows, int n, int kd, int kclass) {
    if (rows > 16 || n % 16 || (ap && (ap->splits < 1 || ap->splits > WS_PRO_SPLITS || kd != ap->heads * 128))) return 0;
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, X, rows, n, kd);
    g.kt_per_split = g.nkt;
    g.xin = x; g.xout = x; g.gain = (const bf16_t *)gain; g.H = A_out; g.ss_out = ss;
    if (ap) {
        g.att_o = ap->o; g.att_m = ap->m; g.att_l = ap->l;
        g.att_splits = ap->splits; g.att_rows = ap->rows; g.att_H = ap->heads;
        return launch_ws_t<1, 1, 1, 16, 4, EPI_RESID, PRO_ATTN>(c, g, 1, 150 * 1024) ? n / 16 : 0;
    }
    return launch_ws_t<1, 1, 1, 16, 4, EPI_RESID>(c, g, 1, 150 * 1024) ? n / 16 : 0;
}

// gate/up with the SwiGLU fused (single split): H[rows][F] = silu(gate) * up.  Every row-block of the
// re-tiled matrix holds 8 gate and 8 up rows.
bool launch_gemm_ws_swiglu(Ctx *c, const void *Wt, const ActBuf &X, const ActBuf &H, int rows, int features, int kd,
                           int kclass, const void *Wh, const float *ss, int n_ss, int planes) {
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, X, rows, features, kd);
    g.nrb = ws_padded_pair_blocks(features);
    g.kt_per_split = g.nkt;
    g.H = H;
    if (n_ss > 0) {   // X holds x * gain: the kernel scales by 1 / rms itself (the streaming kernel only)
        if (rows > 16) return false;
        g.ss_in = ss; g.n_ss_in = n_ss; g.rms_eps = c->cfg.rms_eps;
    }
    if (rows <= 16) {
        // no k-split here, so the workgroup count is fixed by the shape: seven waves per workgroup when that fills
        // whole rounds of 256 CUs better than eight (14336 features: 256 workgroups instead of 224)
        auto fill = [&](int wr) { const int wgs = (g.nrb + wr - 1) / wr; return (double)wgs / ((wgs + 255) / 256 * 256); };
        if (fill(7) > fill(8)) return launch_ws_t<1, 1, 7, 1, 16, EPI_SWIGLU>(c, g, 1, 36 * 1024);
        return launch_ws_t<1, 1, 8, 1, 16, EPI_SWIGLU>(c, g, 1, 36 * 1024);
    }
    // more than 16 rows: H has one consumer, the down projection, and `planes` names the representation it reads;
    // the others (at 512 rows 59 of 73 MB) are not written
    g.H = act_planes(g.H, planes);
    return launch_ws_many<EPI_SWIGLU>(c, g, 1, mm_layout(rows, g.nrb, g.nkt, false, 1), Wh);
}

// LM head with the argmax fused: greedy token of every row in c->amax; logits kept only on request
bool launch_gemm_ws_argmax(Ctx *c, const void *Wt, const ActBuf &X, float *logits, int rows, int n, int kd, int kclass,
                           const void *Wh) {
    GemmArgs g{};
    fill_args(g, Wt, X, rows, n, kd);
    g.kt_per_split = g.nkt;
    g.n_cand = g.nrb;                     // at most one candidate slot per row-block
    g.Yp = logits;
    g.cand_val = c->cand_val; g.cand_idx = c->cand_idx;
    const int slots = rows <= 16 ? g.nrb : (g.nrb + MM_RB - 1) / MM_RB;
    {
        ProfScope ps(c, kclass);
        const bool ok = rows <= 16 ? launch_ws_t<1, 1, 8, 1, 16, EPI_ARGMAX>(c, g, 1, 70 * 1024)
                                   : launch_ws_many<EPI_ARGMAX>(c, g, 1, mm_layout(rows, g.nrb, g.nkt, false, 1), Wh);
        if (!ok) return false;
    }
    {
        ProfScope ps(c, KC_ARGMAX);
        hipLaunchKernelGGL(k_argmax_cand, dim3(rows), dim3(1024), 0, c->stream, c->cand_val, c->cand_idx, slots, g.n_cand, c->amax);
    }
    return true;
}

}  // namespace wisv
