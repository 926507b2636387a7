// Weight-streaming bf16 GEMM for a small number of activation rows (the memory-bound regime of the
// verify round: every weight byte is read once per round and meets at most a few dozen rows).
//
// Y[m, n] = sum_k X[m, k] W[n, k] is computed "swapped": the 16x16x32 MFMA takes a 16-row block of W as
// its A operand and 16 activation rows as its B operand, so the output-feature dimension fills the
// matrix core however few rows there are.  Activations arrive as float and are fed as two bf16 terms
// (x = hi + lo), one MFMA each: the products are then exact to about 2^-17 while the weights stay bf16;
// the second MFMA costs issue slots this memory-bound kernel has to spare.  W is stored re-tiled: tile (rb, kt) holds W[16rb..+16][32kt..+32]
// as 64 lanes x 8 bf16 in exactly the order the MFMA wants, so that one wave-wide 16-byte load fetches a
// contiguous KiB and a wave walking along k reads one contiguous stream.
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------ re-tiling
// out[((rb * nkt + kt) * 64 + lane) * 8 + e] = W[row(rb, lane % 16)][32 kt + 8 (lane / 16) + e]
// pair_rows > 0: W stacks two matrices of pair_rows rows each (gate over up); row-blocks alternate
// between them so that a wave owning blocks 2p and 2p+1 holds gate and up of the same 16 features.
__global__ void k_retile(const bf16_t *__restrict__ W, int n_rows, int kd, int nrb, int nkt, int pair_rows,
                         uint4 *__restrict__ out) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)nrb * nkt * 64) return;
    const int lane = idx & 63;
    const size_t tile = idx >> 6;
    const int kt = tile % nkt, rb = tile / nkt;
    int row;
    if (pair_rows > 0) row = (rb & 1) * pair_rows + (rb >> 1) * 16 + (lane & 15);
    else row = rb * 16 + (lane & 15);
    const bool valid = pair_rows > 0 ? ((rb >> 1) * 16 + (lane & 15)) < pair_rows : row < n_rows;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid) v = *reinterpret_cast<const uint4 *>(W + (size_t)row * kd + 32 * kt + 8 * (lane >> 4));
    out[idx] = v;
}

void launch_retile(Ctx *c, const void *W, int n_rows, int kd, int pair_rows, void *out, int nrb) {
    const int nkt = kd / 32;
    const size_t total = (size_t)nrb * nkt * 64;
    hipLaunchKernelGGL(k_retile, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, (const bf16_t *)W,
                       n_rows, kd, nrb, nkt, pair_rows, (uint4 *)out);
}

// ------------------------------------------------------------------------------------------ the GEMM
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2 };

struct GemmArgs {
    const u32x4 *Wt;      // re-tiled weights [nrb][nkt][64]
    const float *X;       // activations [M][kd], float: split into two bf16 terms while staged
    int M, N, kd, nrb, nkt, kt_per_split;
    int kc;               // k-tiles of X staged in LDS at a time (a multiple of the prefetch depth)
    float *Yp;            // EPI_PARTIAL: [S][m_stride][N];  EPI_ARGMAX with logits != null: [M][N]
    size_t split_stride;  // elements between consecutive split slices of Yp
    float *H;             // EPI_SWIGLU: [M][N/2]
    float *cand_val;      // EPI_ARGMAX: [M][n_cand]
    int32_t *cand_idx;
    int n_cand;
};

// NT: 16-row activation tiles held per wave; RB: row-blocks of W per wave; U: depth of the register prefetch.
// X is staged through LDS in chunks of g.kc k-tiles (double-buffered when there is more than one chunk).
template <int NT, int RB, int U, int EPI>
__global__ __launch_bounds__(256) void k_gemm_ws(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kt0 = blockIdx.y * g.kt_per_split;
    const int ntile = min(g.kt_per_split, g.nkt - kt0);
    const int rb0 = (blockIdx.x * 4 + wave) * RB;
    const bool active = rb0 < g.nrb;   // RB divides nrb by construction of the launch

    // ---- start the weight stream before anything else: it does not depend on the activations
    const u32x4 *wp[RB];
    u32x4 abuf[U][RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) wp[r] = g.Wt + ((size_t)(active ? rb0 + r : 0) * g.nkt + kt0) * 64 + lane;
    if (active) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (u < ntile) abuf[u][r] = __builtin_nontemporal_load(wp[r] + (size_t)u * 64);
    }

    floatx4 acc[RB][NT];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // ---- X chunk c (k-tiles [c kc, (c+1) kc) of this split) lives at lds + (c & 1) * buf_bytes as two
    //      bf16 planes: hi = bf16(x) at row m * pitch, lo = bf16(x - hi) at lo_off + m * pitch
    //      (x = hi + lo to 2^-17 relative); pitch = chunk bytes + 16 spreads rows over the banks
    const int kc = g.kc, pitch = kc * 64 + 16, lo_off = g.M * pitch, buf_bytes = 2 * lo_off;
    const int nchunk = (ntile + kc - 1) / kc;
    auto stage = [&](int ch) {
        unsigned char *dst = lds + (size_t)(ch & 1) * buf_bytes;
        const int tiles = min(kc, ntile - ch * kc), vec_per_row = tiles * 4;
        const float *src = g.X + (size_t)(kt0 + ch * kc) * 32;
        for (int i = tid; i < g.M * vec_per_row; i += 256) {
            const int m = i / vec_per_row, v = i - m * vec_per_row;
            const float4 x0 = *reinterpret_cast<const float4 *>(src + (size_t)m * g.kd + v * 8);
            const float4 x1 = *reinterpret_cast<const float4 *>(src + (size_t)m * g.kd + v * 8 + 4);
            const float xs[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bf16_t h0 = f32_to_bf16(xs[2 * e]), h1 = f32_to_bf16(xs[2 * e + 1]);
                const bf16_t l0 = f32_to_bf16(xs[2 * e] - bf16_to_f32(h0)), l1 = f32_to_bf16(xs[2 * e + 1] - bf16_to_f32(h1));
                hi[e] = h0 | ((uint32_t)h1 << 16);
                lo[e] = l0 | ((uint32_t)l1 << 16);
            }
            *reinterpret_cast<uint4 *>(dst + (size_t)m * pitch + v * 16) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<uint4 *>(dst + lo_off + (size_t)m * pitch + v * 16) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
    };
    const int bj = lane & 15, bg = lane >> 4;
    stage(0);
    for (int ch = 0; ch < nchunk; ++ch) {
        __syncthreads();   // chunk ch is staged; everyone is done with the buffer chunk ch + 1 goes to
        if (ch + 1 < nchunk) stage(ch + 1);
        if (!active) continue;
        const unsigned char *buf = lds + (size_t)(ch & 1) * buf_bytes;
        const int kend = min(ntile, (ch + 1) * kc);
        for (int kt = ch * kc; kt < kend; kt += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kt + u < kend) {
                    u32x4 a[RB];
#pragma unroll
                    for (int r = 0; r < RB; ++r) {
                        a[r] = abuf[u][r];
                        if (kt + u + U < ntile)
                            abuf[u][r] = __builtin_nontemporal_load(wp[r] + (size_t)(kt + u + U) * 64);
                    }
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const int m = t * 16 + bj;
                        uint4 bh = make_uint4(0, 0, 0, 0), bl = bh;
                        if (m < g.M) {
                            const unsigned char *p = buf + (size_t)m * pitch + ((kt + u - ch * kc) * 32 + bg * 8) * 2;
                            bh = *reinterpret_cast<const uint4 *>(p);
                            bl = *reinterpret_cast<const uint4 *>(p + lo_off);
                        }
#pragma unroll
                        for (int r = 0; r < RB; ++r) {
                            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                *reinterpret_cast<bf16x8 *>(&a[r]), *reinterpret_cast<bf16x8 *>(&bh), acc[r][t], 0, 0, 0);
                            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                *reinterpret_cast<bf16x8 *>(&a[r]), *reinterpret_cast<bf16x8 *>(&bl), acc[r][t], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }
    if (!active) return;

    // ---- epilogue.  acc[r][t][e] = Y[m = 16 t + lane % 16][n = 16 (rb0 + r) + 4 (lane / 16) + e]
    if (EPI == EPI_PARTIAL) {
        float *out = g.Yp + (size_t)blockIdx.y * g.split_stride;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = t * 16 + bj;
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
        // blocks rb0 + 2p hold gate, rb0 + 2p + 1 hold up of features 16 (rb0 / 2 + p) ..
        const int F = g.N / 2;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = t * 16 + bj;
            if (m >= g.M) continue;
#pragma unroll
            for (int pr = 0; pr < RB / 2; ++pr) {
                const int f = ((rb0 >> 1) + pr) * 16 + bg * 4;
                floatx4 hv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float gt = acc[2 * pr][t][e], up = acc[2 * pr + (RB > 1 ? 1 : 0)][t][e];
                    hv[e] = gt / (1.0f + expf(-gt)) * up;
                }
                if (f + 3 < F && (F & 3) == 0) *reinterpret_cast<floatx4 *>(g.H + (size_t)m * F + f) = hv;
                else
                    for (int e = 0; e < 4; ++e)
                        if (f + e < F) g.H[(size_t)m * F + f + e] = hv[e];
            }
        }
    } else {   // EPI_ARGMAX: best (value, lowest index) of this wave's 16*RB features for every row
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = t * 16 + bj;
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
                const int slot = blockIdx.x * 4 + wave;   // one slot per wave
                g.cand_val[(size_t)m * g.n_cand + slot] = best;
                g.cand_idx[(size_t)m * g.n_cand + slot] = idx;
            }
        }
    }
}

// final argmax over the per-wave candidates of every row
__global__ void k_argmax_cand(const float *__restrict__ val, const int32_t *__restrict__ idxs, int n_cand, int stride,
                              int32_t *amax) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int i = tid; i < n_cand; i += 256) {
        const float v = val[(size_t)m * stride + i];
        const int n = idxs[(size_t)m * stride + i];
        if (v > best || (v == best && n < idx)) { best = v; idx = n; }
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
        for (int w = 1; w < 4; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        amax[m] = idx == 0x7fffffff ? 0 : idx;
    }
}

// LDS bytes of the X staging (hi and lo planes) for a chunk of kc k-tiles (two buffers unless one chunk
// covers the split)
static size_t ws_lds(int M, int kc, int ntile) { return (size_t)(ntile > kc ? 2 : 1) * 2 * M * (kc * 64 + 16); }

// largest chunk (a multiple of the prefetch depth U) whose staging fits the LDS budget; 0 if none does
static int pick_kc(int M, int ntile, int U, size_t budget) {
    int kc = (ntile + U - 1) / U * U;
    while (kc > U && ws_lds(M, kc, ntile) > budget) kc = (kc / 2 + U - 1) / U * U;
    return ws_lds(M, kc, ntile) <= budget ? kc : 0;
}

// row-blocks are padded to a multiple of 4 so that a wave may own 1, 2 or 4 of them
int ws_padded_row_blocks(int n_rows) { return ((n_rows + 15) / 16 + 3) / 4 * 4; }

template <int NT, int RB, int EPI> static bool launch_ws_t(Ctx *c, GemmArgs &g, int splits) {
    constexpr int U = RB == 1 ? 8 : (RB == 2 ? 4 : 2);
    // small row counts stay within the default 64 KiB of dynamic LDS; more rows opt in to the CU's 160 KiB
    const size_t budget = NT <= 2 ? 60 * 1024 : 144 * 1024;
    g.kc = pick_kc(g.M, g.kt_per_split, U, budget);
    if (!g.kc) return false;
    const size_t lds = ws_lds(g.M, g.kc, g.kt_per_split);
    static bool opted_in = false;     // per instantiation
    if (lds > 64 * 1024 && !opted_in) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_ws<NT, RB, U, EPI>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return false;
        opted_in = true;
    }
    const int waves = g.nrb / RB;
    dim3 grid((waves + 3) / 4, splits);
    hipLaunchKernelGGL((k_gemm_ws<NT, RB, U, EPI>), grid, dim3(256), lds, c->stream, g);
    return true;
}

// few rows: one row-block per wave and a deep prefetch; many rows: more row-blocks per wave so that one
// LDS read of the activations serves several weight tiles
template <int EPI> static bool launch_ws_nt(Ctx *c, GemmArgs &g, int splits) {
    const int nt = (g.M + 15) / 16;
    constexpr int RS = EPI == EPI_SWIGLU ? 2 : 1;   // SwiGLU needs gate and up in the same wave
    switch (nt) {
        case 1: return launch_ws_t<1, RS, EPI>(c, g, splits);
        case 2: return launch_ws_t<2, 2, EPI>(c, g, splits);
        case 3: return launch_ws_t<3, 2, EPI>(c, g, splits);
        case 4: return launch_ws_t<4, 4, EPI>(c, g, splits);
        case 5: return launch_ws_t<5, 4, EPI>(c, g, splits);
        case 6: return launch_ws_t<6, 4, EPI>(c, g, splits);
        default: return false;
    }
}

static int rb_per_wave(int M, int epi) {
    const int nt = (M + 15) / 16;
    return nt == 1 ? (epi == EPI_SWIGLU ? 2 : 1) : (nt <= 3 ? 2 : 4);
}

// Number of k-splits: enough waves to keep every CU streaming, at least 8 k-tiles per split, and no
// more slices than the partial buffer holds.
static int pick_splits(int M, int nkt, int waves_per_split, int max_splits) {
    const int want_waves = M <= 16 ? 2048 : 1024;
    int s = (want_waves + waves_per_split - 1) / waves_per_split;
    s = std::min(s, std::min(max_splits, std::max(1, nkt / 8)));
    return std::max(s, 1);
}

bool ws_supported(const Ctx *c, int rows, int kd) {
    return c->bf16 && kd % 32 == 0 && rows <= 96;
}

static void fill_args(GemmArgs &g, const void *Wt, const void *X, int rows, int n, int kd) {
    g.Wt = (const u32x4 *)Wt;
    g.X = (const float *)X;
    g.M = rows; g.N = n; g.kd = kd;
    g.nrb = ws_padded_row_blocks(n); g.nkt = kd / 32;
}

// Y partial slices: returns the number of slices written to `Yp` ([S][split_stride]), 0 if the shape cannot
// be served (nothing was launched)
int launch_gemm_ws_partial(Ctx *c, const void *Wt, const void *X, float *Yp, size_t split_stride, int max_splits,
                           int rows, int n, int kd, int kclass) {
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, X, rows, n, kd);
    g.Yp = Yp; g.split_stride = split_stride;
    const int s = pick_splits(rows, g.nkt, g.nrb / rb_per_wave(rows, EPI_PARTIAL), max_splits);
    g.kt_per_split = (g.nkt + s - 1) / s;
    const int splits = (g.nkt + g.kt_per_split - 1) / g.kt_per_split;
    return launch_ws_nt<EPI_PARTIAL>(c, g, splits) ? splits : 0;
}

// gate/up with the SwiGLU fused (single split): H[rows][F] = silu(gate) * up.  The re-tiled matrix
// alternates gate and up row-blocks, 2 * padded(F) in all.
bool launch_gemm_ws_swiglu(Ctx *c, const void *Wt, const void *X, void *H, int rows, int two_f, int kd, int kclass) {
    ProfScope ps(c, kclass);
    GemmArgs g{};
    fill_args(g, Wt, X, rows, two_f, kd);
    g.nrb = 2 * ws_padded_row_blocks(two_f / 2);
    g.kt_per_split = g.nkt;
    g.H = (float *)H;
    return launch_ws_nt<EPI_SWIGLU>(c, g, 1);
}

// LM head with the argmax fused: greedy token of every row in c->amax; logits kept only on request
bool launch_gemm_ws_argmax(Ctx *c, const void *Wt, const void *X, float *logits, int rows, int n, int kd, int kclass) {
    GemmArgs g{};
    fill_args(g, Wt, X, rows, n, kd);
    g.kt_per_split = g.nkt;
    g.Yp = logits;
    g.cand_val = c->cand_val; g.cand_idx = c->cand_idx;
    g.n_cand = g.nrb;                     // at most one candidate slot per row-block
    const int slots = g.nrb / rb_per_wave(rows, EPI_ARGMAX);
    {
        ProfScope ps(c, kclass);
        if (!launch_ws_nt<EPI_ARGMAX>(c, g, 1)) return false;
    }
    {
        ProfScope ps(c, KC_ARGMAX);
        hipLaunchKernelGGL(k_argmax_cand, dim3(rows), dim3(256), 0, c->stream, c->cand_val, c->cand_idx, slots, g.n_cand, c->amax);
    }
    return true;
}

}  // namespace wisv
