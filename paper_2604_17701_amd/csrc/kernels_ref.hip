// Generic kernels of the verify round: one straightforward kernel per step, templated on the
// storage type (float or bf16) of weights / cache (WT) and of activations (AT; float in both paths).
// They serve the fp32 configuration and are the fallback wherever no specialised bf16 kernel
// applies (prefill chunks, unusual shapes).
#include "wisv_internal.h"

namespace wisv {

template <typename T> __device__ __forceinline__ void load8(const T *p, float *out);
template <> __device__ __forceinline__ void load8<float>(const float *p, float *out) {
    float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t *p, float *out) {
    uint4 a = *reinterpret_cast<const uint4 *>(p);
    uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// float sum over a block of NT threads (NT multiple of 64); every thread gets the result
template <int NT> __device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) t += red[w];
    return t;
}
template <int NT> __device__ __forceinline__ float block_max(float v, float *red) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) t = fmaxf(t, red[w]);
    return t;
}

// ------------------------------------------------------------------------------------------ rows
// row m = (stream b = m / k, position j = m % k): slot and absolute position L_b + j
__global__ void k_prep_rows(const int32_t *__restrict__ stream_ids, const int32_t *__restrict__ kv_len, int k,
                            int rows, int max_batch, int max_ctx, int32_t *row_slot, int32_t *row_pos) {
    int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= rows) return;
    int b = m / k, j = m - b * k;
    int s = min(max(stream_ids[b], 0), max_batch - 1);
    row_slot[m] = s;
    row_pos[m] = min(max(kv_len[s], 0) + j, max_ctx - 1);
}

void launch_prep_rows(Ctx *c, const Fwd &f) {
    ProfScope ps(c, KC_PREP);
    hipLaunchKernelGGL(k_prep_rows, dim3((f.rows + 63) / 64), dim3(64), 0, c->stream, f.stream_ids, c->d_kv_len, f.k,
                       f.rows, c->cfg.max_batch, c->cfg.max_ctx, c->row_slot, c->row_pos);
}

// ------------------------------------------------------------------------------------------ embedding
template <typename WT>
__global__ void k_embed(const WT *__restrict__ E, const int32_t *__restrict__ tok, int d, int vocab, float *x) {
    int m = blockIdx.x;
    int t = min(max(tok[m], 0), vocab - 1);
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = Elem<WT>::load(E + (size_t)t * d + i);
}

void launch_embed(Ctx *c, const Fwd &f) {
    ProfScope ps(c, KC_EMBED);
    if (c->bf16)
        hipLaunchKernelGGL(k_embed<bf16_t>, dim3(f.rows), dim3(256), 0, c->stream, (const bf16_t *)c->embed, f.tokens,
                           c->cfg.d_model, c->cfg.vocab, c->x);
    else
        hipLaunchKernelGGL(k_embed<float>, dim3(f.rows), dim3(256), 0, c->stream, (const float *)c->embed, f.tokens,
                           c->cfg.d_model, c->cfg.vocab, c->x);
}

// ------------------------------------------------------------------------------------------ RMSNorm
// x[m] += y[0][m] + ... + y[n_partial-1][m] (fixed order), then out[m] = x[m] / sqrt(mean(x^2)+eps) * g
// NP: the most slices a launch may hold (the loads of all NP are issued whatever n_partial is)
template <typename WT, typename AT, int NP>
__global__ __launch_bounds__(1024) void k_rmsnorm(float *x, const float *__restrict__ y, int n_partial, size_t partial_stride,
                          const WT *__restrict__ g, int d, float eps, ActBuf out, float *out_f32) {
    __shared__ float red[16];
    const int m = blockIdx.x;
    float *xr = x + (size_t)m * d;
    float ss = 0.f;
    // 1024 threads, four consecutive elements each per pass.  Every slice is requested before the first is used
    // (no load sits behind a branch: slices past the last re-read it and count as zero) and added in slice order.
    // The first pass's elements stay in registers for the second phase.
    float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = threadIdx.x * 4; i < d; i += 4096) {
        float4 v = *reinterpret_cast<const float4 *>(xr + i);
        float4 part[NP];
        const int np = max(n_partial, 1);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            part[p] = *reinterpret_cast<const float4 *>(y + (size_t)min(p, np - 1) * partial_stride + (size_t)m * d + i);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool on = p < n_partial;   // a select, not a product: the unused re-read may hold anything
            v.x += on ? part[p].x : 0.f; v.y += on ? part[p].y : 0.f; v.z += on ? part[p].z : 0.f; v.w += on ? part[p].w : 0.f;
        }
        if (n_partial) *reinterpret_cast<float4 *>(xr + i) = v;
        if (i < 4096) v0 = v;
        ss += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    ss = block_sum<1024>(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x * 4; i < d; i += 4096) {
        const float4 v = i < 4096 ? v0 : *reinterpret_cast<const float4 *>(xr + i);
        float4 r;
        r.x = v.x * inv * Elem<WT>::load(g + i);
        r.y = v.y * inv * Elem<WT>::load(g + i + 1);
        r.z = v.z * inv * Elem<WT>::load(g + i + 2);
        r.w = v.w * inv * Elem<WT>::load(g + i + 3);
        // a representation whose pointer is null has no reader this round and is not written
        if (out.f) *reinterpret_cast<float4 *>(out.f + (size_t)m * d + i) = r;
        if (out.hi) {
            bf16_t h[4], l[4];
            split2(r.x, h[0], l[0]);
            split2(r.y, h[1], l[1]);
            split2(r.z, h[2], l[2]);
            split2(r.w, h[3], l[3]);
            *reinterpret_cast<uint2 *>(out.hi + (size_t)m * d + i) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
            *reinterpret_cast<uint2 *>(out.lo + (size_t)m * d + i) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
        }
        if (out.h16)
            *reinterpret_cast<uint2 *>(out.h16 + (size_t)m * d + i) = make_uint2(f32_to_f16(r.x) | ((uint32_t)f32_to_f16(r.y) << 16),
                                                                                 f32_to_f16(r.z) | ((uint32_t)f32_to_f16(r.w) << 16));
        if (out_f32) *reinterpret_cast<float4 *>(out_f32 + (size_t)m * d + i) = r;
    }
}

template <int NP>
static void launch_rmsnorm_np(Ctx *c, int rows, int n_partial, const void *g, const ActBuf &out, float *out_f32) {
    const int d = c->cfg.d_model;
    const size_t stride = (size_t)c->rows_max * d;
    if (c->bf16)
        hipLaunchKernelGGL((k_rmsnorm<bf16_t, float, NP>), dim3(rows), dim3(1024), 0, c->stream, c->x, c->y, n_partial,
                           stride, (const bf16_t *)g, d, c->cfg.rms_eps, out, out_f32);
    else
        hipLaunchKernelGGL((k_rmsnorm<float, float, NP>), dim3(rows), dim3(1024), 0, c->stream, c->x, c->y, n_partial,
                           stride, (const float *)g, d, c->cfg.rms_eps, out, out_f32);
}

void launch_rmsnorm(Ctx *c, int rows, int n_partial, const void *g, const ActBuf &out, float *out_f32) {
    ProfScope ps(c, KC_NORM);
    static_assert(MAX_SPLITS <= 16, "the widest instantiation below covers every slice count");
    // the kernel requests as many slices as its instantiation holds: the smallest one that covers n_partial
    if (n_partial <= 4) launch_rmsnorm_np<4>(c, rows, n_partial, g, out, out_f32);
    else if (n_partial <= 8) launch_rmsnorm_np<8>(c, rows, n_partial, g, out, out_f32);
    else launch_rmsnorm_np<16>(c, rows, n_partial, g, out, out_f32);
}

// ------------------------------------------------------------------------------------------ GEMM (fallback)
// Y[r, o] = sum_i A[r, i] W[o, i]; one wave per output feature, MT rows per pass, kd % 8 == 0
template <typename WT, typename AT, int MT>
__global__ void k_gemm_ref(const AT *__restrict__ A, const WT *__restrict__ W, float *__restrict__ Y, int rows, int n,
                           int kd) {
    const int lane = threadIdx.x & 63, o = blockIdx.x * 4 + (threadIdx.x >> 6), r0 = blockIdx.y * MT;
    if (o >= n) return;
    float acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = 0.f;
    const WT *wr = W + (size_t)o * kd;
    for (int i = lane * 8; i < kd; i += 512) {
        float wv[8], av[8];
        load8<WT>(wr + i, wv);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (r0 + t < rows) {
                load8<AT>(A + (size_t)(r0 + t) * kd + i, av);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[t] = fmaf(av[e], wv[e], acc[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        float s = wave_sum(acc[t]);
        if (lane == 0 && r0 + t < rows) Y[(size_t)(r0 + t) * n + o] = s;
    }
}

void launch_gemm_ref(Ctx *c, const float *A, const void *W, float *Y, int rows, int n, int kd, int kclass) {
    ProfScope ps(c, kclass);
    constexpr int MT = 8;
    dim3 grid((n + 3) / 4, (rows + MT - 1) / MT);
    if (c->bf16)
        hipLaunchKernelGGL((k_gemm_ref<bf16_t, float, MT>), grid, dim3(256), 0, c->stream, A,
                           (const bf16_t *)W, Y, rows, n, kd);
    else
        hipLaunchKernelGGL((k_gemm_ref<float, float, MT>), grid, dim3(256), 0, c->stream, A,
                           (const float *)W, Y, rows, n, kd);
}

// ------------------------------------------------------------------------------------------ RoPE + KV append
// grid (rows, H + 2G), block hd/2.  q heads: rotate -> q operand; k heads: rotate -> cache; v heads: copy -> cache
template <typename WT, typename AT>
__global__ void k_rope_append(const float *__restrict__ qkv, int n_partial, size_t partial_stride, int H, int G, int hd, const int32_t *__restrict__ row_slot,
                              const int32_t *__restrict__ row_pos, const float *__restrict__ cs,
                              const float *__restrict__ sn, AT *q_out, WT *kv_layer, size_t slot_stride, int ctx_pad,
                              const float *__restrict__ ss, int n_ss, int d_model, float eps) {
    const int m = blockIdx.x, hh = blockIdx.y, i = threadIdx.x, half = hd >> 1;
    const int d_q = H * hd, d_kv = G * hd, pos = row_pos[m];
    const float *src = qkv + (size_t)m * (d_q + 2 * d_kv) + (size_t)hh * hd;
    float a = src[i], b = src[i + half];
    for (int p = 1; p < n_partial; ++p) {   // fixed order: slice 0 + slice 1 + ...
        a += src[p * partial_stride + i];
        b += src[p * partial_stride + i + half];
    }
    if (n_ss > 0) {   // the slices are products of x * gain: the deferred 1 / rms of the folded RMSNorm
        float t = 0.f;
        for (int p = 0; p < n_ss; ++p) t += ss[(size_t)p * gridDim.x + m];
        const float inv = 1.0f / sqrtf(t / (float)d_model + eps);
        a *= inv;
        b *= inv;
    }
    const float co = cs[(size_t)pos * half + i], si = sn[(size_t)pos * half + i];
    if (hh < H) {
        AT *dst = q_out + (size_t)m * d_q + (size_t)hh * hd;
        Elem<AT>::store(dst + i, a * co - b * si);
        Elem<AT>::store(dst + i + half, b * co + a * si);
    } else if (hh < H + G) {
        WT *dst = kv_layer + (size_t)row_slot[m] * slot_stride + ((size_t)(hh - H) * ctx_pad + pos) * hd;
        Elem<WT>::store(dst + i, a * co - b * si);
        Elem<WT>::store(dst + i + half, b * co + a * si);
    } else {
        WT *dst = kv_layer + (size_t)row_slot[m] * slot_stride + (size_t)(hh - H) * ctx_pad * hd;   // V planes follow the G K planes
        Elem<WT>::store(dst + v_plane_index(pos, i, hd), a);
        Elem<WT>::store(dst + v_plane_index(pos, i + half, hd), b);
    }
}

void launch_rope_append(Ctx *c, const Fwd &f, int layer, int n_partial, int n_ss) {
    const size_t pstride = (size_t)c->rows_max * c->d_qkv;
    ProfScope ps(c, KC_ROPE);
    const wisv_config &g = c->cfg;
    const size_t slot_stride = (size_t)2 * g.n_kv_heads * c->ctx_pad * g.head_dim;
    dim3 grid(f.rows, g.n_heads + 2 * g.n_kv_heads), block(g.head_dim / 2);
    void *kvl = kv_ptr(c, layer, 0, 0);
    if (c->bf16)
        hipLaunchKernelGGL((k_rope_append<bf16_t, float>), grid, block, 0, c->stream, c->qkv, n_partial, pstride, g.n_heads, g.n_kv_heads,
                           g.head_dim, c->row_slot, c->row_pos, c->rope_cos, c->rope_sin, c->q, (bf16_t *)kvl,
                           slot_stride, c->ctx_pad, c->ss, n_ss, g.d_model, g.rms_eps);
    else
        hipLaunchKernelGGL((k_rope_append<float, float>), grid, block, 0, c->stream, c->qkv, n_partial, pstride, g.n_heads, g.n_kv_heads,
                           g.head_dim, c->row_slot, c->row_pos, c->rope_cos, c->rope_sin, c->q, (float *)kvl,
                           slot_stride, c->ctx_pad, c->ss, n_ss, g.d_model, g.rms_eps);
}

// ------------------------------------------------------------------------------------------ attention (fallback)
// one block per (row, query head): scores of the visible keys in LDS, float softmax, then P.V
template <typename WT, typename AT>
__global__ void k_attn_ref(const AT *__restrict__ q, const WT *__restrict__ kv_layer, size_t slot_stride, int H, int G,
                           int hd, int ctx_pad, const int32_t *__restrict__ row_slot,
                           const int32_t *__restrict__ row_pos, ActBuf o) {
    extern __shared__ float smem[];
    float *qs = smem;            // [hd]
    float *red = smem + hd;      // [256 + 4]
    float *sc = red + 260;       // [n_vis]
    const int m = blockIdx.x, h = blockIdx.y, g = h / (H / G), tid = threadIdx.x;
    const int n_vis = row_pos[m] + 1;
    const WT *kc = kv_layer + (size_t)row_slot[m] * slot_stride + (size_t)g * ctx_pad * hd;
    const WT *vc = kc + (size_t)G * ctx_pad * hd;
    if (tid < hd) qs[tid] = Elem<AT>::load(q + (size_t)m * H * hd + (size_t)h * hd + tid);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)hd);
    float mx = -INFINITY;
    for (int s = tid; s < n_vis; s += 256) {
        float acc = 0.f, kvv[8];
        for (int i = 0; i < hd; i += 8) {
            load8<WT>(kc + (size_t)s * hd + i, kvv);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf(qs[i + e], kvv[e], acc);
        }
        acc *= scale;
        sc[s] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = block_max<256>(mx, red + 256);
    float sum = 0.f;
    for (int s = tid; s < n_vis; s += 256) {
        float e = expf(sc[s] - mx);
        sc[s] = e;
        sum += e;
    }
    sum = block_sum<256>(sum, red + 256);   // also makes every sc[] visible
    const int dim = tid % hd, part = tid / hd, nparts = 256 / hd;
    float acc = 0.f;
    for (int s = part; s < n_vis; s += nparts) acc = fmaf(sc[s], Elem<WT>::load(vc + v_plane_index(s, dim, hd)), acc);
    red[tid] = acc;
    __syncthreads();
    if (part == 0) {
        for (int p = 1; p < nparts; ++p) acc += red[p * hd + dim];
        act_store(o, (size_t)m * H * hd + (size_t)h * hd + dim, acc / sum);
    }
}

void launch_attn_ref(Ctx *c, const Fwd &f, int layer) {
    ProfScope ps(c, KC_ATTN);
    const wisv_config &g = c->cfg;
    const size_t slot_stride = (size_t)2 * g.n_kv_heads * c->ctx_pad * g.head_dim;
    // the kernel keeps every visible score in LDS: contexts beyond what a workgroup may hold are not served
    const size_t lds = sizeof(float) * (g.head_dim + 260 + f.max_len_ub);
    static bool allowed_bf16[MAX_DEVICES], allowed_f32[MAX_DEVICES];
    const void *kern = c->bf16 ? reinterpret_cast<const void *>(&k_attn_ref<bf16_t, float>) : reinterpret_cast<const void *>(&k_attn_ref<float, float>);
    if (lds > 150 * 1024 || (lds > 64 * 1024 && !allow_big_lds(c, kern, c->bf16 ? allowed_bf16 : allowed_f32))) {
        c->launch_failed = true;
        c->launch_err = "the generic attention kernel holds one score per visible position in LDS: a context of " +
                        std::to_string(f.max_len_ub) + " positions does not fit (this shape is not served by the MFMA attention kernel)";
        return;
    }
    dim3 grid(f.rows, g.n_heads);
    void *kvl = kv_ptr(c, layer, 0, 0);
    if (c->bf16)
        hipLaunchKernelGGL((k_attn_ref<bf16_t, float>), grid, dim3(256), lds, c->stream, (const float *)c->q,
                           (const bf16_t *)kvl, slot_stride, g.n_heads, g.n_kv_heads, g.head_dim, c->ctx_pad,
                           c->row_slot, c->row_pos, act_planes(c->o, c->o_planes));
    else
        hipLaunchKernelGGL((k_attn_ref<float, float>), grid, dim3(256), lds, c->stream, (const float *)c->q,
                           (const float *)kvl, slot_stride, g.n_heads, g.n_kv_heads, g.head_dim, c->ctx_pad, c->row_slot,
                           c->row_pos, act_planes(c->o, c->o_planes));
}

// ------------------------------------------------------------------------------------------ V plane <-> rows
// rows: [G][len][hd] (what the host hands over); plane: one (layer, slot) V plane [G][ctx_pad / 32][hd][32]
template <typename WT>
__global__ void k_v_reblock(WT *rows, WT *plane, int len, int hd, int ctx_pad, bool to_plane) {
    const int g = blockIdx.y;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)len * hd) return;
    const int pos = i / hd, dim = i % hd;
    WT *r = rows + ((size_t)g * len + pos) * hd + dim, *q = plane + (size_t)g * ctx_pad * hd + v_plane_index(pos, dim, hd);
    if (to_plane) *q = *r;
    else *r = *q;
}

void launch_v_reblock(Ctx *c, void *rows, void *plane, int len, bool to_plane) {
    const wisv_config &g = c->cfg;
    dim3 grid((unsigned)(((size_t)len * g.head_dim + 255) / 256), g.n_kv_heads);
    if (c->bf16)
        hipLaunchKernelGGL(k_v_reblock<bf16_t>, grid, dim3(256), 0, c->stream, (bf16_t *)rows, (bf16_t *)plane, len, g.head_dim,
                           c->ctx_pad, to_plane);
    else
        hipLaunchKernelGGL(k_v_reblock<float>, grid, dim3(256), 0, c->stream, (float *)rows, (float *)plane, len, g.head_dim,
                           c->ctx_pad, to_plane);
}

// ------------------------------------------------------------------------------------------ SwiGLU
__global__ void k_swiglu(const float *__restrict__ gu, int F, ActBuf h) {
    const int m = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= F) return;
    const float g = gu[(size_t)m * 2 * F + i], u = gu[(size_t)m * 2 * F + F + i];
    act_store(h, (size_t)m * F + i, g / (1.0f + expf(-g)) * u);
}

void launch_swiglu(Ctx *c, int rows) {
    ProfScope ps(c, KC_SWIGLU);
    const int F = c->cfg.d_ff;
    dim3 grid((F + 255) / 256, rows);
    hipLaunchKernelGGL(k_swiglu, grid, dim3(256), 0, c->stream, c->gu, F, c->h);
}

// ------------------------------------------------------------------------------------------ argmax over logits rows
__global__ void k_argmax_rows(const float *__restrict__ z, int V, int32_t *amax) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const float *zr = z + (size_t)m * V;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int i = tid; i < V; i += 256) {
        float v = zr[i];
        if (v > best || idx == 0x7fffffff) { best = v; idx = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(best, o, 64);
        int oi = __shfl_xor(idx, o, 64);
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

void launch_argmax(Ctx *c, int rows) {
    ProfScope ps(c, KC_ARGMAX);
    hipLaunchKernelGGL(k_argmax_rows, dim3(rows), dim3(256), 0, c->stream, c->logits, c->cfg.vocab, c->amax);
}

// after a prefill chunk: the slot's length grows by the chunk, pred_next = greedy token of its last row
__global__ void k_set_pred_next(int32_t *kv_len, int32_t *pred_next, const int32_t *amax, int slot, int row,
                                int new_len) {
    pred_next[slot] = amax[row];
    kv_len[slot] = new_len;
}

void launch_set_pred_next(Ctx *c, int slot, int row, int new_len) {
    hipLaunchKernelGGL(k_set_pred_next, dim3(1), dim3(1), 0, c->stream, c->d_kv_len, c->d_pred_next, c->amax, slot, row,
                       new_len);
}

}  // namespace wisv
