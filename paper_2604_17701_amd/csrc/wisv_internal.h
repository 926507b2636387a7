// Internal declarations of the WISV verify-round library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "wisv.h"
#include "wisv_diag.h"

namespace wisv {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

// ---------------------------------------------------------------- device-side scalar helpers
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even; NaN is kept a NaN.  On gfx950 this is one v_cvt_pk_bf16_f32 (two values when the
// compiler pairs them) instead of a dozen integer instructions.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static __forceinline__ float load(const float *p) { return *p; }
    __device__ static __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    __device__ static __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// An activation tensor handed to a matrix product: the float values (read by the generic kernels and by the
// decision head) and, for the MFMA kernels, the same values as two bf16 planes with x = hi + lo to 2^-17.
// Every kernel that produces such a tensor writes all three.
struct ActBuf {
    float *f;
    bf16_t *hi, *lo;
    uint16_t *h16;   // the same values as one IEEE half each (null when the ctx never runs the one-term products)
};
// nearest-even; magnitudes beyond the largest half saturate instead of becoming infinite
__device__ __forceinline__ uint16_t f32_to_f16(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)__builtin_amdgcn_fmed3f(f, -65504.0f, 65504.0f));
}
__device__ __forceinline__ void split2(float v, bf16_t &hi, bf16_t &lo) {
    hi = f32_to_bf16(v);
    lo = f32_to_bf16(v - bf16_to_f32(hi));
}
// A plane whose pointer is null is not written (f; hi and lo together; h16): a producer whose only consumer reads
// one representation leaves the others out.
__device__ __forceinline__ void act_store(const ActBuf &a, size_t i, float v) {
    if (a.f) a.f[i] = v;
    if (a.hi) {
        bf16_t h, l;
        split2(v, h, l);
        a.hi[i] = h;
        a.lo[i] = l;
    }
    if (a.h16) a.h16[i] = f32_to_f16(v);
}

// four consecutive elements, i a multiple of 4: one 16-byte and two 8-byte stores
__device__ __forceinline__ void act_store4(const ActBuf &a, size_t i, float v0, float v1, float v2, float v3) {
    if (a.f) *reinterpret_cast<float4 *>(a.f + i) = make_float4(v0, v1, v2, v3);
    if (a.hi) {
        bf16_t h[4], l[4];
        split2(v0, h[0], l[0]);
        split2(v1, h[1], l[1]);
        split2(v2, h[2], l[2]);
        split2(v3, h[3], l[3]);
        *reinterpret_cast<uint2 *>(a.hi + i) = make_uint2(h[0] | ((unsigned)h[1] << 16), h[2] | ((unsigned)h[3] << 16));
        *reinterpret_cast<uint2 *>(a.lo + i) = make_uint2(l[0] | ((unsigned)l[1] << 16), l[2] | ((unsigned)l[3] << 16));
    }
    if (a.h16)
        *reinterpret_cast<uint2 *>(a.h16 + i) = make_uint2(f32_to_f16(v0) | ((unsigned)f32_to_f16(v1) << 16),
                                                           f32_to_f16(v2) | ((unsigned)f32_to_f16(v3) << 16));
}

// Which representations of an activation buffer a producer writes: all of them, or only the one its single consumer
// reads (beyond 16 rows, where these buffers are tens of megabytes)
enum { ACT_ALL = 0, ACT_TWO_TERM = 1, ACT_HALF = 2 };
// the buffer with the pointers of the representations that `planes` leaves out set to null (producers skip those)
inline ActBuf act_planes(ActBuf a, int planes) {
    if (planes == ACT_HALF && a.h16) a.f = nullptr, a.hi = a.lo = nullptr;
    else if (planes == ACT_TWO_TERM) a.f = nullptr, a.h16 = nullptr;
    return a;
}

// ---------------------------------------------------------------- kernel classes (for per-kernel timing)
enum KernelClass {
    KC_PREP = 0, KC_EMBED, KC_NORM, KC_GEMM_QKV, KC_GEMM_GATEUP, KC_ROPE, KC_ATTN, KC_ATTN_COMBINE, KC_SWIGLU, KC_LMHEAD,
    KC_ARGMAX, KC_HEAD, KC_DECIDE, KC_SS, KC_EMPTY, KC_GEMM_O, KC_GEMM_DOWN, KC_COUNT
};

// ---------------------------------------------------------------- the context
struct LayerW {
    void *attn_norm, *wqkv, *wo, *ffn_norm, *wgu, *wdown;
    void *wqkv_t, *wo_t, *wgu_t, *wdown_t;   // re-tiled copies for the weight-streaming GEMM (bf16 only)
    void *wqkv_h, *wo_h, *wgu_h, *wdown_h;   // the same tiles as IEEE halves, for the one-term products (or null)
};

// product classes whose many-rows kernel may take its activations as one half-precision term (wisv_set_option)
enum { TERM_QKV = 1, TERM_O = 2, TERM_GATE_UP = 4, TERM_DOWN = 8, TERM_LM_HEAD = 16, TERM_ALL = 31 };

struct Ctx {
    wisv_config cfg;
    hipStream_t stream;
    bool stream_owned;   // no stream was given: the ctx made its own (the null stream cannot be captured)

    // the last device-I/O round, captured as a HIP graph when the same call comes a second time
    hipGraphExec_t graph_exec;
    wisv_round_in graph_in;
    wisv_round_out graph_out;
    int graph_len_ub;
    bool bf16;
    size_t esz;          // bytes per weight / cache element
    int d_q, d_kv, d_qkv, rows_max;

    // parameters (private copies)
    void *embed, *lm_head, *final_norm, *lm_head_t, *lm_head_h;
    bool half_ok;              // the half-precision weight tiles exist and every weight fits the half range
    uint32_t one_term_mask;    // TERM_* classes that run with one half-precision term when there are more than 16 rows
    bool ws_ok;          // shapes allow the weight-streaming MFMA GEMM
    std::vector<LayerW> layers;
    void *head_w1, *head_b1, *head_w2, *head_b2;
    void *head_w1_pad, *head_w1_t;   // W1 with its rows zero-padded to din_pad columns; its re-tiled copy (bf16)
    int din_pad;                     // d_draft + d_model + d_csi rounded up to a multiple of 32
    float *rope_cos, *rope_sin;      // [max_ctx][head_dim/2]

    // KV cache [n_layers][max_batch][2][n_kv_heads] planes of ctx_pad * head_dim elements (ctx_pad = max_ctx rounded
    // up to 32): K plane [ctx_pad][head_dim]; V plane in blocks of 32 positions, [ctx_pad / 32][head_dim][32], so
    // that 32 cached values of one feature are contiguous (the k dimension of P.V runs over positions)
    int ctx_pad;
    void *kv;
    bool kv_owned;

    // per-slot state (device) and a host mirror holding an upper bound of kv_len
    int32_t *d_kv_len, *d_pred_next;
    std::vector<int32_t> h_len_ub;

    // round inputs staged on the device (host-pointer mode)
    int32_t *d_stream_ids, *d_tokens, *d_proto, *d_hd_row;
    void *d_hd;
    float *d_csi, *d_tau;
    // round outputs staged on the device
    int32_t *d_alen, *d_ytok, *d_targ;
    float *d_pacc;
    uint32_t *d_mask, *d_status;

    // scratch
    int32_t *row_slot, *row_pos, *amax, *scored;
    float *x, *y, *qkv, *gu, *h_t, *logits;   // y and qkv hold up to MAX_SPLITS partial slices
    float *x_alt;                 // second residual-stream buffer: a product that folds the norm in reads x and writes here
    float *ss;                    // [MAX_SPLITS][rows_max] sums of squares left by such a product
    float *ss2;                   // [d_model / 16][min(rows_max, 16)]: those of the O projection that folds the FFN norm in
    bool graph_refused;           // a capture of the round failed once: later rounds run eagerly without trying again
    float *cand_val;
    int32_t *cand_idx;
    float *q;                     // rotated queries [rows][d_q]
    ActBuf a, o, h;               // normalised activations, attention output, SwiGLU output
    int o_planes;                 // ACT_*: the representations of o that this round's attention kernels write
    float *hu;                    // decision head: second-layer partial sums [row-block of hidden units][row]
    float *att_o, *att_m, *att_l; // split-KV attention partials: [split][rows][heads][head_dim], [split][rows][heads]
    int att_max_splits;
    size_t logits_rows;
    void *ss_ws;                  // speculative-sampling scratch: chunk statistics, normalisers, chunk weights
    float *d_ss_q, *d_ss_u, *d_ss_v;   // its host-mode input staging (d_ss_q is allocated by the first call that needs it)

    // timing
    hipEvent_t ev_round[2];
    bool profiling;
    std::vector<hipEvent_t> ev_pool;
    std::vector<int> ev_class;
    size_t ev_used;
    double prof_ms[KC_COUNT];
    long prof_n[KC_COUNT];
    int last_rows;
    // the round a WISV_FLAG_VERIFY_ONLY call left for its WISV_FLAG_DECIDE_ONLY call
    bool pending_valid;
    int pending_batch, pending_k;
    std::vector<int32_t> pending_ids, pending_tokens;

    // a launcher that cannot serve a shape mid-forward (no kernel fits) says so here; the entry point reports it
    bool launch_failed;
    std::string launch_err;

    std::string err;
    std::vector<void *> owned;    // device allocations to free
};

// what one forward needs to know (rows = batch*k; rows of a stream are consecutive)
struct Fwd {
    int rows, batch, k;
    const int32_t *stream_ids;   // device [batch]
    const int32_t *tokens;       // device [rows]
    bool keep_logits;
    int max_len_ub;              // upper bound of kv_len + k over the streams of this forward
};

// ---------------------------------------------------------------- kernel launchers (kernels_ref.hip)
void launch_prep_rows(Ctx *c, const Fwd &f);
void launch_embed(Ctx *c, const Fwd &f);
void launch_v_reblock(Ctx *c, void *rows, void *plane, int len, bool to_plane);
// x += sum of n_partial slices of y (if n_partial > 0); out = RMSNorm(x) * g; optional second float copy
void launch_rmsnorm(Ctx *c, int rows, int n_partial, const void *g, const ActBuf &out, float *out_f32);
// Y[rows, n] = A[rows, kd] * W[n, kd]^T (float accumulate, float out)
void launch_gemm_ref(Ctx *c, const float *A, const void *W, float *Y, int rows, int n, int kd, int kclass);
// n_ss > 0: the slices are scaled by 1 / rms from the n_ss partial sums of squares in c->ss (folded RMSNorm)
void launch_rope_append(Ctx *c, const Fwd &f, int layer, int n_partial, int n_ss = 0);
void launch_attn_ref(Ctx *c, const Fwd &f, int layer);
void launch_swiglu(Ctx *c, int rows);
void launch_argmax(Ctx *c, int rows);
void launch_set_pred_next(Ctx *c, int slot, int row, int new_len);

// ---------------------------------------------------------------- decision head + scan (kernels_head.hip)
void launch_head_decide(Ctx *c, const Fwd &f, const wisv_round_in &in_dev, const wisv_round_out &out_dev);
void launch_pad_cols(Ctx *c, const void *src, void *dst, int rows, int cols, int cols_pad);

// ---------------------------------------------------------------- speculative-sampling decision (kernels_ss.hip)
struct SsArgs {                    // all device pointers
    int batch, k, vocab;
    const float *logits;           // [batch*k][vocab]
    const int32_t *stream_ids;     // [batch]; pending token = pred_next of the slot (used when pending_tokens is null)
    const int32_t *pending_tokens; // [batch] or null
    const int32_t *tokens;         // [batch*k]
    const float *draft_probs;      // [batch*k][vocab]
    const float *u_accept, *u_sample;
    int32_t *accepted_len, *emitted_token;
    float *alpha;
    bool commit;                   // kv_len += A, pred_next = emitted token (needs stream_ids)
};
constexpr int SS_MAX_VOCAB = 4000 * 2048;   // the sampling kernel keeps one weight per 2048-token chunk in LDS
size_t ss_workspace_bytes(int rows, int vocab, int batch);
void launch_ss(Ctx *c, const SsArgs &a);
// the same kernels on the library's static scratch (no allocation): ss_static_init looks its device address up once
// per device, with that device current; launch_ss_static returns null or why the sizes are not served
hipError_t ss_static_init(int device);
const char *launch_ss_static(Ctx *c, const SsArgs &a);

// ---------------------------------------------------------------- weight-streaming GEMM (kernels_gemm.hip)
constexpr int MAX_SPLITS = 16;
bool ws_supported(const Ctx *c, int rows, int kd);
int ws_padded_row_blocks(int n_rows);
int ws_padded_pair_blocks(int features);
// overflow != null: the tiles are written as IEEE halves (nearest-even) and *overflow is set to 1 if a weight does not
// fit the half range
void launch_retile(Ctx *c, const void *W, int n_rows, int kd, int pair_rows, void *out, int nrb, int32_t *overflow = nullptr);
// the attention output before its k-splits are combined: o [split][rows][heads][128], m and l [split][rows][heads]
struct AttnPartials {
    const float *o, *m, *l;
    int splits, rows, heads;
};
constexpr int WS_PRO_SPLITS = 4;
// ap != null: X is ignored and the activations are combined from the partials while they are staged (at most 16
// rows and WS_PRO_SPLITS splits; 0 is returned otherwise)
// Wh != null: with more than 16 rows the product runs on the half-precision tiles Wh and X.h16 (one MFMA per pair)
int launch_gemm_ws_partial(Ctx *c, const void *Wt, const ActBuf &X, float *Yp, size_t split_stride, int max_splits,
                           int rows, int n, int kd, int kclass, const AttnPartials *ap = nullptr, const void *Wh = nullptr);
int launch_gemm_ws_normfold(Ctx *c, const void *Wt, const float *x_in, float *x_out, int n_partial, const void *gain,
                            float *Yp, size_t split_stride, int max_splits, int rows, int n, int kd, float *ss, int kclass);
// n_ss > 0: X holds x * gain of a folded RMSNorm and ss the n_ss partial sums of squares per row ([n_ss][rows]); the
// kernel applies 1 / rms before the SiLU (at most 16 rows)
// planes: one of ACT_* (more than 16 rows only): the kernel writes no other representation of H
bool launch_gemm_ws_swiglu(Ctx *c, const void *Wt, const ActBuf &X, const ActBuf &H, int rows, int features, int kd,
                           int kclass, const void *Wh = nullptr, const float *ss = nullptr, int n_ss = 0, int planes = ACT_ALL);
int launch_gemm_ws_resid(Ctx *c, const void *Wt, const ActBuf &X, const AttnPartials *ap, float *x, const void *gain,
                         const ActBuf &A_out, float *ss, int rows, int n, int kd, int kclass);
bool launch_gemm_ws_argmax(Ctx *c, const void *Wt, const ActBuf &X, float *logits, int rows, int n, int kd, int kclass,
                           const void *Wh = nullptr);

// ---------------------------------------------------------------- split-KV MFMA attention (kernels_attn.hip)
// true if the shape is served (bf16 cache, head_dim 128, at most 64 query rows per KV head); then c->o holds
// the attention output of every row
// with_combine false leaves the k-split partials in c->att_o / att_m / att_l for a consumer that combines them
// itself (*n_splits tells how many; 1 means c->o is complete all the same)
// n_ss > 0: the QKV product was fed x * gain instead of RMSNorm(x); its slices are scaled by 1 / rms from the n_ss
// partial sums of squares in c->ss (fused RoPE path only)
bool launch_attn_mfma(Ctx *c, const Fwd &f, int layer, int n_partial, bool with_combine = true, int *n_splits = nullptr,
                      int n_ss = 0);
void launch_attn_combine(Ctx *c, const Fwd &f, int n_splits);
// true if launch_attn_mfma(.., n_partial > 0) will do RoPE and the cache append itself from the k-split slices of
// the QKV product (then launch_rope_append must not run)
bool attn_mfma_fuses_rope(const Ctx *c, const Fwd &f);

// A kernel that wants more than 64 KiB of dynamic LDS must be allowed to once per device.  `done` is the caller's
// per-kernel table (one flag per device): a cache of an idempotent call, not state that results depend on.
constexpr int MAX_DEVICES = 64;
inline bool allow_big_lds(const Ctx *c, const void *kernel, bool (&done)[MAX_DEVICES]) {
    const int dev = c->cfg.device_id;
    if (dev < 0 || dev >= MAX_DEVICES) return false;
    if (done[dev]) return true;
    // 150 KiB: what the launchers use at most; the rest of the CU's 160 KiB stays free for a kernel's static LDS
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) != hipSuccess) {
        (void)hipGetLastError();   // the caller falls back to another kernel: the refusal is not the round's error
        return false;
    }
    done[dev] = true;
    return true;
}

// records the event pair of one launch when profiling is on
struct ProfScope {
    Ctx *c;
    int idx;
    ProfScope(Ctx *c, int kclass);
    ~ProfScope();
};

void *kv_ptr(const Ctx *c, int layer, int slot, int which);   // which: 0 = K, 1 = V
// offset of (position, feature) inside one head's V plane
__host__ __device__ __forceinline__ size_t v_plane_index(int pos, int dim, int hd) {
    return ((size_t)(pos >> 5) * hd + dim) * 32 + (pos & 31);
}

}  // namespace wisv
