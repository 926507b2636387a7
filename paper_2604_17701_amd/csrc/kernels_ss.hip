// Speculative-sampling verification of drafted blocks (Sec. II-A: acceptance probability eq. ss_accept_prob,
// residual distribution eq. ss_residual, applied position by position until the first rejection).
//
//   1. stats    per (logits row, chunk of the vocabulary): largest logit and sum of exp(logit - largest)
//   2. accept   per stream: softmax normalisers of its rows, alpha_j of every position, the first rejected
//               position A, and the distribution the emitted token is drawn from
//   3. mass     per (stream, chunk): weight of the chunk under that distribution (residual or target)
//   4. sample   per stream: the chunk, then the token, at which the cumulative weight passes v * total; commit
//
// Probabilities are float exponentials divided by a double normaliser; every sum that decides a token is a
// double sum in a fixed order, so equal inputs give equal tokens.  HBM-bound: the logits are read twice for
// one row per stream and once for the others, the drafter's distribution once for one row per stream.
#include <algorithm>

#include "wisv_internal.h"

namespace wisv {

constexpr int SS_THREADS = 256, SS_PER_THREAD = 8;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// exclusive prefix sum over the block's 256 threads (wave scans, then the wave totals left to right) and the block total
__device__ __forceinline__ double block_scan_excl(double v, double *wave_tot, double &total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    double inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    const double below = __shfl_up(inc, 1, 64);
    if (lane == 63) wave_tot[w] = inc;
    __syncthreads();
    double off = 0.0, tot = 0.0;
#pragma unroll
    for (int i = 0; i < SS_THREADS / 64; ++i) {
        if (i < w) off += wave_tot[i];
        tot += wave_tot[i];
    }
    total = tot;
    __syncthreads();
    return off + (lane ? below : 0.0);
}

// eight consecutive elements of a row starting at i0 (a multiple of 8); elements at or beyond n read as `fill`.
// Every lane issues the same loads (clamped addresses), the selection comes afterwards.
__device__ __forceinline__ void ss_load8(const float *__restrict__ row, int i0, int n, bool vec, float fill, float x[8]) {
    if (vec) {   // n is a multiple of 4 and the row is 16-byte aligned
        const int a = min(i0, n - 4), b = min(i0 + 4, n - 4);
        const float4 lo = *reinterpret_cast<const float4 *>(row + a), hi = *reinterpret_cast<const float4 *>(row + b);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
        x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = i0 + e < n ? x[e] : fill;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = row[min(i0 + e, n - 1)];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = i0 + e < n ? x[e] : fill;
    }
}

__global__ void __launch_bounds__(SS_THREADS)
k_ss_stats(const float *__restrict__ logits, int V, int C, bool vec, float *__restrict__ pm, float *__restrict__ pz) {
    __shared__ float red[SS_THREADS / 64];
    const int c = blockIdx.x, r = blockIdx.y, tid = threadIdx.x;
    float x[8];
    ss_load8(logits + (size_t)r * V, (c * SS_THREADS + tid) * SS_PER_THREAD, V, vec, -INFINITY, x);
    float m = x[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) m = fmaxf(m, x[e]);
    m = wave_max(m);
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float z = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) z += expf(x[e] - m);   // exp(-inf) = 0 beyond the row's end
    z = wave_sum(z);
    if ((tid & 63) == 0) red[tid >> 6] = z;
    __syncthreads();
    if (tid == 0) {
        pm[(size_t)r * C + c] = m;
        pz[(size_t)r * C + c] = (red[0] + red[1]) + (red[2] + red[3]);
    }
}

// one block per stream, one wave per logits row of the stream: wave w reduces the chunk statistics of row w and
// decides position w + 1 (wave 0 also position 0)
__global__ void __launch_bounds__(1024)
k_ss_accept(int k, int V, int C, int max_batch, const float *__restrict__ logits, const float *__restrict__ pm,
            const float *__restrict__ pz, const int32_t *__restrict__ stream_ids, const int32_t *__restrict__ pred_next,
            const int32_t *__restrict__ pending_tokens, const int32_t *__restrict__ tokens, const float *__restrict__ q,
            const float *__restrict__ u, float *__restrict__ row_m, double *__restrict__ row_z, int32_t *__restrict__ sel_row,
            int32_t *__restrict__ sel_mode, int32_t *__restrict__ alen, int32_t *__restrict__ ytok, float *__restrict__ alpha_out) {
    __shared__ int s_reject[WISV_MAX_K];
    const int b = blockIdx.x, w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rp = b * k + w;
    const int pending = pending_tokens ? pending_tokens[b] : pred_next[min(max(stream_ids[b], 0), max_batch - 1)];
    float M = -INFINITY;
    for (int c = lane; c < C; c += 64) M = fmaxf(M, pm[(size_t)rp * C + c]);
    M = wave_max(M);
    double Z = 0.0;
    for (int c = lane; c < C; c += 64) Z += (double)pz[(size_t)rp * C + c] * (double)expf(pm[(size_t)rp * C + c] - M);
    Z = wave_sum_f64(Z);
    if (lane == 0) {
        row_m[rp] = M;
        row_z[rp] = Z;
        if (w + 1 < k) {
            const int t = min(max(tokens[rp + 1], 0), V - 1);
            const double P = (double)expf(logits[(size_t)rp * V + t] - M) / Z, qv = (double)q[(size_t)(rp + 1) * V + t];
            const double alpha = qv <= P ? 1.0 : P / qv;
            alpha_out[rp + 1] = (float)alpha;
            s_reject[w + 1] = !((double)u[rp + 1] < alpha);
        }
        if (w == 0) {
            const double alpha = tokens[b * k] == pending ? 1.0 : 0.0;
            alpha_out[b * k] = (float)alpha;
            s_reject[0] = !((double)u[b * k] < alpha);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int A = k;
        for (int j = k - 1; j >= 0; --j)
            if (s_reject[j]) A = j;
        alen[b] = A;
        sel_row[b] = b * k + max(A, 1) - 1;
        sel_mode[b] = A == 0 ? 0 : A < k ? 1 : 2;    // 0: emit the pending token; 1: residual of position A; 2: target after the block
        if (A == 0) ytok[b] = pending;
    }
}

// weight of element i of the selected row: p_T(i), less min(p_D(i), p_T(i)) for a residual
__device__ __forceinline__ double ss_weight(float x, float q, float M, double Z, bool resid) {
    const double p = (double)expf(x - M) / Z;
    return resid ? fmax(p - (double)q, 0.0) : p;
}

__global__ void __launch_bounds__(SS_THREADS)
k_ss_mass(int V, int C, int rows, bool vec, const float *__restrict__ logits, const float *__restrict__ q,
          const float *__restrict__ row_m, const double *__restrict__ row_z, const int32_t *__restrict__ sel_row,
          const int32_t *__restrict__ sel_mode, double *__restrict__ mass) {
    __shared__ double red[SS_THREADS / 64];
    const int c = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int rs = sel_row[b], mode = sel_mode[b];
    const int i0 = (c * SS_THREADS + tid) * SS_PER_THREAD;
    float x[8], qv[8];
    ss_load8(logits + (size_t)rs * V, i0, V, vec, -INFINITY, x);
    ss_load8(q + (size_t)min(rs + 1, rows - 1) * V, i0, V, vec, 0.f, qv);
    const float M = row_m[rs];
    const double Z = row_z[rs];
    double s = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += ss_weight(x[e], qv[e], M, Z, mode == 1);
    s = wave_sum_f64(s);
    if ((tid & 63) == 0) red[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) mass[(size_t)b * C + c] = mode == 0 ? 0.0 : (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ void __launch_bounds__(SS_THREADS)
k_ss_sample(int V, int C, int rows, int max_batch, bool vec, int commit, const float *__restrict__ logits,
            const float *__restrict__ q, const float *__restrict__ row_m, const double *__restrict__ row_z,
            const int32_t *__restrict__ sel_row, const int32_t *__restrict__ sel_mode, const double *__restrict__ mass,
            const float *__restrict__ v, const int32_t *__restrict__ stream_ids, const int32_t *__restrict__ alen,
            int32_t *__restrict__ ytok, int32_t *kv_len, int32_t *pred_next) {
    extern __shared__ double s_chunks[];   // [C] chunk weights, then [C] their exclusive prefix sums
    __shared__ double wave_tot[SS_THREADS / 64];
    __shared__ int s_chunk, s_lastc, s_first, s_last;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int rs = sel_row[b], mode = sel_mode[b];
    if (mode != 0) {   // the whole block takes the same side
        double *cw = s_chunks, *cex = s_chunks + C;
        if (tid == 0) { s_chunk = 0x7fffffff; s_lastc = 0; s_first = 0x7fffffff; s_last = -1; }
        double carry = 0.0;
        for (int c0 = 0; c0 < C; c0 += SS_THREADS) {   // chunk weights and their exclusive prefix sums, 256 at a time
            const int c = c0 + tid;
            const double m = c < C ? mass[(size_t)b * C + c] : 0.0;
            double tile_total;
            const double ex = carry + block_scan_excl(m, wave_tot, tile_total);
            if (c < C) { cw[c] = m; cex[c] = ex; }
            carry += tile_total;
        }
        const double target = (double)v[b] * carry;
        __syncthreads();
        for (int c = tid; c < C; c += SS_THREADS)
            if (cw[c] > 0.0) {
                atomicMax(&s_lastc, c);
                if (cex[c] + cw[c] > target) atomicMin(&s_chunk, c);
            }
        __syncthreads();
        const int chunk = s_chunk != 0x7fffffff ? s_chunk : s_lastc;   // else: v * total rounded up to the total
        const double base = cex[chunk];
        const int i0 = (chunk * SS_THREADS + tid) * SS_PER_THREAD;
        float x[8], qv[8];
        ss_load8(logits + (size_t)rs * V, i0, V, vec, -INFINITY, x);
        ss_load8(q + (size_t)min(rs + 1, rows - 1) * V, i0, V, vec, 0.f, qv);
        const float M = row_m[rs];
        const double Z = row_z[rs];
        double w[8], ts = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) { w[e] = ss_weight(x[e], qv[e], M, Z, mode == 1); ts += w[e]; }
        double chunk_total;
        double cum = base + block_scan_excl(ts, wave_tot, chunk_total);
        int first = 0x7fffffff, last = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += w[e];
            if (w[e] > 0.0) {
                last = i0 + e;
                if (cum > target) first = min(first, i0 + e);
            }
        }
        if (first != 0x7fffffff) atomicMin(&s_first, first);
        if (last >= 0) atomicMax(&s_last, last);
        __syncthreads();
        if (tid == 0) ytok[b] = s_first != 0x7fffffff ? s_first : max(s_last, 0);
    }
    if (commit && tid == 0) {
        const int slot = min(max(stream_ids[b], 0), max_batch - 1);
        kv_len[slot] += alen[b];
        pred_next[slot] = ytok[b];   // written by this thread or by the accept kernel
    }
}

size_t ss_workspace_bytes(int rows, int vocab, int batch) {
    const size_t C = (vocab + SS_THREADS * SS_PER_THREAD - 1) / (SS_THREADS * SS_PER_THREAD);
    return (size_t)rows * C * 8 + (size_t)rows * 16 + (size_t)batch * 8 + (size_t)batch * C * 8 + 64;
}

// the four kernels on `stream`, with their scratch carved from `ws` (at least ss_workspace_bytes(rows, vocab, batch))
static void enqueue_ss(hipStream_t stream, const SsArgs &a, void *ws, int max_batch, int32_t *d_kv_len, int32_t *d_pred_next) {
    const int rows = a.batch * a.k, V = a.vocab;
    const int C = (V + SS_THREADS * SS_PER_THREAD - 1) / (SS_THREADS * SS_PER_THREAD);
    const bool vec = (V & 3) == 0 && V >= 4 && ((uintptr_t)a.logits & 15) == 0 && ((uintptr_t)a.draft_probs & 15) == 0;
    // carve the workspace: doubles first
    char *p = (char *)ws;
    double *row_z = (double *)p;  p += (size_t)rows * 8;
    double *mass = (double *)p;   p += (size_t)a.batch * C * 8;
    float *pm = (float *)p;       p += (size_t)rows * C * 4;
    float *pz = (float *)p;       p += (size_t)rows * C * 4;
    float *row_m = (float *)p;    p += (size_t)rows * 4;
    int32_t *sel_row = (int32_t *)p;  p += (size_t)a.batch * 4;
    int32_t *sel_mode = (int32_t *)p;
    hipLaunchKernelGGL(k_ss_stats, dim3(C, rows), dim3(SS_THREADS), 0, stream, a.logits, V, C, vec, pm, pz);
    hipLaunchKernelGGL(k_ss_accept, dim3(a.batch), dim3(64 * a.k), 0, stream, a.k, V, C, max_batch, a.logits, pm, pz,
                       a.stream_ids, d_pred_next, a.pending_tokens, a.tokens, a.draft_probs, a.u_accept, row_m, row_z,
                       sel_row, sel_mode, a.accepted_len, a.emitted_token, a.alpha);
    hipLaunchKernelGGL(k_ss_mass, dim3(C, a.batch), dim3(SS_THREADS), 0, stream, V, C, rows, vec, a.logits, a.draft_probs,
                       row_m, row_z, sel_row, sel_mode, mass);
    hipLaunchKernelGGL(k_ss_sample, dim3(a.batch), dim3(SS_THREADS), (size_t)C * 16, stream, V, C, rows, max_batch, vec,
                       a.commit ? 1 : 0, a.logits, a.draft_probs, row_m, row_z, sel_row, sel_mode, mass, a.u_sample,
                       a.stream_ids, a.accepted_len, a.emitted_token, d_kv_len, d_pred_next);
}

void launch_ss(Ctx *c, const SsArgs &a) {
    ProfScope ps(c, KC_SS);
    enqueue_ss(c->stream, a, c->ss_ws, c->cfg.max_batch, c->d_kv_len, c->d_pred_next);
}

// ------------------------------------------------------------------------------------------ no allocation
// The same four kernels for callers that cannot allocate: their scratch is this array, which every device the
// library runs on holds from the moment the library is loaded there.  `scratch` itself is only a host-side handle:
// the device address is looked up once per device (with that device current) and kept.
constexpr int SS_STATIC_MAX_ROWS = 1024, SS_STATIC_MAX_VOCAB = 262144, SS_STATIC_MAX_DEVICES = 64;
constexpr size_t SS_STATIC_CHUNKS = (SS_STATIC_MAX_VOCAB + SS_THREADS * SS_PER_THREAD - 1) / (SS_THREADS * SS_PER_THREAD);
// ss_workspace_bytes(rows, vocab, batch) at its largest (batch <= rows)
constexpr size_t SS_STATIC_BYTES = (size_t)SS_STATIC_MAX_ROWS * SS_STATIC_CHUNKS * 8 + (size_t)SS_STATIC_MAX_ROWS * 16 +
                                   (size_t)SS_STATIC_MAX_ROWS * 8 + (size_t)SS_STATIC_MAX_ROWS * SS_STATIC_CHUNKS * 8 + 64;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[SS_STATIC_BYTES];
static void *scratch_ptr[SS_STATIC_MAX_DEVICES];   // device address of `scratch` on each device, null until looked up

// with `device` current; called when a context is created there.  Calls made concurrently for one device store the
// same address.
hipError_t ss_static_init(int device) {
    if (device < 0 || device >= SS_STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    if (scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[device] = p;
    return hipSuccess;
}

const char *launch_ss_static(Ctx *c, const SsArgs &a) {
    const int dev = c->cfg.device_id;
    if ((size_t)a.batch * a.k > (size_t)SS_STATIC_MAX_ROWS) return "batch * k beyond the static scratch (1024 rows)";
    if (a.vocab > SS_STATIC_MAX_VOCAB) return "vocab beyond the static scratch (262144 tokens)";
    if (dev < 0 || dev >= SS_STATIC_MAX_DEVICES || !scratch_ptr[dev]) return "no static scratch address for this device";
    if (ss_workspace_bytes(a.batch * a.k, a.vocab, a.batch) > SS_STATIC_BYTES) return "static scratch too small for these sizes";
    // no kernel of the four reads scratch it has not written in the same call: nothing needs clearing
    enqueue_ss(c->stream, a, scratch_ptr[dev], c->cfg.max_batch, c->d_kv_len, c->d_pred_next);
    return nullptr;
}

}  // namespace wisv
