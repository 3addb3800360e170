// Row-wise kernels of the verify step: tree preparation, embedding gather, residual add + RMSNorm (which also
// sums the split-K slabs of the producing GEMM), RoPE + paged KV append, SwiGLU for the fp32 path, and the
// per-row argmax / top-2 over the logits.  All are HBM-bound and tiny next to the GEMMs; each row is one block.
#include "fg_common.h"

namespace fg {

// ---- tree preparation ------------------------------------------------------------------------------------
// For every new node: its position (committed length + depth) and the 64-bit set of its in-round
// ancestors-or-self.  Parents are clamped so that a malformed tree cannot loop or index out of range.
__global__ void tree_prep_kernel(const int32_t *slot, const int32_t *parent, const int32_t *seq_len, int B, int N,
                                 int n_prev, int n_slots, int32_t *pos, uint64_t *mask)
{
    int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= B * N) return;
    int b = r / N, j = r % N, n_tot = n_prev + N;
    int u = n_prev + j, depth = 0;
    uint64_t m = 0;
    for (int step = 0; step < FG_MAX_NODES && u >= 0; step++) {
        m |= 1ull << u;
        int p = parent[(size_t)b * n_tot + u];
        if (p >= u) p = -1;
        if (p >= 0) depth++;
        u = p;
    }
    int s = min(max(slot[b], 0), n_slots - 1);
    pos[r] = seq_len[s] + depth;
    mask[r] = m;
}

int32_t launch_tree_prep_ex(const fg_tree *t, const int32_t *seq_len, int n_slots, TreeDev td, hipStream_t st)
{
    int M = t->B * t->N;
    hipLaunchKernelGGL(tree_prep_kernel, dim3((M + 127) / 128), dim3(128), 0, st, t->slot, t->parent, seq_len, t->B, t->N,
                       t->n_prev, n_slots, td.pos, td.mask);
    FG_LAUNCH_CHECK("tree_prep");
    return FG_OK;
}

// ---- embedding -------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_kernel(const T *embed, const int32_t *tokens, int vocab, float *h, int d)
{
    int r = blockIdx.x;
    int tok = min(max(tokens[r], 0), vocab - 1);
    for (int c = threadIdx.x; c < d; c += blockDim.x) h[(size_t)r * d + c] = to_f<T>(embed[(size_t)tok * d + c]);
}

int32_t launch_embed(int32_t dtype, const void *embed, const int32_t *tokens, int vocab, float *h, int M, int d, hipStream_t st)
{
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(embed_kernel<T>, dim3(M), dim3(256), 0, st, (const T *)embed, tokens, vocab, h, d));
    FG_LAUNCH_CHECK("embed");
    return FG_OK;
}

// cat[r] = embed[token r] ++ feat[r]  (the draft head's fc input)
template <typename T>
__global__ void concat_embed_kernel(const T *embed, const int32_t *tokens, int vocab, const T *feat, T *cat, int d)
{
    int r = blockIdx.x;
    int tok = min(max(tokens[r], 0), vocab - 1);
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        cat[(size_t)r * 2 * d + c] = embed[(size_t)tok * d + c];
        cat[(size_t)r * 2 * d + d + c] = feat[(size_t)r * d + c];
    }
}

int32_t launch_concat_embed(int32_t dtype, const void *embed, const int32_t *tokens, int vocab, const void *feat, void *cat,
                            int M, int d, hipStream_t st)
{
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(concat_embed_kernel<T>, dim3(M), dim3(256), 0, st, (const T *)embed, tokens, vocab,
                                             (const T *)feat, (T *)cat, d));
    FG_LAUNCH_CHECK("concat_embed");
    return FG_OK;
}

// ---- residual add + RMSNorm ------------------------------------------------------------------------------
// h[r] = (init ? 0 : h[r]) + sum_s partials[s][r];  a[r] = h[r] / sqrt(mean(h[r]^2) + eps) * gain.
// One block per row; the row stays in registers between the two passes.
constexpr int NORM_THREADS = 256, NORM_MAX_PER_THREAD = 32;  // d <= 8192

template <typename T>
__global__ __launch_bounds__(NORM_THREADS) void add_rmsnorm_kernel(float *h, const float *partials, int S, int init,
                                                                   const T *gain, T *a, T *h_copy, int M, int d, float eps)
{
    __shared__ float red[NORM_THREADS / 64];
    const int r = blockIdx.x, tid = threadIdx.x;
    float v[NORM_MAX_PER_THREAD];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_PER_THREAD; i++) {
        int c = tid + i * NORM_THREADS;
        if (c < d) {
            float x = init ? 0.f : h[(size_t)r * d + c];
            for (int s = 0; s < S; s++) x += partials[((size_t)s * M + r) * d + c];
            v[i] = x;
            ss += x * x;
        } else
            v[i] = 0.f;
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_THREADS / 64; i++) tot += red[i];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int i = 0; i < NORM_MAX_PER_THREAD; i++) {
        int c = tid + i * NORM_THREADS;
        if (c < d) {
            if (S > 0 || init) h[(size_t)r * d + c] = v[i];
            if (a) a[(size_t)r * d + c] = from_f<T>(v[i] * inv * to_f<T>(gain[c]));
            if (h_copy) h_copy[(size_t)r * d + c] = from_f<T>(v[i]);
        }
    }
}

int32_t launch_add_rmsnorm(int32_t dtype, float *h, const float *partials, int S, int init, const void *gain, void *a,
                           void *h_copy, int M, int d, float eps, hipStream_t st)
{
    if (d > NORM_THREADS * NORM_MAX_PER_THREAD) return fail(FG_ERR_SHAPE, "d_model %d too large for the norm kernel", d);
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(add_rmsnorm_kernel<T>, dim3(M), dim3(NORM_THREADS), 0, st, h, partials, S, init,
                                             (const T *)gain, (T *)a, (T *)h_copy, M, d, eps));
    FG_LAUNCH_CHECK("add_rmsnorm");
    return FG_OK;
}

// ---- RoPE + KV append -------------------------------------------------------------------------------------
// Sums the QKV GEMM's split-K slabs, rotates q and k (rotate-half pairing i, i + hd/2; angles from the table
// built in double precision at model creation), writes q rows for the attention kernel and the new node's
// k (token-major) and v (transposed) into its page.
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(const float *qkv, int S, int M, const int32_t *slot,
                                                          const int32_t *pos, const int32_t *seq_len,
                                                          const int32_t *page_table, T *k_pool, T *v_pool, int layer,
                                                          int n_pages, int n_slots, int max_pages, int N, int n_prev,
                                                          int Hq, int Hkv, int hd, const float2 *rope_tab, int max_pos,
                                                          T *q_out)
{
    const int r = blockIdx.x, b = r / N, j = r % N;
    const int QKVD = (Hq + 2 * Hkv) * hd, half = hd >> 1;
    const int s = min(max(slot[b], 0), n_slots - 1);
    const int p = min(max(pos[r], 0), max_pos - 1);
    const int at = seq_len[s] + n_prev + j;                 // cache slot of this node
    const int page_idx = min(at >> 4, max_pages - 1);
    const int page = min(max(page_table[(size_t)s * max_pages + page_idx], 0), n_pages - 1);
    const int t = at & 15;
    auto val = [&](int c) {
        float x = 0.f;
        for (int z = 0; z < S; z++) x += qkv[((size_t)z * M + r) * QKVD + c];
        return x;
    };
    // rotated pairs of q and k heads
    for (int w = threadIdx.x; w < (Hq + Hkv) * half; w += blockDim.x) {
        int head = w / half, i = w % half;
        float a = val(head * hd + i), bb = val(head * hd + i + half);
        float2 cs = rope_tab[(size_t)p * half + i];
        float x0 = a * cs.x - bb * cs.y, x1 = bb * cs.x + a * cs.y;
        if (head < Hq) {
            q_out[(size_t)r * Hq * hd + head * hd + i] = from_f<T>(x0);
            q_out[(size_t)r * Hq * hd + head * hd + i + half] = from_f<T>(x1);
        } else {
            int hk = head - Hq;
            size_t base = ((((size_t)layer * n_pages + page) * Hkv + hk) * 16 + t) * hd;
            k_pool[base + i] = from_f<T>(x0);
            k_pool[base + i + half] = from_f<T>(x1);
        }
    }
    for (int w = threadIdx.x; w < Hkv * hd; w += blockDim.x) {
        int hk = w / hd, e = w % hd;
        size_t base = (((size_t)layer * n_pages + page) * Hkv + hk) * 16 * hd;
        v_pool[base + (size_t)e * 16 + t] = from_f<T>(val((Hq + Hkv) * hd + w));
    }
}

int32_t launch_rope_append(int32_t dtype, const float *qkv_partials, int S, const fg_tree *t, TreeDev td, const fg_kv_cache *kv,
                           int layer, const float *rope_tab, int max_pos, int Hq, void *q_out, hipStream_t st)
{
    int M = t->B * t->N;
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(rope_append_kernel<T>, dim3(M), dim3(256), 0, st, qkv_partials, S, M, t->slot, td.pos,
                                             kv->seq_len, kv->page_table, (T *)kv->k_pool, (T *)kv->v_pool, layer, kv->n_pages,
                                             kv->n_slots, kv->max_pages_per_seq, t->N, t->n_prev, Hq, kv->n_kv_heads,
                                             kv->head_dim, (const float2 *)rope_tab, max_pos, (T *)q_out));
    FG_LAUNCH_CHECK("rope_append");
    return FG_OK;
}

// ---- SwiGLU on the interleaved gate/up output (fp32 path) -------------------------------------------------
__global__ void swiglu_f32_kernel(const float *gu, float *act, int M, int F)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * F) return;
    int m = idx / F, f = idx % F;
    int t = f >> 5, j = f & 31;
    float g = gu[(size_t)m * 2 * F + 64 * t + j], u = gu[(size_t)m * 2 * F + 64 * t + 32 + j];
    act[idx] = g / (1.f + expf(-g)) * u;
}

int32_t launch_swiglu_f32(const float *gu, float *act, int M, int F, hipStream_t st)
{
    size_t total = (size_t)M * F;
    hipLaunchKernelGGL(swiglu_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, gu, act, M, F);
    FG_LAUNCH_CHECK("swiglu_f32");
    return FG_OK;
}

// sum split-K slabs of an interleaved gate/up output and apply SwiGLU: act[m, f] (16-bit)
template <typename T>
__global__ void swiglu_partials_kernel(const float *gu, int S, T *act, int M, int F)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * F) return;
    int m = idx / F, f = idx % F;
    int t = f >> 5, j = f & 31;
    float g = 0.f, u = 0.f;
    for (int s = 0; s < S; s++) {
        const float *row = gu + ((size_t)s * M + m) * 2 * F;
        g += row[64 * t + j];
        u += row[64 * t + 32 + j];
    }
    act[idx] = from_f<T>(g / (1.f + __expf(-g)) * u);
}

int32_t launch_swiglu_partials(int32_t dtype, const float *gu, int S, void *act, int M, int F, hipStream_t st)
{
    size_t total = (size_t)M * F;
    if (dtype == FG_BF16)
        hipLaunchKernelGGL(swiglu_partials_kernel<bf16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, gu, S,
                           (bf16_t *)act, M, F);
    else
        hipLaunchKernelGGL(swiglu_partials_kernel<f16_t>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, gu, S,
                           (f16_t *)act, M, F);
    FG_LAUNCH_CHECK("swiglu_partials");
    return FG_OK;
}

// ---- per-row argmax and top-2 -------------------------------------------------------------------------------
struct Top2 {
    float best, second;
    int idx;
};
__device__ __forceinline__ Top2 top2_merge(Top2 a, Top2 b)
{
    Top2 o;
    bool b_wins = b.best > a.best || (b.best == a.best && b.idx < a.idx);
    if (b_wins) { o.best = b.best; o.idx = b.idx; o.second = fmaxf(a.best, b.second); }
    else { o.best = a.best; o.idx = a.idx; o.second = fmaxf(a.second, b.best); }
    return o;
}

__global__ __launch_bounds__(1024) void argmax_top2_kernel(const float *logits, int V, int32_t *idx, float *top2)
{
    __shared__ Top2 red[1024 / 64];
    const int r = blockIdx.x, tid = threadIdx.x;
    const float *row = logits + (size_t)r * V;
    Top2 t = {-INFINITY, -INFINITY, 0x7fffffff};
    for (int v = tid; v < V; v += blockDim.x) {
        float x = row[v];
        if (x > t.best) { t.second = t.best; t.best = x; t.idx = v; }   // v increases, so ties keep the lower index
        else if (x > t.second) t.second = x;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Top2 u;
        u.best = __shfl_xor(t.best, o, 64);
        u.second = __shfl_xor(t.second, o, 64);
        u.idx = __shfl_xor(t.idx, o, 64);
        t = top2_merge(t, u);
    }
    if ((tid & 63) == 0) red[tid >> 6] = t;
    __syncthreads();
    if (tid == 0) {
        Top2 a = red[0];
        for (int i = 1; i < (int)(blockDim.x >> 6); i++) a = top2_merge(a, red[i]);
        if (idx) idx[r] = a.idx;
        if (top2) { top2[2 * r] = a.best; top2[2 * r + 1] = a.second; }
    }
}

int32_t launch_argmax_top2(const float *logits, int M, int V, int32_t *idx, float *top2, hipStream_t st)
{
    hipLaunchKernelGGL(argmax_top2_kernel, dim3(M), dim3(1024), 0, st, logits, V, idx, top2);
    FG_LAUNCH_CHECK("argmax_top2");
    return FG_OK;
}

}  // namespace fg
