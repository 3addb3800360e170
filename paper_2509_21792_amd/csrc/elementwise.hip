// Row-wise kernels of the verify step: tree preparation, embedding gather, residual add + RMSNorm (which also
// sums the split-K slabs of the producing GEMM), RoPE + paged KV append, SwiGLU for the fp32 path, and the
// per-row argmax / top-2 over the logits.  All are HBM-bound and tiny next to the GEMMs; each row is one block.
#include "fg_common.h"

namespace fg {

// ---- tree preparation ------------------------------------------------------------------------------------
// For every new node: its position (committed length + depth), the 64-bit set of its in-round
// ancestors-or-self, and the cache cell it is appended to (the same in every layer).  Parents are clamped so that
// a malformed tree cannot loop or index out of range.  A node whose slot lies beyond the sequence's page table gets
// cell -1 -- nothing is appended for it -- and raises FG_CACHE_OVERFLOW in the cache's status word; a position the
// RoPE table does not cover raises FG_POS_OVERFLOW (the position is clamped where it is used).
__global__ void tree_prep_kernel(const int32_t *slot, const int32_t *parent, const int32_t *seq_len,
                                 const int32_t *page_table, int B, int N, int n_prev, int n_slots, int max_pages, int n_pages,
                                 int max_pos, int32_t *pos, uint64_t *mask, int32_t *dest, int32_t *status)
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
    const int L = seq_len[s];
    pos[r] = L + depth;
    mask[r] = m;
    const int at = L + n_prev + j;
    if (at < 0 || (at >> 4) >= max_pages) {
        dest[r] = -1;
        if (status) atomicOr(status, (int32_t)FG_CACHE_OVERFLOW);
    } else {
        const int page = min(max(page_table[(size_t)s * max_pages + (at >> 4)], 0), n_pages - 1);
        dest[r] = page * 16 + (at & 15);
    }
    if (status && max_pos > 0 && (L + depth >= max_pos || L + depth < 0)) atomicOr(status, (int32_t)FG_POS_OVERFLOW);
}

int32_t launch_tree_prep_ex(const fg_tree *t, const fg_kv_cache *kv, TreeDev td, int max_pos, hipStream_t st)
{
    int M = t->B * t->N;
    hipLaunchKernelGGL(tree_prep_kernel, dim3((M + 127) / 128), dim3(128), 0, st, t->slot, t->parent, kv->seq_len,
                       kv->page_table, t->B, t->N, t->n_prev, kv->n_slots, kv->max_pages_per_seq, kv->n_pages, max_pos, td.pos,
                       td.mask, td.dest, kv->status);
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

// cat[r] = embed[token r] ++ feat[b][src]  (the draft head's fc input); src = feat_index[r] if given, else j
template <typename T>
__global__ void concat_embed_kernel(const T *embed, const int32_t *tokens, int vocab, const T *feat, const int32_t *feat_index,
                                    int N, int feat_rows, T *cat, int d)
{
    int r = blockIdx.x, b = r / N, j = r % N;
    int tok = min(max(tokens[r], 0), vocab - 1);
    int src = feat_index ? min(max(feat_index[r], 0), feat_rows - 1) : min(j, feat_rows - 1);
    const T *f = feat + ((size_t)b * feat_rows + src) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        cat[(size_t)r * 2 * d + c] = embed[(size_t)tok * d + c];
        cat[(size_t)r * 2 * d + d + c] = f[c];
    }
}

int32_t launch_concat_embed(int32_t dtype, const void *embed, const int32_t *tokens, int vocab, const void *feat,
                            const int32_t *feat_index, int N, int feat_rows, void *cat, int M, int d, hipStream_t st)
{
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(concat_embed_kernel<T>, dim3(M), dim3(256), 0, st, (const T *)embed, tokens, vocab,
                                             (const T *)feat, feat_index, N, feat_rows, (T *)cat, d));
    FG_LAUNCH_CHECK("concat_embed");
    return FG_OK;
}

// ---- residual add + RMSNorm ------------------------------------------------------------------------------
// h[r] = (init ? 0 : h[r]) + sum_s partials[s][r];  a[r] = h[r] / sqrt(mean(h[r]^2) + eps) * gain.
// One block per row; the split-K slabs are read as independent 16-byte loads so that a handful of rows (low
// concurrency) is not a chain of dependent round trips.  The row stays in registers between the two passes.
constexpr int NORM_THREADS = 1024, NORM_VEC_PER_THREAD = 2;  // d <= 8192, d % 4 == 0

template <typename T> __device__ __forceinline__ void store4(T *p, float4 v);
template <> __device__ __forceinline__ void store4<float>(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t *p, float4 v)
{
    uint2 u;
    u.x = (uint32_t)f2bf(v.x) | ((uint32_t)f2bf(v.y) << 16);
    u.y = (uint32_t)f2bf(v.z) | ((uint32_t)f2bf(v.w) << 16);
    *reinterpret_cast<uint2 *>(p) = u;
}
template <> __device__ __forceinline__ void store4<f16_t>(f16_t *p, float4 v)
{
    f16_t h[4] = {(f16_t)v.x, (f16_t)v.y, (f16_t)v.z, (f16_t)v.w};
    *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<uint2 *>(h);
}
template <typename T> __device__ __forceinline__ float4 load4(const T *p);
template <> __device__ __forceinline__ float4 load4<float>(const float *p) { return *reinterpret_cast<const float4 *>(p); }
template <> __device__ __forceinline__ float4 load4<bf16_t>(const bf16_t *p)
{
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                       __uint_as_float(u.y & 0xffff0000u));
}
template <> __device__ __forceinline__ float4 load4<f16_t>(const f16_t *p)
{
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    const f16_t *h = reinterpret_cast<const f16_t *>(&u);
    return make_float4((float)h[0], (float)h[1], (float)h[2], (float)h[3]);
}

// sum of S slabs at one float4 position; the loads are independent of each other
__device__ __forceinline__ float4 slab_sum4(const float *base, size_t slab_stride, int S, float4 x)
{
    int s = 0;
    for (; s + 4 <= S; s += 4) {
        float4 a = *reinterpret_cast<const float4 *>(base + (size_t)s * slab_stride);
        float4 b = *reinterpret_cast<const float4 *>(base + (size_t)(s + 1) * slab_stride);
        float4 c = *reinterpret_cast<const float4 *>(base + (size_t)(s + 2) * slab_stride);
        float4 d = *reinterpret_cast<const float4 *>(base + (size_t)(s + 3) * slab_stride);
        x.x += a.x; x.y += a.y; x.z += a.z; x.w += a.w;
        x.x += b.x; x.y += b.y; x.z += b.z; x.w += b.w;
        x.x += c.x; x.y += c.y; x.z += c.z; x.w += c.w;
        x.x += d.x; x.y += d.y; x.z += d.z; x.w += d.w;
    }
    for (; s < S; s++) {
        float4 a = *reinterpret_cast<const float4 *>(base + (size_t)s * slab_stride);
        x.x += a.x; x.y += a.y; x.z += a.z; x.w += a.w;
    }
    return x;
}

// THREADS x VPT float4 cover a row.  1024 x 2 for few rows, where a row's latency is what counts; 256 x 4 (rows up
// to 4096 wide) when there are hundreds of rows: eight blocks fit a CU instead of two, so 2048 rows are resident at
// once instead of taking four turns (15 -> 9 us per call at 2048 rows of the 7B-class width).
template <typename T, int THREADS, int VPT>
__global__ __launch_bounds__(THREADS) void add_rmsnorm_kernel(float *h, const float *partials, int S, int init,
                                                              const T *gain, T *a, T *h_copy, int M, int d, float eps)
{
    __shared__ float red[THREADS / 64];
    const int r = blockIdx.x, tid = threadIdx.x;
    const int nvec = d >> 2;
    float4 v[VPT];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; i++) {
        int c4 = tid + i * THREADS;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 < nvec) {
            float4 x = init ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4 *>(h + (size_t)r * d + c4 * 4);
            x = slab_sum4(partials + (size_t)r * d + c4 * 4, (size_t)M * d, S, x);
            v[i] = x;
            ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < THREADS / 64; i++) tot += red[i];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int i = 0; i < VPT; i++) {
        int c4 = tid + i * THREADS;
        if (c4 < nvec) {
            size_t at = (size_t)r * d + c4 * 4;
            if (S > 0 || init) *reinterpret_cast<float4 *>(h + at) = v[i];
            if (a) {
                float4 g = load4<T>(gain + c4 * 4);
                store4<T>(a + at, make_float4(v[i].x * inv * g.x, v[i].y * inv * g.y, v[i].z * inv * g.z, v[i].w * inv * g.w));
            }
            if (h_copy) store4<T>(h_copy + at, v[i]);
        }
    }
}

int32_t launch_add_rmsnorm(int32_t dtype, float *h, const float *partials, int S, int init, const void *gain, void *a,
                           void *h_copy, int M, int d, float eps, hipStream_t st)
{
    if (d > NORM_THREADS * NORM_VEC_PER_THREAD * 4 || d % 4)
        return fail(FG_ERR_SHAPE, "d_model %d not supported by the norm kernel (multiple of 4, at most %d)", d,
                    NORM_THREADS * NORM_VEC_PER_THREAD * 4);
    if (M >= 512 && d <= 256 * 4 * 4)
        FG_DISPATCH(dtype, T, hipLaunchKernelGGL((add_rmsnorm_kernel<T, 256, 4>), dim3(M), dim3(256), 0, st, h, partials, S, init,
                                                 (const T *)gain, (T *)a, (T *)h_copy, M, d, eps));
    else
        FG_DISPATCH(dtype, T, hipLaunchKernelGGL((add_rmsnorm_kernel<T, NORM_THREADS, NORM_VEC_PER_THREAD>), dim3(M), dim3(NORM_THREADS),
                                                 0, st, h, partials, S, init, (const T *)gain, (T *)a, (T *)h_copy, M, d, eps));
    FG_LAUNCH_CHECK("add_rmsnorm");
    return FG_OK;
}

// ---- RoPE + KV append -------------------------------------------------------------------------------------
// Sums the QKV GEMM's split-K slabs, rotates q and k (rotate-half pairing i, i + hd/2; angles from the table
// built in double precision at model creation), writes q rows for the attention kernel and the new node's
// k (in the cache's K page layout) and v (transposed) into its cache cell.  A thread owns four consecutive pair indices of one
// head (or four consecutive v elements), all slab loads independent.  A row is cut over gridDim.y blocks: with few
// rows one block per row would pull the whole slab sum through a handful of CUs.
template <typename T>
__global__ __launch_bounds__(1024) void rope_append_kernel(const float *qkv, int S, int M, const int32_t *pos,
                                                           const int32_t *dest, T *k_pool, T *v_pool, int layer,
                                                           int n_pages, int Hq, int Hkv, int hd, const float2 *rope_tab,
                                                           int max_pos, T *q_out, int k_frag)
{
    const int r = blockIdx.x;
    const int QKVD = (Hq + 2 * Hkv) * hd, half = hd >> 1, quads = half >> 2;
    const int n_rot = (Hq + Hkv) * quads, n_v = Hkv * hd / 4;
    const int w = blockIdx.y * blockDim.x + threadIdx.x;
    if (w >= n_rot + n_v) return;
    const size_t slab = (size_t)M * QKVD;
    const float *row = qkv + (size_t)r * QKVD;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    if (w < n_rot) {
        int head = w / quads, i = (w % quads) * 4;
        float4 a = slab_sum4(row + head * hd + i, slab, S, zero);
        float4 bb = slab_sum4(row + head * hd + i + half, slab, S, zero);
        const int p = min(max(pos[r], 0), max_pos - 1);
        const float2 *cs = rope_tab + (size_t)p * half + i;
        float2 c0 = cs[0], c1 = cs[1], c2 = cs[2], c3 = cs[3];
        float4 x0 = make_float4(a.x * c0.x - bb.x * c0.y, a.y * c1.x - bb.y * c1.y, a.z * c2.x - bb.z * c2.y,
                                a.w * c3.x - bb.w * c3.y);
        float4 x1 = make_float4(bb.x * c0.x + a.x * c0.y, bb.y * c1.x + a.y * c1.y, bb.z * c2.x + a.z * c2.y,
                                bb.w * c3.x + a.w * c3.y);
        if (head < Hq) {
            T *o = q_out + (size_t)r * Hq * hd + head * hd + i;
            store4<T>(o, x0);
            store4<T>(o + half, x1);
        } else {
            const int cell = dest[r], page = cell >> 4, t = cell & 15, hk = head - Hq;
            if (cell < 0) return;   // beyond the page table: not appended
            T *o = k_pool + (((size_t)layer * n_pages + page) * Hkv + hk) * 16 * hd;
            store4<T>(o + k_page_offset(k_frag, hd, t, i), x0);
            store4<T>(o + k_page_offset(k_frag, hd, t, i + half), x1);
        }
    } else {
        int e4 = (w - n_rot) * 4, hk = e4 / hd, e = e4 % hd;
        float4 v = slab_sum4(row + (Hq + Hkv) * hd + e4, slab, S, zero);
        const int cell = dest[r], page = cell >> 4, t = cell & 15;
        if (cell < 0) return;
        T *o = v_pool + (((size_t)layer * n_pages + page) * Hkv + hk) * 16 * hd + (size_t)e * 16 + t;
        o[0] = from_f<T>(v.x); o[16] = from_f<T>(v.y); o[32] = from_f<T>(v.z); o[48] = from_f<T>(v.w);
    }
}

int32_t launch_rope_append(int32_t dtype, const float *qkv_partials, int S, const fg_tree *t, TreeDev td, const fg_kv_cache *kv,
                           int layer, const float *rope_tab, int max_pos, int Hq, void *q_out, hipStream_t st)
{
    int M = t->B * t->N;
    const int work = (Hq + kv->n_kv_heads) * (kv->head_dim / 8) + kv->n_kv_heads * kv->head_dim / 4;
    // about 512 blocks in all when there are few rows, whole rows per block when there are many
    int threads = 1024;
    while (threads > 64 && (int64_t)M * ((work + threads - 1) / threads) < 512) threads >>= 1;
    if (threads > (work + 63) / 64 * 64) threads = (work + 63) / 64 * 64;
    FG_DISPATCH(dtype, T, hipLaunchKernelGGL(rope_append_kernel<T>, dim3(M, (work + threads - 1) / threads), dim3(threads), 0, st,
                                             qkv_partials, S, M, td.pos, td.dest, (T *)kv->k_pool, (T *)kv->v_pool, layer,
                                             kv->n_pages, Hq, kv->n_kv_heads, kv->head_dim, (const float2 *)rope_tab, max_pos,
                                             (T *)q_out, (int)k_fragment_major(kv->dtype, kv->head_dim, kv->page_size)));
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

// sum split-K slabs of an interleaved gate/up output and apply SwiGLU: act[m, f] (16-bit); a thread owns four
// consecutive features (one float4 of gate and one of up per slab, all slab loads independent)
template <typename T>
__global__ void swiglu_partials_kernel(const float *gu, int S, T *act, int M, int F)
{
    const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // quad index over [M, F / 4]
    const int fq = F >> 2;
    if (q >= (size_t)M * fq) return;
    const int m = (int)(q / fq), f = (int)(q % fq) * 4;
    const int t = f >> 5, j = f & 31;
    const size_t slab = (size_t)M * 2 * F;
    const float *row = gu + (size_t)m * 2 * F + 64 * t + j;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 g = slab_sum4(row, slab, S, zero), u = slab_sum4(row + 32, slab, S, zero);
    store4<T>(act + (size_t)m * F + f, make_float4(swiglu_f(g.x, u.x), swiglu_f(g.y, u.y),
                                                   swiglu_f(g.z, u.z), swiglu_f(g.w, u.w)));
}

int32_t launch_swiglu_partials(int32_t dtype, const float *gu, int S, void *act, int M, int F, hipStream_t st)
{
    if (F % 32) return fail(FG_ERR_SHAPE, "d_ffn %d is not a multiple of 32", F);
    const size_t total = (size_t)M * (F / 4);
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
    // a thread meets its indices in ascending order, so a strict comparison keeps the lower index on ties
    auto take = [&](float x, int v) {
        const bool gt = x > t.best;
        t.second = gt ? t.best : fmaxf(t.second, x);
        t.idx = gt ? v : t.idx;
        t.best = gt ? x : t.best;
    };
    if ((V & 3) == 0) {
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
#pragma unroll 4
        for (int q = tid; q < (V >> 2); q += 1024) {
            const float4 x = row4[q];
            take(x.x, 4 * q); take(x.y, 4 * q + 1); take(x.z, 4 * q + 2); take(x.w, 4 * q + 3);
        }
    } else {
        for (int v = tid; v < V; v += 1024) take(row[v], v);
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

// dst[b] = src[b * N + clamp(pick[b])]: one row of d elements per sequence, 16 bytes per thread
__global__ void gather_rows_kernel(const uint4 *src, const int32_t *pick, int B, int N, int vec_per_row, uint4 *dst)
{
    const int b = blockIdx.y, v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= vec_per_row) return;
    const int j = min(max(pick[b], 0), N - 1);
    dst[(size_t)b * vec_per_row + v] = src[((size_t)b * N + j) * vec_per_row + v];
}

int32_t launch_gather_rows(int32_t dtype, const void *src, const int32_t *pick, int B, int N, int d, void *dst, hipStream_t st)
{
    const int64_t row_bytes = (int64_t)d * dtype_size(dtype);
    if (row_bytes % 16) return fail(FG_ERR_SHAPE, "row of %lld bytes is not a multiple of 16", (long long)row_bytes);
    const int vec = (int)(row_bytes / 16);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((vec + 255) / 256, B), dim3(256), 0, st, (const uint4 *)src, pick, B, N, vec,
                       (uint4 *)dst);
    FG_LAUNCH_CHECK("gather_rows");
    return FG_OK;
}

// dst[i] = src[clamp(index[i])], rows of `words` 32-bit words
__global__ void select_rows_kernel(const uint32_t *src, int64_t words, int n_src, const int32_t *index, uint32_t *dst)
{
    const int i = blockIdx.y;
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= words) return;
    const int j = min(max(index[i], 0), n_src - 1);
    dst[(int64_t)i * words + w] = src[(int64_t)j * words + w];
}

int32_t launch_select_rows(const void *src, int64_t row_bytes, int n_src, const int32_t *index, int n, void *dst, hipStream_t st)
{
    const int64_t words = row_bytes / 4;
    if (n > 65535) return fail(FG_ERR_CAPACITY, "fg_select_rows: at most 65535 rows per call (got %d)", n);
    hipLaunchKernelGGL(select_rows_kernel, dim3((unsigned)((words + 255) / 256), n), dim3(256), 0, st, (const uint32_t *)src, words,
                       n_src, index, (uint32_t *)dst);
    FG_LAUNCH_CHECK("select_rows");
    return FG_OK;
}

}  // namespace fg
