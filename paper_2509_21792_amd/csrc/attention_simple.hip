// Tree attention over the paged cache, straightforward form: one wave per (node row, query head).
// Used by the fp32 parity configuration and as the shape-agnostic path (any head_dim, any group size); the
// bf16 production shapes go through the MFMA kernel in attention_mfma.hip.  Scores live in LDS, so the cache
// length this kernel accepts is bounded (see launch_attention_simple).
#include "fg_common.h"

namespace fg {

template <typename T>
__global__ __launch_bounds__(64) void attn_simple_kernel(const T *q, T *out, const T *k_pool, const T *v_pool,
                                                         const int32_t *page_table, const int32_t *seq_len,
                                                         const int32_t *slot, const uint64_t *mask, int layer, int n_pages,
                                                         int n_slots, int max_pages, int N, int n_prev, int Hq, int Hkv,
                                                         int hd, int max_keys, float scale, int k_frag)
{
    extern __shared__ float sm[];  // [max_keys] scores / probabilities, then [hd] the query
    const int r = blockIdx.x, hq = blockIdx.y, lane = threadIdx.x;
    const int b = r / N, n_tot = n_prev + N;
    const int s = min(max(slot[b], 0), n_slots - 1);
    const int L = seq_len[s];
    const int nk = min(L + n_tot, min(max_keys, max_pages * 16));
    const int hk = hq / (Hq / Hkv);
    const uint64_t m = mask[r];
    float *qs = sm + max_keys;
    for (int e = lane; e < hd; e += 64) qs[e] = to_f<T>(q[(size_t)r * Hq * hd + (size_t)hq * hd + e]);
    __syncthreads();

    float mx = -INFINITY;
    for (int t = lane; t < nk; t += 64) {
        bool valid = t < L || ((m >> (t - L)) & 1ull);
        float sc = -INFINITY;
        if (valid) {
            int page = min(max(page_table[(size_t)s * max_pages + (t >> 4)], 0), n_pages - 1);
            const T *kr = k_pool + (((size_t)layer * n_pages + page) * Hkv + hk) * 16 * hd;
            float dot = 0.f;
            for (int e = 0; e < hd; e++) dot += qs[e] * to_f<T>(kr[k_page_offset(k_frag, hd, t & 15, e)]);
            sc = dot * scale;
        }
        sm[t] = sc;
        mx = fmaxf(mx, sc);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int t = lane; t < nk; t += 64) {
        float p = sm[t] == -INFINITY ? 0.f : expf(sm[t] - mx);
        sm[t] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    for (int e = lane; e < hd; e += 64) {
        float acc = 0.f;
        for (int t = 0; t < nk; t++) {
            float p = sm[t];
            if (p != 0.f) {
                int page = min(max(page_table[(size_t)s * max_pages + (t >> 4)], 0), n_pages - 1);
                acc += p * to_f<T>(v_pool[(((size_t)layer * n_pages + page) * Hkv + hk) * 16 * hd + (size_t)e * 16 + (t & 15)]);
            }
        }
        out[(size_t)r * Hq * hd + (size_t)hq * hd + e] = from_f<T>(acc / sum);
    }
}

int32_t launch_attention_simple(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q,
                                void *out, int max_keys, hipStream_t st)
{
    const int M = t->B * t->N, hd = kv->head_dim;
    size_t lds = ((size_t)max_keys + hd) * sizeof(float);
    if (lds > 64 * 1024) return fail(FG_ERR_CAPACITY, "simple attention kernel holds at most %d keys in LDS (asked %d)",
                                     (int)(64 * 1024 / sizeof(float)) - hd, max_keys);
    const float scale = 1.0f / sqrtf((float)hd);
    dim3 grid(M, Hq);
    FG_DISPATCH(kv->dtype, T, hipLaunchKernelGGL(attn_simple_kernel<T>, grid, dim3(64), lds, st, (const T *)q, (T *)out,
                                                 (const T *)kv->k_pool, (const T *)kv->v_pool, kv->page_table, kv->seq_len,
                                                 t->slot, td.mask, layer, kv->n_pages, kv->n_slots, kv->max_pages_per_seq,
                                                 t->N, t->n_prev, Hq, kv->n_kv_heads, hd, max_keys, scale,
                                                 (int)k_fragment_major(kv->dtype, hd, kv->page_size)));
    FG_LAUNCH_CHECK("attn_simple");
    return FG_OK;
}

}  // namespace fg
