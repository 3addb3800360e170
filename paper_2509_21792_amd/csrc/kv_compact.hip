// In-place compaction of the accepted path's K/V in the paged cache, the gather of the accepted feature rows,
// and the length update.
//
// Hazard analysis: for sequence b with committed length L, slot L + path[j] moves to L + j, j ascending.
// path increases strictly and path[j] >= j, so a destination L + j is never a later source (every later source
// is > L + j).  One thread owns one element index (head_dim position) of one (layer, kv head) across all j and
// copies in ascending j, so there is no cross-thread dependence at all and no barrier is needed.
// The lengths are bumped by a second kernel, after every block of the first has read them (stream order).
#include "fg_common.h"

namespace fg {

__device__ __forceinline__ bool path_ok(const int32_t *p, int a, int N)
{
    if (a < 0 || a >= N || p[0] != 0) return false;
    for (int j = 1; j <= a; j++)
        if (p[j] <= p[j - 1] || p[j] >= N) return false;
    return true;
}

template <typename T>
__global__ void kv_compact_kernel(T *k_pool, T *v_pool, const int32_t *page_table, const int32_t *seq_len,
                                  const int32_t *slot, const int32_t *accept_len, const int32_t *path, int N, int n_pages,
                                  int n_slots, int max_pages, int Hkv, int hd, int k_frag)
{
    const int b = blockIdx.x, lh = blockIdx.y;  // lh = layer * Hkv + head
    const int layer = lh / Hkv, hk = lh % Hkv;
    const int a = accept_len[b];
    const int32_t *p = path + (size_t)b * N;
    if (!path_ok(p, a, N)) return;
    const int s = min(max(slot[b], 0), n_slots - 1);
    const int L = seq_len[s];
    if (((L + p[a]) >> 4) >= max_pages) return;
    for (int e = threadIdx.x; e < hd; e += blockDim.x) {
        for (int j = 1; j <= a; j++) {
            int src = L + p[j], dst = L + j;
            if (src == dst) continue;
            int ps = min(max(page_table[(size_t)s * max_pages + (src >> 4)], 0), n_pages - 1);
            int pd = min(max(page_table[(size_t)s * max_pages + (dst >> 4)], 0), n_pages - 1);
            size_t bs = (((size_t)layer * n_pages + ps) * Hkv + hk) * 16 * hd;
            size_t bd = (((size_t)layer * n_pages + pd) * Hkv + hk) * 16 * hd;
            k_pool[bd + k_page_offset(k_frag, hd, dst & 15, e)] = k_pool[bs + k_page_offset(k_frag, hd, src & 15, e)];
            v_pool[bd + (size_t)e * 16 + (dst & 15)] = v_pool[bs + (size_t)e * 16 + (src & 15)];
        }
    }
}

// The same conditions as kv_compact_kernel: a path that is malformed, or whose last node lies beyond the page table
// (nothing was moved), leaves the length alone; the latter raises FG_CACHE_OVERFLOW in the cache's status word.
__global__ void bump_len_kernel(int32_t *seq_len, const int32_t *slot, const int32_t *accept_len, const int32_t *path, int B,
                                int N, int n_slots, int max_pages, int32_t *status)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int a = accept_len[b];
    const int32_t *p = path + (size_t)b * N;
    if (!path_ok(p, a, N)) return;
    int s = min(max(slot[b], 0), n_slots - 1);
    const int L = seq_len[s];
    if (((L + p[a]) >> 4) >= max_pages) {
        if (status) atomicOr(status, (int32_t)FG_CACHE_OVERFLOW);
        return;
    }
    seq_len[s] = L + a + 1;
}

template <typename T>
__global__ void gather_feature_kernel(const T *fin, T *fout, const int32_t *accept_len, const int32_t *path, int N, int d)
{
    const int b = blockIdx.x, j = blockIdx.y;
    const int a = accept_len[b];
    const int32_t *p = path + (size_t)b * N;
    const bool ok = path_ok(p, a, N) && j <= a;
    const int src = ok ? p[j] : 0;
    for (int c = threadIdx.x; c < d; c += blockDim.x)
        fout[((size_t)b * N + j) * d + c] = ok ? fin[((size_t)b * N + src) * d + c] : (T)0;
}

int32_t launch_kv_compact(fg_kv_cache *kv, const int32_t *slot, const int32_t *accept_len, const int32_t *path, int B, int N,
                          const void *fin, void *fout, int d, int feat_dtype, hipStream_t st)
{
    dim3 grid(B, kv->n_layers * kv->n_kv_heads);
    int threads = kv->head_dim <= 64 ? 64 : 128;
    // pure data movement: only the element width matters
    if (kv->dtype == FG_F32)
        hipLaunchKernelGGL(kv_compact_kernel<float>, grid, dim3(threads), 0, st, (float *)kv->k_pool, (float *)kv->v_pool,
                           kv->page_table, kv->seq_len, slot, accept_len, path, N, kv->n_pages, kv->n_slots,
                           kv->max_pages_per_seq, kv->n_kv_heads, kv->head_dim, (int)k_fragment_major(kv->dtype, kv->head_dim, kv->page_size));
    else
        hipLaunchKernelGGL(kv_compact_kernel<uint16_t>, grid, dim3(threads), 0, st, (uint16_t *)kv->k_pool,
                           (uint16_t *)kv->v_pool, kv->page_table, kv->seq_len, slot, accept_len, path, N, kv->n_pages,
                           kv->n_slots, kv->max_pages_per_seq, kv->n_kv_heads, kv->head_dim, (int)k_fragment_major(kv->dtype, kv->head_dim, kv->page_size));
    FG_LAUNCH_CHECK("kv_compact");
    if (fin && fout) {
        if (feat_dtype != FG_F32)
            hipLaunchKernelGGL(gather_feature_kernel<uint16_t>, dim3(B, N), dim3(256), 0, st, (const uint16_t *)fin,
                               (uint16_t *)fout, accept_len, path, N, d);
        else
            hipLaunchKernelGGL(gather_feature_kernel<float>, dim3(B, N), dim3(256), 0, st, (const float *)fin, (float *)fout,
                               accept_len, path, N, d);
        FG_LAUNCH_CHECK("gather_feature");
    }
    hipLaunchKernelGGL(bump_len_kernel, dim3((B + 63) / 64), dim3(64), 0, st, kv->seq_len, slot, accept_len, path, B, N,
                       kv->n_slots, kv->max_pages_per_seq, kv->status);
    FG_LAUNCH_CHECK("bump_len");
    return FG_OK;
}

}  // namespace fg
