// Draft-side kernels: top-K tokens with log-probabilities per node, the frontier update between drafting
// steps, the rerank that turns the candidate lists into the verify tree, and the draft cache's length update.
#include "fg_common.h"

namespace fg {

constexpr int TK_THREADS = 1024, TK_MAX = 8;

// Per row: logsumexp over the vocabulary and the K largest logits (ties: lower index), by K block-wide argmax
// passes that skip the tokens already taken.
__global__ __launch_bounds__(TK_THREADS) void topk_logp_kernel(const float *logits, int V, int K, int32_t *tok, float *logp)
{
    __shared__ float rb[TK_THREADS / 64];
    __shared__ int ri[TK_THREADS / 64];
    __shared__ int taken[TK_MAX];
    __shared__ float lse_s;
    const int r = blockIdx.x, tid = threadIdx.x;
    const float *row = logits + (size_t)r * V;
    float mx = -INFINITY;
    for (int v = tid; v < V; v += TK_THREADS) mx = fmaxf(mx, row[v]);
    mx = wave_max(mx);
    if ((tid & 63) == 0) rb[tid >> 6] = mx;
    __syncthreads();
    mx = -INFINITY;
    for (int i = 0; i < TK_THREADS / 64; i++) mx = fmaxf(mx, rb[i]);
    __syncthreads();
    float den = 0.f;
    for (int v = tid; v < V; v += TK_THREADS) den += expf(row[v] - mx);
    den = wave_sum(den);
    if ((tid & 63) == 0) rb[tid >> 6] = den;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int i = 0; i < TK_THREADS / 64; i++) t += rb[i];
        lse_s = mx + logf(t);
    }
    __syncthreads();
    for (int k = 0; k < K; k++) {
        float best = -INFINITY;
        int bi = 0x7fffffff;
        for (int v = tid; v < V; v += TK_THREADS) {
            bool skip = false;
            for (int t = 0; t < k; t++) skip |= (taken[t] == v);
            float x = row[v];
            if (!skip && x > best) { best = x; bi = v; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ob = __shfl_xor(best, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        __syncthreads();
        if ((tid & 63) == 0) { rb[tid >> 6] = best; ri[tid >> 6] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int i = 1; i < TK_THREADS / 64; i++)
                if (rb[i] > best || (rb[i] == best && ri[i] < bi)) { best = rb[i]; bi = ri[i]; }
            taken[k] = bi;
            tok[(size_t)r * K + k] = bi;
            logp[(size_t)r * K + k] = best - lse_s;
        }
        __syncthreads();
    }
}

int32_t launch_topk_logp(const float *logits, int M, int V, int K, int32_t *tok, float *logp, hipStream_t st)
{
    if (K < 1 || K > TK_MAX || K > V) return fail(FG_ERR_INVALID_ARG, "K_draft must be in 1..%d (got %d)", TK_MAX, K);
    hipLaunchKernelGGL(topk_logp_kernel, dim3(M), dim3(TK_THREADS), 0, st, logits, V, K, tok, logp);
    FG_LAUNCH_CHECK("topk_logp");
    return FG_OK;
}

// Frontier update, one thread per sequence (at most 64 children).  With node_pick only the children of node
// node_pick[b] count (the catch-up chain's last valid row is the root; the rows before it are not expanded).
__global__ void frontier_kernel(int B, int K_in, int K, const int32_t *child_tok, const float *child_logp,
                                const int32_t *node_cand, const float *node_score, const int32_t *node_pick,
                                const int32_t *node_tok, int n_cand, int stride, int32_t *cand_tok, int32_t *cand_parent,
                                float *cand_score, int32_t *next_tok, int32_t *next_cand, float *next_score, int32_t *next_src,
                                const int32_t *parent_prev, int n_parent_prev, int32_t *parent_next)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int pick = node_pick ? min(max(node_pick[b], 0), K_in - 1) : -1;
    if (pick >= 0 && node_tok) {   // first step: candidate 0 is the root
        cand_tok[(size_t)b * stride] = node_tok[(size_t)b * K_in + pick];
        cand_parent[(size_t)b * stride] = -1;
        cand_score[(size_t)b * stride] = 0.f;
    }
    const int C = pick >= 0 ? K : K_in * K, base = pick >= 0 ? pick * K : 0;
    for (int i = 0; i < C; i++) {
        int src = (base + i) / K;
        float ps = node_score ? node_score[(size_t)b * K_in + src] : 0.f;
        int pc = node_cand ? node_cand[(size_t)b * K_in + src] : 0;
        cand_tok[(size_t)b * stride + n_cand + i] = child_tok[(size_t)b * K_in * K + base + i];
        cand_parent[(size_t)b * stride + n_cand + i] = pc;
        cand_score[(size_t)b * stride + n_cand + i] = ps + child_logp[(size_t)b * K_in * K + base + i];
    }
    uint64_t used = 0;
    for (int k = 0; k < K; k++) {
        int best = -1;
        float bs = 0.f;
        for (int i = 0; i < C; i++) {
            if ((used >> i) & 1ull) continue;
            float sc = cand_score[(size_t)b * stride + n_cand + i];
            if (best < 0 || sc > bs) { best = i; bs = sc; }
        }
        used |= 1ull << best;
        next_tok[(size_t)b * K + k] = cand_tok[(size_t)b * stride + n_cand + best];
        next_cand[(size_t)b * K + k] = n_cand + best;
        next_score[(size_t)b * K + k] = bs;
        next_src[(size_t)b * K + k] = (base + best) / K;
        // in-round parent of the new frontier node: this step's nodes are the last K_in in-round nodes; the
        // children of the root hang off the committed prefix
        if (parent_next)
            parent_next[(size_t)b * (n_parent_prev + K) + n_parent_prev + k] = pick >= 0 ? -1 : n_parent_prev - K_in + best / K;
    }
    if (parent_next)
        for (int i = 0; i < n_parent_prev; i++)
            parent_next[(size_t)b * (n_parent_prev + K) + i] = parent_prev[(size_t)b * n_parent_prev + i];
}

int32_t launch_frontier(int B, int K_in, int K, const int32_t *child_tok, const float *child_logp, const int32_t *node_cand,
                        const float *node_score, const int32_t *node_pick, const int32_t *node_tok, int n_cand, int stride,
                        int32_t *cand_tok, int32_t *cand_parent, float *cand_score, int32_t *next_tok, int32_t *next_cand,
                        float *next_score, int32_t *next_src, const int32_t *parent_prev, int n_parent_prev,
                        int32_t *parent_next, hipStream_t st)
{
    hipLaunchKernelGGL(frontier_kernel, dim3((B + 63) / 64), dim3(64), 0, st, B, K_in, K, child_tok, child_logp, node_cand,
                       node_score, node_pick, node_tok, n_cand, stride, cand_tok, cand_parent, cand_score, next_tok, next_cand, next_score,
                       next_src, parent_prev, n_parent_prev, parent_next);
    FG_LAUNCH_CHECK("frontier");
    return FG_OK;
}

// Rerank, one thread per sequence; candidate count <= 128.
constexpr int BT_MAX_CAND = 128;

__global__ void build_tree_kernel(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int B, int C,
                                  int stride, int N, int32_t *tokens, int32_t *parent, int32_t *sel)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t *ct = cand_tok + (size_t)b * stride, *cp = cand_parent + (size_t)b * stride;
    const float *cs = cand_score + (size_t)b * stride;
    uint64_t chosen[2] = {1ull, 0ull};  // candidate 0 (the root) is always in
    uint8_t depth[BT_MAX_CAND], newidx[BT_MAX_CAND];
    depth[0] = 0;
    int maxd = 0;
    for (int i = 1; i < C; i++) {
        int p = cp[i];
        p = (p < 0 || p >= i) ? 0 : p;
        depth[i] = depth[p] + 1;
    }
    for (int k = 1; k < N; k++) {
        int best = -1;
        float bs = 0.f;
        for (int i = 1; i < C; i++) {
            if ((chosen[i >> 6] >> (i & 63)) & 1ull) continue;
            if (best < 0 || cs[i] > bs) { best = i; bs = cs[i]; }
        }
        if (best < 0) break;
        chosen[best >> 6] |= 1ull << (best & 63);
        if (depth[best] > maxd) maxd = depth[best];
    }
    int n = 0;
    for (int dd = 0; dd <= maxd; dd++)
        for (int i = 0; i < C; i++) {
            if (!((chosen[i >> 6] >> (i & 63)) & 1ull) || depth[i] != dd) continue;
            newidx[i] = (uint8_t)n;
            tokens[(size_t)b * N + n] = ct[i];
            int par = -1;
            if (i > 0) {
                int p = cp[i];
                p = (p < 0 || p >= i) ? 0 : p;
                par = ((chosen[p >> 6] >> (p & 63)) & 1ull) ? newidx[p] : 0;   // unselected parent: re-attach to the root
            }
            parent[(size_t)b * N + n] = par;
            if (sel) sel[(size_t)b * N + n] = i;
            n++;
        }
}

int32_t launch_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int B, int C, int stride,
                          int N, int32_t *tokens, int32_t *parent, int32_t *sel, hipStream_t st)
{
    if (C > BT_MAX_CAND) return fail(FG_ERR_CAPACITY, "at most %d candidates (got %d)", BT_MAX_CAND, C);
    hipLaunchKernelGGL(build_tree_kernel, dim3((B + 63) / 64), dim3(64), 0, st, cand_tok, cand_parent, cand_score, B, C,
                       stride, N, tokens, parent, sel);
    FG_LAUNCH_CHECK("build_tree");
    return FG_OK;
}

__global__ void commit_len_kernel(int32_t *seq_len, const int32_t *slot, const int32_t *n_commit, int bias, int B, int n_slots)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int s = min(max(slot[b], 0), n_slots - 1);
    seq_len[s] += max(n_commit[b] + bias, 0);
}

int32_t launch_commit_len(int32_t *seq_len, const int32_t *slot, const int32_t *n_commit, int bias, int B, int n_slots,
                          hipStream_t st)
{
    hipLaunchKernelGGL(commit_len_kernel, dim3((B + 63) / 64), dim3(64), 0, st, seq_len, slot, n_commit, bias, B, n_slots);
    FG_LAUNCH_CHECK("commit_len");
    return FG_OK;
}

}  // namespace fg
