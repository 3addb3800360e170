// Draft-side kernels: top-K tokens with log-probabilities per node, the frontier update between drafting
// steps, the rerank that turns the candidate lists into the verify tree, and the draft cache's length update.
#include "fg_common.h"

namespace fg {

constexpr int TK_THREADS = 1024, TK_MAX = 8;
constexpr int TK_REDO = -1;   // first token of a row the selective kernel hands to the general one

// Per row, in ONE pass over the logits: every thread keeps an online (max, sum of exponentials) pair and the
// TK_MAX largest of its own elements, sorted (value descending, index ascending on ties: a thread meets its indices
// in ascending order and a new element is placed behind equal ones).  The block then combines the pairs into the
// row's logsumexp and pops the K overall winners from the heads of the threads' lists, one block-wide
// (value, lowest index) arg-max per winner.
struct TopList {
    float v[TK_MAX];
    int i[TK_MAX];
};

__device__ __forceinline__ void toplist_insert(TopList &t, float x, int idx)
{
    if (!(x > t.v[TK_MAX - 1])) return;
    t.v[TK_MAX - 1] = x;
    t.i[TK_MAX - 1] = idx;
#pragma unroll
    for (int j = TK_MAX - 1; j > 0; j--) {
        const bool up = t.v[j] > t.v[j - 1];
        const float fv = t.v[j - 1];
        const int fi = t.i[j - 1];
        t.v[j - 1] = up ? t.v[j] : fv;
        t.i[j - 1] = up ? t.i[j] : fi;
        t.v[j] = up ? fv : t.v[j];
        t.i[j] = up ? fi : t.i[j];
    }
}

__device__ __forceinline__ void online_add(float &m, float &sum, float x)
{
    if (x > m) {
        sum = sum * __expf(m - x) + 1.f;   // m = -inf: exp(-inf) = 0
        m = x;
    } else {
        sum += __expf(x - m);
    }
}

__global__ __launch_bounds__(TK_THREADS) void topk_logp_kernel(const float *logits, int V, int K, int32_t *tok, float *logp,
                                                               int only_marked)
{
    __shared__ float rb[TK_THREADS / 64];
    __shared__ int ri[TK_THREADS / 64];
    __shared__ float sm[TK_THREADS / 64], ss[TK_THREADS / 64];
    const int r = blockIdx.x, tid = threadIdx.x;
    if (only_marked && tok[(size_t)r * K] != TK_REDO) return;   // the selective kernel finished this row
    const float *row = logits + (size_t)r * V;
    TopList t;
#pragma unroll
    for (int j = 0; j < TK_MAX; j++) { t.v[j] = -INFINITY; t.i[j] = 0x7fffffff; }
    float m = -INFINITY, sum = 0.f;
    if ((V & 3) == 0) {
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
        for (int q = tid; q < (V >> 2); q += TK_THREADS) {
            const float4 x = row4[q];
            const float xs[4] = {x.x, x.y, x.z, x.w};
            const float m4 = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
            if (m4 > m) {   // one rescale per quad
                sum *= __expf(m - m4);
                m = m4;
            }
#pragma unroll
            for (int c = 0; c < 4; c++) sum += __expf(xs[c] - m);
            if (m4 > t.v[TK_MAX - 1]) {
#pragma unroll
                for (int c = 0; c < 4; c++) toplist_insert(t, xs[c], q * 4 + c);
            }
        }
    } else {
        for (int v = tid; v < V; v += TK_THREADS) {
            const float x = row[v];
            online_add(m, sum, x);
            toplist_insert(t, x, v);
        }
    }
    // logsumexp of the row
    const float wm = wave_max(m);
    float wsum = sum * (m == -INFINITY ? 0.f : __expf(m - wm));
    wsum = wave_sum(wsum);
    if ((tid & 63) == 0) { sm[tid >> 6] = wm; ss[tid >> 6] = wsum; }
    __syncthreads();
    float bm = -INFINITY;
    for (int i = 0; i < TK_THREADS / 64; i++) bm = fmaxf(bm, sm[i]);
    float bs = 0.f;
    for (int i = 0; i < TK_THREADS / 64; i++) bs += ss[i] * (sm[i] == -INFINITY ? 0.f : __expf(sm[i] - bm));
    const float lse = bm + logf(bs);
    // K winners
    for (int k = 0; k < K; k++) {
        float best = t.v[0];
        int bi = t.i[0];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ob = __shfl_xor(best, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        __syncthreads();   // the previous round's readers are done with rb / ri
        if ((tid & 63) == 0) { rb[tid >> 6] = best; ri[tid >> 6] = bi; }
        __syncthreads();
        best = rb[0]; bi = ri[0];
        for (int i = 1; i < TK_THREADS / 64; i++)
            if (rb[i] > best || (rb[i] == best && ri[i] < bi)) { best = rb[i]; bi = ri[i]; }
        if (t.i[0] == bi) {   // this thread owned the winner: pop it
#pragma unroll
            for (int j = 0; j + 1 < TK_MAX; j++) { t.v[j] = t.v[j + 1]; t.i[j] = t.i[j + 1]; }
            t.v[TK_MAX - 1] = -INFINITY;
            t.i[TK_MAX - 1] = 0x7fffffff;
        }
        if (tid == 0) {
            tok[(size_t)r * K + k] = bi;
            logp[(size_t)r * K + k] = best - lse;
        }
    }
}

// The same result for rows whose vocabulary is a multiple of four, with far less arithmetic per element.  The
// general kernel keeps a sorted list per thread; some lane of a wave wants an insertion at almost every step, so
// every wave walks the insertion code for all of its elements (70 us for a row of 152 064 whatever the number of
// rows up to 256).  Here the one pass over the row only takes each thread's maximum and its online sum of
// exponentials.  The K-th largest of the 1024 thread maxima, tau, is a lower bound of the row's K-th largest entry,
// and entries >= tau can only sit in threads whose maximum is >= tau -- K of them unless values tie.  Their few
// quads are read again (a few KiB, cooperatively), the entries >= tau are collected in LDS, and K block-wide
// (value, lowest index) arg-max rounds pick the winners as before.  Rows with more tied candidates than the lists
// hold are marked (first token = TK_REDO) and redone by the general kernel, which is launched behind this one and
// returns at once for every other row.
constexpr int TK_HOT_MAX = 64, TK_CAND_MAX = 2 * TK_THREADS;

__global__ __launch_bounds__(TK_THREADS) void topk_logp_select_kernel(const float *logits, int V, int K, int32_t *tok, float *logp)
{
    __shared__ float rb[TK_THREADS / 64];
    __shared__ int ri[TK_THREADS / 64];
    __shared__ float sm[TK_THREADS / 64], ss[TK_THREADS / 64];
    __shared__ int hot[TK_HOT_MAX];
    __shared__ int hot_n, cand_n;
    __shared__ float cv[TK_CAND_MAX];
    __shared__ int ci[TK_CAND_MAX];
    const int r = blockIdx.x, tid = threadIdx.x;
    const float4 *row4 = reinterpret_cast<const float4 *>(logits + (size_t)r * V);
    const int nq = V >> 2, qpt = (nq + TK_THREADS - 1) / TK_THREADS;
    if (tid == 0) { hot_n = 0; cand_n = 0; }

    // pass over the row: thread maximum and online sum of exponentials, four quads requested together
    float m = -INFINITY, sum = 0.f;
    auto take = [&](const float4 x) {
        const float m4 = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
        if (m4 > m) {   // one rescale per quad
            sum *= __expf(m - m4);
            m = m4;
        }
        sum += (__expf(x.x - m) + __expf(x.y - m)) + (__expf(x.z - m) + __expf(x.w - m));
    };
    int q = tid;
    for (; q + 3 * TK_THREADS < nq; q += 4 * TK_THREADS) {
        const float4 x0 = row4[q], x1 = row4[q + TK_THREADS], x2 = row4[q + 2 * TK_THREADS], x3 = row4[q + 3 * TK_THREADS];
        take(x0); take(x1); take(x2); take(x3);
    }
    for (; q < nq; q += TK_THREADS) take(row4[q]);

    // logsumexp of the row
    const float wm = wave_max(m);
    float wsum = sum * (m == -INFINITY ? 0.f : __expf(m - wm));
    wsum = wave_sum(wsum);
    if ((tid & 63) == 0) { sm[tid >> 6] = wm; ss[tid >> 6] = wsum; }
    __syncthreads();
    float bm = -INFINITY;
    for (int i = 0; i < TK_THREADS / 64; i++) bm = fmaxf(bm, sm[i]);
    float bs = 0.f;
    for (int i = 0; i < TK_THREADS / 64; i++) bs += ss[i] * (sm[i] == -INFINITY ? 0.f : __expf(sm[i] - bm));
    const float lse = bm + logf(bs);

    // block-wide (value, lowest index) arg-max over one (value, index) pair per thread
    auto block_argmax = [&](float &best, int &bi) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ob = __shfl_xor(best, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        __syncthreads();   // the previous round's readers are done with rb / ri
        if ((tid & 63) == 0) { rb[tid >> 6] = best; ri[tid >> 6] = bi; }
        __syncthreads();
        best = rb[0]; bi = ri[0];
        for (int i = 1; i < TK_THREADS / 64; i++)
            if (rb[i] > best || (rb[i] == best && ri[i] < bi)) { best = rb[i]; bi = ri[i]; }
    };

    // tau = the K-th largest thread maximum
    float cur = m, tau = -INFINITY;
    for (int k = 0; k < K; k++) {
        float best = cur;
        int bi = tid;
        block_argmax(best, bi);
        if (bi == tid) cur = -INFINITY;
        tau = best;
    }
    // threads that can hold an entry >= tau, then their quads once more
    if (m >= tau) {
        const int p = atomicAdd(&hot_n, 1);
        if (p < TK_HOT_MAX) hot[p] = tid;
    }
    __syncthreads();
    const int n_hot = hot_n;
    bool redo = n_hot > TK_HOT_MAX || !(tau > -INFINITY);
    if (!redo) {
        for (int it = tid; it < n_hot * qpt; it += TK_THREADS) {
            const int qq = hot[it / qpt] + (it % qpt) * TK_THREADS;
            if (qq >= nq) continue;
            const float4 x = row4[qq];
            const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int c = 0; c < 4; c++)
                if (xs[c] >= tau) {
                    const int p = atomicAdd(&cand_n, 1);
                    if (p < TK_CAND_MAX) { cv[p] = xs[c]; ci[p] = qq * 4 + c; }
                }
        }
        __syncthreads();
        redo = cand_n > TK_CAND_MAX;
    }
    if (redo) {
        if (tid == 0) tok[(size_t)r * K] = TK_REDO;
        return;
    }
    // K winners among the candidates: a thread owns candidates tid and tid + TK_THREADS
    const int n_cand = cand_n;
    float v0 = tid < n_cand ? cv[tid] : -INFINITY, v1 = tid + TK_THREADS < n_cand ? cv[tid + TK_THREADS] : -INFINITY;
    int i0 = tid < n_cand ? ci[tid] : 0x7fffffff, i1 = tid + TK_THREADS < n_cand ? ci[tid + TK_THREADS] : 0x7fffffff;
    if (v1 > v0 || (v1 == v0 && i1 < i0)) {
        const float tv = v0; v0 = v1; v1 = tv;
        const int ti = i0; i0 = i1; i1 = ti;
    }
    for (int k = 0; k < K; k++) {
        float best = v0;
        int bi = i0;
        block_argmax(best, bi);
        if (i0 == bi) { v0 = v1; i0 = i1; v1 = -INFINITY; i1 = 0x7fffffff; }   // this thread owned the winner
        if (tid == 0) {
            tok[(size_t)r * K + k] = bi;
            logp[(size_t)r * K + k] = best - lse;
        }
    }
}

int32_t launch_topk_logp(const float *logits, int M, int V, int K, int32_t *tok, float *logp, hipStream_t st)
{
    if (K < 1 || K > TK_MAX || K > V) return fail(FG_ERR_INVALID_ARG, "K_draft must be in 1..%d (got %d)", TK_MAX, K);
    const bool selective = (V & 3) == 0 && V >= 4 * TK_THREADS;
    if (selective) {
        hipLaunchKernelGGL(topk_logp_select_kernel, dim3(M), dim3(TK_THREADS), 0, st, logits, V, K, tok, logp);
        FG_LAUNCH_CHECK("topk_logp_select");
    }
    hipLaunchKernelGGL(topk_logp_kernel, dim3(M), dim3(TK_THREADS), 0, st, logits, V, K, tok, logp, selective ? 1 : 0);
    FG_LAUNCH_CHECK("topk_logp");
    return FG_OK;
}

// ---- merge of the LM head's per-block partials (the GEMM's top-k epilogue) ----------------------------------------
// One block per row: the row's n_blocks x K (value, column) candidates and n_blocks (max, sum exp) pairs become the K
// largest entries of the row (ties to the lower column), their log-softmax values (when the pairs are given) and / or
// the arg-max and the two largest values.
constexpr int TM_THREADS = 256;
__global__ __launch_bounds__(TM_THREADS) void topk_merge_kernel(const float *__restrict__ part_val, const int32_t *__restrict__ part_idx,
                                                                const float *__restrict__ part_ms, int n_blocks, int K,
                                                                int32_t *tok, float *logp, int32_t *row_argmax, float *row_top2)
{
    __shared__ float rb[TM_THREADS / 64];
    __shared__ int ri[TM_THREADS / 64];
    const int r = blockIdx.x, tid = threadIdx.x;
    const int n = n_blocks * K;
    const float *pv = part_val + (size_t)r * n;
    const int32_t *pi = part_idx + (size_t)r * n;
    float lse = 0.f;
    if (part_ms) {
        const float *ms = part_ms + (size_t)r * n_blocks * 2;
        float mx = -INFINITY;
        for (int b = tid; b < n_blocks; b += TM_THREADS) mx = fmaxf(mx, ms[2 * b]);
        mx = wave_max(mx);
        if ((tid & 63) == 0) rb[tid >> 6] = mx;
        __syncthreads();
        mx = rb[0];
        for (int i = 1; i < TM_THREADS / 64; i++) mx = fmaxf(mx, rb[i]);
        __syncthreads();
        float sum = 0.f;
        for (int b = tid; b < n_blocks; b += TM_THREADS) sum += ms[2 * b + 1] * __expf(ms[2 * b] - mx);
        sum = wave_sum(sum);
        if ((tid & 63) == 0) rb[tid >> 6] = sum;
        __syncthreads();
        sum = 0.f;
        for (int i = 0; i < TM_THREADS / 64; i++) sum += rb[i];
        lse = mx + logf(sum);
        __syncthreads();
    }
    float lv = INFINITY;
    int li = -1;
    for (int k = 0; k < K; k++) {
        float best = -INFINITY;
        int bi = 0x7fffffff;
        for (int e = tid; e < n; e += TM_THREADS) {
            const float v = pv[e];
            const int c = pi[e];
            const bool after = lv > v || (lv == v && li < c);
            if (after && (v > best || (v == best && c < bi))) { best = v; bi = c; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ob = __shfl_xor(best, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        __syncthreads();
        if ((tid & 63) == 0) { rb[tid >> 6] = best; ri[tid >> 6] = bi; }
        __syncthreads();
        best = rb[0]; bi = ri[0];
        for (int i = 1; i < TM_THREADS / 64; i++)
            if (rb[i] > best || (rb[i] == best && ri[i] < bi)) { best = rb[i]; bi = ri[i]; }
        lv = best; li = bi;
        if (tid == 0) {
            if (tok) tok[(size_t)r * K + k] = bi;
            if (logp) logp[(size_t)r * K + k] = best - lse;
            if (k == 0 && row_argmax) row_argmax[r] = bi;
            if (k < 2 && row_top2) row_top2[2 * r + k] = best;
        }
    }
}

int32_t launch_topk_merge(const float *part_val, const int32_t *part_idx, const float *part_ms, int M, int n_blocks, int K,
                          int32_t *tok, float *logp, int32_t *row_argmax, float *row_top2, hipStream_t st)
{
    hipLaunchKernelGGL(topk_merge_kernel, dim3(M), dim3(TM_THREADS), 0, st, part_val, part_idx, part_ms, n_blocks, K, tok, logp,
                       row_argmax, row_top2);
    FG_LAUNCH_CHECK("topk_merge");
    return FG_OK;
}

// Frontier update, one thread per sequence (at most 64 children).  With node_pick only the children of node
// node_pick[b] count (the catch-up chain's last valid row is the root; the rows before it are not expanded).
__global__ void frontier_kernel(int B, int K_in, int K, const int32_t *child_tok, const float *child_logp, int child_rows,
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
    // child lists: child_rows rows of K per sequence; with one row it is the picked node's
    const size_t cbase = (size_t)b * child_rows * K + (child_rows == 1 ? 0 : base);
    for (int i = 0; i < C; i++) {
        int src = (base + i) / K;
        float ps = node_score ? node_score[(size_t)b * K_in + src] : 0.f;
        int pc = node_cand ? node_cand[(size_t)b * K_in + src] : 0;
        cand_tok[(size_t)b * stride + n_cand + i] = child_tok[cbase + i];
        cand_parent[(size_t)b * stride + n_cand + i] = pc;
        cand_score[(size_t)b * stride + n_cand + i] = ps + child_logp[cbase + i];
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

int32_t launch_frontier(int B, int K_in, int K, const int32_t *child_tok, const float *child_logp, int child_rows,
                        const int32_t *node_cand, const float *node_score, const int32_t *node_pick, const int32_t *node_tok, int n_cand, int stride,
                        int32_t *cand_tok, int32_t *cand_parent, float *cand_score, int32_t *next_tok, int32_t *next_cand,
                        float *next_score, int32_t *next_src, const int32_t *parent_prev, int n_parent_prev,
                        int32_t *parent_next, hipStream_t st)
{
    hipLaunchKernelGGL(frontier_kernel, dim3((B + 63) / 64), dim3(64), 0, st, B, K_in, K, child_tok, child_logp, child_rows, node_cand,
                       node_score, node_pick, node_tok, n_cand, stride, cand_tok, cand_parent, cand_score, next_tok, next_cand, next_score,
                       next_src, parent_prev, n_parent_prev, parent_next);
    FG_LAUNCH_CHECK("frontier");
    return FG_OK;
}

// Rerank, one wave per sequence; at most 128 candidates, two per lane.  Candidate 0 (the root) is always in; a
// non-root candidate is chosen when fewer than N - 1 others beat it (higher score, or equal score and lower
// index); a chosen candidate's node index is the number of chosen ones before it in (depth, index) order.
constexpr int BT_MAX_CAND = 128;

__global__ __launch_bounds__(64) void build_tree_kernel(const int32_t *cand_tok, const int32_t *cand_parent,
                                                          const float *cand_score, int B, int C, int stride, int N,
                                                          int32_t *tokens, int32_t *parent, int32_t *sel)
{
    __shared__ float sc[BT_MAX_CAND];
    __shared__ int par[BT_MAX_CAND], dep[BT_MAX_CAND], chosen[BT_MAX_CAND], newidx[BT_MAX_CAND];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int32_t *ct = cand_tok + (size_t)b * stride, *cp = cand_parent + (size_t)b * stride;
    const float *cs = cand_score + (size_t)b * stride;
    for (int i = lane; i < C; i += 64) {
        int p = cp[i];
        par[i] = (i == 0) ? -1 : ((p < 0 || p >= i) ? 0 : p);   // malformed parents hang off the root
        sc[i] = cs[i];
    }
    __syncthreads();
    for (int i = lane; i < C; i += 64) {
        int d = 0;
        for (int p = par[i]; p >= 0 && d < BT_MAX_CAND; p = par[p]) d++;
        dep[i] = d;
        int beat = 0;
        const float mine = sc[i];
        for (int j = 1; j < C; j++) beat += (sc[j] > mine) || (sc[j] == mine && j < i);
        chosen[i] = (i == 0) || beat < N - 1;
    }
    __syncthreads();
    for (int i = lane; i < C; i += 64) {
        int before = 0;
        const int d = dep[i];
        for (int j = 0; j < C; j++) before += chosen[j] && (dep[j] < d || (dep[j] == d && j < i));
        newidx[i] = before;
    }
    __syncthreads();
    for (int i = lane; i < C; i += 64) {
        if (!chosen[i]) continue;
        const int n = newidx[i];
        int pn = -1;
        if (i > 0) pn = chosen[par[i]] ? newidx[par[i]] : 0;   // unselected parent: re-attach to the root
        tokens[(size_t)b * N + n] = ct[i];
        parent[(size_t)b * N + n] = pn;
        if (sel) sel[(size_t)b * N + n] = i;
    }
}

int32_t launch_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int B, int C, int stride,
                          int N, int32_t *tokens, int32_t *parent, int32_t *sel, hipStream_t st)
{
    if (C > BT_MAX_CAND) return fail(FG_ERR_CAPACITY, "at most %d candidates (got %d)", BT_MAX_CAND, C);
    if (B <= 0) return FG_OK;
    hipLaunchKernelGGL(build_tree_kernel, dim3(B), dim3(64), 0, st, cand_tok, cand_parent, cand_score, B, C, stride, N, tokens,
                       parent, sel);
    FG_LAUNCH_CHECK("build_tree");
    return FG_OK;
}

// A commit that would run past the page table is not applied and raises FG_CACHE_OVERFLOW in the cache's status word.
__global__ void commit_len_kernel(int32_t *seq_len, const int32_t *slot, const int32_t *n_commit, int bias, int B, int n_slots,
                                  int capacity, int32_t *status)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int s = min(max(slot[b], 0), n_slots - 1);
    const int L = seq_len[s] + max(n_commit[b] + bias, 0);
    if (L > capacity) {
        if (status) atomicOr(status, (int32_t)FG_CACHE_OVERFLOW);
        return;
    }
    seq_len[s] = L;
}

int32_t launch_commit_len(int32_t *seq_len, const int32_t *slot, const int32_t *n_commit, int bias, int B, int n_slots,
                          int capacity, int32_t *status, hipStream_t st)
{
    hipLaunchKernelGGL(commit_len_kernel, dim3((B + 63) / 64), dim3(64), 0, st, seq_len, slot, n_commit, bias, B, n_slots,
                       capacity, status);
    FG_LAUNCH_CHECK("commit_len");
    return FG_OK;
}

}  // namespace fg
