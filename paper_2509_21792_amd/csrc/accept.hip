// Acceptance kernels: the strict-match walk (greedy or one Gumbel-max sample per node) and rejection sampling
// over sibling sets.  Integer work apart from the softmax / residual arithmetic of the rejection mode.
#include "fg_common.h"

namespace fg {

// ---- target token per node by Gumbel-max: argmax_v logits[v] / T + Gumbel(seed, row, v) ---------------------
__global__ __launch_bounds__(1024) void gumbel_argmax_kernel(const float *logits, int V, float T, uint64_t seed,
                                                             int64_t row0, int32_t *idx)
{
    __shared__ float rb[16];
    __shared__ int ri[16];
    const int r = blockIdx.x, tid = threadIdx.x;
    const float *row = logits + (size_t)r * V;
    const uint64_t key = row_key(seed, (uint64_t)(row0 + r));
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = tid; v < V; v += blockDim.x) {
        float s = row[v] / T + gumbel_from_key(key, (uint64_t)v);
        if (s > best) { best = s; bi = v; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ob = __shfl_xor(best, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
    }
    if ((tid & 63) == 0) { rb[tid >> 6] = best; ri[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < (int)(blockDim.x >> 6); i++)
            if (rb[i] > best || (rb[i] == best && ri[i] < bi)) { best = rb[i]; bi = ri[i]; }
        idx[r] = bi;
    }
}

int32_t launch_gumbel_argmax(const float *logits, int M, int V, float T, uint64_t seed, int64_t row0, int32_t *idx, hipStream_t st)
{
    hipLaunchKernelGGL(gumbel_argmax_kernel, dim3(M), dim3(1024), 0, st, logits, V, T, seed, row0, idx);
    FG_LAUNCH_CHECK("gumbel_argmax");
    return FG_OK;
}

// ---- strict-match walk: one thread per sequence -------------------------------------------------------------
__global__ void walk_kernel(int B, int N, const int32_t *tokens, const int32_t *parent, const int32_t *target_tok,
                            int32_t eos, int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int32_t *tok = tokens + (size_t)b * N, *par = parent + (size_t)b * N, *tt = target_tok + (size_t)b * N;
    int32_t *pp = path + (size_t)b * N, *ot = out_tokens + (size_t)b * N;
    for (int j = 0; j < N; j++) { pp[j] = -1; ot[j] = -1; }
    int u = 0, a = 0, fin = 0;
    pp[0] = 0;
    for (int guard = 0; guard < N; guard++) {
        int t = tt[u];
        ot[a] = t;
        if (t == eos) { fin = 1; break; }
        int next = -1;
        for (int ch = u + 1; ch < N; ch++)
            if (par[ch] == u && tok[ch] == t) { next = ch; break; }
        if (next < 0) break;
        u = next;
        a++;
        pp[a] = u;
    }
    accept_len[b] = a;
    finished[b] = fin;
}

int32_t launch_walk(int B, int N, const int32_t *tokens, const int32_t *parent, const int32_t *target_tok, int32_t eos,
                    int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished, hipStream_t st)
{
    hipLaunchKernelGGL(walk_kernel, dim3((B + 63) / 64), dim3(64), 0, st, B, N, tokens, parent, target_tok, eos, accept_len,
                       path, out_tokens, finished);
    FG_LAUNCH_CHECK("walk");
    return FG_OK;
}

// ---- rejection sampling: one block per sequence --------------------------------------------------------------
constexpr int RJ_THREADS = 1024;

__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < RJ_THREADS / 64; i++) t += red[i];
    return t;
}
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = -INFINITY;
    for (int i = 0; i < RJ_THREADS / 64; i++) t = fmaxf(t, red[i]);
    return t;
}

__global__ __launch_bounds__(RJ_THREADS) void reject_kernel(int N, int V, const int32_t *tokens, const int32_t *parent,
                                                            const float *logits, const float *draft_probs,
                                                            const float *unif, float T, uint64_t seed, int64_t row0,
                                                            int32_t eos, float *ws, int32_t *accept_len, int32_t *path,
                                                            int32_t *out_tokens, int32_t *finished)
{
    __shared__ float red[RJ_THREADS / 64];
    __shared__ int redi[RJ_THREADS / 64];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int32_t *tok = tokens + (size_t)b * N, *par = parent + (size_t)b * N;
    int32_t *pp = path + (size_t)b * N, *ot = out_tokens + (size_t)b * N;
    float *p = ws + (size_t)b * 2 * V, *q = p + V;
    for (int j = tid; j < N; j += RJ_THREADS) { pp[j] = -1; ot[j] = -1; }
    __syncthreads();
    int u = 0, a = 0, fin = 0;
    if (tid == 0) pp[0] = 0;
    for (int guard = 0; guard < N; guard++) {
        const float *lg = logits + ((size_t)b * N + u) * V;
        float mx = -INFINITY;
        for (int v = tid; v < V; v += RJ_THREADS) mx = fmaxf(mx, lg[v] / T);
        mx = block_max(mx, red);
        float den = 0.f;
        for (int v = tid; v < V; v += RJ_THREADS) {
            float e = expf(lg[v] / T - mx);
            p[v] = e;
            den += e;
        }
        den = block_sum(den, red);
        const float *dq = draft_probs + ((size_t)b * N + u) * V;
        for (int v = tid; v < V; v += RJ_THREADS) { p[v] = p[v] / den; q[v] = dq[v]; }
        __syncthreads();
        int next = -1;
        for (int ch = u + 1; ch < N; ch++) {
            if (par[ch] != u) continue;
            int x = min(max(tok[ch], 0), V - 1);
            float px = p[x], qx = q[x];
            float ratio = qx > 0.f ? px / qx : (px > 0.f ? INFINITY : 0.f);
            ratio = fminf(ratio, 1.f);
            if (unif[(size_t)b * N + ch] < ratio) { next = ch; break; }
            __syncthreads();  // everyone has read p[x], q[x]
            float sp = 0.f;
            for (int v = tid; v < V; v += RJ_THREADS) {
                float t = fmaxf(p[v] - q[v], 0.f);
                p[v] = t;
                sp += t;
            }
            sp = block_sum(sp, red);
            if (tid == 0) q[x] = 0.f;
            __syncthreads();
            float sq = 0.f;
            for (int v = tid; v < V; v += RJ_THREADS) sq += q[v];
            sq = block_sum(sq, red);
            for (int v = tid; v < V; v += RJ_THREADS) {
                if (sp > 0.f) p[v] = p[v] / sp;
                if (sq > 0.f) q[v] = q[v] / sq;
            }
            __syncthreads();
        }
        if (next >= 0) {
            int t = tok[next];
            if (tid == 0) ot[a] = t;
            if (t == eos) { fin = 1; break; }
            u = next;
            a++;
            if (tid == 0) pp[a] = u;
            __syncthreads();
            continue;
        }
        // bonus token: Gumbel-max over the current p
        const uint64_t key = row_key(seed, (uint64_t)(row0 + (int64_t)b * N + u));
        float best = -INFINITY;
        int bi = 0x7fffffff;
        for (int v = tid; v < V; v += RJ_THREADS) {
            float pv = p[v];
            if (pv > 0.f) {
                float s = logf(pv) + gumbel_from_key(key, (uint64_t)v);
                if (s > best) { best = s; bi = v; }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ob = __shfl_xor(best, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        __syncthreads();
        if ((tid & 63) == 0) { red[tid >> 6] = best; redi[tid >> 6] = bi; }
        __syncthreads();
        for (int i = 0; i < RJ_THREADS / 64; i++)
            if (red[i] > best || (red[i] == best && redi[i] < bi)) { best = red[i]; bi = redi[i]; }
        if (tid == 0) ot[a] = bi;
        if (bi == eos) fin = 1;
        break;
    }
    if (tid == 0) { accept_len[b] = a; finished[b] = fin; }
}

int32_t launch_reject(int B, int N, int V, const int32_t *tokens, const int32_t *parent, const float *logits,
                      const float *draft_probs, const float *unif, float T, uint64_t seed, int64_t row0, int32_t eos,
                      float *ws, int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished, hipStream_t st)
{
    hipLaunchKernelGGL(reject_kernel, dim3(B), dim3(RJ_THREADS), 0, st, N, V, tokens, parent, logits, draft_probs, unif, T,
                       seed, row0, eos, ws, accept_len, path, out_tokens, finished);
    FG_LAUNCH_CHECK("reject");
    return FG_OK;
}

}  // namespace fg
