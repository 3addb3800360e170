/*
 * fg_oracle.c -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of the batched speculative
 * decoding step of FastGRPO's generation phase (Alg. 1, the speculative part of
 * the generation loop; Sec. 2 "Speculative Decoding", "Draft Model
 * Architectures", "Verification Strategies"; Sec. 4.1 Eq. 1-3).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load
 * this library.  It shares no code with the HIP library: no headers, no
 * helpers, no tables.  There is no blocking, fusion or reordering beyond what
 * the definitions state: every matrix product is a loop of dot products, the
 * KV cache is one contiguous array per sequence, attention walks the keys in
 * position order.
 *
 * Precision: `real` is float by default (the fp32 oracle the tolerances are
 * quoted against); build with -DORC_REAL=double for the fp64 twin used by the
 * pins.  Every row of the batch runs the same scalar code whatever the batch
 * is, so results are bitwise independent of batch composition: greedy
 * speculative output equals plain greedy decoding with no tolerance.
 *
 * Parity status of each function (what pins it, see tests/test_oracle_*.py):
 *   orc_plan           Eq. 1-3 worked table (tests/golden/plan_table.txt)
 *   orc_tree_forward   torch fp64 library ops on chain / N=1 cases; tree pass
 *                      == linear passes; RoPE invariants
 *   orc_row_argmax / orc_walk / orc_kv_compact
 *                      speculative greedy == autoregressive greedy
 *   orc_accept_reject  chi-square against the target distribution
 *   orc_gumbel_scores  chi-square against softmax(logits/T)
 *   orc_topk_logp      scipy logsumexp + argsort on small cases
 *   orc_build_tree     brute force on tiny candidate sets
 *   orc_topk_index + the frontier / candidate-list bookkeeping of
 *   oracle/loop.py: draft_expand
 *                      brute force over every token path of a tiny vocabulary
 *                      (tests/test_oracle_draft_expand.py)
 *   orc_knee           exact break point of two-segment curves; invariance
 *                      under affine maps of either axis
 *   draft head internals (fc + one layer, no final norm): fixed by this
 *   build's reading of Sec. 2 only -- "parity unpinned" beyond the shared
 *   layer code.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORC_REAL
#define ORC_REAL float
#endif
typedef ORC_REAL real;

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t pad_;
    double rms_eps, rope_theta;
} orc_cfg;

/* All matrices are [out, in] row-major (in contiguous). */
typedef struct {
    const real *embed;             /* [vocab, d]                                  */
    const real *lm_head;           /* [vocab, d]                                  */
    const real *final_norm;        /* [d] (target only)                           */
    const real *fc;                /* [d, 2d] (draft only): in = embed ++ feature */
    const real *const *wqkv;       /* per layer [(Hq + 2 Hkv) * hd, d]: q, k, v   */
    const real *const *wo;         /* per layer [d, Hq * hd]                      */
    const real *const *w_gate;     /* per layer [F, d]                            */
    const real *const *w_up;       /* per layer [F, d]                            */
    const real *const *w_down;     /* per layer [d, F]                            */
    const real *const *norm_attn;  /* per layer [d]                               */
    const real *const *norm_ffn;   /* per layer [d]                               */
} orc_weights;

enum { ORC_OK = 0, ORC_ERR_ARG = -1, ORC_ERR_TREE = -2, ORC_ERR_CAP = -3 };

int orc_sizeof_real(void) { return (int)sizeof(real); }

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------------ */
/* Eq. 1-3: tree shape from live concurrency.                               */
/* N = floor(C_peak / B) clamped to [1, N_cap]; K = min(N-1, K_max);        */
/* L = min(floor(log2(N / alpha)), L_max) clamped to [0, N-1]; K or L zero   */
/* means plain decoding (N = 1); N cannot exceed the candidate count        */
/* 1 + K + (L-1) K^2 (Sec. 4.1, text after Eq. 2).                           */
/* ------------------------------------------------------------------------ */
int orc_plan(int32_t B_cur, double C_peak, double alpha, int32_t K_max, int32_t L_max, int32_t N_cap,
             int32_t *N_verify, int32_t *K_draft, int32_t *L_draft)
{
    if (B_cur < 1 || !(C_peak > 0) || !(alpha > 0) || K_max < 0 || L_max < 0 || N_cap < 1) return ORC_ERR_ARG;
    double n = floor(C_peak / (double)B_cur);
    int64_t N = (int64_t)n;
    if (N < 1) N = 1;
    if (N > N_cap) N = N_cap;
    int64_t K = N - 1 < K_max ? N - 1 : K_max;
    /* floor(log2(N/alpha)) by exact comparison, no libm rounding at powers of two */
    int64_t L = 0;
    double ratio = (double)N / alpha;
    if (ratio < 1.0) L = 0;
    else { while (ldexp(1.0, (int)(L + 1)) <= ratio) L++; }
    if (L > L_max) L = L_max;
    if (L > N - 1) L = N - 1;
    if (L < 0) L = 0;
    if (K <= 0 || L <= 0) { K = 0; L = 0; N = 1; }
    else {
        int64_t cand = 1 + K + (L - 1) * K * K;
        if (N > cand) N = cand;
    }
    *N_verify = (int32_t)N; *K_draft = (int32_t)K; *L_draft = (int32_t)L;
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Knee of a latency curve (appendix, empirical measurement of C_peak: the   */
/* batch size at which latency stops being flat).  The paper names no        */
/* detector; the reading taken: scale both axes to [0, 1] and return the     */
/* sample that lies farthest below the chord through the first and the last  */
/* sample (first such sample on ties).  x must increase strictly.            */
/* ------------------------------------------------------------------------ */
int orc_knee(const double *x, const double *y, int64_t n, int64_t *knee)
{
    if (!x || !y || !knee || n < 3) return ORC_ERR_ARG;
    double ylo = y[0], yhi = y[0];
    for (int64_t i = 1; i < n; i++) {
        if (!(x[i] > x[i - 1])) return ORC_ERR_ARG;
        if (y[i] < ylo) ylo = y[i];
        if (y[i] > yhi) yhi = y[i];
    }
    const double xs = x[n - 1] - x[0], ys = yhi - ylo;
    int64_t best = 0;
    double best_d = 0.0;
    if (ys > 0) {
        const double y0 = (y[0] - ylo) / ys, y1 = (y[n - 1] - ylo) / ys;
        for (int64_t i = 0; i < n; i++) {
            const double xn = (x[i] - x[0]) / xs, yn = (y[i] - ylo) / ys;
            const double chord = y0 + (y1 - y0) * xn;
            const double d = chord - yn;
            if (d > best_d) { best_d = d; best = i; }
        }
    }
    *knee = best;
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Building blocks                                                          */
/* ------------------------------------------------------------------------ */

/* out[m, n] = sum_k x[m, k] * W[n, k] */
static void matmul_nt(real *out, const real *x, const real *W, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        const real *w = W + n * K;
        for (int64_t m = 0; m < M; m++) {
            const real *a = x + m * K;
            real acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int64_t k = 0; k < K; k++) acc += a[k] * w[k];
            out[m * N + n] = acc;
        }
    }
}

/* y = x / sqrt(mean(x^2) + eps) * g, row by row */
static void rmsnorm(real *y, const real *x, const real *g, int64_t M, int64_t d, double eps)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++) {
        real ss = 0;
        for (int64_t k = 0; k < d; k++) ss += x[m * d + k] * x[m * d + k];
        real inv = (real)1 / (real)sqrt((double)(ss / (real)d) + eps);
        for (int64_t k = 0; k < d; k++) y[m * d + k] = x[m * d + k] * inv * g[k];
    }
}

/* rotate-half RoPE of one head vector at integer position pos */
static void rope_head(real *v, int hd, int64_t pos, double theta)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

void orc_rope_head(real *v, int32_t hd, int64_t pos, double theta) { rope_head(v, hd, pos, theta); }

static int check_parents(const int32_t *parent, int B, int n_tot)
{
    for (int b = 0; b < B; b++)
        for (int i = 0; i < n_tot; i++) {
            int p = parent[b * n_tot + i];
            if (p < -1 || p >= i) return ORC_ERR_TREE;
        }
    return ORC_OK;
}

/*
 * The decoder layers over B * N_new rows.  Row (b, j) is in-round node
 * i = n_prev + j of sequence b.  In-round node i lives in cache slot
 * len[b] + i and at position len[b] + depth(i), depth(i) = 0 if parent is -1
 * else depth(parent) + 1.  It attends to the committed prefix 0..len[b]-1 and
 * to its in-round ancestors and itself (Sec. 2, tree-structured attention).
 * kc / vc: [n_layers][n_slots][cap][Hkv][hd]; sequence b of the call uses cache
 * slot slot[b] (identity when slot is NULL) and length len_of_slot[slot[b]].
 */
static int decoder_layers(const orc_cfg *c, const orc_weights *w, int B, int n_prev, int N_new,
                          const int32_t *parent, real *kc, real *vc, int64_t cap, int n_slots, const int32_t *slot,
                          const int32_t *len_of_slot, real *h)
{
    const int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim, F = c->d_ffn;
    const int n_tot = n_prev + N_new, M = B * N_new, grp = Hq / Hkv;
    const int qkv_dim = (Hq + 2 * Hkv) * hd;
    int *depth = (int *)malloc(sizeof(int) * (size_t)B * n_tot);
    real *a = (real *)malloc(sizeof(real) * (size_t)M * d);
    real *qkv = (real *)malloc(sizeof(real) * (size_t)M * qkv_dim);
    real *att = (real *)malloc(sizeof(real) * (size_t)M * Hq * hd);
    real *proj = (real *)malloc(sizeof(real) * (size_t)M * d);
    real *gate = (real *)malloc(sizeof(real) * (size_t)M * F);
    real *up = (real *)malloc(sizeof(real) * (size_t)M * F);
    int64_t max_keys = 0;
    int *len = (int *)malloc(sizeof(int) * (size_t)(B > 0 ? B : 1));
    int *sl = (int *)malloc(sizeof(int) * (size_t)(B > 0 ? B : 1));
    for (int b = 0; b < B; b++) {
        sl[b] = slot ? slot[b] : b;
        if (sl[b] < 0 || sl[b] >= n_slots) { max_keys = -1; break; }
        len[b] = len_of_slot[sl[b]];
        if (len[b] < 0 || (int64_t)len[b] + n_tot > cap) { max_keys = -1; break; }
        if (len[b] + n_tot > max_keys) max_keys = len[b] + n_tot;
        for (int i = 0; i < n_tot; i++) {
            int p = parent[b * n_tot + i];
            depth[b * n_tot + i] = p < 0 ? 0 : depth[b * n_tot + p] + 1;
        }
    }
    int rc = ORC_OK;
    if (max_keys < 0) { rc = ORC_ERR_CAP; goto done; }

    for (int l = 0; l < c->n_layers; l++) {
        real *kl = kc + (size_t)l * n_slots * cap * Hkv * hd;
        real *vl = vc + (size_t)l * n_slots * cap * Hkv * hd;
        rmsnorm(a, h, w->norm_attn[l], M, d, c->rms_eps);
        matmul_nt(qkv, a, w->wqkv[l], M, qkv_dim, d);
        /* RoPE on q and k heads; write k, v of each new node into its slot */
        for (int b = 0; b < B; b++)
            for (int j = 0; j < N_new; j++) {
                int i = n_prev + j;
                int64_t pos = (int64_t)len[b] + depth[b * n_tot + i];
                real *row = qkv + (size_t)(b * N_new + j) * qkv_dim;
                for (int hh = 0; hh < Hq + Hkv; hh++) rope_head(row + (size_t)hh * hd, hd, pos, c->rope_theta);
                size_t at = ((size_t)sl[b] * cap + (size_t)len[b] + i) * Hkv * hd;
                memcpy(kl + at, row + (size_t)Hq * hd, sizeof(real) * Hkv * hd);
                memcpy(vl + at, row + (size_t)(Hq + Hkv) * hd, sizeof(real) * Hkv * hd);
            }
        /* attention */
#pragma omp parallel
        {
            real *sc = (real *)malloc(sizeof(real) * (size_t)max_keys);
            int64_t *key = (int64_t *)malloc(sizeof(int64_t) * (size_t)max_keys);
#pragma omp for schedule(dynamic, 1)
            for (int r = 0; r < M; r++) {
                int b = r / N_new, j = r % N_new, i = n_prev + j;
                int64_t L = len[b], nk = 0;
                for (int64_t t = 0; t < L; t++) key[nk++] = t;
                {   /* in-round ancestors-or-self, ascending */
                    int chain[4096], nc = 0;
                    for (int u = i; u >= 0; u = parent[b * n_tot + u]) chain[nc++] = u;
                    for (int t = nc - 1; t >= 0; t--) key[nk++] = L + chain[t];
                }
                real scale = (real)1 / (real)sqrt((double)hd);
                for (int hq = 0; hq < Hq; hq++) {
                    int hk = hq / grp;
                    const real *q = qkv + (size_t)r * qkv_dim + (size_t)hq * hd;
                    real mx = 0;
                    for (int64_t t = 0; t < nk; t++) {
                        const real *kk = kl + (((size_t)sl[b] * cap + (size_t)key[t]) * Hkv + hk) * hd;
                        real s = 0;
                        for (int e = 0; e < hd; e++) s += q[e] * kk[e];
                        s *= scale;
                        sc[t] = s;
                        if (t == 0 || s > mx) mx = s;
                    }
                    real den = 0;
                    for (int64_t t = 0; t < nk; t++) { sc[t] = (real)exp((double)(sc[t] - mx)); den += sc[t]; }
                    real *o = att + (size_t)r * Hq * hd + (size_t)hq * hd;
                    for (int e = 0; e < hd; e++) o[e] = 0;
                    for (int64_t t = 0; t < nk; t++) {
                        const real *vv = vl + (((size_t)sl[b] * cap + (size_t)key[t]) * Hkv + hk) * hd;
                        real p = sc[t] / den;
                        for (int e = 0; e < hd; e++) o[e] += p * vv[e];
                    }
                }
            }
            free(sc); free(key);
        }
        matmul_nt(proj, att, w->wo[l], M, d, (int64_t)Hq * hd);
        for (size_t t = 0; t < (size_t)M * d; t++) h[t] += proj[t];
        rmsnorm(a, h, w->norm_ffn[l], M, d, c->rms_eps);
        matmul_nt(gate, a, w->w_gate[l], M, F, d);
        matmul_nt(up, a, w->w_up[l], M, F, d);
        for (size_t t = 0; t < (size_t)M * F; t++) {
            real g = gate[t];
            real silu = g / ((real)1 + (real)exp((double)-g));
            gate[t] = silu * up[t];
        }
        matmul_nt(proj, gate, w->w_down[l], M, d, F);
        for (size_t t = 0; t < (size_t)M * d; t++) h[t] += proj[t];
    }
done:
    free(len); free(sl);
    free(depth); free(a); free(qkv); free(att); free(proj); free(gate); free(up);
    return rc;
}

/*
 * One forward of the target (is_draft = 0) or the draft head (is_draft = 1)
 * over the new in-round nodes of B sequences.
 *   tokens   [B, N_new]         token of each new node
 *   feat_in  [B, N_new, d]      draft only: the feature paired with the token
 *   parent   [B, n_prev+N_new]  in-round parent index, -1 = child of the prefix
 * Target: hidden = RMSNorm_final(h) (the LM head's input); draft: hidden = h.
 * logits (optional) = hidden . lm_head^T.
 */
int orc_tree_forward(const orc_cfg *c, const orc_weights *w, int32_t is_draft, int32_t B, int32_t n_prev,
                     int32_t N_new, const int32_t *tokens, const real *feat_in, const int32_t *parent, real *kc,
                     real *vc, int64_t cap, int32_t n_slots, const int32_t *slot, const int32_t *len,
                     real *hidden /*[B*N_new, d]*/,
                     real *logits /*[B*N_new, V] or NULL*/)
{
    if (B < 0 || N_new < 0 || n_prev < 0 || n_prev + N_new > 4096) return ORC_ERR_ARG;
    if (B == 0 || N_new == 0) return ORC_OK;
    if (c->n_q_heads % c->n_kv_heads || c->head_dim % 2) return ORC_ERR_ARG;
    int rc = check_parents(parent, B, n_prev + N_new);
    if (rc) return rc;
    const int d = c->d_model, M = B * N_new;
    for (int r = 0; r < M; r++)
        if (tokens[r] < 0 || tokens[r] >= c->vocab) return ORC_ERR_ARG;
    real *h = (real *)malloc(sizeof(real) * (size_t)M * d);
    if (!is_draft) {
        for (int r = 0; r < M; r++) memcpy(h + (size_t)r * d, w->embed + (size_t)tokens[r] * d, sizeof(real) * d);
    } else {
        real *cat = (real *)malloc(sizeof(real) * (size_t)M * 2 * d);
        for (int r = 0; r < M; r++) {
            memcpy(cat + (size_t)r * 2 * d, w->embed + (size_t)tokens[r] * d, sizeof(real) * d);
            memcpy(cat + (size_t)r * 2 * d + d, feat_in + (size_t)r * d, sizeof(real) * d);
        }
        matmul_nt(h, cat, w->fc, M, d, 2 * d);
        free(cat);
    }
    rc = decoder_layers(c, w, B, n_prev, N_new, parent, kc, vc, cap, n_slots, slot, len, h);
    if (rc == ORC_OK) {
        if (!is_draft) rmsnorm(hidden, h, w->final_norm, M, d, c->rms_eps);
        else memcpy(hidden, h, sizeof(real) * (size_t)M * d);
        if (logits) matmul_nt(logits, hidden, w->lm_head, M, c->vocab, d);
    }
    free(h);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Counter-based random numbers (SplitMix64 finaliser as a hash).           */
/* u(seed, row, v) = (k + 1/2) / 2^23, k the top 23 bits: exact in fp32.       */
/* ------------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
static double uniform01(uint64_t seed, uint64_t row, uint64_t v)
{
    uint64_t bits = mix64(mix64(seed ^ (row * 0xD1B54A32D192ED03ULL)) + v);
    return ((double)(bits >> 41) + 0.5) / 8388608.0;
}
double orc_uniform01(uint64_t seed, uint64_t row, uint64_t v) { return uniform01(seed, row, v); }

/* scores[r, v] = logits[r, v] / T + Gumbel(seed, row0 + r, v);  argmax of a row is one exact
 * sample of softmax(logits / T) (Gumbel-max).  T <= 0 is an error. */
int orc_gumbel_scores(const real *logits, int64_t M, int64_t V, double T, uint64_t seed, int64_t row0, real *scores)
{
    if (!(T > 0)) return ORC_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++)
        for (int64_t v = 0; v < V; v++) {
            real u = (real)uniform01(seed, (uint64_t)(row0 + r), (uint64_t)v);
            real g = -(real)log(-(real)log(u));
            scores[r * V + v] = logits[r * V + v] / (real)T + g;
        }
    return ORC_OK;
}

/* argmax of each row (lowest index on exact ties) and the top-1 minus top-2 margin */
int orc_row_argmax(const real *scores, int64_t M, int64_t V, int32_t *idx, real *margin)
{
    if (V < 1) return ORC_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        const real *s = scores + r * V;
        int64_t best = 0;
        for (int64_t v = 1; v < V; v++) if (s[v] > s[best]) best = v;
        real second = 0; int have = 0;
        for (int64_t v = 0; v < V; v++) if (v != best && (!have || s[v] > second)) { second = s[v]; have = 1; }
        idx[r] = (int32_t)best;
        if (margin) margin[r] = have ? s[best] - second : (real)INFINITY;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Acceptance by strict token match (Sec. 2, "Verification Strategies").    */
/* target_tok[b, u] is the token the target emits after node u (greedy       */
/* argmax, or one Gumbel-max sample).  Walk from the root: move to the child */
/* (lowest index first) whose token equals target_tok of the current node;   */
/* stop when there is none.  Emits path[b, 0..a], out_tokens[b, 0..a] with   */
/* out_tokens[b, j] = target_tok[b, path[j]] (accepted drafts, then the      */
/* bonus token).  The first EOS among the emitted tokens cuts the walk there */
/* and sets finished.                                                        */
/* ------------------------------------------------------------------------ */
int orc_walk(int32_t B, int32_t N, const int32_t *tokens, const int32_t *parent, const int32_t *target_tok,
             int32_t eos_id, int32_t *accept_len, int32_t *path /*[B,N]*/, int32_t *out_tokens /*[B,N]*/,
             int32_t *finished)
{
    if (B < 0 || N < 1) return ORC_ERR_ARG;
    int rc = check_parents(parent, B, N);
    if (rc) return rc;
    for (int b = 0; b < B; b++) {
        const int32_t *tok = tokens + (size_t)b * N, *par = parent + (size_t)b * N;
        const int32_t *tt = target_tok + (size_t)b * N;
        int32_t *pp = path + (size_t)b * N, *ot = out_tokens + (size_t)b * N;
        for (int j = 0; j < N; j++) { pp[j] = -1; ot[j] = -1; }
        int u = 0, a = 0, fin = 0;
        pp[0] = 0;
        for (;;) {
            int t = tt[u];
            ot[a] = t;
            if (t == eos_id) { fin = 1; break; }
            int next = -1;
            for (int ch = u + 1; ch < N; ch++)
                if (par[ch] == u && tok[ch] == t) { next = ch; break; }
            if (next < 0) break;
            u = next; a++; pp[a] = u;
        }
        accept_len[b] = a;
        finished[b] = fin;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Acceptance by rejection sampling over sibling sets (the scheme of the     */
/* speculative-decoding work Sec. 2 builds on, extended to a tree).  At node */
/* u: p = softmax(logits[u] / T), q = draft_probs[u].  For each child c of u */
/* in index order with token x: accept if unif[c] < min(1, p(x) / q(x));     */
/* else p <- normalise(max(p - q, 0)), q(x) <- 0, q <- normalise(q).  When    */
/* no child is accepted the bonus token is a Gumbel-max draw from the        */
/* current p (argmax_v log p(v) + Gumbel(seed, row of u, v), zero-mass        */
/* tokens excluded).  bonus_margin[b] = top-1 minus top-2 of those scores.    */
/* min_gap[b] = the smallest |unif - min(1, p/q)| met on the walk.            */
/* ------------------------------------------------------------------------ */
int orc_accept_reject(int32_t B, int32_t N, int32_t V, const int32_t *tokens, const int32_t *parent,
                      const real *logits /*[B*N,V]*/, const real *draft_probs /*[B*N,V]*/,
                      const real *unif /*[B,N]*/, double T, uint64_t seed, int64_t row0, int32_t eos_id,
                      int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished,
                      real *bonus_margin /*[B] or NULL*/, real *min_gap /*[B] or NULL*/)
{
    if (B < 0 || N < 1 || V < 1 || !(T > 0)) return ORC_ERR_ARG;
    int rc = check_parents(parent, B, N);
    if (rc) return rc;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        const int32_t *tok = tokens + (size_t)b * N, *par = parent + (size_t)b * N;
        int32_t *pp = path + (size_t)b * N, *ot = out_tokens + (size_t)b * N;
        real *p = (real *)malloc(sizeof(real) * (size_t)V), *q = (real *)malloc(sizeof(real) * (size_t)V);
        for (int j = 0; j < N; j++) { pp[j] = -1; ot[j] = -1; }
        int u = 0, a = 0, fin = 0;
        real gap = (real)INFINITY, bm = (real)INFINITY;
        pp[0] = 0;
        for (;;) {
            const real *lg = logits + ((size_t)b * N + u) * V;
            real mx = lg[0] / (real)T;
            for (int v = 1; v < V; v++) if (lg[v] / (real)T > mx) mx = lg[v] / (real)T;
            real den = 0;
            for (int v = 0; v < V; v++) { p[v] = (real)exp((double)(lg[v] / (real)T - mx)); den += p[v]; }
            for (int v = 0; v < V; v++) p[v] /= den;
            memcpy(q, draft_probs + ((size_t)b * N + u) * V, sizeof(real) * (size_t)V);
            int next = -1;
            for (int ch = u + 1; ch < N && next < 0; ch++) {
                if (par[ch] != u) continue;
                int x = tok[ch];
                real ratio = q[x] > 0 ? p[x] / q[x] : (p[x] > 0 ? (real)INFINITY : (real)0);
                if (ratio > 1) ratio = 1;
                real r = unif[(size_t)b * N + ch];
                real g = (real)fabs((double)(r - ratio));
                if (g < gap) gap = g;
                if (r < ratio) { next = ch; break; }
                real sp = 0, sq = 0;
                for (int v = 0; v < V; v++) { real t = p[v] - q[v]; p[v] = t > 0 ? t : 0; sp += p[v]; }
                q[x] = 0;
                for (int v = 0; v < V; v++) sq += q[v];
                if (sp > 0) for (int v = 0; v < V; v++) p[v] /= sp;
                if (sq > 0) for (int v = 0; v < V; v++) q[v] /= sq;
            }
            if (next >= 0) {
                ot[a] = tok[next];
                if (tok[next] == eos_id) { fin = 1; break; }
                u = next; a++; pp[a] = u;
                continue;
            }
            /* bonus token from the current p */
            int best = -1; real s1 = 0, s2 = 0; int have2 = 0;
            for (int v = 0; v < V; v++) {
                if (!(p[v] > 0)) continue;
                real uu = (real)uniform01(seed, (uint64_t)(row0 + (int64_t)b * N + u), (uint64_t)v);
                real s = (real)log((double)p[v]) - (real)log(-(real)log(uu));
                if (best < 0) { best = v; s1 = s; }
                else if (s > s1) { s2 = s1; have2 = 1; s1 = s; best = v; }
                else if (!have2 || s > s2) { s2 = s; have2 = 1; }
            }
            ot[a] = best;
            bm = have2 ? s1 - s2 : (real)INFINITY;
            if (best == eos_id) fin = 1;
            break;
        }
        accept_len[b] = a;
        finished[b] = fin;
        if (bonus_margin) bonus_margin[b] = bm;
        if (min_gap) min_gap[b] = gap;
        free(p); free(q);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Keep the accepted path's K/V: in-round slot path[j] -> slot j, j = 0..a,  */
/* then len += a + 1 (Alg. 1, "extract accepted tokens ..."; the rejected     */
/* nodes' entries are dropped).  Also gathers the path's feature rows.        */
/* ------------------------------------------------------------------------ */
int orc_kv_compact(int32_t n_layers, int32_t B, int32_t N, int32_t Hkv, int32_t hd, real *kc, real *vc, int64_t cap,
                   int32_t n_slots, const int32_t *slot, int32_t *len, const int32_t *accept_len,
                   const int32_t *path /*[B,N]*/)
{
    size_t row = (size_t)Hkv * hd;
    for (int b = 0; b < B; b++) {
        int a = accept_len[b];
        int sb = slot ? slot[b] : b;
        if (sb < 0 || sb >= n_slots) return ORC_ERR_ARG;
        if (a < 0 || a >= N || (int64_t)len[sb] + N > cap) return ORC_ERR_ARG;
        for (int j = 0; j <= a; j++) {
            int s = path[(size_t)b * N + j];
            if (s < j || s >= N || (j > 0 && s <= path[(size_t)b * N + j - 1])) return ORC_ERR_TREE;
        }
    }
    for (int l = 0; l < n_layers; l++)
        for (int b = 0; b < B; b++) {
            int sb = slot ? slot[b] : b;
            real *kb = kc + ((size_t)l * n_slots + sb) * cap * row, *vb = vc + ((size_t)l * n_slots + sb) * cap * row;
            for (int j = 0; j <= accept_len[b]; j++) {
                size_t src = (size_t)len[sb] + path[(size_t)b * N + j], dst = (size_t)len[sb] + j;
                if (src != dst) {
                    memcpy(kb + dst * row, kb + src * row, sizeof(real) * row);
                    memcpy(vb + dst * row, vb + src * row, sizeof(real) * row);
                }
            }
        }
    for (int b = 0; b < B; b++) len[slot ? slot[b] : b] += accept_len[b] + 1;
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Draft side: top-K children with log-probabilities, frontier selection,    */
/* rerank into the verify tree (Alg. 1, draft expansion and reranking).      */
/* ------------------------------------------------------------------------ */

/* Per row: the K largest logits (ties: lower index first) and their log-softmax values. */
int orc_topk_logp(const real *logits, int64_t M, int64_t V, int32_t K, int32_t *tok /*[M,K]*/, real *logp /*[M,K]*/)
{
    if (K < 1 || K > V) return ORC_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; r++) {
        const real *s = logits + r * V;
        real mx = s[0];
        for (int64_t v = 1; v < V; v++) if (s[v] > mx) mx = s[v];
        real den = 0;
        for (int64_t v = 0; v < V; v++) den += (real)exp((double)(s[v] - mx));
        real lse = mx + (real)log((double)den);
        for (int k = 0; k < K; k++) {
            int64_t best = -1;
            for (int64_t v = 0; v < V; v++) {
                int taken = 0;
                for (int t = 0; t < k; t++) if (tok[r * K + t] == v) taken = 1;
                if (taken) continue;
                if (best < 0 || s[v] > s[best]) best = v;
            }
            tok[r * K + k] = (int32_t)best;
            logp[r * K + k] = s[best] - lse;
        }
    }
    return ORC_OK;
}

/* Indices of the K largest entries of each row of scores [B, C] (ties: lower index first), in rank order. */
int orc_topk_index(const float *scores, int32_t B, int32_t C, int32_t K, int32_t *idx /*[B,K]*/)
{
    if (K < 0 || K > C) return ORC_ERR_ARG;
    for (int b = 0; b < B; b++) {
        const float *s = scores + (size_t)b * C;
        for (int k = 0; k < K; k++) {
            int best = -1;
            for (int i = 0; i < C; i++) {
                int taken = 0;
                for (int t = 0; t < k; t++) if (idx[(size_t)b * K + t] == i) taken = 1;
                if (taken) continue;
                if (best < 0 || s[i] > s[best]) best = i;
            }
            idx[(size_t)b * K + k] = best;
        }
    }
    return ORC_OK;
}

/*
 * Rerank: candidate 0 is the root (cand_parent -1); cand_parent[i] < i.  Select the root and the N-1
 * non-root candidates of highest score (ties: lower index first), order them by (depth, candidate index)
 * and emit tokens / parent of the verify tree (parent[0] = -1, parent[i] < i).  Scores must not increase
 * from parent to child (they are sums of log-probabilities), which makes the selection ancestor-closed;
 * a selection that is not closed is ORC_ERR_TREE.  sel[b, i] = candidate index of tree node i.
 */
int orc_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int32_t B,
                   int32_t C, int32_t N, int32_t *tokens /*[B,N]*/, int32_t *parent /*[B,N]*/, int32_t *sel /*[B,N]*/)
{
    if (N < 1 || N > C) return ORC_ERR_ARG;
    int *chosen = (int *)malloc(sizeof(int) * (size_t)C), *depth = (int *)malloc(sizeof(int) * (size_t)C);
    int *newidx = (int *)malloc(sizeof(int) * (size_t)C);
    int rc = ORC_OK;
    for (int b = 0; b < B && rc == ORC_OK; b++) {
        const int32_t *ct = cand_tok + (size_t)b * C, *cp = cand_parent + (size_t)b * C;
        const float *cs = cand_score + (size_t)b * C;
        if (cp[0] != -1) { rc = ORC_ERR_TREE; break; }
        for (int i = 0; i < C; i++) {
            if (i > 0 && (cp[i] < 0 || cp[i] >= i)) { rc = ORC_ERR_TREE; break; }
            chosen[i] = (i == 0);
            depth[i] = i == 0 ? 0 : depth[cp[i]] + 1;
        }
        if (rc) break;
        for (int k = 1; k < N; k++) {
            int best = -1;
            for (int i = 1; i < C; i++) if (!chosen[i] && (best < 0 || cs[i] > cs[best])) best = i;
            chosen[best] = 1;
        }
        for (int i = 1; i < C; i++) if (chosen[i] && !chosen[cp[i]]) rc = ORC_ERR_TREE;
        if (rc) break;
        int n = 0, maxd = 0;
        for (int i = 0; i < C; i++) if (chosen[i] && depth[i] > maxd) maxd = depth[i];
        for (int dd = 0; dd <= maxd; dd++)
            for (int i = 0; i < C; i++)
                if (chosen[i] && depth[i] == dd) {
                    newidx[i] = n;
                    tokens[(size_t)b * N + n] = ct[i];
                    parent[(size_t)b * N + n] = i == 0 ? -1 : newidx[cp[i]];
                    if (sel) sel[(size_t)b * N + n] = i;
                    n++;
                }
    }
    free(chosen); free(depth); free(newidx);
    return rc;
}
