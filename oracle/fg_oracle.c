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
 *   orc_draft_train    central finite differences (fp64 build) and torch
 *                      autograd on the same forward written with torch ops;
 *                      the loss itself (the paper names none) is this build's
 *                      reading -- "parity unpinned" as to which loss
 *   orc_adamw          torch.optim.AdamW
 *   draft head internals (fc + one layer, no final norm): fixed by this
 *   build's reading of Sec. 2 only -- "parity unpinned" beyond the shared
 *   layer code.
 *
 * Rounding twin (cfg.act_round = 1: bf16, 2: fp16; 0 = the oracle proper, which
 * every tolerance is quoted against).  The paper fixes no arithmetic; a 16-bit
 * pipeline stores its activations in 16 bits between the steps of a layer, and
 * the twin does the same with exact arithmetic in between: the outputs of both
 * RMS norms, q / k / v after RoPE (hence the cached K and V), the attention
 * output, the SwiGLU output and the vector handed to the LM head are rounded to
 * nearest-even; the residual stream, scores, softmax weights and all sums are
 * not.  It is a second reference for 16-bit implementations, tight where the
 * first cannot be (bf16 rounding alone moves a 28-layer model's logits by 0.2).
 * Pins: orc_round_act against torch's casts (ties, subnormals, range ends); the
 * twin against the torch decoder of the chain pin with casts at the same places.
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
    int32_t act_round;   /* 0: none (the oracle proper); 1 / 2: activations rounded to bf16 / fp16 between the layer's steps */
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

/* ------------------------------------------------------------------------ */
/* Round to the nearest bf16 / fp16 value, ties to even (the rounding twin). */
/* ------------------------------------------------------------------------ */
static real round_act(real x, int mode)
{
    if (mode == 0) return x;
    float f = (float)x;
    if (!(f == f) || f == 0.0f) return (real)f;
    if (mode == 1) {                       /* bf16: the top 16 bits of the fp32 pattern */
        uint32_t u;
        memcpy(&u, &f, 4);
        u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
        memcpy(&f, &u, 4);
        return (real)f;
    }
    /* fp16 (from the fp32 value, as a cast does): 11 significant bits down to 2^-14, multiples of 2^-24 below,
       infinity from 65504 + half an ulp on */
    double a = fabs((double)f);
    if (a >= 65520.0) return (real)(f > 0 ? INFINITY : -INFINITY);
    int e;
    frexp(a, &e);                          /* a = m 2^e, m in [0.5, 1) */
    double ulp = ldexp(1.0, (e - 11 > -24) ? e - 11 : -24);
    double r = nearbyint((double)f / ulp) * ulp;   /* default rounding mode: ties to even */
    return (real)r;
}
int orc_round_act(real *x, int64_t n, int32_t mode)
{
    if (mode < 0 || mode > 2) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; i++) x[i] = round_act(x[i], mode);
    return ORC_OK;
}
static void round_all(real *x, size_t n, int mode)
{
    if (mode)
        for (size_t i = 0; i < n; i++) x[i] = round_act(x[i], mode);
}

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
        round_all(a, (size_t)M * d, c->act_round);
        matmul_nt(qkv, a, w->wqkv[l], M, qkv_dim, d);
        /* RoPE on q and k heads; write k, v of each new node into its slot */
        for (int b = 0; b < B; b++)
            for (int j = 0; j < N_new; j++) {
                int i = n_prev + j;
                int64_t pos = (int64_t)len[b] + depth[b * n_tot + i];
                real *row = qkv + (size_t)(b * N_new + j) * qkv_dim;
                for (int hh = 0; hh < Hq + Hkv; hh++) rope_head(row + (size_t)hh * hd, hd, pos, c->rope_theta);
                round_all(row, (size_t)qkv_dim, c->act_round);
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
                    round_all(o, (size_t)hd, c->act_round);
                }
            }
            free(sc); free(key);
        }
        matmul_nt(proj, att, w->wo[l], M, d, (int64_t)Hq * hd);
        for (size_t t = 0; t < (size_t)M * d; t++) h[t] += proj[t];
        rmsnorm(a, h, w->norm_ffn[l], M, d, c->rms_eps);
        round_all(a, (size_t)M * d, c->act_round);
        matmul_nt(gate, a, w->w_gate[l], M, F, d);
        matmul_nt(up, a, w->w_up[l], M, F, d);
        for (size_t t = 0; t < (size_t)M * F; t++) {
            real g = gate[t];
            real silu = g / ((real)1 + (real)exp((double)-g));
            gate[t] = round_act(silu * up[t], c->act_round);
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
        round_all(hidden, (size_t)M * d, c->act_round);
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

/* ------------------------------------------------------------------------ */
/* Online draft learning (Sec. 4.2 "Draft Model Learning with Online Target  */
/* Feedback"; Alg. 1, the draft training phase).  The draft head is trained  */
/* on what the generation phase left behind: the tokens the target emitted   */
/* and the target's hidden states ("logits and hidden states", which are     */
/* cached).  The paper names no loss; the reading taken is the one of the    */
/* draft-head work it follows for pre-training (Sec. 5.1): per position,     */
/*   L = mean_e smooth_l1(h_hat[e] - f_next[e])                               */
/*     + w_ce * CE(softmax(lm_head f_next), softmax(lm_head h_hat)),          */
/* h_hat = the head's output for the entry (token t+1, target feature t),    */
/* f_next = the target's feature t+1, averaged over the valid entries.       */
/* Each sequence is one teacher-forced chain from an empty draft cache        */
/* (causal attention inside the chain).  This function returns the loss and  */
/* the gradient of every draft parameter; embedding and LM head are the      */
/* target's and frozen.                                                       */
/* Pins: central finite differences in the fp64 build, and the same forward  */
/* written with torch ops differentiated by autograd (tests/test_oracle_      */
/* train.py).                                                                 */
/* ------------------------------------------------------------------------ */

/* out[m, k] = sum_n dy[m, n] * W[n, k] */
static void matmul_nn(real *out, const real *dy, const real *W, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++) {
        real *o = out + m * K;
        for (int64_t k = 0; k < K; k++) o[k] = 0;
        for (int64_t n = 0; n < N; n++) {
            const real g = dy[m * N + n];
            const real *w = W + n * K;
            for (int64_t k = 0; k < K; k++) o[k] += g * w[k];
        }
    }
}

/* dW[n, k] = sum_m dy[m, n] * x[m, k] */
static void matmul_tn(real *dW, const real *dy, const real *x, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        real *o = dW + n * K;
        for (int64_t k = 0; k < K; k++) o[k] = 0;
        for (int64_t m = 0; m < M; m++) {
            const real g = dy[m * N + n];
            const real *a = x + m * K;
            for (int64_t k = 0; k < K; k++) o[k] += g * a[k];
        }
    }
}

/* y = x * inv * g with inv = (mean(x^2) + eps)^(-1/2):
 * dx = inv * (g . dy) - x * inv^3 * sum_k (g . dy)_k x_k / d;  dg += sum over rows of dy * x * inv */
static void rmsnorm_backward(real *dx, real *dg, const real *dy, const real *x, const real *g, int64_t M, int64_t d, double eps)
{
    for (int64_t k = 0; k < d; k++) dg[k] = 0;
    for (int64_t m = 0; m < M; m++) {
        real ss = 0;
        for (int64_t k = 0; k < d; k++) ss += x[m * d + k] * x[m * d + k];
        const real inv = (real)1 / (real)sqrt((double)(ss / (real)d) + eps);
        real dot = 0;
        for (int64_t k = 0; k < d; k++) dot += g[k] * dy[m * d + k] * x[m * d + k];
        for (int64_t k = 0; k < d; k++) {
            dx[m * d + k] = inv * g[k] * dy[m * d + k] - x[m * d + k] * inv * inv * inv * dot / (real)d;
            dg[k] += dy[m * d + k] * x[m * d + k] * inv;
        }
    }
}

/* the transpose of rope_head's rotation (it is orthogonal) */
static void rope_head_backward(real *dv, int hd, int64_t pos, double theta)
{
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = dv[i], b = dv[i + half];
        dv[i] = a * c + b * s;
        dv[i + half] = b * c - a * s;
    }
}

/*
 * tokens [B, T], feat_in / feat_tgt [B, T, d], n_valid [B]: entries t < n_valid[b] carry loss (the rest is padding
 * behind them, which causal attention keeps from influencing them).  loss[0] = regression term, loss[1] = cross-entropy
 * term (before the weight); the total is loss[0] + w_ce * loss[1].  Gradients of the total: g_* in the shapes of the
 * weights.  One decoder layer (n_layers must be 1).
 */
int orc_draft_train(const orc_cfg *c, const orc_weights *w, int32_t B, int32_t T, const int32_t *tokens, const real *feat_in,
                    const real *feat_tgt, const int32_t *n_valid, double w_ce, real *loss, real *g_fc, real *g_wqkv, real *g_wo,
                    real *g_gate, real *g_up, real *g_down, real *g_norm_attn, real *g_norm_ffn)
{
    if (c->n_layers != 1 || B < 1 || T < 1 || c->n_q_heads % c->n_kv_heads || c->head_dim % 2) return ORC_ERR_ARG;
    const int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim, F = c->d_ffn, V = c->vocab;
    const int grp = Hq / Hkv, qkvd = (Hq + 2 * Hkv) * hd, M = B * T;
    int64_t n_tot = 0;
    for (int b = 0; b < B; b++) {
        if (n_valid[b] < 0 || n_valid[b] > T) return ORC_ERR_ARG;
        n_tot += n_valid[b];
    }
    if (n_tot == 0) return ORC_ERR_ARG;
    for (int r = 0; r < M; r++)
        if (tokens[r] < 0 || tokens[r] >= V) return ORC_ERR_ARG;
#define ALLOC(n) ((real *)calloc((size_t)(n), sizeof(real)))
    real *cat = ALLOC((size_t)M * 2 * d), *h0 = ALLOC((size_t)M * d), *a1 = ALLOC((size_t)M * d), *qkv = ALLOC((size_t)M * qkvd);
    real *P = ALLOC((size_t)B * Hq * T * T), *att = ALLOC((size_t)M * Hq * hd), *proj = ALLOC((size_t)M * d), *h1 = ALLOC((size_t)M * d);
    real *a2 = ALLOC((size_t)M * d), *gate = ALLOC((size_t)M * F), *up = ALLOC((size_t)M * F), *act = ALLOC((size_t)M * F);
    real *h2 = ALLOC((size_t)M * d), *z = ALLOC((size_t)M * V), *zt = ALLOC((size_t)M * V);
    /* ---- forward ---- */
    for (int r = 0; r < M; r++) {
        memcpy(cat + (size_t)r * 2 * d, w->embed + (size_t)tokens[r] * d, sizeof(real) * d);
        memcpy(cat + (size_t)r * 2 * d + d, feat_in + (size_t)r * d, sizeof(real) * d);
    }
    matmul_nt(h0, cat, w->fc, M, d, 2 * d);
    rmsnorm(a1, h0, w->norm_attn[0], M, d, c->rms_eps);
    matmul_nt(qkv, a1, w->wqkv[0], M, qkvd, d);
    for (int b = 0; b < B; b++)
        for (int t = 0; t < T; t++)
            for (int hh = 0; hh < Hq + Hkv; hh++) rope_head(qkv + (size_t)(b * T + t) * qkvd + (size_t)hh * hd, hd, t, c->rope_theta);
    const real scale = (real)1 / (real)sqrt((double)hd);
    for (int b = 0; b < B; b++)
        for (int hq = 0; hq < Hq; hq++) {
            const int hk = hq / grp;
            for (int t = 0; t < T; t++) {
                const real *q = qkv + (size_t)(b * T + t) * qkvd + (size_t)hq * hd;
                real *p = P + (((size_t)b * Hq + hq) * T + t) * T;
                real mx = 0;
                for (int s = 0; s <= t; s++) {
                    const real *k = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd;
                    real sc = 0;
                    for (int e = 0; e < hd; e++) sc += q[e] * k[e];
                    p[s] = sc * scale;
                    if (s == 0 || p[s] > mx) mx = p[s];
                }
                real den = 0;
                for (int s = 0; s <= t; s++) { p[s] = (real)exp((double)(p[s] - mx)); den += p[s]; }
                real *o = att + (size_t)(b * T + t) * Hq * hd + (size_t)hq * hd;
                for (int s = 0; s <= t; s++) {
                    p[s] /= den;
                    const real *v = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd;
                    for (int e = 0; e < hd; e++) o[e] += p[s] * v[e];
                }
            }
        }
    matmul_nt(proj, att, w->wo[0], M, d, (int64_t)Hq * hd);
    for (size_t i = 0; i < (size_t)M * d; i++) h1[i] = h0[i] + proj[i];
    rmsnorm(a2, h1, w->norm_ffn[0], M, d, c->rms_eps);
    matmul_nt(gate, a2, w->w_gate[0], M, F, d);
    matmul_nt(up, a2, w->w_up[0], M, F, d);
    for (size_t i = 0; i < (size_t)M * F; i++) act[i] = gate[i] / ((real)1 + (real)exp((double)-gate[i])) * up[i];
    matmul_nt(proj, act, w->w_down[0], M, d, F);
    for (size_t i = 0; i < (size_t)M * d; i++) h2[i] = h1[i] + proj[i];
    matmul_nt(z, h2, w->lm_head, M, V, d);
    matmul_nt(zt, feat_tgt, w->lm_head, M, V, d);
    /* ---- loss and its gradient with respect to h2 (dh2) and z (dz, kept in z) ---- */
    real *dh2 = ALLOC((size_t)M * d);
    double l_reg = 0, l_ce = 0;
    for (int b = 0; b < B; b++)
        for (int t = 0; t < T; t++) {
            const int r = b * T + t;
            real *zr = z + (size_t)r * V, *ztr = zt + (size_t)r * V;
            if (t >= n_valid[b]) {
                for (int v = 0; v < V; v++) zr[v] = 0;
                continue;
            }
            for (int e = 0; e < d; e++) {
                const real df = h2[(size_t)r * d + e] - feat_tgt[(size_t)r * d + e];
                const real ad = df < 0 ? -df : df;
                l_reg += (double)(ad < 1 ? (real)0.5 * df * df : ad - (real)0.5) / d;
                dh2[(size_t)r * d + e] = (ad < 1 ? df : (df < 0 ? (real)-1 : (real)1)) / (real)d / (real)n_tot;
            }
            real mq = zr[0], mp = ztr[0];
            for (int v = 1; v < V; v++) { if (zr[v] > mq) mq = zr[v]; if (ztr[v] > mp) mp = ztr[v]; }
            double sq = 0, sp = 0;
            for (int v = 0; v < V; v++) { sq += exp((double)(zr[v] - mq)); sp += exp((double)(ztr[v] - mp)); }
            const double lq = (double)mq + log(sq), lp = (double)mp + log(sp);
            for (int v = 0; v < V; v++) {
                const double pv = exp((double)ztr[v] - lp), qv = exp((double)zr[v] - lq);
                l_ce -= pv * ((double)zr[v] - lq);
                zr[v] = (real)(w_ce * (qv - pv) / (double)n_tot);     /* d loss / d z */
            }
        }
    loss[0] = (real)(l_reg / (double)n_tot);
    loss[1] = (real)(l_ce / (double)n_tot);
    /* ---- backward ---- */
    real *tmp = ALLOC((size_t)M * d), *dact = ALLOC((size_t)M * F), *dgate = ALLOC((size_t)M * F), *dup = ALLOC((size_t)M * F);
    real *da = ALLOC((size_t)M * d), *dh1 = ALLOC((size_t)M * d), *datt = ALLOC((size_t)M * Hq * hd), *dqkv = ALLOC((size_t)M * qkvd);
    real *dh0 = ALLOC((size_t)M * d);
    matmul_nn(tmp, z, w->lm_head, M, V, d);                       /* through the frozen LM head */
    for (size_t i = 0; i < (size_t)M * d; i++) dh2[i] += tmp[i];
    matmul_tn(g_down, dh2, act, M, d, F);
    matmul_nn(dact, dh2, w->w_down[0], M, d, F);
    for (size_t i = 0; i < (size_t)M * F; i++) {
        const real g = gate[i], sg = (real)1 / ((real)1 + (real)exp((double)-g));
        dup[i] = dact[i] * g * sg;
        dgate[i] = dact[i] * up[i] * (sg + g * sg * ((real)1 - sg));
    }
    matmul_tn(g_gate, dgate, a2, M, F, d);
    matmul_tn(g_up, dup, a2, M, F, d);
    matmul_nn(da, dgate, w->w_gate[0], M, F, d);
    matmul_nn(tmp, dup, w->w_up[0], M, F, d);
    for (size_t i = 0; i < (size_t)M * d; i++) da[i] += tmp[i];
    rmsnorm_backward(tmp, g_norm_ffn, da, h1, w->norm_ffn[0], M, d, c->rms_eps);
    for (size_t i = 0; i < (size_t)M * d; i++) dh1[i] = dh2[i] + tmp[i];
    matmul_tn(g_wo, dh1, att, M, d, (int64_t)Hq * hd);
    matmul_nn(datt, dh1, w->wo[0], M, d, (int64_t)Hq * hd);
    for (int b = 0; b < B; b++)
        for (int hq = 0; hq < Hq; hq++) {
            const int hk = hq / grp;
            for (int t = 0; t < T; t++) {
                const real *p = P + (((size_t)b * Hq + hq) * T + t) * T;
                const real *dout = datt + (size_t)(b * T + t) * Hq * hd + (size_t)hq * hd;
                const real *q = qkv + (size_t)(b * T + t) * qkvd + (size_t)hq * hd;
                real *dq = dqkv + (size_t)(b * T + t) * qkvd + (size_t)hq * hd;
                real dot = 0;
                for (int s = 0; s <= t; s++) {
                    const real *v = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd;
                    real dp = 0;
                    for (int e = 0; e < hd; e++) dp += dout[e] * v[e];
                    dot += dp * p[s];
                }
                for (int s = 0; s <= t; s++) {
                    const real *k = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd;
                    const real *v = qkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd;
                    real *dk = dqkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + hk) * hd;
                    real *dv = dqkv + (size_t)(b * T + s) * qkvd + (size_t)(Hq + Hkv + hk) * hd;
                    real dp = 0;
                    for (int e = 0; e < hd; e++) dp += dout[e] * v[e];
                    const real ds = p[s] * (dp - dot) * scale;
                    for (int e = 0; e < hd; e++) {
                        dq[e] += ds * k[e];
                        dk[e] += ds * q[e];
                        dv[e] += p[s] * dout[e];
                    }
                }
            }
        }
    for (int b = 0; b < B; b++)
        for (int t = 0; t < T; t++)
            for (int hh = 0; hh < Hq + Hkv; hh++) rope_head_backward(dqkv + (size_t)(b * T + t) * qkvd + (size_t)hh * hd, hd, t, c->rope_theta);
    matmul_tn(g_wqkv, dqkv, a1, M, qkvd, d);
    matmul_nn(da, dqkv, w->wqkv[0], M, qkvd, d);
    rmsnorm_backward(tmp, g_norm_attn, da, h0, w->norm_attn[0], M, d, c->rms_eps);
    for (size_t i = 0; i < (size_t)M * d; i++) dh0[i] = dh1[i] + tmp[i];
    matmul_tn(g_fc, dh0, cat, M, d, 2 * d);
#undef ALLOC
    free(cat); free(h0); free(a1); free(qkv); free(P); free(att); free(proj); free(h1); free(a2); free(gate); free(up); free(act);
    free(h2); free(z); free(zt); free(dh2); free(tmp); free(dact); free(dgate); free(dup); free(da); free(dh1); free(datt);
    free(dqkv); free(dh0);
    return ORC_OK;
}

/* One AdamW step (the optimiser Sec. 5.1 names), decoupled weight decay, bias-corrected moments:
 * m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  p -= lr (m / (1 - b1^t) / (sqrt(v / (1 - b2^t)) + eps) + wd p). */
int orc_adamw(real *p, const real *g, real *m, real *v, int64_t n, double lr, double b1, double b2, double eps, double wd, int32_t step)
{
    if (n < 0 || step < 1) return ORC_ERR_ARG;
    const double c1 = 1.0 - pow(b1, step), c2 = 1.0 - pow(b2, step);
    for (int64_t i = 0; i < n; i++) {
        m[i] = (real)(b1 * m[i] + (1.0 - b1) * g[i]);
        v[i] = (real)(b2 * v[i] + (1.0 - b2) * (double)g[i] * g[i]);
        const double upd = ((double)m[i] / c1) / (sqrt((double)v[i] / c2) + eps) + wd * (double)p[i];
        p[i] = (real)((double)p[i] - lr * upd);
    }
    return ORC_OK;
}
