// The C ABI of libfastgrpo: argument checking, workspace carving and the launch sequence of each entry point.
// Every numeric step is a kernel in the sibling .hip files; nothing here touches tensor contents on the host.
#include <math.h>
#include <string.h>

#include <array>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "fg_common.h"

namespace fg {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// launchers defined in the other translation units and not listed in fg_common.h
int32_t launch_tree_prep_ex(const fg_tree *t, const fg_kv_cache *kv, TreeDev td, int max_pos, hipStream_t st);
int32_t launch_swiglu_partials(int32_t dtype, const float *gu, int S, void *act, int M, int F, hipStream_t st);
int32_t launch_attention_simple(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q, void *out,
                                int max_keys, hipStream_t st);
int32_t launch_attention_mfma(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q, void *out,
                              int max_keys, void *ws, int64_t ws_bytes, int reuse_order, hipStream_t st);
int64_t attention_mfma_ws_bytes(int B, int N, int Hq, int Hkv, int hd, int max_keys);
bool attention_mfma_supported(const fg_kv_cache *kv, int Hq, int N);
int32_t launch_gumbel_argmax(const float *logits, int M, int V, float T, uint64_t seed, int64_t row0, int32_t *idx, hipStream_t st);
int32_t launch_walk(int B, int N, const int32_t *tokens, const int32_t *parent, const int32_t *target_tok, int32_t eos,
                    int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished, hipStream_t st);
int32_t launch_reject(int B, int N, int V, const int32_t *tokens, const int32_t *parent, const float *logits,
                      const float *draft_probs, const float *unif, float T, uint64_t seed, int64_t row0, int32_t eos, float *ws,
                      int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished, hipStream_t st);
int32_t launch_kv_compact(fg_kv_cache *kv, const int32_t *slot, const int32_t *accept_len, const int32_t *path, int B, int N,
                          const void *fin, void *fout, int d, int feat_dtype, hipStream_t st);
int32_t launch_topk_logp(const float *logits, int M, int V, int K, int32_t *tok, float *logp, hipStream_t st);
int32_t launch_topk_merge(const float *part_val, const int32_t *part_idx, const float *part_ms, int M, int n_blocks, int K,
                          int32_t *tok, float *logp, int32_t *row_argmax, float *row_top2, hipStream_t st);
int32_t launch_select_rows(const void *src, int64_t row_bytes, int n_src, const int32_t *index, int n, void *dst, hipStream_t st);
int32_t launch_gather_rows(int32_t dtype, const void *src, const int32_t *pick, int B, int N, int d, void *dst, hipStream_t st);
int32_t launch_frontier(int B, int K_in, int K, const int32_t *child_tok, const float *child_logp, int child_rows,
                        const int32_t *node_cand, const float *node_score, const int32_t *node_pick, const int32_t *node_tok, int n_cand, int stride,
                        int32_t *cand_tok, int32_t *cand_parent, float *cand_score, int32_t *next_tok, int32_t *next_cand,
                        float *next_score, int32_t *next_src, const int32_t *parent_prev, int n_parent_prev,
                        int32_t *parent_next, hipStream_t st);
int32_t launch_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int B, int C, int stride,
                          int N, int32_t *tokens, int32_t *parent, int32_t *sel, hipStream_t st);
int32_t launch_commit_len(int32_t *seq_len, const int32_t *slot, const int32_t *n_commit, int bias, int B, int n_slots,
                          int capacity, int32_t *status, hipStream_t st);
int gemm_mfma_split_for(int M, int N, int K);
bool gemm_mfma_fuses_swiglu(int M, int N, int K);
int32_t launch_probe_read(const void *src, int64_t bytes, int nontemporal, int blocks, void *sink, hipStream_t st);
int32_t launch_probe_copy(const void *src, void *dst, int64_t bytes, int blocks, hipStream_t st);
int32_t launch_probe_mfma(int32_t dtype, int iters, int random, int blocks, void *sink, hipStream_t st);
const char *gemm_mfma_kernel_name(int M, int N, int K, int epilogue);
int64_t draft_train_ws_bytes(const fg_model_cfg &c, int B, int T);
int32_t launch_draft_train_grad(const fg_model_cfg &c, const float *embed, const float *lm_head, const fg_draft_params *w,
                                const int32_t *tokens, const float *feat_in, const float *feat_tgt, const int32_t *n_valid, int B,
                                int T, float w_ce, fg_draft_params *g, float *loss, const void *head_packed, void *ws,
                                int64_t ws_bytes, hipStream_t st);
int64_t draft_train_head_bytes(const fg_model_cfg &c);
int32_t launch_draft_train_pack_head(const fg_model_cfg &c, const float *lm_head, void *packed, hipStream_t st);
int32_t launch_adamw(float *p, const float *g, float *m, float *v, int64_t n, float lr, float b1, float b2, float eps, float wd,
                     int step, hipStream_t st);

}  // namespace fg

using namespace fg;

// Stage timing of one model (fg_model_profile): an event is recorded before every launch group of the entry points
// that run this model, and one at their end; the time between two consecutive events belongs to the stage the
// first one announces.
struct StageProf {
    bool on = false;
    int only = -1;               // >= 0: only this stage is bracketed
    std::vector<hipEvent_t> ev;
    std::vector<int8_t> stage;   // stage[i]: what runs after event i (-1: nothing, the end of an entry point)
    size_t used = 0;
};

struct fg_model {
    fg_model_cfg cfg;
    const void *embed, *lm_head, *final_norm, *fc;
    std::vector<const void *> wqkv, wo, wgu, wdown, norm_attn, norm_ffn;
    float2 *rope_tab;  // device [max_pos][head_dim / 2] (cos, sin), angles evaluated in double
    int device;
    StageProf prof;
};

namespace {

inline void mark(const fg_model *m, int stage, hipStream_t st)
{
    StageProf &p = const_cast<fg_model *>(m)->prof;
    if (!p.on || p.used >= p.ev.size()) return;
    if (p.only >= 0 && stage != p.only && !(p.used > 0 && p.stage[p.used - 1] == p.only)) return;
    (void)hipEventRecord(p.ev[p.used], st);
    p.stage[p.used++] = (int8_t)stage;
}

struct Carver {
    char *base;
    int64_t off, cap;
    bool ok;
    Carver(void *b, int64_t c) : base((char *)b), off(0), cap(c), ok(true) {}
    template <typename T> T *take(int64_t n)
    {
        off = align_up(off, 256);
        T *p = (T *)(base + off);
        off += n * (int64_t)sizeof(T);
        if (off > cap) ok = false;
        return p;
    }
};

// split-K factor the library will use for each GEMM of the step (0 = not a partial-sum GEMM)
int split_for(const fg_model_cfg &c, int M, int N, int K) { return is16(c.dtype) ? gemm_mfma_split_for(M, N, K) : 1; }

// gate/up with the SwiGLU epilogue (no split-K slabs) whenever the pipelined kernel runs it
bool gate_up_fused(const fg_model_cfg &c, int M) { return is16(c.dtype) && gemm_mfma_fuses_swiglu(M, 2 * c.d_ffn, c.d_model); }

int64_t partial_floats(const fg_model_cfg &c, int M, bool is_draft)
{
    const int d = c.d_model, F = c.d_ffn, qkvd = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, hq = c.n_q_heads * c.head_dim;
    int64_t m = 0;
    // the split factors (and whether gate/up needs slabs at all) step with the row count, so S * rows is not
    // monotone: size for the worst row count up to M
    auto need = [&](int mm) {
        auto upd = [&](int N, int K) {
            int64_t v = (int64_t)split_for(c, mm, N, K) * mm * N;
            if (v > m) m = v;
        };
        upd(qkvd, d);
        upd(d, hq);
        upd(d, F);
        if (!gate_up_fused(c, mm)) upd(2 * F, d);
        if (is_draft) upd(d, 2 * d);
    };
    // every row count is tried once per (shape, M); the result is remembered
    static std::mutex mu;
    static std::map<std::array<int64_t, 9>, int64_t> memo;
    const std::array<int64_t, 9> key = {c.dtype, d, F, qkvd, hq, M, is_draft, c.n_layers, c.vocab};
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = memo.find(key);
        if (it != memo.end()) return it->second;
    }
    for (int mm = M; mm > 0; mm--) need(mm);
    std::lock_guard<std::mutex> lock(mu);
    memo[key] = m;
    return m;
}

struct StepWs {
    TreeDev td;
    float *h, *partials, *logits;
    void *a, *q, *att, *act, *feat, *cat;
    void *attn_ws;
    int64_t attn_ws_bytes;
};

// attn_bytes_override >= 0: size the attention workspace with that figure instead of the one of this (B, N)
int64_t carve_step(const fg_model_cfg &c, int M, int max_keys, int B, int N, bool is_draft, void *base, int64_t cap, StepWs *w,
                   bool need_logits, int64_t attn_bytes_override = -1)
{
    Carver cv(base, cap);
    const int64_t es = dtype_size(c.dtype);
    const int d = c.d_model, hq = c.n_q_heads * c.head_dim;
    StepWs s;
    s.td.pos = cv.take<int32_t>(M);
    s.td.mask = cv.take<uint64_t>(M);
    s.td.dest = cv.take<int32_t>(M);
    s.h = cv.take<float>((int64_t)M * d);
    s.partials = cv.take<float>(partial_floats(c, M, is_draft));
    s.a = cv.take<char>((int64_t)M * d * es);
    s.q = cv.take<char>((int64_t)M * hq * es);
    s.att = cv.take<char>((int64_t)M * hq * es);
    s.act = cv.take<char>((int64_t)M * c.d_ffn * es);
    s.feat = cv.take<char>((int64_t)M * d * es);
    s.cat = is_draft ? (void *)cv.take<char>((int64_t)M * 2 * d * es) : nullptr;
    s.logits = need_logits ? cv.take<float>((int64_t)M * c.vocab) : nullptr;
    s.attn_ws_bytes = attn_bytes_override >= 0 ? attn_bytes_override
                                               : attention_mfma_ws_bytes(B, N, c.n_q_heads, c.n_kv_heads, c.head_dim, max_keys);
    s.attn_ws = cv.take<char>(s.attn_ws_bytes);
    if (w) *w = s;
    if (base && !cv.ok) return -1;
    return align_up(cv.off, 256);
}

// The largest attention workspace any call of at most max_rows rows can need: the figure depends on how the keys of
// a (sequence, kv head) pair are cut into chunks, which is monotone neither in B nor in N, so every shape
// (N = 1 .. FG_MAX_NODES, B = 1 .. max_rows / N) is evaluated once and the result remembered.
int64_t max_attention_ws(const fg_model_cfg &c, int max_rows, int max_keys)
{
    static std::mutex mu;
    static std::map<std::array<int64_t, 5>, int64_t> memo;
    const std::array<int64_t, 5> key = {c.n_q_heads, c.n_kv_heads, c.head_dim, max_rows, max_keys};
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = memo.find(key);
        if (it != memo.end()) return it->second;
    }
    int64_t best = 0;
    for (int N = 1; N <= FG_MAX_NODES && N <= max_rows; N++)
        for (int B = 1; B * N <= max_rows; B++) {
            const int64_t v = attention_mfma_ws_bytes(B, N, c.n_q_heads, c.n_kv_heads, c.head_dim, max_keys);
            if (v > best) best = v;
        }
    std::lock_guard<std::mutex> lock(mu);
    memo[key] = best;
    return best;
}

int32_t gemm_any(const fg_model_cfg &c, const void *x, const void *w, float *partials, int M, int N, int K, int *S, hipStream_t st)
{
    if (is16(c.dtype)) return launch_gemm_mfma(c.dtype, x, w, partials, M, N, K, 0, 0, S, st);
    *S = 1;
    return launch_gemm_f32((const float *)x, (const float *)w, partials, M, N, K, st);
}

// LM head with the selection in the GEMM's epilogue: x [M, d] . W^T -> per-block top-k / (max, sum exp) partials in
// `scratch` (the region a materialised [M, V] fp32 logits tensor would take: the partials need under a third of it) ->
// the K best tokens of each row with their log-probabilities, and / or the row arg-max and top-2 values.
int64_t lm_head_topk_bytes(int M, int V, int K) { return (int64_t)M * ((V + 255) / 256) * (K * 8 + 8) + 1024; }

int32_t lm_head_topk(int32_t dtype, const void *x, const void *lm_head, int M, int V, int d, int K, bool want_logp, void *scratch,
                     int32_t *tok, float *logp, int32_t *row_argmax, float *row_top2, hipStream_t st)
{
    const int nb = (V + 255) / 256;
    GemmEpi ep;
    ep.topk = K;
    ep.part_val = (float *)scratch;
    ep.part_idx = (int32_t *)(ep.part_val + (size_t)M * nb * K);
    ep.part_ms = want_logp ? (float *)(ep.part_idx + (size_t)M * nb * K) : nullptr;
    int32_t rc;
    if ((rc = launch_gemm_mfma(dtype, x, lm_head, nullptr, M, V, d, EPI_TOPK, 1, nullptr, st, &ep))) return rc;
    return launch_topk_merge(ep.part_val, ep.part_idx, ep.part_ms, M, nb, K, tok, logp, row_argmax, row_top2, st);
}

int32_t check_cache(const fg_model *m, const fg_kv_cache *kv)
{
    if (!kv || !kv->k_pool || !kv->v_pool || !kv->page_table || !kv->seq_len)
        return fail(FG_ERR_INVALID_ARG, "KV cache or one of its members is NULL");
    if (kv->page_size != 16) return fail(FG_ERR_SHAPE, "page_size must be 16 (got %d)", kv->page_size);
    if (kv->n_slots < 1 || kv->n_pages < 1 || kv->max_pages_per_seq < 1)
        return fail(FG_ERR_INVALID_ARG, "KV cache sizes must be positive");
    if (m) {
        const fg_model_cfg &c = m->cfg;
        if (kv->dtype != c.dtype) return fail(FG_ERR_INVALID_ARG, "dtype mismatch: model %d, cache %d", c.dtype, kv->dtype);
        if (kv->n_layers != c.n_layers || kv->n_kv_heads != c.n_kv_heads || kv->head_dim != c.head_dim)
            return fail(FG_ERR_SHAPE, "cache geometry (%d layers, %d kv heads, head_dim %d) does not match the model (%d, %d, %d)",
                        kv->n_layers, kv->n_kv_heads, kv->head_dim, c.n_layers, c.n_kv_heads, c.head_dim);
    }
    return FG_OK;
}

int32_t check_tree(const fg_tree *t, bool need_tokens)
{
    if (!t) return fail(FG_ERR_INVALID_ARG, "tree is NULL");
    if (t->B < 0 || t->N < 0 || t->n_prev < 0) return fail(FG_ERR_INVALID_ARG, "negative B / N / n_prev");
    if (t->n_prev + t->N > FG_MAX_NODES)
        return fail(FG_ERR_CAPACITY, "n_prev + N = %d exceeds %d in-round nodes", t->n_prev + t->N, (int)FG_MAX_NODES);
    if (t->B > 0 && t->N > 0 && (!t->parent || (need_tokens && (!t->tokens || !t->slot))))
        return fail(FG_ERR_INVALID_ARG, "tree slot / tokens / parent is NULL");
    return FG_OK;
}

int max_keys_of(const fg_kv_cache *kv, const fg_tree *t, int32_t *rc)
{
    int cap = kv->max_pages_per_seq * kv->page_size;
    int mk = t->max_seq_len > 0 ? t->max_seq_len : cap;
    if (mk > cap) { *rc = fail(FG_ERR_CAPACITY, "max_seq_len %d exceeds the cache capacity %d", mk, cap); return 0; }
    *rc = FG_OK;
    return mk;
}

// reuse_order: the workspace still holds the item order an earlier layer of the same step built
int32_t attention_any(const fg_kv_cache *kv, int layer, const fg_tree *t, TreeDev td, int Hq, const void *q, void *out,
                      int max_keys, void *ws, int64_t ws_bytes, int reuse_order, hipStream_t st)
{
    if (attention_mfma_supported(kv, Hq, t->N))
        return launch_attention_mfma(kv, layer, t, td, Hq, q, out, max_keys, ws, ws_bytes, reuse_order, st);
    return launch_attention_simple(kv, layer, t, td, Hq, q, out, max_keys, st);
}

// The decoder layers shared by the target's verify step and the draft head.  On entry h holds the layer
// input when first_S == 0, otherwise `partials` holds first_S slabs whose sum is the layer input (h is
// initialised from them).  On exit `partials` holds *last_S slabs that still have to be added to h (0: h is complete).
// With enough rows for the pipelined GEMM to run without a k split, the row-wise steps ride in the GEMM epilogues: the
// QKV projection rotates q / k and appends k / v itself, the O and down projections add into h, and the norms read h
// alone.
int32_t run_layers(const fg_model *m, fg_kv_cache *kv, const fg_tree *t, const StepWs &w, int max_keys, int first_S,
                   int *last_S, hipStream_t st)
{
    const fg_model_cfg &c = m->cfg;
    const int M = t->B * t->N, d = c.d_model, F = c.d_ffn, hq = c.n_q_heads * c.head_dim;
    const int qkvd = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const bool f16 = is16(c.dtype);
    const bool fuse_rope = f16 && gemm_mfma_fusable(M, qkvd, d, EPI_ROPE) && qkvd % 256 == 0 && kv->page_size == 16;
    const bool fuse_o = f16 && gemm_mfma_fusable(M, d, hq, EPI_RESIDUAL);
    const bool fuse_down = f16 && gemm_mfma_fusable(M, d, F, EPI_RESIDUAL);
    GemmEpi rope;
    rope.pos = w.td.pos; rope.dest = w.td.dest; rope.k_pool = kv->k_pool; rope.v_pool = kv->v_pool; rope.q_out = w.q;
    rope.rope_tab = m->rope_tab; rope.n_pages = kv->n_pages; rope.Hq = c.n_q_heads; rope.Hkv = c.n_kv_heads; rope.hd = c.head_dim;
    rope.max_pos = c.max_pos; rope.k_frag = (int)k_fragment_major(kv->dtype, kv->head_dim, kv->page_size);
    GemmEpi resid;
    resid.h = w.h;
    int S = first_S, init = first_S > 0 ? 1 : 0;
    int32_t rc;
    for (int l = 0; l < c.n_layers; l++) {
        mark(m, FG_STAGE_NORM, st);
        if ((rc = launch_add_rmsnorm(c.dtype, w.h, w.partials, S, init, m->norm_attn[l], w.a, nullptr, M, d, c.rms_eps, st))) return rc;
        init = 0;
        mark(m, FG_STAGE_QKV, st);
        if (fuse_rope) {
            rope.layer = l;
            if ((rc = launch_gemm_mfma(c.dtype, w.a, m->wqkv[l], nullptr, M, qkvd, d, EPI_ROPE, 1, nullptr, st, &rope))) return rc;
        } else {
            if ((rc = gemm_any(c, w.a, m->wqkv[l], w.partials, M, qkvd, d, &S, st))) return rc;
            mark(m, FG_STAGE_ROPE, st);
            if ((rc = launch_rope_append(c.dtype, w.partials, S, t, w.td, kv, l, (const float *)m->rope_tab, c.max_pos, c.n_q_heads, w.q, st))) return rc;
        }
        mark(m, FG_STAGE_ATTENTION, st);
        if ((rc = attention_any(kv, l, t, w.td, c.n_q_heads, w.q, w.att, max_keys, w.attn_ws, w.attn_ws_bytes, l > 0, st))) return rc;
        mark(m, FG_STAGE_O, st);
        if (fuse_o) {
            if ((rc = launch_gemm_mfma(c.dtype, w.att, m->wo[l], nullptr, M, d, hq, EPI_RESIDUAL, 1, nullptr, st, &resid))) return rc;
            S = 0;
        } else if ((rc = gemm_any(c, w.att, m->wo[l], w.partials, M, d, hq, &S, st))) return rc;
        mark(m, FG_STAGE_NORM, st);
        if ((rc = launch_add_rmsnorm(c.dtype, w.h, w.partials, S, 0, m->norm_ffn[l], w.a, nullptr, M, d, c.rms_eps, st))) return rc;
        mark(m, FG_STAGE_GATE_UP, st);
        if (gate_up_fused(c, M)) {
            if ((rc = launch_gemm_mfma(c.dtype, w.a, m->wgu[l], w.act, M, 2 * F, d, EPI_SWIGLU, 1, nullptr, st))) return rc;
        } else {
            if ((rc = gemm_any(c, w.a, m->wgu[l], w.partials, M, 2 * F, d, &S, st))) return rc;
            mark(m, FG_STAGE_SWIGLU, st);
            if (f16) rc = launch_swiglu_partials(c.dtype, w.partials, S, w.act, M, F, st);
            else rc = launch_swiglu_f32(w.partials, (float *)w.act, M, F, st);
            if (rc) return rc;
        }
        mark(m, FG_STAGE_DOWN, st);
        if (fuse_down) {
            if ((rc = launch_gemm_mfma(c.dtype, w.act, m->wdown[l], nullptr, M, d, F, EPI_RESIDUAL, 1, nullptr, st, &resid))) return rc;
            S = 0;
        } else if ((rc = gemm_any(c, w.act, m->wdown[l], w.partials, M, d, F, &S, st))) return rc;
    }
    *last_S = S;
    return FG_OK;
}

// ---- scratch of the allocation-free entry point -----------------------------------------------------------------
// A file-scope device array: every GPU the library runs on holds its own copy from the moment the code object is
// loaded until the process ends.  In host code the array's name is only a handle for the runtime; its device
// address is looked up once per device and kept, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[FG_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES] = {};

int32_t scratch_of_current_device(void **out)
{
    int dev = -1;
    FG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(FG_ERR_CAPACITY, "device index %d beyond %d", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        FG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(FG_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FG_OK;
}

}  // namespace

extern "C" {

const char *fg_last_error(void) { return g_err; }

int32_t fg_plan(int32_t B_cur, float C_peak, float alpha, int32_t K_max, int32_t L_max, int32_t N_cap, int32_t *N_verify,
                int32_t *K_draft, int32_t *L_draft)
{
    if (!N_verify || !K_draft || !L_draft) return fail(FG_ERR_INVALID_ARG, "fg_plan: NULL output");
    if (B_cur < 1 || !(C_peak > 0.f) || !(alpha > 0.f) || K_max < 0 || L_max < 0 || N_cap < 1 || N_cap > FG_MAX_NODES)
        return fail(FG_ERR_INVALID_ARG, "fg_plan: B_cur=%d C_peak=%g alpha=%g K_max=%d L_max=%d N_cap=%d", B_cur, (double)C_peak,
                    (double)alpha, K_max, L_max, N_cap);
    // Eq. 1: N = C_peak / B, floored, at least the root, at most the mask width
    long long N = (long long)floor((double)C_peak / (double)B_cur);
    N = N < 1 ? 1 : (N > N_cap ? N_cap : N);
    // Eq. 2
    long long K = N - 1 < K_max ? N - 1 : K_max;
    // Eq. 3: the largest L with 2^L <= N / alpha, found by doubling (no libm rounding at powers of two)
    long long L = 0;
    const double ratio = (double)N / (double)alpha;
    if (ratio >= 1.0) {
        double pw = 2.0;
        while (pw <= ratio && L < 62) { L++; pw *= 2.0; }
    }
    if (L > L_max) L = L_max;
    if (L > N - 1) L = N - 1;
    if (K <= 0 || L <= 0) { N = 1; K = 0; L = 0; }
    else {
        long long cand = 1 + K + (L - 1) * K * K;  // all candidates the expansion produces
        if (N > cand) N = cand;
    }
    *N_verify = (int32_t)N; *K_draft = (int32_t)K; *L_draft = (int32_t)L;
    return FG_OK;
}

int32_t fg_knee(const double *x_in, const double *y, int32_t n, int32_t log2_axis, int32_t *knee_index)
{
    if (!x_in || !y || !knee_index || n < 3) return fail(FG_ERR_INVALID_ARG, "fg_knee: NULL pointer or fewer than 3 samples");
    std::vector<double> xs(x_in, x_in + n);
    if (log2_axis)
        for (int i = 0; i < n; i++) {
            if (!(xs[i] > 0.0)) return fail(FG_ERR_INVALID_ARG, "fg_knee: a log2 axis needs positive x (sample %d)", i);
            xs[i] = log2(xs[i]);
        }
    const double *x = xs.data();
    double lo = y[0], hi = y[0];
    for (int i = 1; i < n; i++) {
        if (!(x[i] > x[i - 1])) return fail(FG_ERR_INVALID_ARG, "fg_knee: x must increase strictly (sample %d)", i);
        lo = fmin(lo, y[i]);
        hi = fmax(hi, y[i]);
    }
    int arg = 0;
    if (hi > lo) {
        // height of the chord above the curve, in units of the curve's range, with x mapped to [0, 1]
        const double span = x[n - 1] - x[0], rise = y[n - 1] - y[0];
        double far = 0.0;
        for (int i = 0; i < n; i++) {
            const double gap = (y[0] + rise * ((x[i] - x[0]) / span) - y[i]) / (hi - lo);
            if (gap > far) { far = gap; arg = i; }
        }
    }
    *knee_index = arg;
    return FG_OK;
}

int32_t fg_select_rows(const void *src, int64_t row_bytes, int32_t n_src, const int32_t *index, int32_t n, void *dst, void *stream)
{
    if (n < 0 || n_src < 1 || row_bytes < 4 || row_bytes % 4) return fail(FG_ERR_INVALID_ARG, "fg_select_rows: bad sizes");
    if (n == 0) return FG_OK;
    if (!src || !index || !dst) return fail(FG_ERR_INVALID_ARG, "fg_select_rows: NULL pointer");
    return launch_select_rows(src, row_bytes, n_src, index, n, dst, (hipStream_t)stream);
}

int64_t fg_packed_bytes(int32_t dtype, int64_t n_out_total, int64_t n_in) { return n_out_total * n_in * (int64_t)dtype_size(dtype); }

int32_t fg_pack_weight(int32_t dtype, const void *src, const void *src2, void *dst, int64_t n_out, int64_t n_in, void *stream)
{
    if (!src || !dst || n_out <= 0 || n_in <= 0) return fail(FG_ERR_INVALID_ARG, "fg_pack_weight: NULL pointer or empty matrix");
    return launch_pack(dtype, src, src2, dst, n_out, n_in, (hipStream_t)stream);
}

int32_t fg_model_create(const fg_model_cfg *cfg, const fg_weights *w, fg_model **out)
{
    if (!cfg || !w || !out) return fail(FG_ERR_INVALID_ARG, "fg_model_create: NULL argument");
    const fg_model_cfg &c = *cfg;
    if (!dtype_ok(c.dtype)) return fail(FG_ERR_INVALID_ARG, "unknown dtype %d", c.dtype);
    if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.d_ffn < 1 || c.vocab < 1 || c.max_pos < 1)
        return fail(FG_ERR_INVALID_ARG, "model sizes must be positive");
    if (c.head_dim != 64 && c.head_dim != 128) return fail(FG_ERR_SHAPE, "head_dim must be 64 or 128 (got %d)", c.head_dim);
    if (c.n_q_heads % c.n_kv_heads || c.n_q_heads / c.n_kv_heads > 8)
        return fail(FG_ERR_SHAPE, "n_q_heads must be a multiple (at most 8x) of n_kv_heads");
    if (c.d_model % 64 || c.d_ffn % 64 || c.vocab % 32 || (c.n_q_heads * c.head_dim) % 64)
        return fail(FG_ERR_SHAPE, "d_model, d_ffn and Hq*hd must be multiples of 64, vocab of 32");
    if (!w->embed || !w->lm_head || !w->wqkv || !w->wo || !w->w_gate_up || !w->w_down || !w->norm_attn || !w->norm_ffn)
        return fail(FG_ERR_INVALID_ARG, "a weight pointer is NULL");
    if (!w->final_norm && !w->fc) return fail(FG_ERR_INVALID_ARG, "need final_norm (target) or fc (draft head)");
    fg_model *m = new (std::nothrow) fg_model();
    if (!m) return fail(FG_ERR_INVALID_ARG, "out of host memory");
    m->cfg = c;
    m->embed = w->embed; m->lm_head = w->lm_head; m->final_norm = w->final_norm; m->fc = w->fc;
    for (int l = 0; l < c.n_layers; l++) {
        if (!w->wqkv[l] || !w->wo[l] || !w->w_gate_up[l] || !w->w_down[l] || !w->norm_attn[l] || !w->norm_ffn[l]) {
            delete m;
            return fail(FG_ERR_INVALID_ARG, "a weight pointer of layer %d is NULL", l);
        }
        m->wqkv.push_back(w->wqkv[l]); m->wo.push_back(w->wo[l]); m->wgu.push_back(w->w_gate_up[l]);
        m->wdown.push_back(w->w_down[l]); m->norm_attn.push_back(w->norm_attn[l]); m->norm_ffn.push_back(w->norm_ffn[l]);
    }
    const int half = c.head_dim / 2;
    std::vector<float2> tab((size_t)c.max_pos * half);
    for (int p = 0; p < c.max_pos; p++)
        for (int i = 0; i < half; i++) {
            double ang = (double)p * pow((double)c.rope_theta, -2.0 * (double)i / (double)c.head_dim);
            tab[(size_t)p * half + i] = make_float2((float)cos(ang), (float)sin(ang));
        }
    m->rope_tab = nullptr;
    hipError_t e = hipGetDevice(&m->device);
    if (e == hipSuccess) e = hipMalloc((void **)&m->rope_tab, tab.size() * sizeof(float2));
    if (e == hipSuccess) e = hipMemcpy(m->rope_tab, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (m->rope_tab) (void)hipFree(m->rope_tab);
        delete m;
        return fail(FG_ERR_HIP, "RoPE table: %s", hipGetErrorString(e));
    }
    void *scratch_ptr = nullptr;
    (void)scratch_of_current_device(&scratch_ptr);   // set-up: the allocation-free entry point finds its address resolved
    *out = m;
    return FG_OK;
}

int32_t fg_model_destroy(fg_model *m)
{
    if (!m) return FG_OK;
    if (m->rope_tab) (void)hipFree(m->rope_tab);
    for (hipEvent_t e : m->prof.ev) (void)hipEventDestroy(e);
    delete m;
    return FG_OK;
}

int64_t fg_workspace_bytes_for(const fg_model_cfg *cfg, int32_t is_draft, int32_t max_rows, int32_t max_seq_len)
{
    if (!cfg || max_rows < 1 || max_seq_len < 1 || !dtype_ok(cfg->dtype) || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return 0;
    // every piece but the attention workspace grows with the row count; that one takes its maximum over all shapes
    const int64_t attn = max_attention_ws(*cfg, max_rows, max_seq_len);
    return carve_step(*cfg, max_rows, max_seq_len, max_rows, 1, is_draft != 0, nullptr, 0, nullptr, true, attn) + (1 << 20);
}

int64_t fg_step_workspace_bytes(const fg_model_cfg *cfg, int32_t is_draft, int32_t B, int32_t N, int32_t max_seq_len, int32_t with_logits)
{
    if (!cfg || B < 1 || N < 1 || max_seq_len < 1 || !dtype_ok(cfg->dtype) || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return 0;
    return carve_step(*cfg, B * N, max_seq_len, B, N, is_draft != 0, nullptr, 0, nullptr, with_logits != 0);
}

int64_t fg_workspace_bytes(const fg_model *m, int32_t max_rows, int32_t max_seq_len)
{
    if (!m) return 0;
    return fg_workspace_bytes_for(&m->cfg, m->fc != nullptr, max_rows, max_seq_len);
}

int32_t fg_spec_verify(fg_model *m, fg_kv_cache *kv, const fg_tree *tree, float *logits, void *feature, int32_t *row_argmax,
                       float *row_top2, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (!m) return fail(FG_ERR_INVALID_ARG, "fg_spec_verify: model is NULL");
    int32_t rc;
    if ((rc = check_cache(m, kv))) return rc;
    if ((rc = check_tree(tree, true))) return rc;
    if (!m->final_norm) return fail(FG_ERR_INVALID_ARG, "fg_spec_verify needs a target model (final_norm)");
    if (tree->B == 0 || tree->N == 0) return FG_OK;
    if (!workspace) return fail(FG_ERR_INVALID_ARG, "workspace is NULL");
    const fg_model_cfg &c = m->cfg;
    const int M = tree->B * tree->N;
    const int mk = max_keys_of(kv, tree, &rc);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    StepWs w;
    const bool need_logits = !logits && (row_argmax || row_top2);
    if (carve_step(c, M, mk, tree->B, tree->N, false, workspace, workspace_bytes, &w, need_logits) < 0)
        return fail(FG_ERR_CAPACITY, "workspace too small: have %lld bytes", (long long)workspace_bytes);
    mark(m, FG_STAGE_PREP, st);
    if ((rc = launch_tree_prep_ex(tree, kv, w.td, c.max_pos, st))) return rc;
    if ((rc = launch_embed(c.dtype, m->embed, tree->tokens, c.vocab, w.h, M, c.d_model, st))) return rc;
    int S = 0;
    if ((rc = run_layers(m, kv, tree, w, mk, 0, &S, st))) return rc;
    void *feat = feature ? feature : w.feat;
    mark(m, FG_STAGE_NORM, st);
    if ((rc = launch_add_rmsnorm(c.dtype, w.h, w.partials, S, 0, m->final_norm, feat, nullptr, M, c.d_model, c.rms_eps, st))) return rc;
    float *lg = logits ? logits : w.logits;
    if (!logits && lg && is16(c.dtype) && gemm_mfma_fusable(M, c.vocab, c.d_model, EPI_TOPK)) {
        // only the decisions are wanted: the LM head selects in its epilogue and no [M, V] tensor is written
        mark(m, FG_STAGE_LM_HEAD, st);
        if ((rc = lm_head_topk(c.dtype, feat, m->lm_head, M, c.vocab, c.d_model, 2, false, w.logits, nullptr, nullptr, row_argmax,
                               row_top2, st))) return rc;
    } else if (lg) {
        mark(m, FG_STAGE_LM_HEAD, st);
        if (is16(c.dtype)) rc = launch_gemm_mfma(c.dtype, feat, m->lm_head, lg, M, c.vocab, c.d_model, 0, 1, nullptr, st);
        else rc = launch_gemm_f32((const float *)feat, (const float *)m->lm_head, lg, M, c.vocab, c.d_model, st);
        if (rc) return rc;
        if (row_argmax || row_top2) {
            mark(m, FG_STAGE_SELECT, st);
            if ((rc = launch_argmax_top2(lg, M, c.vocab, row_argmax, row_top2, st))) return rc;
        }
    }
    mark(m, FG_STAGE_END, st);
    return FG_OK;
}

int32_t fg_spec_accept(const fg_tree *tree, int32_t mode, const float *logits, const int32_t *row_argmax, int32_t vocab,
                       float temperature, const float *draft_probs, const float *uniforms, uint64_t seed, int64_t row0,
                       int32_t eos_id, int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished,
                       void *workspace, int64_t workspace_bytes, void *stream)
{
    int32_t rc;
    if ((rc = check_tree(tree, false))) return rc;
    if (!tree->tokens) return fail(FG_ERR_INVALID_ARG, "fg_spec_accept: tokens is NULL");
    if (tree->n_prev != 0) return fail(FG_ERR_INVALID_ARG, "fg_spec_accept works on a whole tree (n_prev must be 0)");
    if (!accept_len || !path || !out_tokens || !finished) return fail(FG_ERR_INVALID_ARG, "fg_spec_accept: NULL output");
    if (tree->B == 0) return FG_OK;
    if (tree->N < 1) return fail(FG_ERR_INVALID_ARG, "fg_spec_accept: N must be at least 1");
    const int B = tree->B, N = tree->N, M = B * N;
    hipStream_t st = (hipStream_t)stream;
    if (mode == FG_ACCEPT_GREEDY || mode == FG_ACCEPT_SAMPLE_MATCH) {
        const int32_t *tt = row_argmax;
        if (mode == FG_ACCEPT_SAMPLE_MATCH || !tt) {
            if (!logits || vocab < 1) return fail(FG_ERR_INVALID_ARG, "fg_spec_accept: logits needed");
            if (!workspace || workspace_bytes < (int64_t)M * 4)
                return fail(FG_ERR_CAPACITY, "fg_spec_accept: workspace of %lld bytes needed", (long long)M * 4);
            int32_t *buf = (int32_t *)workspace;
            if (mode == FG_ACCEPT_GREEDY) rc = launch_argmax_top2(logits, M, vocab, buf, nullptr, st);
            else {
                if (!(temperature > 0.f)) return fail(FG_ERR_INVALID_ARG, "temperature must be positive");
                rc = launch_gumbel_argmax(logits, M, vocab, temperature, seed, row0, buf, st);
            }
            if (rc) return rc;
            tt = buf;
        }
        return launch_walk(B, N, tree->tokens, tree->parent, tt, eos_id, accept_len, path, out_tokens, finished, st);
    }
    if (mode == FG_ACCEPT_REJECT) {
        if (!logits || !draft_probs || !uniforms || vocab < 1) return fail(FG_ERR_INVALID_ARG, "rejection mode needs logits, draft_probs, uniforms");
        if (!(temperature > 0.f)) return fail(FG_ERR_INVALID_ARG, "temperature must be positive");
        int64_t need = (int64_t)B * 2 * vocab * 4;
        if (!workspace || workspace_bytes < need) return fail(FG_ERR_CAPACITY, "fg_spec_accept: workspace of %lld bytes needed", (long long)need);
        return launch_reject(B, N, vocab, tree->tokens, tree->parent, logits, draft_probs, uniforms, temperature, seed, row0,
                             eos_id, (float *)workspace, accept_len, path, out_tokens, finished, st);
    }
    return fail(FG_ERR_INVALID_ARG, "unknown acceptance mode %d", mode);
}

int32_t fg_spec_accept_static(const fg_tree *tree, int32_t mode, const float *logits, const int32_t *row_argmax, int32_t vocab,
                              float temperature, const float *draft_probs, const float *uniforms, uint64_t seed, int64_t row0,
                              int32_t eos_id, int32_t *accept_len, int32_t *path, int32_t *out_tokens, int32_t *finished,
                              void *stream)
{
    if (!tree) return fail(FG_ERR_INVALID_ARG, "tree is NULL");
    if (tree->B < 0 || tree->N < 0) return fail(FG_ERR_INVALID_ARG, "negative B / N");
    int64_t need = 0;
    if (mode == FG_ACCEPT_REJECT) need = (int64_t)tree->B * 2 * (vocab > 0 ? vocab : 0) * 4;
    else if (mode == FG_ACCEPT_SAMPLE_MATCH || !row_argmax) need = (int64_t)tree->B * tree->N * 4;
    if (need > FG_STATIC_SCRATCH_BYTES)
        return fail(FG_ERR_CAPACITY, "fg_spec_accept_static: this call needs %lld bytes of scratch, the static array holds %d "
                                     "(use fg_spec_accept with a caller-provided workspace)", (long long)need, (int)FG_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    int32_t rc;
    if ((rc = scratch_of_current_device(&ptr))) return rc;
    return fg_spec_accept(tree, mode, logits, row_argmax, vocab, temperature, draft_probs, uniforms, seed, row0, eos_id,
                          accept_len, path, out_tokens, finished, ptr, FG_STATIC_SCRATCH_BYTES, stream);
}

int32_t fg_kv_compact(fg_kv_cache *kv, const int32_t *slot, const int32_t *accept_len, const int32_t *path, int32_t B, int32_t N,
                      const void *feature_in, void *feature_out, int32_t d_model, int32_t feat_dtype, void *stream)
{
    int32_t rc;
    if ((rc = check_cache(nullptr, kv))) return rc;
    if (B < 0 || N < 1 || N > FG_MAX_NODES) return fail(FG_ERR_INVALID_ARG, "fg_kv_compact: bad B / N");
    if (B == 0) return FG_OK;
    if (!slot || !accept_len || !path) return fail(FG_ERR_INVALID_ARG, "fg_kv_compact: NULL input");
    if ((feature_in != nullptr) != (feature_out != nullptr)) return fail(FG_ERR_INVALID_ARG, "feature_in and feature_out go together");
    if (!dtype_ok(kv->dtype)) return fail(FG_ERR_INVALID_ARG, "unknown cache dtype");
    return launch_kv_compact(kv, slot, accept_len, path, B, N, feature_in, feature_out, d_model, feat_dtype, (hipStream_t)stream);
}

int32_t fg_draft_step(fg_model *target, fg_model *draft, fg_kv_cache *draft_kv, const fg_tree *tree, const void *in_feature,
                      const int32_t *feat_index, int32_t feat_rows, const int32_t *n_commit, int32_t commit_bias,
                      int32_t K_draft, const int32_t *expand_row, int32_t *child_tok, float *child_logp, void *out_feature,
                      void *workspace, int64_t workspace_bytes, void *stream)
{
    if (!target || !draft) return fail(FG_ERR_INVALID_ARG, "fg_draft_step: model is NULL");
    if (!draft->fc) return fail(FG_ERR_INVALID_ARG, "fg_draft_step needs a draft head (fc)");
    int32_t rc;
    if ((rc = check_cache(draft, draft_kv))) return rc;
    if ((rc = check_tree(tree, true))) return rc;
    const fg_model_cfg &c = draft->cfg;
    if (c.d_model != target->cfg.d_model || c.vocab != target->cfg.vocab || c.dtype != target->cfg.dtype)
        return fail(FG_ERR_SHAPE, "draft head and target differ in width, vocabulary or dtype");
    if (tree->B == 0 || tree->N == 0) return FG_OK;
    if (!in_feature || !workspace) return fail(FG_ERR_INVALID_ARG, "fg_draft_step: NULL input");
    if (feat_rows < 1 || (!feat_index && feat_rows < tree->N)) return fail(FG_ERR_INVALID_ARG, "fg_draft_step: bad feat_rows");
    if ((child_tok != nullptr) != (child_logp != nullptr)) return fail(FG_ERR_INVALID_ARG, "child_tok and child_logp go together");
    const int M = tree->B * tree->N, d = c.d_model;
    const int mk = max_keys_of(draft_kv, tree, &rc);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    StepWs w;
    if (carve_step(c, M, mk, tree->B, tree->N, true, workspace, workspace_bytes, &w, child_tok != nullptr) < 0)
        return fail(FG_ERR_CAPACITY, "workspace too small: have %lld bytes", (long long)workspace_bytes);
    mark(draft, FG_STAGE_PREP, st);
    if ((rc = launch_tree_prep_ex(tree, draft_kv, w.td, c.max_pos, st))) return rc;
    if ((rc = launch_concat_embed(c.dtype, target->embed, tree->tokens, c.vocab, in_feature, feat_index, tree->N, feat_rows, w.cat, M, d, st))) return rc;
    int S = 0;
    mark(draft, FG_STAGE_FC, st);
    if ((rc = gemm_any(c, w.cat, draft->fc, w.partials, M, d, 2 * d, &S, st))) return rc;
    if ((rc = run_layers(draft, draft_kv, tree, w, mk, S, &S, st))) return rc;
    void *hid = out_feature ? out_feature : w.feat;
    mark(draft, FG_STAGE_NORM, st);
    if ((rc = launch_add_rmsnorm(c.dtype, w.h, w.partials, S, 0, draft->norm_attn[0], nullptr, hid, M, d, c.rms_eps, st))) return rc;
    if (child_tok) {
        int rows = M;
        if (expand_row) {   // only the picked row of each sequence goes through the LM head
            rows = tree->B;
            mark(draft, FG_STAGE_PREP, st);
            if ((rc = launch_gather_rows(c.dtype, hid, expand_row, tree->B, tree->N, d, w.cat, st))) return rc;
            hid = w.cat;
        }
        if (K_draft < 1 || K_draft > 8 || K_draft > c.vocab) return fail(FG_ERR_INVALID_ARG, "K_draft must be in 1..8 (got %d)", K_draft);
        mark(draft, FG_STAGE_LM_HEAD, st);
        if (is16(c.dtype) && gemm_mfma_fusable(rows, c.vocab, d, EPI_TOPK)) {
            if ((rc = lm_head_topk(c.dtype, hid, target->lm_head, rows, c.vocab, d, K_draft, true, w.logits, child_tok, child_logp,
                                   nullptr, nullptr, st))) return rc;
        } else {
            if (is16(c.dtype)) rc = launch_gemm_mfma(c.dtype, hid, target->lm_head, w.logits, rows, c.vocab, d, 0, 1, nullptr, st);
            else rc = launch_gemm_f32((const float *)hid, (const float *)target->lm_head, w.logits, rows, c.vocab, d, st);
            if (rc) return rc;
            mark(draft, FG_STAGE_SELECT, st);
            if ((rc = launch_topk_logp(w.logits, rows, c.vocab, K_draft, child_tok, child_logp, st))) return rc;
        }
    }
    if (n_commit) {
        mark(draft, FG_STAGE_PREP, st);
        if ((rc = launch_commit_len(draft_kv->seq_len, tree->slot, n_commit, commit_bias, tree->B, draft_kv->n_slots,
                                    draft_kv->max_pages_per_seq * draft_kv->page_size, draft_kv->status, st))) return rc;
    }
    mark(draft, FG_STAGE_END, st);
    return FG_OK;
}

int32_t fg_draft_frontier(int32_t B, int32_t K_in, int32_t K, const int32_t *child_tok, const float *child_logp,
                          int32_t child_rows, const int32_t *node_cand, const float *node_score, const int32_t *node_pick,
                          const int32_t *node_tok, int32_t n_cand, int32_t cand_stride,
                          int32_t *cand_tok, int32_t *cand_parent, float *cand_score, int32_t *next_tok, int32_t *next_cand,
                          float *next_score, int32_t *next_src, const int32_t *parent_prev, int32_t n_parent_prev,
                          int32_t *parent_next, void *stream)
{
    if (B < 0 || K_in < 1 || K < 1 || K_in * K > 64 || K > K_in * K) return fail(FG_ERR_INVALID_ARG, "fg_draft_frontier: bad K_in / K");
    if (child_rows != K_in && !(child_rows == 1 && node_pick)) return fail(FG_ERR_INVALID_ARG, "fg_draft_frontier: child_rows must be K_in, or 1 with node_pick");
    if (n_cand < 0 || n_cand + (node_pick ? K : K_in * K) > cand_stride) return fail(FG_ERR_CAPACITY, "candidate lists too short");
    if (B == 0) return FG_OK;
    if ((!node_pick && (!node_cand || !node_score)) || !child_tok || !child_logp || !cand_tok || !cand_parent || !cand_score || !next_tok ||
        !next_cand || !next_score || !next_src)
        return fail(FG_ERR_INVALID_ARG, "fg_draft_frontier: NULL pointer");
    if (n_parent_prev < 0 || n_parent_prev + K > FG_MAX_NODES || (parent_next && n_parent_prev > 0 && !parent_prev) ||
        (parent_next && !node_pick && n_parent_prev < K_in))
        return fail(FG_ERR_INVALID_ARG, "fg_draft_frontier: bad parent list");
    return launch_frontier(B, K_in, K, child_tok, child_logp, child_rows, node_cand, node_score, node_pick, node_tok, n_cand, cand_stride, cand_tok, cand_parent,
                           cand_score, next_tok, next_cand, next_score, next_src, parent_prev, n_parent_prev, parent_next,
                           (hipStream_t)stream);
}

int32_t fg_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int32_t B, int32_t n_cand,
                      int32_t cand_stride, int32_t N, int32_t *tokens, int32_t *parent, int32_t *sel, void *stream)
{
    if (B < 0 || n_cand < 1 || N < 1 || N > n_cand || N > FG_MAX_NODES || cand_stride < n_cand)
        return fail(FG_ERR_INVALID_ARG, "fg_build_tree: bad sizes (n_cand %d, N %d)", n_cand, N);
    if (B == 0) return FG_OK;
    if (!cand_tok || !cand_parent || !cand_score || !tokens || !parent) return fail(FG_ERR_INVALID_ARG, "fg_build_tree: NULL pointer");
    return launch_build_tree(cand_tok, cand_parent, cand_score, B, n_cand, cand_stride, N, tokens, parent, sel, (hipStream_t)stream);
}

int32_t fg_gemm(int32_t dtype, const void *x, const void *w_packed, void *out, int32_t M, int32_t n_out, int32_t n_in,
                int32_t epilogue, int32_t split_k, int32_t *split_k_used, int32_t variant, void *stream)
{
    if (!x || !w_packed || !out || M < 0 || n_out < 1 || n_in < 1) return fail(FG_ERR_INVALID_ARG, "fg_gemm: bad argument");
    if (epilogue != EPI_SLABS && epilogue != EPI_SWIGLU && epilogue != EPI_RESIDUAL) return fail(FG_ERR_INVALID_ARG, "fg_gemm: epilogue %d", epilogue);
    if (M == 0) return FG_OK;
    if (is16(dtype)) {
        GemmEpi ep;
        ep.h = (float *)out;
        if (epilogue == EPI_RESIDUAL && (variant == 1 || variant == 2)) return fail(FG_ERR_INVALID_ARG, "fg_gemm: the residual epilogue needs the pipelined kernel");
        return launch_gemm_mfma(dtype, x, w_packed, out, M, n_out, n_in, epilogue, epilogue == EPI_SLABS ? split_k : 1, split_k_used,
                                (hipStream_t)stream, &ep, variant);
    }
    if (dtype == FG_F32) {
        if (epilogue != 0) return fail(FG_ERR_UNIMPLEMENTED, "fp32 GEMM has no fused epilogue");
        if (split_k_used) *split_k_used = 1;
        return launch_gemm_f32((const float *)x, (const float *)w_packed, (float *)out, M, n_out, n_in, (hipStream_t)stream);
    }
    return fail(FG_ERR_INVALID_ARG, "unknown dtype %d", dtype);
}

const char *fg_gemm_kernel_name(int32_t M, int32_t n_out, int32_t n_in, int32_t epilogue)
{
    if (M < 1 || n_out < 1 || n_in < 1 || epilogue < 0 || epilogue > EPI_RESIDUAL) return "";
    return gemm_mfma_kernel_name(M, n_out, n_in, epilogue);
}

int32_t fg_topk_logp(const float *logits, int32_t M, int32_t vocab, int32_t K, int32_t *tok, float *logp, void *stream)
{
    if (M < 0 || vocab < 1) return fail(FG_ERR_INVALID_ARG, "fg_topk_logp: bad sizes (M %d, vocab %d)", M, vocab);
    if (M == 0) return FG_OK;
    if (!logits || !tok || !logp) return fail(FG_ERR_INVALID_ARG, "fg_topk_logp: null pointer");
    return launch_topk_logp(logits, M, vocab, K, tok, logp, (hipStream_t)stream);
}

static int32_t check_train_cfg(const fg_model_cfg *c)
{
    if (!c) return fail(FG_ERR_INVALID_ARG, "draft training: configuration is NULL");
    if (c->n_layers != 1) return fail(FG_ERR_SHAPE, "draft training: the head has one decoder layer (got %d)", c->n_layers);
    if (c->d_model < 4 || c->d_ffn < 4 || c->vocab < 4 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads ||
        c->head_dim < 2 || c->head_dim % 2)
        return fail(FG_ERR_INVALID_ARG, "draft training: bad model sizes");
    if (c->d_model % 4 || c->d_ffn % 4 || c->vocab % 4 || (c->n_q_heads * c->head_dim) % 4 || (c->n_kv_heads * c->head_dim) % 4)
        return fail(FG_ERR_SHAPE, "draft training: d_model, d_ffn, vocab, Hq*hd and Hkv*hd must be multiples of 4");
    return FG_OK;
}

static bool params_ok(const fg_draft_params *p)
{
    return p && p->fc && p->wqkv && p->wo && p->w_gate && p->w_up && p->w_down && p->norm_attn && p->norm_ffn;
}

int64_t fg_draft_train_workspace_bytes(const fg_model_cfg *cfg, int32_t B, int32_t T)
{
    if (check_train_cfg(cfg) || !dtype_ok(cfg->dtype) || B < 1 || T < 1) return 0;
    return draft_train_ws_bytes(*cfg, B, T);
}

int32_t fg_draft_train_grad(const fg_model_cfg *cfg, const float *embed, const float *lm_head, const fg_draft_params *w,
                            const int32_t *tokens, const float *feat_in, const float *feat_tgt, const int32_t *n_valid, int32_t B,
                            int32_t T, float w_ce, fg_draft_params *grad, float *loss, const void *head_packed, void *workspace,
                            int64_t workspace_bytes, void *stream)
{
    int32_t rc;
    if ((rc = check_train_cfg(cfg))) return rc;
    if (cfg->dtype == FG_F16) return fail(FG_ERR_INVALID_ARG, "fg_draft_train_grad: FG_F32 (exact) or FG_BF16 (matrix cores); fp16 would flush the gradients");
    if (cfg->dtype == FG_BF16 && (((int64_t)B * T) % 64 || cfg->d_model % 64 || cfg->d_ffn % 64 || cfg->vocab % 64 ||
                                  (cfg->n_q_heads * cfg->head_dim) % 64 || ((cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim) % 64))
        return fail(FG_ERR_SHAPE, "fg_draft_train_grad: the matrix-core path needs B * T and every model width in multiples of 64");
    if (B < 0 || T < 0) return fail(FG_ERR_INVALID_ARG, "fg_draft_train_grad: negative B / T");
    if (B == 0 || T == 0) return FG_OK;
    if (T > 8192) return fail(FG_ERR_CAPACITY, "fg_draft_train_grad: chains of at most 8192 entries (got %d)", T);
    if ((int64_t)B * T * (int64_t)cfg->vocab >= (1LL << 31) * 4) return fail(FG_ERR_CAPACITY, "fg_draft_train_grad: B * T * vocab too large");
    if (!embed || !lm_head || !params_ok(w) || !params_ok(grad) || !tokens || !feat_in || !feat_tgt || !n_valid || !loss || !workspace)
        return fail(FG_ERR_INVALID_ARG, "fg_draft_train_grad: NULL pointer");
    return launch_draft_train_grad(*cfg, embed, lm_head, w, tokens, feat_in, feat_tgt, n_valid, B, T, w_ce, grad, loss, head_packed,
                                   workspace, workspace_bytes, (hipStream_t)stream);
}

int64_t fg_draft_train_head_bytes(const fg_model_cfg *cfg)
{
    if (check_train_cfg(cfg)) return 0;
    return draft_train_head_bytes(*cfg);
}

int32_t fg_draft_train_pack_head(const fg_model_cfg *cfg, const float *lm_head, void *packed, int64_t packed_bytes, void *stream)
{
    int32_t rc;
    if ((rc = check_train_cfg(cfg))) return rc;
    if (!lm_head || !packed) return fail(FG_ERR_INVALID_ARG, "fg_draft_train_pack_head: NULL pointer");
    if (cfg->vocab % 64 || cfg->d_model % 64) return fail(FG_ERR_SHAPE, "fg_draft_train_pack_head: vocab and d in multiples of 64");
    if (packed_bytes < draft_train_head_bytes(*cfg)) return fail(FG_ERR_CAPACITY, "fg_draft_train_pack_head: buffer too small");
    return launch_draft_train_pack_head(*cfg, lm_head, packed, (hipStream_t)stream);
}

int32_t fg_draft_adamw(const fg_model_cfg *cfg, fg_draft_params *w, const fg_draft_params *grad, fg_draft_params *m,
                       fg_draft_params *v, float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step,
                       void *stream)
{
    int32_t rc;
    if ((rc = check_train_cfg(cfg))) return rc;
    if (!params_ok(w) || !params_ok(grad) || !params_ok(m) || !params_ok(v)) return fail(FG_ERR_INVALID_ARG, "fg_draft_adamw: NULL pointer");
    if (step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f))
        return fail(FG_ERR_INVALID_ARG, "fg_draft_adamw: step >= 1, betas in [0, 1), eps > 0");
    const int64_t d = cfg->d_model, F = cfg->d_ffn, hq = (int64_t)cfg->n_q_heads * cfg->head_dim;
    const int64_t qkvd = (int64_t)(cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
    const int64_t sizes[8] = {d * 2 * d, qkvd * d, d * hq, F * d, F * d, d * F, d, d};
    float *pw[8] = {w->fc, w->wqkv, w->wo, w->w_gate, w->w_up, w->w_down, w->norm_attn, w->norm_ffn};
    const float *pg[8] = {grad->fc, grad->wqkv, grad->wo, grad->w_gate, grad->w_up, grad->w_down, grad->norm_attn, grad->norm_ffn};
    float *pm[8] = {m->fc, m->wqkv, m->wo, m->w_gate, m->w_up, m->w_down, m->norm_attn, m->norm_ffn};
    float *pv[8] = {v->fc, v->wqkv, v->wo, v->w_gate, v->w_up, v->w_down, v->norm_attn, v->norm_ffn};
    for (int i = 0; i < 8; i++)
        if ((rc = launch_adamw(pw[i], pg[i], pm[i], pv[i], sizes[i], lr, beta1, beta2, eps, weight_decay, step, (hipStream_t)stream))) return rc;
    return FG_OK;
}

int64_t fg_lm_head_topk_workspace_bytes(int32_t M, int32_t vocab, int32_t K)
{
    if (M < 1 || vocab < 1 || K < 1 || K > 8) return 0;
    return lm_head_topk_bytes(M, vocab, K);
}

int32_t fg_lm_head_topk(int32_t dtype, const void *x, const void *lm_head_packed, int32_t M, int32_t vocab, int32_t d_model, int32_t K,
                        int32_t *tok, float *logp, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (!x || !lm_head_packed || !tok || !logp || !workspace || M < 0 || vocab < 1 || d_model < 1)
        return fail(FG_ERR_INVALID_ARG, "fg_lm_head_topk: bad argument");
    if (K < 1 || K > 8 || K > vocab) return fail(FG_ERR_INVALID_ARG, "fg_lm_head_topk: K must be in 1..8 (got %d)", K);
    if (M == 0) return FG_OK;
    if (!is16(dtype) || vocab % 32 || d_model % 64) return fail(FG_ERR_SHAPE, "fg_lm_head_topk: 16-bit dtypes, vocab %% 32 == 0, d_model %% 64 == 0");
    if (!gemm_mfma_fusable(M, vocab, d_model, EPI_TOPK))
        return fail(FG_ERR_SHAPE, "fg_lm_head_topk: the selecting epilogue runs from 129 rows and 16384 tokens on, from 65 rows and 32544 tokens on (got %d, %d)", M, vocab);
    if (workspace_bytes < lm_head_topk_bytes(M, vocab, K)) return fail(FG_ERR_CAPACITY, "fg_lm_head_topk: workspace too small");
    return lm_head_topk(dtype, x, lm_head_packed, M, vocab, d_model, K, true, workspace, tok, logp, nullptr, nullptr, (hipStream_t)stream);
}

int32_t fg_model_profile(fg_model *m, int32_t enable, int32_t max_marks)
{
    if (!m) return fail(FG_ERR_INVALID_ARG, "fg_model_profile: model is NULL");
    StageProf &p = m->prof;
    p.on = false;
    p.used = 0;
    p.only = -1;
    if (!enable) return FG_OK;
    if (enable < 0 || enable >= 2 + FG_STAGE_COUNT) return fail(FG_ERR_INVALID_ARG, "fg_model_profile: enable is 0, 1 or 2 + a stage");
    if (enable >= 2) p.only = enable - 2;
    if (max_marks < 2 || max_marks > (1 << 22)) return fail(FG_ERR_INVALID_ARG, "fg_model_profile: bad max_marks");
    while ((int)p.ev.size() < max_marks) {
        hipEvent_t e;
        FG_HIP(hipEventCreate(&e));
        p.ev.push_back(e);
    }
    p.stage.resize(p.ev.size());
    p.on = true;
    return FG_OK;
}

int32_t fg_model_profile_read(fg_model *m, double *ms, int32_t *launches)
{
    if (!m || !ms || !launches) return fail(FG_ERR_INVALID_ARG, "fg_model_profile_read: NULL argument");
    StageProf &p = m->prof;
    for (int i = 0; i < FG_STAGE_COUNT; i++) { ms[i] = 0.0; launches[i] = 0; }
    if (p.used > 0) FG_HIP(hipEventSynchronize(p.ev[p.used - 1]));
    for (size_t i = 0; i + 1 < p.used; i++) {
        const int sg = p.stage[i];
        if (sg < 0 || sg >= FG_STAGE_COUNT || (p.only >= 0 && sg != p.only)) continue;
        float t = 0.f;
        FG_HIP(hipEventElapsedTime(&t, p.ev[i], p.ev[i + 1]));
        ms[sg] += t;
        launches[sg]++;
    }
    p.used = 0;
    return FG_OK;
}

int32_t fg_probe_read(const void *src, int64_t bytes, int32_t nontemporal, int32_t blocks, void *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || bytes % 16 || blocks < 1 || nontemporal < 0 || nontemporal > 6)
        return fail(FG_ERR_INVALID_ARG, "fg_probe_read: bad argument");
    if (nontemporal == 3 && (bytes < 32768 || bytes > (64 << 20) || (bytes & (bytes - 1))))
        return fail(FG_ERR_INVALID_ARG, "fg_probe_read: the L2-resident pattern needs a power-of-two size of 32 KiB to 64 MiB");
    if (nontemporal == 2 && (bytes < 4096 || (bytes & (bytes - 1)))) return fail(FG_ERR_INVALID_ARG, "fg_probe_read: the paged pattern needs a power-of-two size");
    return launch_probe_read(src, bytes, nontemporal, blocks, sink, (hipStream_t)stream);
}

int32_t fg_probe_copy(const void *src, void *dst, int64_t bytes, int32_t blocks, void *stream)
{
    if (!src || !dst || bytes < 16 || bytes % 16 || blocks < 1) return fail(FG_ERR_INVALID_ARG, "fg_probe_copy: bad argument");
    return launch_probe_copy(src, dst, bytes, blocks, (hipStream_t)stream);
}

int32_t fg_probe_mfma(int32_t dtype, int32_t iters, int32_t random_operands, int32_t blocks, void *sink, void *stream)
{
    if (!is16(dtype) || !sink || iters < 1 || blocks < 1) return fail(FG_ERR_INVALID_ARG, "fg_probe_mfma: bad argument");
    return launch_probe_mfma(dtype, iters, random_operands, blocks, sink, (hipStream_t)stream);
}

int64_t fg_attention_workspace_bytes(int32_t B, int32_t N, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     int32_t max_seq_len)
{
    if (B < 1 || N < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads) return 0;
    return 2 * align_up((int64_t)B * N * 4, 256) + align_up((int64_t)B * N * 8, 256) +
           attention_mfma_ws_bytes(B, N, n_q_heads, n_kv_heads, head_dim, max_seq_len) + 1024;
}

int32_t fg_attention(const fg_kv_cache *kv, int32_t layer, const fg_tree *tree, int32_t n_q_heads, const void *q, void *out,
                     void *workspace, int64_t workspace_bytes, void *stream)
{
    int32_t rc;
    if ((rc = check_cache(nullptr, kv))) return rc;
    if ((rc = check_tree(tree, false))) return rc;
    if (!tree->slot) return fail(FG_ERR_INVALID_ARG, "fg_attention: slot is NULL");
    if (tree->B == 0 || tree->N == 0) return FG_OK;
    if (!q || !out || !workspace) return fail(FG_ERR_INVALID_ARG, "fg_attention: NULL pointer");
    if (layer < 0 || layer >= kv->n_layers || n_q_heads < 1 || n_q_heads % kv->n_kv_heads)
        return fail(FG_ERR_INVALID_ARG, "fg_attention: bad layer or head count");
    const int mk = max_keys_of(kv, tree, &rc);
    if (rc) return rc;
    const int M = tree->B * tree->N;
    Carver cv(workspace, workspace_bytes);
    TreeDev td;
    td.pos = cv.take<int32_t>(M);
    td.mask = cv.take<uint64_t>(M);
    td.dest = cv.take<int32_t>(M);
    int64_t ab = attention_mfma_ws_bytes(tree->B, tree->N, n_q_heads, kv->n_kv_heads, kv->head_dim, mk);
    void *aws = cv.take<char>(ab);
    if (!cv.ok) return fail(FG_ERR_CAPACITY, "fg_attention: workspace too small");
    hipStream_t st = (hipStream_t)stream;
    if ((rc = launch_tree_prep_ex(tree, kv, td, 0, st))) return rc;
    return attention_any(kv, layer, tree, td, n_q_heads, q, out, mk, aws, ab, 0, st);
}

}  // extern "C"
