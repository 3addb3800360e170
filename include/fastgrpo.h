/*
 * fastgrpo.h -- C ABI of the MI355X speculative-verify library (libfastgrpo.so).
 *
 * The hot path of FastGRPO's generation phase (Alg. 1, the concurrency-aware speculative decoding block of
 * the generation loop): plan the tree shape from the live concurrency (Sec. 4.1 Eq. 1-3), expand and rerank
 * the draft tree (Alg. 1 drafting loop and reranking; Sec. 2 "Draft Model Architectures", "Verification
 * Strategies"), verify all nodes in one target forward with tree attention, accept the longest matching
 * path, and keep its K/V.
 *
 * Conventions
 *  - Every function returns int32_t: FG_OK (0) or a negative fg_status.  fg_last_error() gives the message
 *    of the calling thread's last failure.  Nothing throws or aborts.
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers are read before return.
 *  - All device work is enqueued on the caller's stream (a hipStream_t passed as void*); calls are
 *    asynchronous and outputs are valid once the caller has synchronised that stream.  The library never
 *    allocates or frees device memory after fg_model_create (which allocates one RoPE table).
 *  - dtype FG_F32: every tensor fp32.  dtype FG_BF16 / FG_F16: weights, activations and KV are bf16 / fp16,
 *    accumulation, the residual stream, softmax and norm statistics are fp32.  The two 16-bit modes run the
 *    same kernels at the same MFMA rate and move the same bytes; fp16 keeps 3 more mantissa bits per
 *    activation rounding (bf16-valued weights and KV are exactly representable in fp16 down to 6e-5).
 *  - A sequence's cache holds the K/V of all its tokens but the last emitted one, which is the root
 *    (node 0) of the next step's tree.  In-round node i of a sequence of committed length L lives in cache
 *    slot L + i at position L + depth(i), and attends to positions 0..L-1 and to its in-round ancestors
 *    and itself.
 */
#ifndef FASTGRPO_H
#define FASTGRPO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FG_OK = 0,
    FG_ERR_INVALID_ARG = -1,   /* NULL required pointer, negative size, unknown mode or dtype          */
    FG_ERR_SHAPE = -2,         /* a dimension the kernels do not support (see each function)           */
    FG_ERR_CAPACITY = -3,      /* N > FG_MAX_NODES, workspace too small, page table too short          */
    FG_ERR_HIP = -4,           /* a HIP runtime call failed                                            */
    FG_ERR_UNIMPLEMENTED = -5
} fg_status;

enum { FG_F32 = 0, FG_BF16 = 1, FG_F16 = 2 };
enum { FG_MAX_NODES = 64 };                 /* in-round nodes per sequence (ancestor sets are 64-bit masks) */
enum { FG_ACCEPT_GREEDY = 0, FG_ACCEPT_SAMPLE_MATCH = 1, FG_ACCEPT_REJECT = 2 };

typedef struct fg_model fg_model;           /* opaque */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;                          /* FG_F32, FG_BF16 or FG_F16                                    */
    int32_t max_pos;                        /* positions 0..max_pos-1 get a RoPE table entry                */
    float rms_eps, rope_theta;
} fg_model_cfg;

/*
 * Weights: device pointers the caller owns and keeps alive while the model exists.  Every matrix is the
 * output of fg_pack_weight (its logical shape is [out, in]).  embed, the norm gains: plain row-major in the
 * model's dtype.  The per-layer members are HOST arrays of n_layers device pointers (copied at create).
 * A draft head (Sec. 2, "Draft Model Architectures": one decoder layer that reads the target's feature and
 * is decoded by the target's LM head) has fc ([d, 2d], input = token embedding ++ feature), n_layers = 1,
 * final_norm = NULL, and embed / lm_head pointing at the target's.
 */
typedef struct {
    const void *embed;              /* [vocab, d] row-major                                                */
    const void *lm_head;            /* packed [vocab, d]                                                   */
    const void *final_norm;         /* [d] or NULL (draft head)                                            */
    const void *fc;                 /* packed [d, 2d] or NULL (target)                                     */
    const void *const *wqkv;        /* packed [(Hq + 2 Hkv) * hd, d]: q rows, then k rows, then v rows     */
    const void *const *wo;          /* packed [d, Hq * hd]                                                 */
    const void *const *w_gate_up;   /* packed, gate and up interleaved (fg_pack_weight with src2)          */
    const void *const *w_down;      /* packed [d, F]                                                       */
    const void *const *norm_attn;   /* [d]                                                                 */
    const void *const *norm_ffn;    /* [d]                                                                 */
} fg_weights;

/*
 * Paged KV cache, caller-owned.  Page p of layer l, kv head h starts at element
 * ((l * n_pages + p) * n_kv_heads + h) * page_size * head_dim of either pool; within it, token t, dim e is at
 *   v_pool: e * page_size + t                                                     (transposed)
 *   k_pool: t * head_dim + e                                                      (token-major: FG_F32, or
 *                                                                                  head_dim % 32 != 0)
 *   k_pool: (((r / 8) * 4 + g) * 16 + t) * 8 + r % 8, g = e / (head_dim / 4),     (16-bit, head_dim % 32 == 0:
 *           r = e % (head_dim / 4)                                                 MFMA operand order, so that the
 *                                                                                  attention kernel reads 1 KiB
 *                                                                                  runs)
 * The library fills the cache itself (fg_spec_verify / fg_draft_step append, fg_kv_compact moves); a caller only
 * needs the formulas to plant or inspect contents.
 * Token t of a sequence in cache slot s is entry t % page_size of page page_table[s][t / page_size].
 * page_size must be 16.  seq_len[s] is the committed length; only fg_kv_compact (and fg_draft_step's n_commit) change it.
 *
 * Capacity.  Lengths live on the device, so the host cannot know that a call runs past a sequence's page table
 * (max_pages_per_seq * page_size tokens) or past the RoPE table (max_pos); the kernels then do no harm and say so in
 * `status` (device int32, zeroed by the caller, optional): a new node whose slot lies beyond the page table is not
 * appended (FG_CACHE_OVERFLOW; its logits are still computed, without itself among its keys), a commit or compaction
 * that would run past the page table is not applied and the length stays (FG_CACHE_OVERFLOW), a position beyond max_pos
 * is rotated as max_pos - 1 (FG_POS_OVERFLOW).  Committed tokens are never overwritten.  A caller that knows its
 * lengths on the host should check before the call; the flags are the backstop.
 */
typedef enum { FG_CACHE_OVERFLOW = 1, FG_POS_OVERFLOW = 2 } fg_cache_flags;
typedef struct {
    void *k_pool, *v_pool;          /* device                                                               */
    const int32_t *page_table;      /* device [n_slots][max_pages_per_seq]                                  */
    int32_t *seq_len;               /* device [n_slots]                                                     */
    int32_t *status;                /* device [1] or NULL: sticky fg_cache_flags the kernels OR in          */
    int32_t n_layers, n_kv_heads, head_dim, dtype;
    int32_t page_size, max_pages_per_seq, n_pages, n_slots;
} fg_kv_cache;

/*
 * The nodes one call works on.  B sequences, N new in-round nodes each, after n_prev nodes that earlier
 * calls of the same round already appended (0 for the target's verify step).
 *   parent[b][i], i < n_prev + N: in-round index of node i's parent, -1 for a child of the committed prefix
 *   (the root); parent[b][i] < i.  n_prev + N <= FG_MAX_NODES.
 * max_seq_len: a host-side upper bound on seq_len[slot[b]] + n_prev + N over the batch, used to size the
 * attention grid (0 = the cache's capacity).  A bound that is too small is FG_ERR_CAPACITY only if it
 * exceeds the capacity; sequences longer than the bound are not detected (their tail would be ignored).
 */
typedef struct {
    const int32_t *slot;            /* device [B]: cache slot of each sequence                              */
    const int32_t *tokens;          /* device [B, N]                                                        */
    const int32_t *parent;          /* device [B, n_prev + N]                                               */
    int32_t B, N, n_prev, max_seq_len;
} fg_tree;

const char *fg_last_error(void);

/*
 * The concurrency rule (Sec. 4.1 Eq. 1-3).  Host only.  N = floor(C_peak / B_cur) clamped to [1, N_cap];
 * K = min(N - 1, K_max); L = min(floor(log2(N / alpha)), L_max) clamped to [0, N - 1]; K = 0 or L = 0 gives
 * plain decoding (N = 1, K = L = 0); N is capped by the candidate count 1 + K + (L - 1) K^2.
 * Errors: B_cur < 1, C_peak <= 0, alpha <= 0, negative caps, N_cap < 1 or > FG_MAX_NODES -> FG_ERR_INVALID_ARG.
 */
int32_t fg_plan(int32_t B_cur, float C_peak, float alpha, int32_t K_max, int32_t L_max, int32_t N_cap,
                int32_t *N_verify, int32_t *K_draft, int32_t *L_draft);

/*
 * Knee of a latency curve (appendix, "Empirical Measurement of C_peak": forward latency against batch size is
 * flat while the pass is bound by weight traffic and rises once it is bound by compute; C_peak is the batch size
 * at the knee).  Host only.  x[n] strictly increasing batch sizes, y[n] latencies (host pointers).  log2_axis != 0
 * takes the abscissa as log2(x) (batch sizes sampled geometrically), 0 as x itself (the appendix plots latency against
 * the batch size).  Both axes are scaled to [0, 1]; *knee_index is the sample farthest below the chord through the
 * first and last sample (the first such sample on ties; 0 when the curve never dips below the chord).
 * Errors: NULL pointers, n < 3, x not strictly increasing (or not positive with log2_axis) -> FG_ERR_INVALID_ARG.
 */
int32_t fg_knee(const double *x, const double *y, int32_t n, int32_t log2_axis, int32_t *knee_index);

/*
 * Row selection for the live set (Alg. 1, the update of the live batch size: finished sequences leave the batch):
 * dst[i] = src[index[i]] for i < n, rows of row_bytes bytes (a multiple of 4), all device pointers; index values
 * are clamped into [0, n_src - 1].  dst must not overlap src.
 */
int32_t fg_select_rows(const void *src, int64_t row_bytes, int32_t n_src, const int32_t *index, int32_t n, void *dst,
                       void *stream);

/*
 * Weight packing (one-time, on the stream).  src is [n_out, n_in] row-major in `dtype`; with src2 != NULL
 * the logical matrix is [2 n_out, n_in] with rows interleaved in blocks of 32 (32 of src, 32 of src2, ...),
 * which is how gate and up are fused.  FG_F32: dst is that logical matrix row-major.  16-bit dtypes: dst holds it
 * as MFMA operand fragments: tile (n / 32, k / 16) is 1 KiB, lane ((k % 16) / 8) * 32 + n % 32 holds 8
 * consecutive k; the tiles of one 32-row band are contiguous in k.  Needs n_out % 32 == 0 and
 * n_in % 64 == 0 (FG_ERR_SHAPE).  dst has fg_packed_bytes(...) bytes and must not alias src.
 */
int64_t fg_packed_bytes(int32_t dtype, int64_t n_out_total, int64_t n_in);
int32_t fg_pack_weight(int32_t dtype, const void *src, const void *src2, void *dst, int64_t n_out, int64_t n_in,
                       void *stream);

/* Creates the model descriptor (copies cfg and the pointer tables; allocates the RoPE table on the current
 * device).  Shape limits: head_dim 64 or 128, n_q_heads % n_kv_heads == 0, d_model / d_ffn / vocab multiples
 * of 32, inner dimensions multiples of 64, (n_q_heads / n_kv_heads) <= 8.  fg_model_destroy frees the table. */
int32_t fg_model_create(const fg_model_cfg *cfg, const fg_weights *w, fg_model **out);
int32_t fg_model_destroy(fg_model *m);

/* Bytes of caller-provided device workspace that suffice for every fg_spec_verify / fg_draft_step call on this model
 * with B * N <= max_rows rows (any B, any N <= FG_MAX_NODES, logits kept in the workspace) and caches of at most
 * max_seq_len tokens.  256-byte aligned base expected.  Host only.  fg_workspace_bytes_for is the same from a
 * configuration (is_draft: the model has an fc matrix); fg_step_workspace_bytes is what one call of a given shape
 * carves (with_logits: logits == NULL while row_argmax / row_top2 / child lists are asked for).  0 on bad arguments. */
int64_t fg_workspace_bytes(const fg_model *m, int32_t max_rows, int32_t max_seq_len);
int64_t fg_workspace_bytes_for(const fg_model_cfg *cfg, int32_t is_draft, int32_t max_rows, int32_t max_seq_len);
int64_t fg_step_workspace_bytes(const fg_model_cfg *cfg, int32_t is_draft, int32_t B, int32_t N, int32_t max_seq_len,
                                int32_t with_logits);

/*
 * Verification (Alg. 1, the verification step; Sec. 2 "Verification Strategies"): one target forward over the B * N new
 * nodes with tree attention against the paged cache.  Appends K/V of every node at slots seq_len + n_prev + j
 * (lengths are NOT changed; fg_kv_compact commits).  Outputs, each optional (NULL to skip), row r = b * N + j:
 *   logits      fp32 [B*N, vocab]
 *   feature     model dtype [B*N, d]: the final-norm output, i.e. the LM head's input
 *   row_argmax  int32 [B*N]: argmax of each logits row, lowest index on ties
 *   row_top2    fp32 [B*N, 2]: the largest and second-largest logit of the row
 * Errors: NULL model / cache / tree members, B or N < 0, n_prev + N > FG_MAX_NODES, dtype mismatch between
 * model and cache, workspace too small, max_seq_len beyond the cache's capacity.  B == 0 or N == 0 is FG_OK
 * and does nothing.  Tokens and parents are not validated on the device beyond clamping into range.
 */
int32_t fg_spec_verify(fg_model *m, fg_kv_cache *kv, const fg_tree *tree, float *logits, void *feature,
                       int32_t *row_argmax, float *row_top2, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Acceptance (Alg. 1, the step after verification; Sec. 2 "Verification Strategies": the longest root path whose
 * draft tokens each equal the token the target itself emits at the parent survives).  Per sequence, from the root: the
 * target's token t
 * after the current node u is
 *   FG_ACCEPT_GREEDY        row_argmax[u] if given, else the argmax of logits[u];
 *   FG_ACCEPT_SAMPLE_MATCH  argmax_v logits[u][v] / temperature + Gumbel(seed, row0 + row of u, v);
 * move to the lowest-indexed child of u whose token equals t, stop when there is none.
 *   FG_ACCEPT_REJECT        rejection sampling over the sibling set: for each child c of u in index order with
 *   token x, accept when uniforms[c] < min(1, p(x) / q(x)), p = softmax(logits[u] / temperature),
 *   q = draft_probs[u]; on rejection p <- normalise(max(p - q, 0)), q(x) <- 0, q <- normalise(q); with no child
 *   accepted the bonus token is the Gumbel-max draw from the current p.
 * Outputs (device): accept_len [B] = a, the number of accepted drafts; path [B, N] node indices path[0..a]
 * (path[0] = 0, rest -1); out_tokens [B, N]: out_tokens[0..a] = the emitted tokens (accepted drafts then the
 * bonus token; rest -1); finished [B] = 1 when an emitted token equals eos_id, in which case the walk is cut
 * at that token.  The uniform/Gumbel generator is SplitMix64-based: u = ((mix(mix(seed ^ row * 0xD1B54A32D192ED03)
 * + v) >> 41) + 0.5) / 2^23.  workspace: FG_ACCEPT_REJECT needs 2 * B * vocab floats, other modes none.
 * Errors: missing inputs for the mode, temperature <= 0 in modes 1-2, N > FG_MAX_NODES.
 */
int32_t fg_spec_accept(const fg_tree *tree, int32_t mode, const float *logits, const int32_t *row_argmax,
                       int32_t vocab, float temperature, const float *draft_probs, const float *uniforms,
                       uint64_t seed, int64_t row0, int32_t eos_id, int32_t *accept_len, int32_t *path,
                       int32_t *out_tokens, int32_t *finished, void *workspace, int64_t workspace_bytes,
                       void *stream);

/*
 * fg_spec_accept for callers that cannot allocate device memory or hand over a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and errors as
 * fg_spec_accept minus the workspace: the per-row target tokens (greedy from logits, sample match) or the p / q
 * vectors (rejection mode) live in a static device array of FG_STATIC_SCRATCH_BYTES that each GPU holds from the
 * first use of the library until the process ends.  Calls that need more (B * N * 4 bytes, or B * 2 * vocab * 4 in
 * rejection mode) fail with FG_ERR_CAPACITY.  It calls no allocator.  The array's device address is looked up once
 * per device (at fg_model_create, else at the first call on that device; do that first call outside a capture).
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different streams or threads) race;
 * calls on one stream are ordered and every call rewrites what it reads, so nothing needs clearing between calls.
 */
enum { FG_STATIC_SCRATCH_BYTES = 4 << 20 };
int32_t fg_spec_accept_static(const fg_tree *tree, int32_t mode, const float *logits, const int32_t *row_argmax,
                              int32_t vocab, float temperature, const float *draft_probs, const float *uniforms,
                              uint64_t seed, int64_t row0, int32_t eos_id, int32_t *accept_len, int32_t *path,
                              int32_t *out_tokens, int32_t *finished, void *stream);

/*
 * KV compaction in place (implied by Alg. 1, the update of the generated sequences: rejected nodes are dropped).  For sequence b
 * with committed length L: in-round slot L + path[b][j] moves to L + j for j = 0..accept_len[b], K and V of
 * every layer and head; then seq_len += accept_len[b] + 1.  path rows must increase strictly with
 * path[j] >= j (what fg_spec_accept emits); rows that do not are left untouched and their length unchanged.
 * N is the row stride of path.  If feature_in / feature_out are given, feature_out[b][j] = feature_in[b][path[j]]
 * for j <= accept_len[b] ([B, N, d] both; rows beyond are zero-filled) -- the accepted hidden states the draft
 * head reads next.  d_model and feat_dtype describe those rows.
 */
int32_t fg_kv_compact(fg_kv_cache *kv, const int32_t *slot, const int32_t *accept_len, const int32_t *path,
                      int32_t B, int32_t N, const void *feature_in, void *feature_out, int32_t d_model,
                      int32_t feat_dtype, void *stream);

/*
 * One drafting step (Alg. 1, the drafting loop's child generation; Sec. 2 "Draft Model Architectures"): the
 * draft head runs on B * tree->N new in-round nodes.  Node input = fc(embed(token) ++ feature row); one decoder
 * layer against the draft's own paged cache with tree attention; the output hidden state is decoded by the
 * target's LM head; per node the K_draft most likely tokens and their log-probabilities come back.
 *   in_feature   model dtype [B, feat_rows, d]; node (b, j) is paired with row feat_index[b][j] of sequence b
 *                (feat_index device int32 [B, N], NULL = row j, which needs feat_rows >= N)
 *   child_tok    int32 [B, N, K_draft]; child_logp fp32 [B, N, K_draft] (log-softmax, descending, ties by
 *                index); both NULL skips the LM head
 *   expand_row   device int32 [B] or NULL: when given, only node expand_row[b] of each sequence is decoded by the
 *                LM head (the root of a catch-up chain; the rows before it are history), and child_tok /
 *                child_logp are [B, 1, K_draft]
 *   out_feature  model dtype [B, N, d]: the head's output hidden state of each node (NULL to skip)
 * n_commit (device [B] or NULL): after the step seq_len[slot[b]] += n_commit[b] + commit_bias -- used for the
 * catch-up chain of accepted tokens, which stays in the draft cache (pass the verify step's accept_len with bias
 * 1); NULL leaves lengths alone.  Rows of a catch-up chain beyond the committed count are padding: they are
 * computed and written past the committed length, where the next nodes overwrite them.
 */
int32_t fg_draft_step(fg_model *target, fg_model *draft, fg_kv_cache *draft_kv, const fg_tree *tree,
                      const void *in_feature, const int32_t *feat_index, int32_t feat_rows, const int32_t *n_commit,
                      int32_t commit_bias, int32_t K_draft, const int32_t *expand_row, int32_t *child_tok,
                      float *child_logp, void *out_feature, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Frontier update between drafting steps (Alg. 1, the drafting loop's update of the candidate set).  The K_in expanded nodes
 * of this step have candidate indices node_cand [B, K_in] and scores node_score [B, K_in]; their K_in * K
 * children (child_tok / child_logp from fg_draft_step) are appended to the candidate lists at index n_cand
 * (cand_* are [B, cand_stride]) with score = parent score + log-probability, and the K best children (ties:
 * lower index) become the next frontier: next_tok / next_cand / next_score / next_src [B, K], next_src being
 * the position (0..K_in-1) of the frontier node's parent among this step's nodes.
 * node_pick (device [B] or NULL): only node node_pick[b] is expanded (its K children are appended); this is the
 * first step, where the last valid row of the catch-up chain is the root and the rows before it are history.
 * With node_pick, NULL node_cand / node_score mean candidate 0 (the root) and score 0, and node_tok [B, K_in]
 * (the step's node tokens), if given, initialises candidate 0 = (token of the picked node, parent -1, score 0).
 * parent_next (optional, device [B, n_parent_prev + K]): the in-round parent list for the next drafting step =
 * parent_prev [B, n_parent_prev] (the round's nodes so far, this step's K_in nodes last) followed by the K new
 * frontier nodes' parents (-1 with node_pick: children of the root attend the committed prefix only).
 * child_rows: rows per sequence in child_tok / child_logp: K_in, or 1 with node_pick when fg_draft_step decoded the
 * picked row only (expand_row).
 */
int32_t fg_draft_frontier(int32_t B, int32_t K_in, int32_t K, const int32_t *child_tok, const float *child_logp,
                          int32_t child_rows, const int32_t *node_cand, const float *node_score, const int32_t *node_pick,
                          const int32_t *node_tok, int32_t n_cand, int32_t cand_stride, int32_t *cand_tok,
                          int32_t *cand_parent, float *cand_score, int32_t *next_tok, int32_t *next_cand,
                          float *next_score, int32_t *next_src, const int32_t *parent_prev, int32_t n_parent_prev,
                          int32_t *parent_next, void *stream);

/*
 * Rerank (Alg. 1, the selection of the N_verify most confident candidates).  Candidate 0 is the root;
 * cand_parent[i] < i.  Selects the root and the N - 1 best-scoring other candidates (ties: lower index), orders
 * them by (depth, candidate index) and writes tokens [B, N], parent [B, N] (parent[0] = -1, parent[i] < i) and
 * sel [B, N] (candidate index of each node; optional).  Scores must not increase from parent to child; a
 * selected node whose parent was not selected is re-attached to the root.  n_cand <= 128, N <= FG_MAX_NODES.
 */
int32_t fg_build_tree(const int32_t *cand_tok, const int32_t *cand_parent, const float *cand_score, int32_t B,
                      int32_t n_cand, int32_t cand_stride, int32_t N, int32_t *tokens, int32_t *parent,
                      int32_t *sel, void *stream);

/*
 * Online draft learning (Sec. 4.2 "Draft Model Learning with Online Target Feedback"; Alg. 1, the draft training phase):
 * the draft head is trained on what the generation phase cached -- the tokens the target emitted and the target's
 * features.  Parameters, gradients, activations and the optimiser state are fp32, whatever type the generation path
 * runs in; the updated head reaches it by casting and re-packing the matrices (fg_pack_weight) into a new draft model.
 * cfg->dtype chooses how the step's matrix products are computed: FG_F32 exactly, in an fp32 GEMM (the parity mode);
 * FG_BF16 on the matrix cores, both operands rounded to bf16 and accumulated in fp32 (6.4 times faster on the 7B-class
 * head; gradients within a few per cent of the exact ones; B * T, d, F, Hq hd, (Hq + 2 Hkv) hd and vocab multiples of 64,
 * FG_ERR_SHAPE otherwise); FG_F16 is refused: backward values underflow fp16.
 *
 * fg_draft_params: the head's parameters, row-major [out, in] fp32 device arrays the caller owns: fc [d, 2d],
 * wqkv [(Hq + 2 Hkv) hd, d] (q rows, k rows, v rows), wo [d, Hq hd], w_gate / w_up [F, d], w_down [d, F], the two norm
 * gains [d].  The same struct describes gradients and the optimiser's two moment sets.
 *
 * fg_draft_train_grad: B sequences, each one teacher-forced chain of T entries from an empty draft cache (causal
 * attention inside the chain, positions 0 .. T-1); entry t pairs tokens[b][t] (token t + 1) with feat_in[b][t] (the
 * target's feature t) and is trained towards feat_tgt[b][t] (the target's feature t + 1); entries t >= n_valid[b] are
 * padding.  With h the head's output, per valid entry
 *   L = mean_e smooth_l1(h[e] - feat_tgt[e]) + w_ce * CE(softmax(lm_head . feat_tgt), softmax(lm_head . h)),
 * averaged over the valid entries (the paper names no loss: this is the one of the draft-head pre-training it follows,
 * Sec. 5.1).  Outputs: loss (device, 2 floats: the regression and the cross-entropy term, unweighted) and the gradient
 * of the total in `grad`.  embed, lm_head: the target's, fp32 row-major [vocab, d], frozen.  tokens int32 [B, T],
 * feat_in / feat_tgt fp32 [B, T, d], n_valid int32 [B], all device.  cfg: the draft head's (n_layers must be 1).  d, F, Hq hd, vocab multiples of 4; T * 4 bytes of LDS per block (T <= 8192).
 * workspace: fg_draft_train_workspace_bytes(cfg, B, T).  Deterministic: no atomics, fixed summation orders.
 * head_packed (optional, NULL allowed; used in the FG_BF16 mode only): the frozen lm_head already rounded to bf16 and
 * packed for the step's two kinds of product with it, written once by fg_draft_train_pack_head into a device buffer of
 * fg_draft_train_head_bytes(cfg) bytes that the caller keeps for as long as lm_head does not change (vocab and d
 * multiples of 64); without it every step packs the head again (1.3 of 16 ms on the 7B-class head).  The results are
 * bitwise the same either way.
 *
 * fg_draft_adamw: one AdamW step on every parameter (decoupled weight decay, bias-corrected moments; step counts
 * from 1): m = b1 m + (1 - b1) g; v = b2 v + (1 - b2) g^2; p -= lr (m / (1 - b1^step) / (sqrt(v / (1 - b2^step)) + eps)
 * + weight_decay p).
 */
typedef struct {
    float *fc, *wqkv, *wo, *w_gate, *w_up, *w_down, *norm_attn, *norm_ffn;
} fg_draft_params;
int64_t fg_draft_train_workspace_bytes(const fg_model_cfg *cfg, int32_t B, int32_t T);
int32_t fg_draft_train_grad(const fg_model_cfg *cfg, const float *embed, const float *lm_head, const fg_draft_params *w,
                            const int32_t *tokens, const float *feat_in, const float *feat_tgt, const int32_t *n_valid,
                            int32_t B, int32_t T, float w_ce, fg_draft_params *grad, float *loss, const void *head_packed,
                            void *workspace, int64_t workspace_bytes, void *stream);
int64_t fg_draft_train_head_bytes(const fg_model_cfg *cfg);
int32_t fg_draft_train_pack_head(const fg_model_cfg *cfg, const float *lm_head, void *packed, int64_t packed_bytes, void *stream);
int32_t fg_draft_adamw(const fg_model_cfg *cfg, fg_draft_params *w, const fg_draft_params *grad, fg_draft_params *m,
                       fg_draft_params *v, float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step,
                       void *stream);

/*
 * Kernel-level entry points (unit parity and per-kernel measurement).
 * fg_gemm: out = x . W^T for packed W [n_out, n_in]; x is [M, n_in] row-major in dtype.
 *   epilogue 0: out fp32 [split_k][M][n_out] partial sums (split_k >= 1; 0 lets the library choose and
 *               returns the value through *split_k_used); the caller adds the slabs.
 *   epilogue 1: W is a gate/up interleaved matrix; out[M, n_out / 2] in dtype = silu(gate) * up.
 *   epilogue 3: out fp32 [M, n_out] += x . W^T in place (the residual add of the O and down projections; 16-bit
 *               dtypes, pipelined kernel only).
 *   variant: 0 = the kernel the library picks for the shape; 1 = weight-streaming kernel, 2 = few-row kernel (at most
 *               512 rows), 3 / 4 / 5 = pipelined kernel with 256- / 128- / 160-row blocks, 6 = decode kernel (at most 16
 *               rows, epilogues 0 and 1), 7 / 8 / 9 = pipelined kernel with 128- / 160- / 256-row blocks of 192 columns instead of
 *               256, 10 = 128-row blocks of 128 columns (epilogues 0 and 1; variant 0 runs the narrowest of these that
 *               gives at most 256 blocks for one row block of a wide output), 11 / 12 = 192-row blocks of 256 / 192
 *               columns, 13 / 14 = 224-row blocks of 256 / 192 columns (epilogues 0 and 1).  16-bit dtypes only.
 * fg_gemm_kernel_name: the kernel the library picks for a 16-bit GEMM of this shape and epilogue (a static string).
 * fg_attention: tree attention of already-rotated queries q [B*N, Hq*hd] (dtype) over the cache, which must
 *   already hold the in-round nodes' K/V; out [B*N, Hq*hd] (dtype).
 * fg_topk_logp: the draft's per-node expansion (Sec. 2, draft tree construction): for each of the M rows of
 *   logits [M, vocab] (fp32, device) the K largest entries, ties to the lower token id, as tok [M, K] (int32)
 *   and their log-softmax values logp [M, K] (fp32).  1 <= K <= 8, K <= vocab.
 * fg_lm_head_topk: the same lists straight from the hidden states x [M, d_model] (dtype) and the packed LM head
 *   [vocab, d_model], the selection done in the GEMM's epilogue, so that no [M, vocab] tensor is written: per row and
 *   256-token block the K best (value, token) and (max, sum exp), then a merge.  What fg_spec_verify (K = 2, for the row
 *   arg-max and top-2) and fg_draft_step do when no logits are asked for; from 129 rows and 16384 tokens on,
 *   and from 65 rows for vocabularies of at least 128 blocks of 256 tokens (FG_ERR_SHAPE below).  workspace: fg_lm_head_topk_workspace_bytes(M, vocab, K) bytes, device.
 */
int32_t fg_gemm(int32_t dtype, const void *x, const void *w_packed, void *out, int32_t M, int32_t n_out,
                int32_t n_in, int32_t epilogue, int32_t split_k, int32_t *split_k_used, int32_t variant, void *stream);
const char *fg_gemm_kernel_name(int32_t M, int32_t n_out, int32_t n_in, int32_t epilogue);
int32_t fg_attention(const fg_kv_cache *kv, int32_t layer, const fg_tree *tree, int32_t n_q_heads, const void *q,
                     void *out, void *workspace, int64_t workspace_bytes, void *stream);
int64_t fg_attention_workspace_bytes(int32_t B, int32_t N, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                     int32_t max_seq_len);
int32_t fg_topk_logp(const float *logits, int32_t M, int32_t vocab, int32_t K, int32_t *tok, float *logp, void *stream);
int64_t fg_lm_head_topk_workspace_bytes(int32_t M, int32_t vocab, int32_t K);
int32_t fg_lm_head_topk(int32_t dtype, const void *x, const void *lm_head_packed, int32_t M, int32_t vocab, int32_t d_model,
                        int32_t K, int32_t *tok, float *logp, void *workspace, int64_t workspace_bytes, void *stream);

/*
 * Stage timing of one model (measurement only, off by default).  While enabled, the entry points that run this model
 * (fg_spec_verify for a target, fg_draft_step for a draft head) record a HIP event on their stream before every group
 * of launches and one at their end, at most max_marks in all; the time between two consecutive events is charged to
 * the stage the first announces, so the stages of a call add up to the call.  fg_model_profile_read waits for the last
 * event, fills ms[FG_STAGE_COUNT] and launches[FG_STAGE_COUNT] (host arrays) and starts a new collection.  A model is
 * driven from one thread (one stream) at a time, and so is its timing.  Not to be enabled under graph capture.
 * enable: 0 off; 1 every stage; 2 + s only stage s (one event before its launches and one after: the cheapest way to time
 * one kernel inside a timed region -- an event costs a microsecond or two of the stream's time).
 */
enum { FG_STAGE_END = -1, FG_STAGE_PREP = 0, FG_STAGE_NORM, FG_STAGE_QKV, FG_STAGE_ROPE, FG_STAGE_ATTENTION, FG_STAGE_O,
       FG_STAGE_GATE_UP, FG_STAGE_SWIGLU, FG_STAGE_DOWN, FG_STAGE_LM_HEAD, FG_STAGE_SELECT, FG_STAGE_FC, FG_STAGE_COUNT };
int32_t fg_model_profile(fg_model *m, int32_t enable, int32_t max_marks);
int32_t fg_model_profile_read(fg_model *m, double *ms, int32_t *launches);

/*
 * Ceiling probes (measurement only): what the GPU sustains for the two resources the path is bound by.
 * fg_probe_read: `blocks` blocks of 256 threads stream `bytes` (a multiple of 16) from src with 16-byte loads, four in
 *   flight per lane; nontemporal 0: ordinary loads, 1: non-temporal loads, 2: non-temporal loads of 4 KiB pages visited
 *   in a hashed order, one page per wave at a time (the pattern of a paged KV cache; bytes a power of two); 3: EVERY
 *   block streams the whole region 256 times (bytes a power of two from 32 KiB to 64 MiB: choose it to fit in L2 and
 *   not in a 32 KiB L1), eight loads in flight per lane -- blocks * 256 * bytes are read in all, as L2 -> L1 fills;
 *   4 / 5 / 6: every block streams its own contiguous slice (bytes / blocks, rounded down to whole rounds) with 8 / 16 /
 *   32 non-temporal loads per lane in flight -- with at most one block per CU, what a single CU draws from HBM;
 *   sink: device, blocks * 4 bytes (written only on a magic checksum).
 * fg_probe_copy: the same stream written to dst (the plain copy whose FETCH_SIZE / WRITE_SIZE counter readings scale
 *   the traffic figures of the other kernels).
 * fg_probe_mfma: blocks x 4 waves each issue iters * 16 v_mfma_f32_32x32x16 (dtype FG_BF16 or FG_F16) on operands that
 *   never leave registers: iters * 16 * 32768 flop per wave; random_operands != 0 rotates four hashed fragment pairs
 *   (operand buses toggle as on real data, which sets the power draw and so the sustained clock), 0 uses one constant
 *   pair; sink: device, blocks * 1024 bytes (practically never written).
 */
int32_t fg_probe_read(const void *src, int64_t bytes, int32_t nontemporal, int32_t blocks, void *sink, void *stream);
int32_t fg_probe_copy(const void *src, void *dst, int64_t bytes, int32_t blocks, void *stream);
int32_t fg_probe_mfma(int32_t dtype, int32_t iters, int32_t random_operands, int32_t blocks, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTGRPO_H */
