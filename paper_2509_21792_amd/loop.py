"""Host driver of one speculative round and of the generation loop (Alg. 1, the generation loop).

Host bookkeeping only: it strings the library's entry points together (plan -> draft steps -> frontier updates ->
rerank -> verify -> accept -> compact), keeps every intermediate on the device, and crosses to the host once
per round for the accepted tokens, as the method requires to update the live set.
"""
import numpy as np
import torch

from . import binding as fg


class SpecState:
    """Per-batch device state carried between rounds: the entries the draft head has not seen yet."""

    def __init__(self, catch_tok, catch_feat, n_valid_minus1):
        self.catch_tok = catch_tok          # int32 [B, Kin]  token t+1 of each pending entry (padding beyond n_valid)
        self.catch_feat = catch_feat        # dtype [B, Kin, d] the target's feature t paired with it
        self.last = n_valid_minus1          # int32 [B] index of the last valid entry (= the root's entry)


def chain_parent(B, n, device):
    return torch.arange(-1, n - 1, dtype=torch.int32, device=device).repeat(B, 1)


def draft_expand(target, draft, dkv, slot, st, K, L, ws, max_seq_len=0):
    """L drafting steps, K paths kept per step.  Returns the candidate lists (tok, parent, score) [B, 1+K+(L-1)K^2]."""
    B, Kin = st.catch_tok.shape
    dev = st.catch_tok.device
    n_total = 1 + K + (L - 1) * K * K
    cand_tok = torch.empty((B, n_total), dtype=torch.int32, device=dev)
    cand_parent = torch.empty((B, n_total), dtype=torch.int32, device=dev)
    cand_score = torch.empty((B, n_total), dtype=torch.float32, device=dev)
    # step 1: the catch-up chain; its last valid row is the root, whose K best children open the tree
    ctok, clogp, ofeat = fg.fg_draft_step(target, draft, dkv, slot, st.catch_tok, chain_parent(B, Kin, dev), st.catch_feat, ws,
                                          K, n_commit=st.last, commit_bias=1, max_seq_len=max_seq_len, expand_row=st.last)
    f_tok, f_cand, f_score, f_src, parents = fg.fg_draft_frontier(ctok, clogp, 1, cand_tok, cand_parent, cand_score,
                                                                 node_pick=st.last, node_tok=st.catch_tok)
    n_cand = 1 + K
    feat_base = ofeat                      # [B, rows, d]: hidden states of the previous step's nodes
    for step in range(2, L + 1):
        n_prev = (step - 2) * K
        ctok, clogp, ofeat = fg.fg_draft_step(target, draft, dkv, slot, f_tok, parents, feat_base, ws, K, n_prev=n_prev,
                                              feat_index=f_src, max_seq_len=max_seq_len)
        f_tok, f_cand, f_score, f_src, parents = fg.fg_draft_frontier(ctok, clogp, n_cand, cand_tok, cand_parent, cand_score,
                                                                     node_cand=f_cand, node_score=f_score,
                                                                     parent_prev=parents)
        feat_base = ofeat
        n_cand += K * K
    return cand_tok, cand_parent, cand_score


def spec_round(target, draft, kv, dkv, slot, st, N, K, L, ws_t, ws_d, eos_id=-1, max_seq_len=0, replant=None, decide=None):
    """One round on the live batch.  Returns (accept_len, out_tokens, finished) on the device and the next SpecState.
    replant(tokens, parent) -> tokens: a measurement hook for synthetic workloads, where no trained draft head
    exists and the agreement between draft and target is planted into the reranked tree at a controlled rate.
    decide(tokens, parent, row_argmax) -> row_argmax: the same purpose from the other side: the target's decisions
    are overridden (throughput experiments whose token values do not matter)."""
    ct, cp, cs = draft_expand(target, draft, dkv, slot, st, K, L, ws_d, max_seq_len=max_seq_len)
    tokens, parent, _ = fg.fg_build_tree(ct, cp, cs, ct.shape[1], N)
    if replant is not None:
        tokens = replant(tokens, parent)
    out = fg.fg_spec_verify(target, kv, slot, tokens, parent, ws_t, max_seq_len=max_seq_len)
    amax = out["argmax"] if decide is None else decide(tokens, parent, out["argmax"])
    acc, path, otok, fin = fg.fg_spec_accept(tokens, parent, row_argmax=amax, eos_id=eos_id)
    B = tokens.shape[0]
    d = target.cfg["d_model"]
    feat = fg.fg_kv_compact(kv, slot, acc, path, feature_in=out["feature"].view(B, N, d), d_model=d)
    Kin = L + 1
    nxt = SpecState(otok[:, :Kin].contiguous(), feat[:, :Kin].contiguous(), acc)
    return acc, otok, fin, nxt


def plain_round(target, draft, kv, dkv, slot, st, root, ws_t, ws_d, eos_id=-1, max_seq_len=0):
    """A round with N_verify = 1 (Eq. 1 when the live batch alone fills C_peak): plain decoding of the root.  The
    draft head still consumes its pending entries (no LM head) so that its cache stays in step with the target's."""
    B = root.shape[0]
    dev = root.device
    Kin = st.catch_tok.shape[1]
    fg.fg_draft_step(target, draft, dkv, slot, st.catch_tok, chain_parent(B, Kin, dev), st.catch_feat, ws_d, 1,
                     n_commit=st.last, commit_bias=1, max_seq_len=max_seq_len, want_children=False)
    tokens = root.view(B, 1)
    parent = torch.full((B, 1), -1, dtype=torch.int32, device=dev)
    out = fg.fg_spec_verify(target, kv, slot, tokens, parent, ws_t, max_seq_len=max_seq_len)
    acc, path, otok, fin = fg.fg_spec_accept(tokens, parent, row_argmax=out["argmax"], eos_id=eos_id)
    d = target.cfg["d_model"]
    feat = fg.fg_kv_compact(kv, slot, acc, path, feature_in=out["feature"].view(B, 1, d), d_model=d)
    return acc, otok, fin, SpecState(otok[:, :1].contiguous(), feat[:, :1].contiguous(), acc)


class RoundGraph:
    """One round of a fixed shape (B, N, K, L, pending entries per sequence) recorded once as a HIP graph and replayed:
    at a small live batch a round is some 350 short launches, and the host's launch rate, not the GPU, sets its
    pace.  The round's inputs live in buffers the graph owns; `run` copies the caller's state in and replays.  The
    outputs are graph-owned tensors that the next replay overwrites (the caller reads or copies them first -- the
    generation loop copies them into the next round's inputs).  Record only after the same calls have run eagerly
    once (code objects are loaded at a kernel's first launch, which a capture cannot do)."""

    replays = 0     # over all instances (tests and measurements read it)

    def __init__(self, target, draft, kv, dkv, B, N, K, L, kin, ws_t, ws_d, eos_id, max_seq_len):
        dev = kv.k_pool.device
        d = target.cfg["d_model"]
        self.slot = torch.zeros(B, dtype=torch.int32, device=dev)
        self.st = SpecState(torch.zeros((B, kin), dtype=torch.int32, device=dev),
                            torch.zeros((B, kin, d), dtype=kv.k_pool.dtype, device=dev),
                            torch.zeros(B, dtype=torch.int32, device=dev))
        self.root = torch.zeros(B, dtype=torch.int32, device=dev)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            if N == 1:
                self.out = plain_round(target, draft, kv, dkv, self.slot, self.st, self.root, ws_t, ws_d, eos_id, max_seq_len)
            else:
                self.out = spec_round(target, draft, kv, dkv, self.slot, self.st, N, K, L, ws_t, ws_d, eos_id, max_seq_len)

    def run(self, slot, st, root=None):
        self.slot.copy_(slot)
        self.st.catch_tok.copy_(st.catch_tok)
        self.st.catch_feat.copy_(st.catch_feat)
        self.st.last.copy_(st.last)
        if root is not None:
            self.root.copy_(root)
        self.graph.replay()
        RoundGraph.replays += 1
        return self.out


def generate(target, draft, kv, dkv, slot, st, first, budgets, c_peak, ws_t, ws_d, alpha=0.5, K_max=4, L_max=6, N_cap=64,
             eos_id=-1, max_seq_len=0, plan=None, max_rounds=10 ** 9, replant=None, decide=None, graphs=False):
    """The concurrency-aware generation loop (Alg. 1): every round (N, K, L) is re-planned from the number of live
    sequences (Eq. 1-3; `plan(B_cur) -> (N, K, L)` overrides the rule, e.g. a fixed shape for comparison), finished
    sequences leave the batch (device rows are re-selected with fg_select_rows), and the host sees only the accepted
    tokens of each round.

    slot int32 [B] (device), st: the draft head's pending entries after the prefill, first int32 [B] (host): the
    token already emitted per sequence, budgets [B] (host): tokens per sequence, first included.
    replant(tokens, parent, live, outs) -> tokens and decide(tokens, parent, row_argmax) -> row_argmax: see spec_round.
    graphs: replay each round shape as a HIP graph from its second use on (RoundGraph; not with the two hooks, which
    run host code inside the round; max_seq_len should then be a bound that holds for the whole rollout).
    Returns (token lists, per-round history of dicts B, N, K, L, emitted).
    """
    B = len(first)
    dev = slot.device
    outs = [[int(first[b])] for b in range(B)]
    # committed lengths at the start (one copy, before the loop): with the tokens emitted since, the host knows every
    # sequence's length and refuses a round that would run past a page table or the RoPE table
    len0 = kv.seq_len[slot.long()].cpu().numpy().astype(np.int64)
    dlen0 = dkv.seq_len[slot.long()].cpu().numpy().astype(np.int64)
    limit = min(kv.capacity, dkv.capacity, target.max_pos, draft.max_pos)
    keep = [b for b in range(B) if budgets[b] > 1]
    live = list(range(B))
    hist = []
    seen, recorded = {}, {}      # round shapes met so far, and their recorded graphs

    def reselect(rows):
        nonlocal slot, st
        idx = torch.as_tensor(np.asarray(rows, dtype=np.int32)).to(dev)
        slot = fg.fg_select_rows(slot, idx)
        st = SpecState(fg.fg_select_rows(st.catch_tok, idx), fg.fg_select_rows(st.catch_feat, idx), fg.fg_select_rows(st.last, idx))

    if len(keep) < B:
        reselect(keep)
        live = keep
    while live and len(hist) < max_rounds:
        Bc = len(live)
        N, K, L = plan(Bc) if plan else fg.fg_plan(Bc, c_peak, alpha, K_max, L_max, N_cap)
        # the round appends N nodes behind the committed tokens (the draft cache: its pending entries and K (L - 1) nodes)
        longest = max(max(len0[b], dlen0[b]) + len(outs[b]) - 1 for b in live)
        need = longest + max(N, st.catch_tok.shape[1] + K * max(L - 1, 0))
        if need > limit:
            raise fg.FgError(-3, f"round of N = {N} nodes needs {need} cache positions, the caches / RoPE tables hold {limit}")
        root = torch.as_tensor(np.array([outs[b][-1] for b in live], dtype=np.int32)).to(dev) if N == 1 else None
        key = (Bc, N, K, L, st.catch_tok.shape[1])
        if graphs and replant is None and decide is None and seen.get(key, 0) >= 1:
            if key not in recorded:
                recorded[key] = RoundGraph(target, draft, kv, dkv, Bc, N, K, L, key[4], ws_t, ws_d, eos_id, max_seq_len)
            acc, otok, fin, st = recorded[key].run(slot, st, root)
        elif N == 1:
            acc, otok, fin, st = plain_round(target, draft, kv, dkv, slot, st, root, ws_t, ws_d, eos_id, max_seq_len)
        else:
            hook = (lambda tk, pr: replant(tk, pr, live, outs)) if replant else None
            acc, otok, fin, st = spec_round(target, draft, kv, dkv, slot, st, N, K, L, ws_t, ws_d, eos_id, max_seq_len, hook, decide)
        seen[key] = seen.get(key, 0) + 1
        a, t, f = acc.cpu().numpy(), otok.cpu().numpy(), fin.cpu().numpy()     # the round's one trip to the host
        rows, nxt_live, emitted_round = [], [], 0
        for j, b in enumerate(live):
            emitted = [int(x) for x in t[j, :a[j] + 1]]
            room = int(budgets[b]) - len(outs[b])
            done = bool(f[j]) or len(emitted) >= room
            emitted = emitted[:room]
            outs[b].extend(emitted)
            emitted_round += len(emitted)
            if not done:
                rows.append(j)
                nxt_live.append(b)
        hist.append(dict(B=Bc, N=N, K=K, L=L, emitted=emitted_round))
        if len(nxt_live) < Bc and nxt_live:
            reselect(rows)
        live = nxt_live
    kv.check()      # the device-side backstop: raises if any call ran past a page table after all
    dkv.check()
    return outs, hist


def measure_c_peak(target, kv, ws, batch_sizes, warmup=2, reps=5, log2_axis=True):
    """Empirical C_peak (appendix): latency of one forward pass over B single-token inputs, for each B in
    batch_sizes, timed with events on the current stream; the knee of the curve is C_peak.  Batch sizes are meant
    to be spaced geometrically and the knee is taken on the log2(B) axis, where the flat weight-bound part and the
    rising compute-bound part have comparable extent.  The sequences start from empty caches (the cache must have
    at least max(batch_sizes) slots); nothing is committed.  log2_axis=False takes the knee on the batch-size axis
    itself, as the appendix plots it (fg_knee(times) can be called again on the returned latencies for the other axis).
    Returns (C_peak, latencies in ms)."""
    dev = kv.k_pool.device
    times = []
    kv.seq_len.zero_()
    for B in batch_sizes:
        slot = torch.arange(B, dtype=torch.int32, device=dev)
        tokens = torch.zeros((B, 1), dtype=torch.int32, device=dev)
        parent = torch.full((B, 1), -1, dtype=torch.int32, device=dev)
        for _ in range(warmup):
            fg.fg_spec_verify(target, kv, slot, tokens, parent, ws, max_seq_len=16, want_feature=False)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fg.fg_spec_verify(target, kv, slot, tokens, parent, ws, max_seq_len=16, want_feature=False)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / reps)
    k = fg.fg_knee(batch_sizes, times, log2_axis=log2_axis)
    return int(batch_sizes[k]), times


def prefill(target, draft, kv, dkv, slot, prompts, ws_t, ws_d, chunk=64, max_seq_len=0):
    """Run the prompts [B, P] (device int32) through the target and commit them, in chain steps of at most `chunk`
    tokens (a chain of n tokens is a tree whose node i has parent i - 1, so one verify step prefills n positions
    against everything committed before; n <= 64, the width of the ancestor masks).  The draft head consumes the
    matching entries (token t + 1 paired with the target's feature t) as it goes, except the last one, whose token
    is the first generated one.  Returns (first [B] int32 on the device: the arg-max after the last prompt token,
    SpecState holding that last pending entry)."""
    B, P = prompts.shape
    dev = prompts.device
    d = target.cfg["d_model"]
    prev_feat = None          # feature of the last position of the previous chunk, waiting for its token
    first = None
    for p0 in range(0, P, chunk):
        n = min(chunk, P - p0)
        tok = prompts[:, p0:p0 + n].contiguous()
        par = chain_parent(B, n, dev)
        last = p0 + n >= P      # only the last chunk's logits are needed (the first generated token)
        out = fg.fg_spec_verify(target, kv, slot, tok, par, ws_t, max_seq_len=max_seq_len, want_argmax=last)
        ident = torch.arange(n, dtype=torch.int32, device=dev).repeat(B, 1)
        feat = fg.fg_kv_compact(kv, slot, torch.full((B,), n - 1, dtype=torch.int32, device=dev), ident,
                                feature_in=out["feature"].view(B, n, d), d_model=d)
        # draft entries completed by this chunk: (prompt token t + 1, feature t) for t = p0 - 1 .. p0 + n - 2
        if draft is not None:
            if prev_feat is None:
                e_tok, e_feat = tok[:, 1:].contiguous(), feat[:, :n - 1].contiguous()
            else:
                e_tok, e_feat = tok, torch.cat([prev_feat, feat[:, :n - 1]], dim=1).contiguous()
            m = e_tok.shape[1]
            if m > 0:
                fg.fg_draft_step(target, draft, dkv, slot, e_tok, chain_parent(B, m, dev), e_feat, ws_d, 1,
                                 n_commit=torch.full((B,), m, dtype=torch.int32, device=dev), commit_bias=0,
                                 max_seq_len=max_seq_len, want_children=False)
        prev_feat = feat[:, n - 1:n].contiguous()
        if last:
            first = out["argmax"].view(B, n)[:, -1].contiguous()
    st = SpecState(first.view(B, 1).contiguous(), prev_feat, torch.zeros(B, dtype=torch.int32, device=dev))
    return first, st


class DraftTrainer:
    """Online draft learning (Sec. 4.2; Alg. 1, the draft training phase): fp32 master parameters of the draft head, their
    AdamW state, and the two library calls of a step.  Host bookkeeping only -- the loss, the gradients and the update are
    fg_draft_train_grad / fg_draft_adamw; `export` hands the updated head to the generation path by casting and re-packing
    the matrices (binding.Model).

    weights: dict fc, layers[0]{wqkv, wo, w_gate, w_up, w_down, norm_attn, norm_ffn} (tensors, any float type);
    target_weights: dict with the target's embed and lm_head (row-major [vocab, d])."""

    def __init__(self, draft_cfg, weights, target_weights, device="cuda", lr=1e-4, w_ce=0.1, betas=(0.9, 0.999), eps=1e-8,
                 weight_decay=0.01, compute="fp32"):
        self.cfg = dict(draft_cfg)
        self.compute = compute          # "fp32": exact; "bf16": the step's matrix products on the matrix cores
        f32 = lambda t: t.detach().to(device=device, dtype=torch.float32).contiguous().clone()
        lay = weights["layers"][0]
        self.w = {"fc": f32(weights["fc"])}
        self.w.update({k: f32(lay[k]) for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")})
        self.m = {k: torch.zeros_like(t) for k, t in self.w.items()}
        self.v = {k: torch.zeros_like(t) for k, t in self.w.items()}
        self.grad = {k: torch.empty_like(t) for k, t in self.w.items()}
        self.embed, self.lm_head = f32(target_weights["embed"]), f32(target_weights["lm_head"])
        self.lr, self.w_ce, self.betas, self.eps, self.weight_decay = lr, w_ce, betas, eps, weight_decay
        self.steps = 0
        self._ws = None
        # the head is frozen: in the matrix-core mode it is rounded and packed here, once, not in every step
        self._head = fg.fg_draft_train_pack_head(self.cfg, self.lm_head) if compute == "bf16" and self._head_packable() else None

    def _head_packable(self):
        return self.cfg["vocab"] % 64 == 0 and self.cfg["d_model"] % 64 == 0

    def step(self, tokens, feat_in, feat_tgt, n_valid):
        """One update on a batch of chains: tokens int32 [B, T], feat_in / feat_tgt [B, T, d] (cast to fp32 here), n_valid
        int32 [B].  Returns the device tensor [2] of the loss terms before the update (regression, cross-entropy)."""
        B, T = tokens.shape
        if self._ws is None or self._ws[0] != (B, T):      # one workspace per batch shape, kept between steps
            self._ws = ((B, T), torch.empty(fg.fg_draft_train_workspace_bytes(self.cfg, B, T, self.compute), dtype=torch.uint8,
                                            device=tokens.device))
        loss, _ = fg.fg_draft_train_grad(self.cfg, self.embed, self.lm_head, self.w, tokens, feat_in.float().contiguous(),
                                         feat_tgt.float().contiguous(), n_valid, self.w_ce, grad=self.grad, workspace=self._ws[1],
                                         compute=self.compute, head_packed=self._head)
        self.steps += 1
        fg.fg_draft_adamw(self.cfg, self.w, self.grad, self.m, self.v, lr=self.lr, step=self.steps, beta1=self.betas[0],
                          beta2=self.betas[1], eps=self.eps, weight_decay=self.weight_decay)
        return loss

    def weights(self):
        """The current parameters in the dict layout binding.Model takes for a draft head."""
        return {"fc": self.w["fc"], "layers": [{k: self.w[k] for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")}]}

    def export(self, target_model, max_pos=8192):
        """A draft Model of the generation path from the current parameters (cast to its type, packed)."""
        return fg.Model(self.cfg, self.weights(), target=target_model, max_pos=max_pos)


def training_chains(feature, tokens):
    """Training entries from what a pass of the target over whole sequences leaves behind: feature [B, P, d] (the target's
    feature at every position) and tokens [B, P] give, per sequence, the chain of P - 1 entries (token t + 1, feature t)
    with targets feature t + 1.  Returns (tokens [B, P-1], feat_in, feat_tgt)."""
    return tokens[:, 1:].contiguous(), feature[:, :-1].contiguous(), feature[:, 1:].contiguous()
