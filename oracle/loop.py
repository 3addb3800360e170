"""Generation loops on top of the CPU oracle (Alg. 1, the generation loop).  TEST INFRASTRUCTURE ONLY.

Host bookkeeping only (appending tokens, the live set, the candidate lists); every numeric step is a call
into fg_oracle.c.  Conventions: a sequence's cache holds the K/V of all tokens but the last emitted one
(the "root" of the next step).  The draft head's entry t pairs the embedding of token t+1 with the target's
feature at position t.
"""
import numpy as np


def chain_parent(B, n):
    return np.tile(np.arange(-1, n - 1, dtype=np.int32), (B, 1))


def prefill(orc, model, cache, prompts, slot=None):
    """Run the prompt through the target as one chain and commit it.  Returns (feature [B,P,d], logits [B,P,V])."""
    B, P = prompts.shape
    hidden, logits = orc.tree_forward(model, cache, prompts, chain_parent(B, P), slot=slot)
    idx = np.arange(B) if slot is None else np.asarray(slot)
    cache.len[idx] += P
    d, V = model.cfg["d_model"], model.cfg["vocab"]
    return hidden.reshape(B, P, d), logits.reshape(B, P, V)


def greedy_ar(orc, model, cache, root, n_new, slot=None):
    """Plain greedy autoregressive decoding: n_new tokens after `root` [B].  Commits as it goes.
    Returns (tokens [B, n_new], margins [B, n_new])."""
    B = root.shape[0]
    out = np.zeros((B, n_new), dtype=np.int32)
    mar = np.zeros((B, n_new), dtype=np.float64)
    idx = np.arange(B) if slot is None else np.asarray(slot)
    cur = root.astype(np.int32).copy()
    par = np.full((B, 1), -1, dtype=np.int32)
    for t in range(n_new):
        _, logits = orc.tree_forward(model, cache, cur.reshape(B, 1), par, slot=slot)
        nxt, margin = orc.row_argmax(logits)
        cache.len[idx] += 1
        out[:, t] = nxt
        mar[:, t] = margin
        cur = nxt
    return out, mar


def draft_expand(orc, target, draft, dcache, catch_tok, catch_feat, n_valid, K, L, slot=None):
    """Draft expansion (Alg. 1, the drafting loop): L sequential steps of the draft head, K paths kept per step.

    catch_tok [B, Kin], catch_feat [B, Kin, d], n_valid [B]: the entries the draft head has not yet seen
    (token t+1 with the target's feature t), the last valid one being the root.  They are committed to the
    draft cache.  Returns candidate lists cand_tok / cand_parent / cand_score [B, 1 + K + (L-1) K^2];
    candidate 0 is the root.
    """
    B, Kin = catch_tok.shape
    d = target.cfg["d_model"]
    idx = np.arange(B) if slot is None else np.asarray(slot)
    hidden, logits = orc.tree_forward(draft, dcache, catch_tok, chain_parent(B, Kin), feat_in=catch_feat,
                                      is_draft=True, slot=slot)
    dcache.len[idx] += n_valid
    hidden = hidden.reshape(B, Kin, d)
    V = logits.shape[-1]
    logits = logits.reshape(B, Kin, V)
    last = n_valid - 1
    root_hidden = hidden[np.arange(B), last]            # [B, d]
    tok, logp = orc.topk_logp(logits[np.arange(B), last], K)
    root_tok = catch_tok[np.arange(B), last]
    cand_tok = [root_tok.reshape(B, 1), tok]
    cand_parent = [np.full((B, 1), -1, np.int32), np.zeros((B, K), np.int32)]
    cand_score = [np.zeros((B, 1), np.float32), logp.astype(np.float32)]
    n_cand = 1 + K
    # frontier: K nodes; for each: token, candidate index, score, the feature it is paired with, in-round parent
    f_tok, f_cand, f_score = tok.copy(), np.tile(np.arange(1, K + 1, dtype=np.int32), (B, 1)), logp.astype(np.float32)
    f_feat = np.repeat(root_hidden[:, None, :], K, axis=1)
    f_par = np.full((B, K), -1, dtype=np.int32)
    inround_parent = np.zeros((B, 0), dtype=np.int32)
    for step in range(2, L + 1):
        n_prev = (step - 2) * K
        inround_parent = np.concatenate([inround_parent, f_par], axis=1)
        hidden, logits = orc.tree_forward(draft, dcache, f_tok, inround_parent, feat_in=f_feat, n_prev=n_prev,
                                          is_draft=True, slot=slot)
        hidden = hidden.reshape(B, K, d)
        ctok, clogp = orc.topk_logp(logits, K)                       # [B*K, K]
        ctok = ctok.reshape(B, K * K)
        cscore = (f_score[:, :, None] + clogp.reshape(B, K, K).astype(np.float32)).astype(np.float32).reshape(B, K * K)
        cpar = np.repeat(f_cand, K, axis=1)                           # candidate index of the parent
        cand_tok.append(ctok); cand_parent.append(cpar); cand_score.append(cscore)
        pick = orc.topk_index(cscore, K)                              # [B, K] into the K*K children
        rows = np.arange(B)[:, None]
        f_tok = ctok[rows, pick]
        f_score = cscore[rows, pick]
        f_cand = (n_cand + pick).astype(np.int32)
        f_feat = hidden[rows, pick // K]
        f_par = (n_prev + pick // K).astype(np.int32)
        n_cand += K * K
    return (np.concatenate(cand_tok, axis=1).astype(np.int32), np.concatenate(cand_parent, axis=1).astype(np.int32),
            np.concatenate(cand_score, axis=1).astype(np.float32))


def spec_generate(orc, target, cache, root, n_new, make_tree, eos_id=-1, max_rounds=10 ** 9):
    """Greedy speculative decoding of n_new tokens per sequence with a caller-supplied tree maker.

    make_tree(live_slots, roots, round_index, outs) -> (tokens [b,N], parent [b,N]) with tokens[:,0] == roots.
    Sequences leave the live set when they have n_new tokens or emit EOS (Alg. 1, the update of B_cur).
    Returns (list of per-sequence token lists, stats dict with accepted / verifications for tau).
    """
    B = root.shape[0]
    outs = [[] for _ in range(B)]
    live = list(range(B))
    cur = root.astype(np.int32).copy()
    accepted = 0
    verifs = 0
    rnd = 0
    hist = []
    while live and rnd < max_rounds:
        slot = np.array(live, dtype=np.int32)
        tokens, parent = make_tree(slot, cur[slot], rnd, outs)
        hidden, logits = orc.tree_forward(target, cache, tokens, parent, slot=slot)
        acc, path, out, fin, _, _ = orc.accept_greedy(tokens, parent, logits, eos_id)
        orc.kv_compact(cache, target.cfg, acc, path, slot=slot)
        verifs += len(live)
        hist.append(len(live))
        nxt_live = []
        for j, b in enumerate(live):
            emitted = [int(t) for t in out[j, :acc[j] + 1]]
            room = n_new - len(outs[b])
            if len(emitted) > room:
                # the sequence hit its length budget inside the path: keep only what fits, roll the cache back
                drop = len(emitted) - room
                emitted = emitted[:room]
                cache.len[b] -= drop
            outs[b].extend(emitted)
            accepted += len(emitted)
            cur[b] = emitted[-1]
            if not fin[j] and len(outs[b]) < n_new:
                nxt_live.append(b)
        live = nxt_live
        rnd += 1
    return outs, dict(accepted=accepted, verifications=verifs, live_history=hist)


def adaptive_generate(orc, target, draft, cache, dcache, catch_tok, catch_feat, n_valid, first, budgets, c_peak,
                      alpha=0.5, K_max=4, L_max=6, N_cap=64, eos_id=-1, max_rounds=10 ** 9):
    """The concurrency-aware generation loop (Alg. 1): every round the tree shape (N, K, L) is re-planned from the
    number of live sequences by Eq. 1-3; a round with N = 1 is plain decoding (the draft head still consumes its
    pending entries, so that its cache stays in step); sequences leave the live set at EOS or when they have
    budgets[b] tokens (first[b], already emitted, counts).

    catch_tok [B, Kin], catch_feat [B, Kin, d], n_valid [B]: the draft head's pending entries after the prefill, the
    last valid one being first[b]'s.  Returns (token lists, per-round history of dicts B, N, K, L, emitted).
    """
    B = len(first)
    d = target.cfg["d_model"]
    outs = [[int(first[b])] for b in range(B)]
    pend_tok = {b: [int(t) for t in catch_tok[b, :n_valid[b]]] for b in range(B)}
    pend_feat = {b: np.array(catch_feat[b, :n_valid[b]], dtype=np.float32) for b in range(B)}
    live = [b for b in range(B) if budgets[b] > 1]
    hist = []
    while live and len(hist) < max_rounds:
        slot = np.array(live, dtype=np.int32)
        Bc = len(live)
        N, K, L = orc.plan(Bc, c_peak, alpha, K_max, L_max, N_cap)
        kin = max(len(pend_tok[b]) for b in live)
        ct = np.zeros((Bc, kin), dtype=np.int32)
        cf = np.zeros((Bc, kin, d), dtype=np.float32)
        nv = np.zeros(Bc, dtype=np.int32)
        for j, b in enumerate(live):
            nv[j] = len(pend_tok[b])
            ct[j, :nv[j]] = pend_tok[b]
            cf[j, :nv[j]] = pend_feat[b]
        if N == 1:
            orc.tree_forward(draft, dcache, ct, chain_parent(Bc, kin), feat_in=cf, is_draft=True, slot=slot, want_logits=False)
            dcache.len[slot] += nv
            tokens = np.array([[outs[b][-1]] for b in live], dtype=np.int32)
            parent = np.full((Bc, 1), -1, dtype=np.int32)
        else:
            cand = draft_expand(orc, target, draft, dcache, ct, cf, nv, K, L, slot=slot)
            tokens, parent, _ = orc.build_tree(cand[0], cand[1], cand[2], N)
        hidden, logits = orc.tree_forward(target, cache, tokens, parent, slot=slot)
        acc, path, out, fin, _, _ = orc.accept_greedy(tokens, parent, logits, eos_id)
        orc.kv_compact(cache, target.cfg, acc, path, slot=slot)
        hidden = hidden.reshape(Bc, tokens.shape[1], d)
        nxt_live, emitted_round = [], 0
        for j, b in enumerate(live):
            a = int(acc[j])
            emitted = [int(t) for t in out[j, :a + 1]]
            room = int(budgets[b]) - len(outs[b])
            done = bool(fin[j]) or len(emitted) >= room
            emitted = emitted[:room]
            outs[b].extend(emitted)
            emitted_round += len(emitted)
            if not done:
                pend_tok[b] = emitted
                pend_feat[b] = hidden[j, path[j, :a + 1]]
                nxt_live.append(b)
        hist.append(dict(B=Bc, N=N, K=K, L=L, emitted=emitted_round))
        live = nxt_live
    return outs, hist
