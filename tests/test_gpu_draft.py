"""GPU parity of the draft side (drafting step, frontier update, rerank) and of the whole generation loop on
config 1 against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import loop as oloop
from synth import configs, gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import harness
    assert torch.cuda.is_available()
    return harness


def topk_agree(g_tok, g_logp, o_tok, o_logp, o_logits, tol, margin):
    """Top-K tokens equal rank by rank except where the oracle's neighbouring logits are within `margin`."""
    assert np.abs(g_logp - o_logp)[g_tok == o_tok].max() <= tol
    bad = 0
    for r in range(o_tok.shape[0]):
        for k in range(o_tok.shape[1]):
            if g_tok[r, k] != o_tok[r, k]:
                srt = np.sort(o_logits[r])[::-1]
                assert srt[k] - srt[k + 1] < margin or (k > 0 and srt[k - 1] - srt[k] < margin), (r, k)
                bad += 1
    return bad


@pytest.mark.parametrize("dtype", ["fp32", "fp16", "bf16"])
def test_draft_step_with_in_round_nodes(H, dtype):
    import paper_2509_21792_amd as fg
    base = configs.TINY if dtype == "fp32" else configs.with_dtype(configs.scaled(configs.Q1P5B, 1), dtype)
    model = configs.scaled(base, 1) if dtype == "fp32" else base
    pair = H.Pair(model, seed=3, with_draft=True)
    dcfg = pair.dcfg
    B, n_prev, N, K = 4, 3, 5, 4
    lengths = np.array([9, 40, 16, 100], dtype=np.int32)
    st = H.State(pair, dcfg, lengths, n_prev + N + 1, seed=4)
    rng = np.random.default_rng(5)
    n_tot = n_prev + N
    parent = np.stack([np.array([-1] + [int(rng.integers(-1, i)) for i in range(1, n_tot)], dtype=np.int32) for _ in range(B)])
    tok_all = rng.integers(0, model["vocab"], size=(B, n_tot)).astype(np.int32)
    td = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}[dtype]
    feat_all = (torch.randn((B, n_tot, model["d_model"]), generator=torch.Generator().manual_seed(6)) * 1.0).to(td)
    ws = pair.gd.workspace(B * n_tot, st.cap)
    fa = feat_all.cuda()
    # first the n_prev nodes, then the N new ones that see them
    fg.fg_draft_step(pair.gm, pair.gd, st.kv, st.slot, tok_all[:, :n_prev], parent[:, :n_prev], fa[:, :n_prev].contiguous(), ws, K)
    ctok, clogp, ofeat = fg.fg_draft_step(pair.gm, pair.gd, st.kv, st.slot, tok_all[:, n_prev:], parent, fa, ws, K,
                                          n_prev=n_prev, feat_index=np.tile(np.arange(n_prev, n_tot, dtype=np.int32), (B, 1)))
    torch.cuda.synchronize()
    orc = pair.orc
    fnp = feat_all.float().numpy()
    orc.tree_forward(pair.od, st.ocache, tok_all[:, :n_prev], parent[:, :n_prev], feat_in=fnp[:, :n_prev], is_draft=True)
    oh, ol = orc.tree_forward(pair.od, st.ocache, tok_all[:, n_prev:], parent, feat_in=fnp[:, n_prev:], n_prev=n_prev, is_draft=True)
    o_tok, o_logp = orc.topk_logp(ol, K)
    herr = np.abs(ofeat.float().cpu().numpy().reshape(B * N, -1) - oh).max()
    tol = {"fp32": 1e-4, "fp16": 5e-3, "bf16": 4e-2}[dtype]
    assert herr <= tol, herr
    n_bad = topk_agree(ctok.cpu().numpy().reshape(B * N, K), clogp.cpu().numpy().reshape(B * N, K), o_tok, o_logp, ol,
                       tol=max(tol, 1e-4) * 3, margin={"fp32": 1e-3, "fp16": 0.05, "bf16": 0.15}[dtype])
    assert (st.kv.seq_len.cpu().numpy() == lengths).all()
    # decoding one picked row per sequence gives that row's lists, bit for bit (the cache slots are rewritten alike)
    pick = np.array([0, N - 1, 2, 1], dtype=np.int32)
    ctok1, clogp1, ofeat1 = fg.fg_draft_step(pair.gm, pair.gd, st.kv, st.slot, tok_all[:, n_prev:], parent, fa, ws, K, n_prev=n_prev,
                                             feat_index=np.tile(np.arange(n_prev, n_tot, dtype=np.int32), (B, 1)), expand_row=pick)
    torch.cuda.synchronize()
    assert ctok1.shape == (B, 1, K) and torch.equal(ofeat1, ofeat)
    rows = torch.arange(B, device="cuda")
    assert torch.equal(ctok1[:, 0], ctok[rows, torch.as_tensor(pick).cuda().long()])
    assert torch.equal(clogp1[:, 0], clogp[rows, torch.as_tensor(pick).cuda().long()])
    print(f"draft step {dtype}: hidden err {herr:.3g}, {n_bad} exempt top-K swaps", flush=True)


def test_frontier_and_rerank_are_bit_exact(H):
    """Integer / comparison work: candidate lists, frontier choice, parent lists and the reranked tree against the oracle."""
    import paper_2509_21792_amd as fg
    orc = H.Oracle("f32")
    rng = np.random.default_rng(2)
    B, K, L = 37, 4, 5
    n_total = 1 + K + (L - 1) * K * K
    ct = torch.zeros((B, n_total), dtype=torch.int32, device="cuda")
    cp = torch.zeros((B, n_total), dtype=torch.int32, device="cuda")
    cs = torch.zeros((B, n_total), dtype=torch.float32, device="cuda")
    Kin = 3
    catch_tok = rng.integers(0, 1000, size=(B, Kin)).astype(np.int32)
    pick = rng.integers(0, Kin, size=B).astype(np.int32)
    # log-probabilities on a coarse grid so that equal scores (ties) occur
    ctok = rng.integers(0, 1000, size=(B, Kin, K)).astype(np.int32)
    clogp = -(rng.integers(1, 6, size=(B, Kin, K)).astype(np.float32)) * 0.5
    o_tok = [catch_tok[np.arange(B), pick].reshape(B, 1), ctok[np.arange(B), pick]]
    o_par = [np.full((B, 1), -1, np.int32), np.zeros((B, K), np.int32)]
    o_sc = [np.zeros((B, 1), np.float32), clogp[np.arange(B), pick]]
    nt, nc, ns, nsrc, parents = fg.fg_draft_frontier(torch.as_tensor(ctok).cuda(), torch.as_tensor(clogp).cuda(), 1, ct, cp, cs,
                                                     node_pick=torch.as_tensor(pick).cuda(), node_tok=torch.as_tensor(catch_tok).cuda())
    torch.cuda.synchronize()
    # the same first step from child lists that hold the picked row only (what a draft step with expand_row returns)
    ct2, cp2, cs2 = torch.zeros_like(ct), torch.zeros_like(cp), torch.zeros_like(cs)
    g2 = fg.fg_draft_frontier(torch.as_tensor(ctok[np.arange(B), pick][:, None]).cuda(),
                              torch.as_tensor(clogp[np.arange(B), pick][:, None]).cuda(), 1, ct2, cp2, cs2,
                              node_pick=torch.as_tensor(pick).cuda(), node_tok=torch.as_tensor(catch_tok).cuda())
    torch.cuda.synchronize()
    for a, b in zip((nt, nc, ns, nsrc, parents), g2):
        assert torch.equal(a, b)
    assert torch.equal(ct2[:, :1 + K], ct[:, :1 + K]) and torch.equal(cs2[:, :1 + K], cs[:, :1 + K])
    assert (parents.cpu().numpy() == -1).all() and parents.shape == (B, K)
    assert np.array_equal(nsrc.cpu().numpy(), np.repeat(pick[:, None], K, axis=1))
    f_score = o_sc[1].copy(); f_cand = np.tile(np.arange(1, K + 1, dtype=np.int32), (B, 1))
    # the root's K children come back best-first (stable) as the first frontier
    order = np.argsort(-f_score, axis=1, kind="stable")
    assert np.array_equal(nc.cpu().numpy(), 1 + order)
    f_tok, f_cand, f_score = nt.cpu().numpy(), nc.cpu().numpy(), ns.cpu().numpy()
    n_cand, o_parents = 1 + K, np.full((B, K), -1, np.int32)
    for step in range(2, L + 1):
        ctok = rng.integers(0, 1000, size=(B, K, K)).astype(np.int32)
        clogp = -(rng.integers(1, 6, size=(B, K, K)).astype(np.float32)) * 0.5
        g = fg.fg_draft_frontier(torch.as_tensor(ctok).cuda(), torch.as_tensor(clogp).cuda(), n_cand, ct, cp, cs,
                                 node_cand=torch.as_tensor(f_cand).cuda(), node_score=torch.as_tensor(f_score).cuda(),
                                 parent_prev=torch.as_tensor(o_parents).cuda())
        torch.cuda.synchronize()
        cscore = (f_score[:, :, None] + clogp).astype(np.float32).reshape(B, K * K)
        o_tok.append(ctok.reshape(B, K * K)); o_par.append(np.repeat(f_cand, K, axis=1)); o_sc.append(cscore)
        pickk = orc.topk_index(cscore, K)
        rows = np.arange(B)[:, None]
        want_tok, want_score, want_cand = ctok.reshape(B, K * K)[rows, pickk], cscore[rows, pickk], (n_cand + pickk).astype(np.int32)
        assert np.array_equal(g[0].cpu().numpy(), want_tok) and np.array_equal(g[1].cpu().numpy(), want_cand)
        assert np.array_equal(g[2].cpu().numpy(), want_score) and np.array_equal(g[3].cpu().numpy(), pickk // K)
        n_prev = (step - 2) * K
        o_parents = np.concatenate([o_parents, (n_prev + pickk // K).astype(np.int32)], axis=1)
        assert np.array_equal(g[4].cpu().numpy(), o_parents)
        f_tok, f_cand, f_score = want_tok, want_cand, want_score
        n_cand += K * K
    ot, op, os_ = np.concatenate(o_tok, 1), np.concatenate(o_par, 1), np.concatenate(o_sc, 1)
    assert np.array_equal(ct.cpu().numpy(), ot) and np.array_equal(cp.cpu().numpy(), op) and np.array_equal(cs.cpu().numpy(), os_)
    for N in (1, 2, 8, 24, 64):
        tokens, parent, sel = fg.fg_build_tree(ct, cp, cs, n_total, N)
        torch.cuda.synchronize()
        wt, wp, wsel = orc.build_tree(ot, op, os_, N)
        assert np.array_equal(tokens.cpu().numpy(), wt) and np.array_equal(parent.cpu().numpy(), wp)
        assert np.array_equal(sel.cpu().numpy(), wsel)


def test_config1_generation_loop_matches_plain_greedy_decoding(H):
    """Config 1 end to end on the GPU (fp32, 8 sequences, prompts of 32 tokens, chain draft depth 4 from the 1-layer
    head, 64 new tokens, greedy) against the oracle's plain autoregressive tokens.  A sequence may leave the
    comparison only at a position whose oracle top-2 margin is below 0.05."""
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    cfg = configs.CONFIGS["cfg1"]
    model = configs.TINY
    pair = H.Pair(model, seed=cfg["seed"], with_draft=True)
    orc = pair.orc
    B, P, n_new, N = cfg["B"], cfg["prompt_len"], cfg["new_tokens"], cfg["N"]
    K, L = 1, N - 1
    prompts = gen.make_prompts(B, cfg["group"], P, model["vocab"], cfg["seed"])
    # oracle: plain greedy decoding
    ocache = orc.cache(model, B, P + n_new + 8)
    _, ologits = oloop.prefill(orc, pair.om, ocache, prompts)
    oroot, m0 = orc.row_argmax(ologits[:, -1])
    orest, omar = oloop.greedy_ar(orc, pair.om, ocache, oroot, n_new - 1)
    ref = np.concatenate([oroot[:, None], orest], axis=1)
    margins = np.concatenate([m0[:, None], omar], axis=1)
    # GPU: prefill = one chain verify step from an empty cache, committed whole
    cap = P + n_new + N + 8
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
    dkv = fg.KVCache(pair.dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t = pair.gm.workspace(B * P, cap)
    ws_d = pair.gd.workspace(B * P, cap)
    ptok = torch.as_tensor(prompts).cuda()
    out = fg.fg_spec_verify(pair.gm, kv, slot, ptok, gloop.chain_parent(B, P, "cuda"), ws_t, want_logits=False)
    ident = torch.arange(P, dtype=torch.int32, device="cuda").repeat(B, 1)
    feat = fg.fg_kv_compact(kv, slot, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"), ident,
                            feature_in=out["feature"].view(B, P, -1), d_model=model["d_model"])
    root = out["argmax"].view(B, P)[:, -1].contiguous()
    catch_tok = torch.cat([ptok[:, 1:], root.view(B, 1)], dim=1).contiguous()
    st = gloop.SpecState(catch_tok, feat, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"))
    outs = [[int(t)] for t in root.cpu().numpy()]
    rounds, accepted = 0, 0
    while min(len(o) for o in outs) < n_new and rounds < 200:
        acc, otok, fin, st = gloop.spec_round(pair.gm, pair.gd, kv, dkv, slot, st, N, K, L, ws_t, ws_d)
        a, t = acc.cpu().numpy(), otok.cpu().numpy()
        for b in range(B):
            outs[b].extend(int(x) for x in t[b, :a[b] + 1])
        accepted += int(a.sum()) + B
        rounds += 1
    got = np.array([o[:n_new] for o in outs])
    n_exempt = 0
    for b in range(B):
        diff = np.nonzero(got[b] != ref[b])[0]
        if len(diff):
            assert margins[b, diff[0]] < H.MARGIN, (b, diff[0], margins[b, diff[0]])
            n_exempt += 1
    assert n_exempt <= 1
    # target and draft caches advance together: the draft holds one entry per committed target position
    assert torch.equal(kv.seq_len, dkv.seq_len + 0) or (kv.seq_len - dkv.seq_len).abs().max().item() <= N
    print(f"config 1 loop: {rounds} rounds, tau = {accepted / (rounds * B):.3f}, sequences exempt {n_exempt}", flush=True)


@pytest.mark.parametrize("V,K", [(16, 3), (1000, 4), (1003, 8), (152064, 4), (152066, 1)])
def test_topk_logp_ties_and_ragged_vocabulary(H, V, K):
    """The top-K kernels against the oracle: token ids exact, with planted ties inside a thread's stride, across
    threads and across waves (lower id first), vocabularies that are and are not multiples of four."""
    import paper_2509_21792_amd as fg
    rng = np.random.default_rng(V + K)
    M = 7
    lg = (rng.standard_normal((M, V)) * 2).astype(np.float32)
    top = lg.max() + 1.0
    for r in range(M):      # ties among the winners
        pos = rng.choice(V, size=min(5, V), replace=False)
        lg[r, pos[:3]] = top + r
        if V > 2100:
            lg[r, [5, 5 + 1024, 5 + 2048]] = top + r        # same thread, later strides
    from oracle.oracle import Oracle
    o_tok, o_logp = Oracle("f64").topk_logp(lg, K)   # the fp32 build's sequential sum is itself off by ~7e-4 at this width
    g_tok, g_logp = fg.fg_topk_logp(torch.as_tensor(lg).cuda(), K)
    torch.cuda.synchronize()
    assert np.array_equal(g_tok.cpu().numpy(), o_tok)
    assert np.abs(g_logp.cpu().numpy() - o_logp).max() < 2e-5


def test_topk_logp_many_ties(H):
    """Rows where the selective top-K kernel cannot decide from a few threads' entries -- every logit equal, or a
    plateau of equal maxima wider than its candidate lists -- are redone by the general kernel; a plateau that still
    fits stays on the selective path.  Token ids exact (lowest ids first)."""
    import paper_2509_21792_amd as fg
    from oracle.oracle import Oracle
    V, K = 8192, 5
    rng = np.random.default_rng(5)
    lg = (rng.standard_normal((4, V))).astype(np.float32)
    lg[0, :] = 0.25                                     # all equal: every thread ties
    lg[1, rng.choice(V, size=3000, replace=False)] = 9.0   # a plateau of 3000 maxima
    lg[2, rng.choice(V, size=30, replace=False)] = 9.0     # a plateau of 30 maxima
    o_tok, o_logp = Oracle("f64").topk_logp(lg, K)
    g_tok, g_logp = fg.fg_topk_logp(torch.as_tensor(lg).cuda(), K)
    torch.cuda.synchronize()
    assert np.array_equal(g_tok.cpu().numpy(), o_tok)
    assert np.abs(g_logp.cpu().numpy() - o_logp).max() < 2e-5


def test_adaptive_generation_loop_follows_the_oracle(H):
    """Alg. 1 with the concurrency rule in the loop, on the device: ragged budgets make the live set decay from 8
    to 1, (N, K, L) is re-planned every round, N = 1 rounds are plain decoding, finished sequences leave the batch.
    Tokens, the live-set history and the per-round plans must equal the oracle loop's (fp32; a sequence is exempt
    only from the first position whose oracle top-2 margin is below the decision margin)."""
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    cfg = configs.CONFIGS["cfg1"]
    model = configs.TINY
    pair = H.Pair(model, seed=cfg["seed"], with_draft=True)
    orc = pair.orc
    B, P = cfg["B"], cfg["prompt_len"]
    budgets = np.array([6, 40, 17, 64, 9, 25, 33, 12], dtype=np.int32)[:B]
    n_new = int(budgets.max())
    c_peak, alpha, K_max, L_max = 12.0, 0.5, 2, 4
    prompts = gen.make_prompts(B, cfg["group"], P, model["vocab"], cfg["seed"])
    # oracle
    ocache = orc.cache(model, B, P + n_new + 72)
    odcache = orc.cache(pair.dcfg, B, P + n_new + 72)
    ofeat, ologits = oloop.prefill(orc, pair.om, ocache, prompts)
    oroot, _ = orc.row_argmax(ologits[:, -1])
    ocatch = np.concatenate([prompts[:, 1:], oroot[:, None]], axis=1).astype(np.int32)
    want, want_hist = oloop.adaptive_generate(orc, pair.om, pair.od, ocache, odcache, ocatch, ofeat, np.full(B, P, np.int32), oroot,
                                              budgets, c_peak, alpha=alpha, K_max=K_max, L_max=L_max)
    # device: prefill = one chain verify step from an empty cache, committed whole
    cap = P + n_new + 72
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
    dkv = fg.KVCache(pair.dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t = pair.gm.workspace(B * P, cap)
    ws_d = pair.gd.workspace(B * P, cap)
    ptok = torch.as_tensor(prompts).cuda()
    out = fg.fg_spec_verify(pair.gm, kv, slot, ptok, gloop.chain_parent(B, P, "cuda"), ws_t, want_logits=False)
    ident = torch.arange(P, dtype=torch.int32, device="cuda").repeat(B, 1)
    feat = fg.fg_kv_compact(kv, slot, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"), ident,
                            feature_in=out["feature"].view(B, P, -1), d_model=model["d_model"])
    root = out["argmax"].view(B, P)[:, -1].contiguous()
    catch_tok = torch.cat([ptok[:, 1:], root.view(B, 1)], dim=1).contiguous()
    st = gloop.SpecState(catch_tok, feat, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"))
    got, hist = gloop.generate(pair.gm, pair.gd, kv, dkv, slot, st, root.cpu().numpy(), budgets, c_peak, ws_t, ws_d,
                               alpha=alpha, K_max=K_max, L_max=L_max, max_seq_len=cap)
    assert np.array_equal(root.cpu().numpy(), oroot)
    for b in range(B):
        assert got[b] == want[b], (b, got[b], want[b])
    assert hist == want_hist
    assert any(h["N"] == 1 for h in hist) and any(h["N"] > 1 for h in hist) and hist[-1]["B"] == 1
    print(f"adaptive loop: {len(hist)} rounds, live set {[h['B'] for h in hist][::4]}, N {[h['N'] for h in hist][::4]}", flush=True)
    # the same rollout with every round shape replayed as a HIP graph from its second use on: fresh caches, same
    # prefill; replays alternate with the loop's eager work (row re-selection, first uses of new shapes, host copies)
    kv2, dkv2 = fg.KVCache(model, table, n_pages), fg.KVCache(pair.dcfg, dtable, dn)
    out2 = fg.fg_spec_verify(pair.gm, kv2, slot, ptok, gloop.chain_parent(B, P, "cuda"), ws_t, want_logits=False)
    feat2 = fg.fg_kv_compact(kv2, slot, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"), ident,
                             feature_in=out2["feature"].view(B, P, -1), d_model=model["d_model"])
    st2 = gloop.SpecState(catch_tok.clone(), feat2, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"))
    before = gloop.RoundGraph.replays
    got2, hist2 = gloop.generate(pair.gm, pair.gd, kv2, dkv2, slot, st2, root.cpu().numpy(), budgets, c_peak, ws_t, ws_d,
                                 alpha=alpha, K_max=K_max, L_max=L_max, max_seq_len=cap, graphs=True)
    n_replays = gloop.RoundGraph.replays - before
    assert got2 == got and hist2 == hist
    assert n_replays >= len(hist) // 3, (n_replays, len(hist))
    assert torch.equal(kv2.seq_len, kv.seq_len) and torch.equal(dkv2.seq_len, dkv.seq_len)
    print(f"adaptive loop with recorded rounds: {n_replays} of {len(hist)} rounds replayed", flush=True)


def test_select_rows_and_knee(H):
    import paper_2509_21792_amd as fg
    g = torch.Generator().manual_seed(0)
    src = torch.randn((37, 5, 12), generator=g).cuda()
    idx = torch.tensor([36, 0, 5, 5, 17], dtype=torch.int32, device="cuda")
    assert torch.equal(fg.fg_select_rows(src, idx), src[idx.long()])
    s1 = torch.arange(50, dtype=torch.int32, device="cuda")
    assert torch.equal(fg.fg_select_rows(s1, idx), s1[idx.long()])
    h = src.to(torch.bfloat16).contiguous()
    assert torch.equal(fg.fg_select_rows(h, idx), h[idx.long()])


def test_adaptive_loop_with_planted_agreement_still_equals_plain_decoding(H):
    """The synthetic-workload hook: the reranked tree's first-child chain is overwritten with the sequence's true
    continuation (here the oracle's plain greedy decoding) at rate 0.8.  Accepted paths of several tokens, ragged
    budgets and a shrinking live set together must still reproduce plain decoding exactly, with tau well above 1."""
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    cfg = configs.CONFIGS["cfg1"]
    model = configs.TINY
    pair = H.Pair(model, seed=cfg["seed"], with_draft=True)
    orc = pair.orc
    B, P = cfg["B"], cfg["prompt_len"]
    budgets = np.array([6, 40, 17, 64, 9, 25, 33, 12], dtype=np.int32)[:B]
    n_new = int(budgets.max())
    prompts = gen.make_prompts(B, cfg["group"], P, model["vocab"], cfg["seed"])
    ocache = orc.cache(model, B, P + n_new + 8)
    _, ologits = oloop.prefill(orc, pair.om, ocache, prompts)
    oroot, _ = orc.row_argmax(ologits[:, -1])
    orest, _ = oloop.greedy_ar(orc, pair.om, ocache, oroot, n_new - 1)
    ref = np.concatenate([oroot[:, None], orest], axis=1)
    cap = P + n_new + 72
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
    dkv = fg.KVCache(pair.dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t = pair.gm.workspace(B * P, cap)
    ws_d = pair.gd.workspace(B * P, cap)
    ptok = torch.as_tensor(prompts).cuda()
    out = fg.fg_spec_verify(pair.gm, kv, slot, ptok, gloop.chain_parent(B, P, "cuda"), ws_t, want_logits=False)
    ident = torch.arange(P, dtype=torch.int32, device="cuda").repeat(B, 1)
    feat = fg.fg_kv_compact(kv, slot, torch.full((B,), P - 1, dtype=torch.int32, device="cuda"), ident,
                            feature_in=out["feature"].view(B, P, -1), d_model=model["d_model"])
    root = out["argmax"].view(B, P)[:, -1].contiguous()
    st = gloop.SpecState(torch.cat([ptok[:, 1:], root.view(B, 1)], dim=1).contiguous(), feat,
                         torch.full((B,), P - 1, dtype=torch.int32, device="cuda"))
    rng = np.random.default_rng(3)

    def replant(tokens, parent, live, outs):
        par, tok = parent.cpu().numpy(), tokens.cpu().numpy().copy()
        for j, b in enumerate(live):
            node, depth, done = 0, 0, len(outs[b])
            while done + depth < n_new:
                kids = np.nonzero(par[j] == node)[0]
                if len(kids) == 0:
                    break
                node = int(kids[0])
                if rng.random() >= 0.8:
                    tok[j, node] = (ref[b, done + depth] + 1) % model["vocab"]
                    break
                tok[j, node] = ref[b, done + depth]
                depth += 1
        return torch.as_tensor(tok).cuda()

    got, hist = gloop.generate(pair.gm, pair.gd, kv, dkv, slot, st, root.cpu().numpy(), budgets, 12.0, ws_t, ws_d,
                               alpha=0.5, K_max=2, L_max=4, max_seq_len=cap, replant=replant)
    for b in range(B):
        assert got[b] == [int(t) for t in ref[b, :budgets[b]]], (b, got[b], list(ref[b, :budgets[b]]))
    spec = [h for h in hist if h["N"] > 1]
    tau = sum(h["emitted"] for h in spec) / sum(h["B"] for h in spec)
    print(f"planted adaptive loop: {len(hist)} rounds, tau over speculative rounds {tau:.2f}", flush=True)
    assert tau > 1.5


def test_chunked_prefill_then_adaptive_generation(H):
    """Prompts of 150 tokens prefilled in chain steps of 64, 64 and 22 positions (target and draft caches), then the
    concurrency-aware loop: first tokens, emitted tokens, round history and both cache lengths equal the oracle's,
    which prefills the whole prompt in one pass."""
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    model = configs.TINY
    pair = H.Pair(model, seed=21, with_draft=True)
    orc = pair.orc
    B, P = 3, 150
    budgets = np.array([5, 30, 14], dtype=np.int32)
    n_new = int(budgets.max())
    c_peak, alpha, K_max, L_max = 6.0, 0.5, 2, 3
    prompts = gen.make_prompts(B, 1, P, model["vocab"], 21)
    ocache = orc.cache(model, B, P + n_new + 72)
    odcache = orc.cache(pair.dcfg, B, P + n_new + 72)
    ofeat, ologits = oloop.prefill(orc, pair.om, ocache, prompts)
    oroot, _ = orc.row_argmax(ologits[:, -1])
    ocatch = np.concatenate([prompts[:, 1:], oroot[:, None]], axis=1).astype(np.int32)
    want, want_hist = oloop.adaptive_generate(orc, pair.om, pair.od, ocache, odcache, ocatch, ofeat, np.full(B, P, np.int32), oroot,
                                              budgets, c_peak, alpha=alpha, K_max=K_max, L_max=L_max)
    cap = P + n_new + 72
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
    dkv = fg.KVCache(pair.dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t = pair.gm.workspace(B * 64, cap)
    ws_d = pair.gd.workspace(B * 64, cap)
    first, st = gloop.prefill(pair.gm, pair.gd, kv, dkv, slot, torch.as_tensor(prompts).cuda(), ws_t, ws_d, max_seq_len=cap)
    torch.cuda.synchronize()
    assert np.array_equal(first.cpu().numpy(), oroot)
    assert (kv.seq_len.cpu().numpy() == P).all() and (dkv.seq_len.cpu().numpy() == P - 1).all()
    got, hist = gloop.generate(pair.gm, pair.gd, kv, dkv, slot, st, first.cpu().numpy(), budgets, c_peak, ws_t, ws_d,
                               alpha=alpha, K_max=K_max, L_max=L_max, max_seq_len=cap)
    for b in range(B):
        assert got[b] == want[b], (b, got[b], want[b])
    assert hist == want_hist


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_draft_step_frontier_and_rerank_at_the_benchmarked_shape(H, dtype):
    """One drafting step of the 7B-class draft head (its real depth: one layer) for 256 sequences x 4 frontier nodes
    behind 4 earlier in-round nodes -- 1024 rows through the pipelined GEMMs with their fused epilogues, the LM head and
    the selective top-K in one fg_draft_step, the shape the benchmark times -- then the frontier update and the rerank,
    against the oracle on a subset of the sequences."""
    import paper_2509_21792_amd as fg
    model = configs.with_dtype(configs.scaled(configs.Q7B, 1), dtype)
    pair = H.Pair(model, seed=31, with_draft=True)
    dcfg = pair.dcfg
    B, K, n_prev = 256, 4, 4
    N = K
    lengths = gen.make_kv_lengths(B, 1024, 4096, 31)
    lengths[0], lengths[-1] = 1024, 4096
    subset = [0, 77, 141, B - 1]
    S = len(subset)
    st = H.State(pair, dcfg, lengths, n_prev + N + 1, seed=32, subset=subset)
    rng = np.random.default_rng(33)
    n_tot = n_prev + N
    # the earlier nodes are the root's four children, the new ones their children (a step-3 shape of the expansion)
    parent = np.tile(np.array([-1, -1, -1, -1, 0, 1, 2, 3], np.int32), (B, 1))
    tok_all = rng.integers(0, model["vocab"], size=(B, n_tot)).astype(np.int32)
    td = torch.float16 if dtype == "fp16" else torch.bfloat16
    feat_all = torch.randn((B, n_tot, model["d_model"]), generator=torch.Generator().manual_seed(34)).to(td)
    fa = feat_all.cuda()
    ws = pair.gd.workspace(B * N, st.cap)
    msl = int(lengths.max()) + n_tot
    fg.fg_draft_step(pair.gm, pair.gd, st.kv, st.slot, tok_all[:, :n_prev], parent[:, :n_prev], fa[:, :n_prev].contiguous(), ws, K,
                     max_seq_len=msl, want_children=False)
    fidx = np.tile(np.arange(n_prev, n_tot, dtype=np.int32), (B, 1))
    ctok, clogp, ofeat = fg.fg_draft_step(pair.gm, pair.gd, st.kv, st.slot, tok_all[:, n_prev:], parent, fa, ws, K, n_prev=n_prev,
                                          feat_index=fidx, max_seq_len=msl)
    torch.cuda.synchronize()
    orc = pair.orc
    fnp = feat_all.float().numpy()[subset]
    orc.tree_forward(pair.od, st.ocache, tok_all[subset, :n_prev], parent[subset, :n_prev], feat_in=fnp[:, :n_prev], is_draft=True,
                     want_logits=False)
    oh, ol = orc.tree_forward(pair.od, st.ocache, tok_all[subset, n_prev:], parent[subset], feat_in=fnp[:, n_prev:], n_prev=n_prev,
                              is_draft=True)
    o_tok, o_logp = orc.topk_logp(ol, K)
    sub_t = torch.as_tensor(subset).cuda()
    herr = np.abs(ofeat[sub_t].float().cpu().numpy().reshape(S * N, -1) - oh).max()
    # the head's output is the un-normalised residual stream: a few roundings of the 16-bit activations that feed it,
    # each 2^-11 (fp16) or 2^-8 (bf16) of values of the stream's own size
    htol = {"fp16": 2e-3, "bf16": 1.6e-2}[dtype] * float(np.abs(oh).max())
    assert herr <= htol, (herr, htol)
    g_tok, g_logp = ctok[sub_t].cpu().numpy().reshape(S * N, K), clogp[sub_t].cpu().numpy().reshape(S * N, K)
    n_bad = topk_agree(g_tok, g_logp, o_tok, o_logp, ol, tol={"fp16": 3e-2, "bf16": 0.12}[dtype],
                       margin={"fp16": 0.05, "bf16": 0.15}[dtype])
    assert n_bad <= S * N * K // 4
    # frontier update and rerank: integer / comparison work on the GPU's own child lists -- the oracle, given the same
    # lists, must pick the same K children and build the same tree
    n_total = 1 + K + 2 * K * K
    cand = [torch.zeros((B, n_total), dtype=t, device="cuda") for t in (torch.int32, torch.int32, torch.float32)]
    node_cand = torch.as_tensor(np.tile(np.arange(1 + K, 1 + 2 * K, dtype=np.int32), (B, 1))).cuda()
    node_score = torch.as_tensor(-rng.random((B, K)).astype(np.float32)).cuda()
    nt, nc, ns, nsrc, pnext = fg.fg_draft_frontier(ctok, clogp, 1 + K + K * K, cand[0], cand[1], cand[2], node_cand=node_cand,
                                                   node_score=node_score, parent_prev=torch.as_tensor(parent).cuda())
    torch.cuda.synchronize()
    cscore = (node_score[sub_t].cpu().numpy()[:, :, None] + clogp[sub_t].cpu().numpy()).astype(np.float32).reshape(S, K * K)
    pick = orc.topk_index(cscore, K)
    rows = np.arange(S)[:, None]
    assert np.array_equal(nt[sub_t].cpu().numpy(), ctok[sub_t].cpu().numpy().reshape(S, K * K)[rows, pick])
    assert np.array_equal(ns[sub_t].cpu().numpy(), cscore[rows, pick]) and np.array_equal(nsrc[sub_t].cpu().numpy(), pick // K)
    assert np.array_equal(pnext[sub_t].cpu().numpy()[:, n_tot:], n_prev + pick // K)
    print(f"draft step at 7B geometry {dtype}, 1024 rows: hidden err {herr:.3g}, {n_bad} exempt top-K swaps of {S * N * K}", flush=True)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_16bit_prefill_in_chunks_against_one_pass(H, dtype):
    """The 16-bit prefill the benchmark times: prompts of 150 tokens through chain verify steps of 64, 64 and 22 positions
    (7B-class geometry, two layers, target and draft head), against the oracle's one-pass prefill: both caches' contents
    and lengths, the last position's feature, and the first generated token outside the margin exemption."""
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    model = configs.with_dtype(configs.scaled(configs.Q7B, 2), dtype)
    pair = H.Pair(model, seed=41, with_draft=True)
    orc = pair.orc
    B, P = 3, 150
    prompts = gen.make_prompts(B, 1, P, model["vocab"], 41)
    prompts[1] = np.random.default_rng(42).integers(0, model["vocab"], size=P)     # not all the same prompt
    cap = P + 80
    ocache, odcache = orc.cache(model, B, cap), orc.cache(pair.dcfg, B, cap)
    ofeat, ologits = oloop.prefill(orc, pair.om, ocache, prompts)
    oroot, omargin = orc.row_argmax(ologits[:, -1])
    # the draft head's entries during a prefill: (prompt token t + 1, feature t) for t = 0 .. P - 2
    orc.tree_forward(pair.od, odcache, prompts[:, 1:], oloop.chain_parent(B, P - 1), feat_in=ofeat[:, :P - 1], is_draft=True,
                     want_logits=False)
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
    dkv = fg.KVCache(pair.dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t, ws_d = pair.gm.workspace(B * 64, cap), pair.gd.workspace(B * 64, cap)
    first, st = gloop.prefill(pair.gm, pair.gd, kv, dkv, slot, torch.as_tensor(prompts).cuda(), ws_t, ws_d, max_seq_len=cap)
    torch.cuda.synchronize()
    assert (kv.seq_len.cpu().numpy() == P).all() and (dkv.seq_len.cpu().numpy() == P - 1).all()
    tol = {"fp16": 2e-2, "bf16": 0.15}[dtype]
    for b in range(B):
        k, v = kv.read(b, P)
        assert np.abs(k.float().cpu().numpy() - ocache.k[:, b, :P]).max() <= tol
        assert np.abs(v.float().cpu().numpy() - ocache.v[:, b, :P]).max() <= tol
        dk, dv = dkv.read(b, P - 1)
        assert np.abs(dk.float().cpu().numpy() - odcache.k[:, b, :P - 1]).max() <= 2 * tol
        assert np.abs(dv.float().cpu().numpy() - odcache.v[:, b, :P - 1]).max() <= 2 * tol
    ferr = np.abs(st.catch_feat[:, 0].float().cpu().numpy() - ofeat[:, -1]).max()
    assert ferr <= {"fp16": 2e-2, "bf16": 0.1}[dtype], ferr
    margin = H.decision_margin(model)
    for b in range(B):
        assert int(first[b]) == int(oroot[b]) or omargin[b] < margin, (b, omargin[b])
    print(f"16-bit prefill {dtype}: last feature err {ferr:.3g}, first-token margins {np.round(omargin, 3).tolist()}", flush=True)
