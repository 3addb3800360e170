"""Pin of the oracle's draft expansion (Alg. 1, the drafting loop "generate children for K_draft paths and update
T_candi"; Sec. 2 "Draft Model Architectures") against a brute-force enumeration (CPU only).

On a tiny vocabulary every token path of depth <= L is enumerated: the draft head is run on each path as a plain
chain (one linear pass per path, which the oracle's forward is pinned to agree with bit for bit), giving the
cumulative log-probability of EVERY path.  From that table the expansion is written out as its definition --
level 1 = the K most likely tokens after the root; level l = the K most likely children of each of the K frontier
paths; the frontier of level l = the K highest cumulative scores among that level's K^2 children, ties to the
earlier candidate -- with Python sorts, and compared with what oracle/loop.py: draft_expand returns.  A planted
mistake (the frontier keeps some other K children) must fail the same comparison.
"""
import numpy as np
import pytest
import scipy.special

from oracle import loop

MODEL = dict(name="pin", n_layers=1, d_model=16, n_q_heads=2, n_kv_heads=1, head_dim=8, d_ffn=32, vocab=8,
             rms_eps=1e-6, rope_theta=10000.0, dtype="fp32")


def make_models(orc, seed):
    rng = np.random.default_rng(seed)
    d, F, V = MODEL["d_model"], MODEL["d_ffn"], MODEL["vocab"]
    qkvd = (MODEL["n_q_heads"] + 2 * MODEL["n_kv_heads"]) * MODEL["head_dim"]
    hq = MODEL["n_q_heads"] * MODEL["head_dim"]

    def mat(o, i, s):
        return (rng.standard_normal((o, i)) * s).astype(np.float32)

    def layer():
        return dict(wqkv=mat(qkvd, d, 0.4), wo=mat(d, hq, 0.4), w_gate=mat(F, d, 0.4), w_up=mat(F, d, 0.4),
                    w_down=mat(d, F, 0.4), norm_attn=1 + mat(1, d, 0.1)[0], norm_ffn=1 + mat(1, d, 0.1)[0])

    tw = dict(embed=mat(V, d, 1.0), lm_head=mat(V, d, 0.6), final_norm=1 + mat(1, d, 0.1)[0], layers=[layer()])
    dw = dict(fc=mat(d, 2 * d, 0.4), layers=[layer()])
    target = orc.model(MODEL, tw)
    draft = orc.model(MODEL, dw, embed_from=target)
    return target, draft, rng


def definition(score, root_logp, K, L):
    """The candidate list of Alg. 1's drafting loop written from the score table: [(path, score)] in list order."""
    V = len(root_logp)
    full = score

    def best_children(path):
        kids = sorted(range(V), key=lambda t: (-full[path + (t,)], t))[:K]
        return [path + (t,) for t in kids]

    cands = best_children(())
    frontier = list(cands)
    out = [(p, full[p]) for p in cands]
    for _ in range(2, L + 1):
        level = [c for p in frontier for c in best_children(p)]
        out += [(p, full[p]) for p in level]
        order = sorted(range(len(level)), key=lambda i: (-full[level[i]], i))[:K]
        frontier = [level[i] for i in order]
    return out


def run_case(orc, seed, K, L, topk_index=None):
    target, draft, rng = make_models(orc, seed)
    B, Kin = 2, 3
    d, V = MODEL["d_model"], MODEL["vocab"]
    catch_tok = rng.integers(0, V, size=(B, Kin)).astype(np.int32)
    catch_feat = rng.standard_normal((B, Kin, d)).astype(np.float32)
    n_valid = np.array([3, 2], dtype=np.int32)
    dcache = orc.cache(MODEL, B, 32)
    saved = orc.topk_index
    if topk_index is not None:
        orc.topk_index = topk_index
    try:
        ct, cp, cs = loop.draft_expand(orc, target, draft, dcache.copy(), catch_tok, catch_feat, n_valid, K, L)
    finally:
        orc.topk_index = saved
    # the committed state the enumeration starts from: the catch-up chain run once, n_valid entries kept
    hid, lg = orc.tree_forward(draft, dcache, catch_tok, loop.chain_parent(B, Kin), feat_in=catch_feat, is_draft=True)
    dcache.len += n_valid
    hid, lg = hid.reshape(B, Kin, d), lg.reshape(B, Kin, V)
    for b in range(B):
        last = n_valid[b] - 1
        root_logp = scipy.special.log_softmax(lg[b, last].astype(np.float64))
        sc = enumerate_paths_from_root(orc, draft, dcache, b, hid[b, last], root_logp, L)
        want = definition(sc, root_logp, K, L)
        assert ct.shape[1] == 1 + len(want) == 1 + K + (L - 1) * K * K
        assert ct[b, 0] == catch_tok[b, last] and cp[b, 0] == -1 and cs[b, 0] == 0.0

        def path_of(i):
            p = []
            while i > 0:
                p.append(int(ct[b, i]))
                i = int(cp[b, i])
            return tuple(reversed(p))

        got = [(path_of(i), float(cs[b, i])) for i in range(1, ct.shape[1])]
        assert [p for p, _ in got] == [p for p, _ in want], (b, got, want)
        assert np.allclose([s for _, s in got], [s for _, s in want], atol=2e-5)


def enumerate_paths_from_root(orc, draft, dcache, b, root_hidden, root_logp, L):
    """score[path] = cumulative draft log-probability of the token path (t_1 .. t_m), m = 1 .. L, for EVERY path:
    each path is run as one chain of single nodes against a copy of sequence b's committed draft cache; node j of
    the chain reads the hidden state the head produced at node j - 1 (the root's for j = 0)."""
    V = len(root_logp)
    score = {(t,): float(root_logp[t]) for t in range(V)}
    hidden_of = {(): root_hidden}
    frontier = [(t,) for t in range(V)]
    for m in range(1, L):
        nxt = []
        for path in frontier:
            c = dcache.copy()
            feats = np.stack([hidden_of[path[:j]] for j in range(m)])[None]
            hid, lg = orc.tree_forward(draft, c, np.array([path], np.int32), loop.chain_parent(1, m), feat_in=feats,
                                       is_draft=True, slot=np.array([b], np.int32))
            hidden_of[path] = hid[-1]
            lp = scipy.special.log_softmax(lg[-1].astype(np.float64))
            for t in range(V):
                score[path + (t,)] = score[path] + float(lp[t])
                nxt.append(path + (t,))
        frontier = nxt
    assert len(score) == sum(V ** m for m in range(1, L + 1))
    return score


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("K,L", [(2, 3), (3, 2), (2, 4)])
def test_draft_expansion_equals_brute_force_over_all_paths(orc32, seed, K, L):
    run_case(orc32, seed, K, L)


def test_frontier_is_not_trivially_the_first_parent(orc32):
    """The cases above exercise the choice: the kept K children are not always the first K of the level's list."""
    differs = 0
    for seed in range(3):
        target, draft, rng = make_models(orc32, seed)
        catch_tok = rng.integers(0, MODEL["vocab"], size=(2, 3)).astype(np.int32)
        catch_feat = rng.standard_normal((2, 3, MODEL["d_model"])).astype(np.float32)
        ct, cp, cs = loop.draft_expand(orc32, target, draft, orc32.cache(MODEL, 2, 32), catch_tok, catch_feat,
                                       np.array([3, 2], np.int32), 2, 3)
        # level-3 candidates (indices 7..10) hang off the level-2 frontier; level-2 candidates are 3..6
        differs += sum(set(cp[b, 7:].tolist()) != {3, 4} for b in range(2))
    assert differs > 0


@pytest.mark.parametrize("mistake", ["worst", "first", "unordered"])
def test_a_wrong_frontier_fails_the_pin(orc32, mistake):
    real = orc32.topk_index

    def wrong(scores, K):
        if mistake == "worst":
            return real(-np.asarray(scores, dtype=np.float32), K)
        if mistake == "first":
            return np.tile(np.arange(K, dtype=np.int32), (np.shape(scores)[0], 1))
        return real(scores, K)[:, ::-1].copy()
    failed = 0
    for seed in range(3):
        try:
            run_case(orc32, seed, 2, 3, topk_index=wrong)
        except AssertionError:
            failed += 1
    assert failed == 3


def test_topk_index_ties_go_to_the_lower_index(orc32):
    s = np.array([[0.5, 2.0, 2.0, -1.0, 2.0, 0.5], [1.0, 1.0, 1.0, 1.0, 1.0, 1.0]], dtype=np.float32)
    assert orc32.topk_index(s, 4).tolist() == [[1, 2, 4, 0], [0, 1, 2, 3]]
    rng = np.random.default_rng(5)
    q = rng.integers(0, 4, size=(50, 16)).astype(np.float32)          # many exact ties
    want = np.array([sorted(range(16), key=lambda i: (-row[i], i))[:5] for row in q])
    assert np.array_equal(orc32.topk_index(q, 5), want)
