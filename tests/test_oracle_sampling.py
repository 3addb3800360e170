"""Pins of the oracle's sampling and draft-side functions (CPU only).

Rejection sampling must reproduce the target distribution (chi-square, p > 0.01, tiny vocabulary); the
strict-match rule at temperature T must too (one Gumbel-max sample per node is an exact sample); the draft
side's top-K / log-probabilities / rerank are checked against library routines and brute force.
"""
import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import loop
from synth import configs, gen

V = 16


def softmax(x):
    return scipy.special.softmax(np.asarray(x, dtype=np.float64), axis=-1)


def test_uniform01_is_uniform_on_a_23_bit_grid(orc32):
    u = np.array([orc32.uniform01(7, r, v) for r in range(40) for v in range(500)])
    assert u.min() > 0 and u.max() < 1
    assert np.allclose((u * 2 ** 23 - 0.5), np.round(u * 2 ** 23 - 0.5))          # exactly representable in fp32
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert scipy.stats.kstest(u, "uniform").pvalue > 0.001
    assert len(set(u)) > 0.99 * len(u)
    assert orc32.uniform01(7, 3, 5) != orc32.uniform01(8, 3, 5) != orc32.uniform01(7, 5, 3)


def test_gumbel_max_sample_follows_softmax(orc32):
    rng = np.random.default_rng(0)
    T = 1.3
    logits = rng.standard_normal(V) * 1.5
    trials = 200000
    scores = orc32.gumbel_scores(np.tile(logits.astype(np.float32), (trials, 1)), T, seed=123)
    idx, margin = orc32.row_argmax(scores)
    obs = np.bincount(idx, minlength=V)
    exp = softmax(logits / T) * trials
    assert scipy.stats.chisquare(obs, exp).pvalue > 0.01
    # a different seed gives different draws, same law
    idx2, _ = orc32.row_argmax(orc32.gumbel_scores(np.tile(logits.astype(np.float32), (trials, 1)), T, seed=124))
    assert (idx != idx2).mean() > 0.5
    assert scipy.stats.chisquare(np.bincount(idx2, minlength=V), exp).pvalue > 0.01


def test_row_argmax_margin_and_ties(orc32):
    s = np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 1.0, 2.0, 4.5]], dtype=np.float32)
    idx, margin = orc32.row_argmax(s)
    assert list(idx) == [1, 0] and margin[0] == 0.0 and margin[1] == 0.5


def draw_without_replacement(rng, q, k):
    """k distinct tokens: the first from q, the next from q renormalised without the earlier ones."""
    out = np.zeros((q.shape[0], k), dtype=np.int32)
    q = q.copy()
    for j in range(k):
        cdf = np.cumsum(q / q.sum(axis=1, keepdims=True), axis=1)
        x = (rng.random((q.shape[0], 1)) > cdf).sum(axis=1).clip(0, q.shape[1] - 1)
        out[:, j] = x
        q[np.arange(q.shape[0]), x] = 0
    return out


@pytest.mark.parametrize("T", [1.0, 0.7])
def test_rejection_sampling_reproduces_target_distribution(orc32, T):
    """Depth-2 tree, 3 children of the root and 2 of each of them, all drawn from the draft distribution
    without replacement.  The first emitted token must follow p = softmax(logits / T) whatever q is, and
    the second, when there is one, must follow the target's distribution at the accepted node."""
    rng = np.random.default_rng(11)
    trials = 200000
    lg_root = rng.standard_normal(V) * 1.5
    base2 = rng.standard_normal(V) * 1.5
    q1 = softmax(rng.standard_normal(V))
    q2 = softmax(rng.standard_normal(V) * 2)
    parent = np.tile(np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32), (trials, 1))
    N = parent.shape[1]
    tokens = np.zeros((trials, N), dtype=np.int32)
    tokens[:, 1:4] = draw_without_replacement(rng, np.tile(q1, (trials, 1)), 3)
    for c in range(3):
        tokens[:, 4 + 2 * c: 6 + 2 * c] = draw_without_replacement(rng, np.tile(q2, (trials, 1)), 2)
    logits = np.zeros((trials, N, V), dtype=np.float32)
    logits[:, 0] = lg_root
    for c in (1, 2, 3):      # the target's distribution after token x is base2 rolled by x
        logits[:, c] = base2[(np.arange(V)[None, :] - tokens[:, c:c + 1]) % V]
    logits[:, 4:] = rng.standard_normal((trials, N - 4, V))
    dq = np.zeros((trials, N, V), dtype=np.float32)
    dq[:, 0] = q1
    dq[:, 1:4] = q2
    dq[:, 4:] = 1.0 / V
    unif = rng.random((trials, N), dtype=np.float32)
    acc, path, out, fin, bm, gap = orc32.accept_reject(tokens, parent, logits.reshape(trials * N, V),
                                                       dq.reshape(trials * N, V), unif, T, seed=99)
    p1 = softmax(lg_root / T)
    obs1 = np.bincount(out[:, 0], minlength=V)
    assert scipy.stats.chisquare(obs1, p1 * trials).pvalue > 0.01
    two = acc >= 1
    assert two.mean() > 0.2                     # drafts do get accepted
    assert (out[two, 0] == tokens[np.arange(trials)[two], path[two, 1]]).all()
    shift = (out[two, 1] - out[two, 0]) % V
    p2 = softmax(base2 / T)
    assert scipy.stats.chisquare(np.bincount(shift, minlength=V), p2 * two.sum()).pvalue > 0.01
    # joint law of the first two tokens on the trials that emit two: p(x1 accepted-or-not is not p, but
    # given x1 the second is p2(. | x1)); check one heavy x1 explicitly
    x1 = int(np.argmax(np.bincount(out[two, 0], minlength=V)))
    sel = two & (out[:, 0] == x1)
    exp = softmax(base2[(np.arange(V) - x1) % V] / T) * sel.sum()
    assert scipy.stats.chisquare(np.bincount(out[sel, 1], minlength=V), exp).pvalue > 0.01
    assert (acc <= 2).all() and (path[:, 0] == 0).all()


def test_rejection_with_q_equal_p_always_accepts_first_child(orc32):
    rng = np.random.default_rng(5)
    B = 500
    lg = rng.standard_normal((B, 2, V)).astype(np.float32)
    q = softmax(lg).astype(np.float32)
    parent = np.tile(np.array([-1, 0], dtype=np.int32), (B, 1))
    tokens = np.zeros((B, 2), np.int32)
    tokens[:, 1] = rng.integers(0, V, B)
    unif = rng.random((B, 2), dtype=np.float32) * 0.999
    acc, path, out, *_ = orc32.accept_reject(tokens, parent, lg.reshape(-1, V), q.reshape(-1, V), unif, 1.0, seed=1)
    assert (acc == 1).all() and (out[:, 0] == tokens[:, 1]).all()


def test_rejected_token_is_never_the_bonus_when_q_exceeds_p(orc32):
    """After rejecting x (p(x) < q(x)) the residual max(p - q, 0) has no mass on x."""
    B = 2000
    rng = np.random.default_rng(6)
    lg = np.tile(np.log(np.array([0.1] + [0.9 / (V - 1)] * (V - 1))), (B, 2, 1)).astype(np.float32)
    q = np.zeros((B, 2, V), np.float32)
    q[:, :, 0] = 0.9
    q[:, :, 1:] = 0.1 / (V - 1)
    parent = np.tile(np.array([-1, 0], dtype=np.int32), (B, 1))
    tokens = np.zeros((B, 2), np.int32)
    unif = rng.random((B, 2), dtype=np.float32)
    acc, path, out, *_ = orc32.accept_reject(tokens, parent, lg.reshape(-1, V), q.reshape(-1, V), unif, 1.0, seed=2)
    rej = acc == 0
    assert abs(rej.mean() - (1 - 0.1 / 0.9)) < 0.03
    assert (out[rej, 0] != 0).all()


def test_topk_logp_against_scipy(orc64):
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((7, 300)) * 3
    tok, logp = orc64.topk_logp(lg, 5)
    ref = scipy.special.log_softmax(lg, axis=-1)
    order = np.argsort(-lg, axis=-1, kind="stable")[:, :5]
    assert np.array_equal(tok, order)
    assert np.abs(logp - np.take_along_axis(ref, order, axis=-1)).max() < 1e-12
    tie = np.array([[1.0, 2.0, 2.0, 0.0]])
    assert list(orc64.topk_logp(tie, 3)[0][0]) == [1, 2, 0]


def test_topk_index_against_stable_sort(orc32):
    rng = np.random.default_rng(4)
    s = rng.integers(0, 6, size=(50, 16)).astype(np.float32)       # many ties
    idx = orc32.topk_index(s, 4)
    assert np.array_equal(idx, np.argsort(-s, axis=1, kind="stable")[:, :4])


def brute_tree(ct, cp, cs, N):
    C = len(ct)
    depth = [0] * C
    for i in range(1, C):
        depth[i] = depth[cp[i]] + 1
    rest = sorted(range(1, C), key=lambda i: (-cs[i], i))[:N - 1]
    chosen = sorted([0] + rest, key=lambda i: (depth[i], i))
    new = {c: n for n, c in enumerate(chosen)}
    return [ct[c] for c in chosen], [-1 if c == 0 else new[cp[c]] for c in chosen], chosen


def test_build_tree_against_brute_force(orc32):
    rng = np.random.default_rng(8)
    for trial in range(200):
        C = int(rng.integers(2, 12))
        N = int(rng.integers(1, C + 1))
        cp = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, C)], dtype=np.int32)
        cs = np.zeros(C, dtype=np.float32)
        for i in range(1, C):     # log-probabilities: a child never scores above its parent; ties happen
            cs[i] = cs[cp[i]] - float(rng.integers(0, 3)) * 0.5
        ct = rng.integers(0, 100, C).astype(np.int32)
        tokens, parent, sel = orc32.build_tree(ct[None], cp[None], cs[None], N)
        bt, bp, bc = brute_tree(list(ct), list(cp), list(cs), N)
        assert list(tokens[0]) == bt and list(parent[0]) == bp and list(sel[0]) == bc
        assert parent[0, 0] == -1 and all(parent[0, i] < i for i in range(1, N))


def test_build_tree_rejects_unclosed_selection(orc32):
    from oracle.oracle import OracleError
    ct = np.array([[0, 1, 2]], np.int32)
    cp = np.array([[-1, 0, 1]], np.int32)
    cs = np.array([[0.0, -5.0, -1.0]], np.float32)        # child scores above its parent
    with pytest.raises(OracleError):
        orc32.build_tree(ct, cp, cs, 2)


@pytest.mark.parametrize("K,L,count", [(4, 5, 69), (4, 6, 85), (3, 3, 22), (1, 4, 5)])
def test_draft_expansion_candidate_count_and_structure(orc32, K, L, count):
    """1 + K + (L - 1) K^2 candidates (Sec. 4.1, after Eq. 2); scores are cumulative log-probabilities."""
    TINY = configs.TINY
    w = gen.weights_to_numpy(gen.make_weights(TINY, seed=0))
    dw = gen.weights_to_numpy(gen.make_weights(configs.draft_of(TINY), seed=0, draft=True))
    target = orc32.model(TINY, w)
    draft = orc32.model(configs.draft_of(TINY), dw, embed_from=target)
    B, P = 2, 6
    prompts = gen.make_prompts(B, 1, P, TINY["vocab"], seed=1)
    cache = orc32.cache(TINY, B, 64)
    dcache = orc32.cache(draft.cfg, B, 64)
    feat, logits = loop.prefill(orc32, target, cache, prompts)
    root, _ = orc32.row_argmax(logits[:, -1])
    catch_tok = np.concatenate([prompts[:, 1:], root[:, None]], axis=1).astype(np.int32)
    ct, cp, cs = loop.draft_expand(orc32, target, draft, dcache, catch_tok, feat, np.full(B, P, np.int32), K, L)
    assert ct.shape == (B, count) and count == 1 + K + (L - 1) * K * K
    assert (dcache.len == P).all()
    for b in range(B):
        assert cp[b, 0] == -1 and (cp[b, 1:] < np.arange(1, count)).all() and (cp[b, 1:] >= 0).all()
        assert (cs[b, 1:] <= cs[b, cp[b, 1:]] + 1e-6).all() and (cs[b, 1:] < 0).all()
        # siblings are distinct tokens, K per expanded parent
        for u in set(cp[b, 1:]):
            kids = ct[b, 1:][cp[b, 1:] == u]
            assert len(kids) == K and len(set(kids)) == K
        # the first K candidates' probabilities are the draft's top-K at the root: they sum to < 1
        assert np.exp(cs[b, 1:K + 1].astype(np.float64)).sum() < 1.0
    N = min(count, 24)
    tokens, parent, sel = orc32.build_tree(ct, cp, cs, N)
    assert (tokens[:, 0] == root).all()
