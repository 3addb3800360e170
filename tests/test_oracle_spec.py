"""Pins of the oracle's speculative step (CPU only): what the paper and the mathematics fix.

- Speculative decoding is accuracy-preserving (Sec. 1, Sec. 2): greedy speculative output equals plain greedy
  autoregressive output token for token, whatever the draft proposes.
- The average acceptance length (appendix, "Average Acceptance Length") has a closed form under planted agreement.
- The compacted cache is the cache plain decoding would have written.
"""
import numpy as np
import pytest

from oracle import loop
from synth import configs, gen

TINY = configs.TINY


@pytest.fixture(scope="module")
def tiny(orc32):
    cfg = configs.CONFIGS["cfg1"]
    w = gen.weights_to_numpy(gen.make_weights(TINY, seed=cfg["seed"]))
    dw = gen.weights_to_numpy(gen.make_weights(configs.draft_of(TINY), seed=cfg["seed"], draft=True))
    target = orc32.model(TINY, w)
    draft = orc32.model(configs.draft_of(TINY), dw, embed_from=target)
    prompts = gen.make_prompts(cfg["B"], cfg["group"], cfg["prompt_len"], TINY["vocab"], cfg["seed"])
    return cfg, target, draft, prompts


def ar_reference(orc, target, prompts, n_new):
    B, P = prompts.shape
    cache = orc.cache(target.cfg, B, P + n_new + 8)
    feat, logits = loop.prefill(orc, target, cache, prompts)
    root, _ = orc.row_argmax(logits[:, -1])
    rest, margins = loop.greedy_ar(orc, target, cache, root, n_new - 1)
    return np.concatenate([root[:, None], rest], axis=1), cache, feat


def test_config1_spec_with_real_draft_equals_ar(orc32, tiny):
    """Config 1 end to end: chain depth 4 from the 1-layer draft head, greedy, 64 new tokens, seed 0."""
    cfg, target, draft, prompts = tiny
    B, P, n_new, N = cfg["B"], cfg["prompt_len"], cfg["new_tokens"], cfg["N"]
    ref, ref_cache, _ = ar_reference(orc32, target, prompts, n_new)

    cache = orc32.cache(TINY, B, P + n_new + N + 8)
    dcache = orc32.cache(draft.cfg, B, P + n_new + N + 8)
    feat, logits = loop.prefill(orc32, target, cache, prompts)
    root, _ = orc32.row_argmax(logits[:, -1])
    outs = [[int(root[b])] for b in range(B)]
    # entries the draft has not seen: (token t+1, feature t) for the whole prompt
    catch_tok = np.concatenate([prompts[:, 1:], root[:, None]], axis=1).astype(np.int32)
    catch_feat = feat
    n_valid = np.full(B, P, dtype=np.int32)
    cur = root.copy()
    total_acc = 0
    rounds = 0
    while min(len(o) for o in outs) < n_new:
        ct, cp, cs = loop.draft_expand(orc32, target, draft, dcache, catch_tok, catch_feat, n_valid, K=1, L=N - 1)
        assert ct.shape[1] == 1 + 1 + (N - 2) * 1          # 1 + K + (L-1) K^2 candidates
        tokens, parent, sel = orc32.build_tree(ct, cp, cs, N)
        assert (tokens[:, 0] == cur).all()
        hidden, lg = orc32.tree_forward(target, cache, tokens, parent)
        acc, path, out, fin, _, _ = orc32.accept_greedy(tokens, parent, lg)
        orc32.kv_compact(cache, TINY, acc, path)
        hidden = hidden.reshape(B, N, -1)
        kin = int(acc.max()) + 1
        catch_tok = np.zeros((B, kin), np.int32)
        catch_feat = np.zeros((B, kin, TINY["d_model"]), np.float32)
        for b in range(B):
            a = acc[b]
            outs[b].extend(int(t) for t in out[b, :a + 1])
            catch_tok[b, :a + 1] = out[b, :a + 1]
            catch_feat[b, :a + 1] = hidden[b, path[b, :a + 1]]
            cur[b] = out[b, a]
        n_valid = (acc + 1).astype(np.int32)
        total_acc += int(acc.sum())
        rounds += 1
    got = np.array([o[:n_new] for o in outs])
    assert np.array_equal(got, ref)
    assert rounds <= n_new


def planted_tree_maker(ref_tokens, N, spec, p, vocab, seed):
    """Trees whose principal path carries the true continuation with probability p per node."""
    def make(slot, roots, rnd, outs):
        b_n = len(slot)
        parent, principal = gen.make_trees(spec, b_n, N, seed + 1000 * rnd)
        nxt = np.zeros((b_n, principal.shape[1]), dtype=np.int32)
        for j, b in enumerate(slot):
            done = len(outs[b])            # tokens already emitted after the first (root) one
            cont = ref_tokens[b, done + 1: done + 1 + principal.shape[1]]
            nxt[j, :len(cont)] = cont
        tokens, _ = gen.plant_tokens(parent, principal, roots, nxt, p, vocab, seed + 77 * rnd)
        return tokens, parent
    return make


@pytest.mark.parametrize("spec,N,p", [(("chain", 4), 5, 0.7), (("tree", 3, 4, 12), 12, 0.6),
                                      (("tree", 4, 5, 24), 24, 1.0), (("chain", 1), 2, 0.0)])
def test_spec_with_planted_trees_equals_ar(orc32, tiny, spec, N, p):
    """Accepted paths of every length occur (planted agreement) and the output is still the AR output."""
    cfg, target, _, prompts = tiny
    B, P, n_new = 4, cfg["prompt_len"], 40
    prompts = prompts[[0, 1, 4, 5]]
    ref, ref_cache, _ = ar_reference(orc32, target, prompts, n_new + 1)
    cache = orc32.cache(TINY, B, P + n_new + N + 8)
    _, logits = loop.prefill(orc32, target, cache, prompts)
    root, _ = orc32.row_argmax(logits[:, -1])
    assert np.array_equal(root, ref[:, 0])
    outs, stats = loop.spec_generate(orc32, target, cache, root, n_new,
                                     planted_tree_maker(ref, N, spec, p, TINY["vocab"], seed=5))
    got = np.array(outs)
    assert np.array_equal(got, ref[:, 1:n_new + 1])
    if p == 1.0:
        assert stats["verifications"] < B * n_new / 3
    if p == 0.0:
        assert stats["accepted"] == stats["verifications"]      # one token (the bonus) per verification
    # the cache left behind equals the cache plain decoding wrote (same tokens at the same positions)
    L = int(cache.len.min())
    assert L >= P + n_new - 1
    for b in range(B):
        Lb = min(int(cache.len[b]), int(ref_cache.len[b]))
        assert np.array_equal(cache.k[:, b, :Lb], ref_cache.k[:, b, :Lb])
        assert np.array_equal(cache.v[:, b, :Lb], ref_cache.v[:, b, :Lb])


def test_live_set_shrinks_on_eos(orc32, tiny):
    cfg, target, _, prompts = tiny
    B, P, n_new, N = 4, cfg["prompt_len"], 24, 5
    prompts = prompts[[0, 1, 4, 5]]
    ref, _, _ = ar_reference(orc32, target, prompts, n_new + 1)
    eos = int(ref[2, 7])                       # sequence 2 ends at its 7th generated token
    cache = orc32.cache(TINY, B, P + n_new + N + 8)
    _, logits = loop.prefill(orc32, target, cache, prompts)
    root, _ = orc32.row_argmax(logits[:, -1])
    outs, stats = loop.spec_generate(orc32, target, cache, root, n_new,
                                     planted_tree_maker(ref, N, ("chain", 4), 0.8, TINY["vocab"], seed=9), eos_id=eos)
    for b in range(B):
        want = list(ref[b, 1:n_new + 1])
        if eos in want:
            want = want[:want.index(eos) + 1]
        assert outs[b] == want
    hist = stats["live_history"]
    assert hist[0] == B and hist[-1] < B and all(x >= y for x, y in zip(hist, hist[1:]))
    # tau = accepted tokens / sum of live sequences over the verification steps
    assert stats["verifications"] == sum(hist)
    assert stats["accepted"] == sum(len(o) for o in outs)


@pytest.mark.parametrize("p,L,want", [(0.7, 5, 2.941), (0.65, 6, 2.717), (0.6, 3, 2.176), (0.6, 1, 1.6)])
def test_tau_closed_form(orc32, p, L, want):
    """With agreement planted at rate p along a principal path of depth L, E[emitted tokens per verification]
    = 1 + p (1 - p^L) / (1 - p)."""
    closed = 1 + p * (1 - p ** L) / (1 - p)
    assert abs(closed - want) < 5e-4
    B, V = 20000, 5000
    N = L + 3
    rng = np.random.default_rng(4)
    parent, principal = gen.make_trees(("tree", 3, L, N), B, N, seed=1)
    truth = rng.integers(0, V, size=(B, L)).astype(np.int32)
    tokens, hit = gen.plant_tokens(parent, principal, np.zeros(B, np.int32), truth, p, V, seed=2)
    # the target's token after a node on the principal path is the next true token; elsewhere anything
    target_tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    target_tok[:, 0] = truth[:, 0]
    for l in range(L - 1):
        target_tok[np.arange(B), principal[:, l]] = truth[:, l + 1]
    acc, path, out, fin = orc32.walk(tokens, parent, target_tok)
    tau = (acc + 1).mean()
    sd = np.sqrt((acc + 1).var() / B)
    assert abs(tau - closed) < 5 * sd + 2e-3
    # what the walk returns is a valid root-to-node path whose tokens are the target's
    for b in range(0, B, 97):
        a = acc[b]
        assert path[b, 0] == 0 and all(parent[b, path[b, j]] == path[b, j - 1] for j in range(1, a + 1))
        assert all(tokens[b, path[b, j]] == target_tok[b, path[b, j - 1]] for j in range(1, a + 1))
        assert out[b, a] == target_tok[b, path[b, a]]
        assert all(path[b, j] > path[b, j - 1] for j in range(1, a + 1))


def test_walk_takes_lowest_child_on_duplicates_and_cuts_at_eos(orc32):
    parent = np.array([[-1, 0, 0, 1, 2]], dtype=np.int32)
    tokens = np.array([[9, 5, 5, 7, 8]], dtype=np.int32)         # two children of the root carry token 5
    tt = np.array([[5, 7, 8, 3, 4]], dtype=np.int32)
    acc, path, out, fin = orc32.walk(tokens, parent, tt)
    assert acc[0] == 2 and list(path[0, :3]) == [0, 1, 3] and list(out[0, :3]) == [5, 7, 3] and fin[0] == 0
    acc, path, out, fin = orc32.walk(tokens, parent, tt, eos_id=7)
    assert acc[0] == 1 and list(out[0, :2]) == [5, 7] and fin[0] == 1
    acc, path, out, fin = orc32.walk(tokens, parent, tt, eos_id=5)
    assert acc[0] == 0 and out[0, 0] == 5 and fin[0] == 1


def test_kv_compact_moves_path_and_bumps_length(orc32):
    cfg = dict(n_layers=2, n_kv_heads=2, head_dim=4)
    cache = orc32.cache(cfg, 3, 16)
    rng = np.random.default_rng(0)
    cache.k[:] = rng.standard_normal(cache.k.shape)
    cache.v[:] = rng.standard_normal(cache.v.shape)
    cache.len[:] = [3, 5, 0]
    before = cache.copy()
    path = np.array([[0, 2, 5, -1, -1, -1], [0, -1, -1, -1, -1, -1]], dtype=np.int32)
    orc32.kv_compact(cache, cfg, np.array([2, 0]), path, slot=np.array([1, 0]))
    assert list(cache.len) == [4, 8, 0]
    for j, s in enumerate([0, 2, 5]):
        assert np.array_equal(cache.k[:, 1, 5 + j], before.k[:, 1, 5 + s])
        assert np.array_equal(cache.v[:, 1, 5 + j], before.v[:, 1, 5 + s])
    assert np.array_equal(cache.k[:, 0, :4], before.k[:, 0, :4])
    assert np.array_equal(cache.k[:, 2], before.k[:, 2])
    from oracle.oracle import OracleError
    with pytest.raises(OracleError):      # a path must increase
        orc32.kv_compact(cache, cfg, np.array([2]), np.array([[0, 3, 2, -1]], np.int32), slot=np.array([2]))


def test_adaptive_loop_equals_ar_and_follows_the_rule(orc32, tiny):
    """Alg. 1 with the concurrency rule in the loop: ragged budgets make the live set decay from 8 to 1, the plan is
    re-derived every round, rounds with N = 1 are plain decoding; the emitted tokens are still exactly the
    autoregressive ones, cut at each sequence's budget."""
    cfg, target, draft, prompts = tiny
    B, P = cfg["B"], cfg["prompt_len"]
    budgets = np.array([6, 40, 17, 64, 9, 25, 33, 12], dtype=np.int32)[:B]
    n_new = int(budgets.max())
    ref, _, _ = ar_reference(orc32, target, prompts, n_new)
    cache = orc32.cache(TINY, B, P + n_new + 72)
    dcache = orc32.cache(draft.cfg, B, P + n_new + 72)
    feat, logits = loop.prefill(orc32, target, cache, prompts)
    root, _ = orc32.row_argmax(logits[:, -1])
    catch_tok = np.concatenate([prompts[:, 1:], root[:, None]], axis=1).astype(np.int32)
    c_peak = 12.0                               # N = floor(12 / B_cur): 1, 1, 2, 2, 3, 4, 6, 12 as B_cur falls from 8 to 1
    outs, hist = loop.adaptive_generate(orc32, target, draft, cache, dcache, catch_tok, feat, np.full(B, P, np.int32), root,
                                        budgets, c_peak, alpha=0.5, K_max=2, L_max=4)
    for b in range(B):
        assert outs[b] == [int(t) for t in ref[b, :budgets[b]]], b
    live = [h["B"] for h in hist]
    assert live[0] == B and live[-1] >= 1 and all(x >= y for x, y in zip(live, live[1:]))
    for h in hist:
        assert (h["N"], h["K"], h["L"]) == orc32.plan(h["B"], c_peak, 0.5, 2, 4, 64)
    assert any(h["N"] == 1 for h in hist) and any(h["N"] > 1 for h in hist)
    assert sum(h["emitted"] for h in hist) == int(budgets.sum()) - B
