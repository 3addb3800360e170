"""Pins of the oracle's forward pass (CPU only).

The oracle is checked against things other than itself: torch's fp64 library routines on the special cases
that reduce to a textbook decoder (a chain tree is ordinary causal attention, N = 1 is a plain decode
step), the equivalence of one tree pass with separate passes over each root-to-node path (Sec. 2,
"Verification Strategies"), RoPE's invariants, and independence from batch composition.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import loop
from synth import gen

SMALL = dict(name="small", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50,
             rms_eps=1e-6, rope_theta=10000.0, dtype="fp32")


def torch_chain_logits(cfg, w, tokens, store=None):
    """A Llama-style decoder over full sequences with torch library ops in fp64: tokens [B, T] -> logits, feature.
    store: None, or the 16-bit torch dtype the activations are stored in between the steps of a layer (a cast and back
    at the outputs of both norms, q / k / v after RoPE, the attention output, the SwiGLU output, the LM head's input)."""
    st = (lambda t: t) if store is None else (lambda t: t.to(store).to(torch.float64))
    d, Hq, Hkv, hd = cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    t64 = lambda a: torch.as_tensor(np.asarray(a), dtype=torch.float64)
    B, T = tokens.shape
    h = F.embedding(torch.as_tensor(tokens, dtype=torch.long), t64(w["embed"]))
    pos = torch.arange(T, dtype=torch.float64)
    inv = cfg["rope_theta"] ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang), torch.sin(ang)

    def rope(x):  # x [B, H, T, hd]; pairs (i, i + hd/2)
        x1, x2 = x[..., : hd // 2], x[..., hd // 2:]
        return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)

    for lay in w["layers"]:
        a = st(F.rms_norm(h, (d,), t64(lay["norm_attn"]), cfg["rms_eps"]))
        qkv = F.linear(a, t64(lay["wqkv"]))
        q, k, v = qkv.split([Hq * hd, Hkv * hd, Hkv * hd], dim=-1)
        q = st(rope(q.view(B, T, Hq, hd).transpose(1, 2)))
        k = st(rope(k.view(B, T, Hkv, hd).transpose(1, 2)))
        v = st(v.view(B, T, Hkv, hd).transpose(1, 2))
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        o = st(F.scaled_dot_product_attention(q, k, v, is_causal=True))
        h = h + F.linear(o.transpose(1, 2).reshape(B, T, Hq * hd), t64(lay["wo"]))
        f = st(F.rms_norm(h, (d,), t64(lay["norm_ffn"]), cfg["rms_eps"]))
        h = h + F.linear(st(F.silu(F.linear(f, t64(lay["w_gate"]))) * F.linear(f, t64(lay["w_up"]))), t64(lay["w_down"]))
    feat = st(F.rms_norm(h, (d,), t64(w["final_norm"]), cfg["rms_eps"]))
    return F.linear(feat, t64(w["lm_head"])).numpy(), feat.numpy()


@pytest.fixture(scope="module")
def small_w():
    w = gen.weights_to_numpy(gen.make_weights(SMALL, seed=3))
    # make the weights large enough that attention is far from uniform
    for lay in w["layers"]:
        lay["wqkv"] = lay["wqkv"] * 8
    return w


def test_chain_equals_torch_causal_decoder(orc64, small_w):
    B, T = 3, 11
    tokens = gen.make_prompts(B, 1, T, SMALL["vocab"], seed=5)
    model = orc64.model(SMALL, small_w)
    cache = orc64.cache(SMALL, B, T + 4)
    feat, logits = loop.prefill(orc64, model, cache, tokens)
    ref_logits, ref_feat = torch_chain_logits(SMALL, small_w, tokens)
    assert np.abs(logits - ref_logits).max() < 1e-11
    assert np.abs(feat - ref_feat).max() < 1e-11
    assert (cache.len == T).all()


@pytest.mark.parametrize("kind,store", [("bf16", torch.bfloat16), ("fp16", torch.float16)])
def test_round_act_equals_torch_casts(orc32, orc64, kind, store):
    """The rounding the twin applies is torch's cast: random values over the format's range, exact ties (which go to the
    even neighbour), fp16 subnormals and the ends of its range."""
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-18, 11, 20000))).astype(np.float32)
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -24,
                     65504.0, 65519.0, 65520.0, 70000.0, -65520.0, 0.0, -0.0, 1e-8, 6.1e-5, 5.96e-8], dtype=np.float32)
    x = np.concatenate([x, ties, -ties])
    want = torch.as_tensor(x).to(store).to(torch.float32).numpy()
    for orc in (orc32, orc64):
        got = orc.round_act(x, kind).astype(np.float32)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("kind,store", [("bf16", torch.bfloat16), ("fp16", torch.float16)])
def test_rounding_twin_equals_torch_decoder_with_casts(orc64, small_w, kind, store):
    """The twin rounds at exactly the places the torch decoder with casts does: same logits, same feature, to the fp64
    noise of the arithmetic in between; it differs from the oracle proper by about what that many roundings predict; what
    it hands to the LM head is representable in the format."""
    B, T = 3, 11
    tokens = gen.make_prompts(B, 1, T, SMALL["vocab"], seed=5)
    model = orc64.model(SMALL, small_w, act_round=kind)
    cache = orc64.cache(SMALL, B, T + 4)
    feat, logits = loop.prefill(orc64, model, cache, tokens)
    ref_logits, ref_feat = torch_chain_logits(SMALL, small_w, tokens, store=store)
    assert np.abs(logits - ref_logits).max() < 1e-10
    assert np.abs(feat - ref_feat).max() < 1e-10
    assert np.array_equal(orc64.round_act(feat, kind), feat)
    k = np.asarray(cache.k)[:, :, :T]
    assert np.array_equal(orc64.round_act(k, kind), k)
    plain_logits, _ = torch_chain_logits(SMALL, small_w, tokens)
    rel = np.sqrt(np.mean((logits - plain_logits) ** 2)) / np.sqrt(np.mean(plain_logits ** 2))
    u = (2.0 ** -8 if kind == "bf16" else 2.0 ** -11) / np.sqrt(3.0)
    assert 0.3 * u < rel < 6 * u * np.sqrt(5 * SMALL["n_layers"] + 1), rel


def test_incremental_decode_equals_torch(orc64, small_w):
    """Prefill part of a sequence, then N = 1 decode steps against the cache: same logits as the full pass."""
    B, T, P = 2, 9, 4
    tokens = gen.make_prompts(B, 1, T, SMALL["vocab"], seed=6)
    model = orc64.model(SMALL, small_w)
    cache = orc64.cache(SMALL, B, T)
    loop.prefill(orc64, model, cache, tokens[:, :P])
    ref_logits, _ = torch_chain_logits(SMALL, small_w, tokens)
    for t in range(P, T):
        _, lg = orc64.tree_forward(model, cache, tokens[:, t:t + 1], np.full((B, 1), -1, np.int32))
        cache.len += 1
        assert np.abs(lg - ref_logits[:, t]).max() < 1e-11


def test_f32_oracle_close_to_f64(orc32, orc64, small_w):
    B, T = 2, 12
    tokens = gen.make_prompts(B, 1, T, SMALL["vocab"], seed=7)
    outs = []
    for orc in (orc32, orc64):
        model = orc.model(SMALL, small_w)
        cache = orc.cache(SMALL, B, T)
        outs.append(loop.prefill(orc, model, cache, tokens)[1].astype(np.float64))
    assert np.abs(outs[0] - outs[1]).max() < 2e-5


def random_tree(rng, N):
    return np.array([-1] + [int(rng.integers(0, i)) for i in range(1, N)], dtype=np.int32)


@pytest.mark.parametrize("kind", ["f32", "f64"])
def test_tree_pass_equals_linear_passes(kind, small_w, orc32, orc64):
    """Logits at node i of one tree pass == the last row of a chain pass over root -> i, bit for bit."""
    orc = orc32 if kind == "f32" else orc64
    rng = np.random.default_rng(0)
    B, P, N = 2, 5, 9
    model = orc.model(SMALL, small_w)
    cache = orc.cache(SMALL, B, P + N)
    prompts = gen.make_prompts(B, 1, P, SMALL["vocab"], seed=8)
    loop.prefill(orc, model, cache, prompts)
    parent = np.stack([random_tree(rng, N) for _ in range(B)])
    tokens = rng.integers(0, SMALL["vocab"], size=(B, N)).astype(np.int32)
    base = cache.copy()
    feat, logits = orc.tree_forward(model, cache, tokens, parent)
    logits = logits.reshape(B, N, -1)
    feat = feat.reshape(B, N, -1)
    for b in range(B):
        for i in range(N):
            chain = []
            u = i
            while u >= 0:
                chain.append(u)
                u = parent[b, u]
            chain = chain[::-1]
            c2 = base.copy()
            sl = np.array([b], dtype=np.int32)
            f2, l2 = orc.tree_forward(model, c2, tokens[b, chain].reshape(1, -1), loop.chain_parent(1, len(chain)),
                                      slot=sl)
            assert np.array_equal(l2[-1], logits[b, i])
            assert np.array_equal(f2[-1], feat[b, i])


def test_batch_invariance(orc32, small_w):
    """A sequence's result does not depend on what else is in the batch or on its slot."""
    rng = np.random.default_rng(1)
    P, N = 6, 5
    model = orc32.model(SMALL, small_w)
    prompts = gen.make_prompts(4, 1, P, SMALL["vocab"], seed=9)
    parent = np.stack([random_tree(rng, N) for _ in range(4)])
    tokens = rng.integers(0, SMALL["vocab"], size=(4, N)).astype(np.int32)
    cache = orc32.cache(SMALL, 4, P + N)
    loop.prefill(orc32, model, cache, prompts)
    _, full = orc32.tree_forward(model, cache, tokens, parent)
    full = full.reshape(4, N, -1)
    c2 = orc32.cache(SMALL, 7, P + N)
    slot = np.array([5, 2], dtype=np.int32)
    loop.prefill(orc32, model, c2, prompts[[3, 1]], slot=slot)
    _, part = orc32.tree_forward(model, c2, tokens[[3, 1]], parent[[3, 1]], slot=slot)
    assert np.array_equal(part.reshape(2, N, -1), full[[3, 1]])


def test_rope_invariants(orc64):
    rng = np.random.default_rng(2)
    hd = 16
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    for pos in (0, 1, 17, 4095):
        assert abs(np.linalg.norm(orc64.rope_head(q, pos)) - np.linalg.norm(q)) < 1e-12
    assert np.allclose(orc64.rope_head(q, 0), q)
    # the rotated dot product depends on the position difference only
    d0 = orc64.rope_head(q, 40) @ orc64.rope_head(k, 33)
    d1 = orc64.rope_head(q, 1007) @ orc64.rope_head(k, 1000)
    assert abs(d0 - d1) < 1e-9
    # first pair rotates by exactly pos radians: (1, 0) -> (cos, sin)
    e = np.zeros(hd); e[0] = 1.0
    r = orc64.rope_head(e, 3)
    assert abs(r[0] - np.cos(3.0)) < 1e-15 and abs(r[hd // 2] - np.sin(3.0)) < 1e-15
    # last pair rotates by pos * theta^(-(hd-2)/hd)
    e = np.zeros(hd); e[hd // 2 - 1] = 1.0
    r = orc64.rope_head(e, 5, theta=10000.0)
    ang = 5 * 10000.0 ** (-(hd - 2) / hd)
    assert abs(r[hd // 2 - 1] - np.cos(ang)) < 1e-15 and abs(r[hd - 1] - np.sin(ang)) < 1e-15


def test_in_round_nodes_over_several_calls(orc64, small_w):
    """Nodes appended over two calls (n_prev > 0) give the same rows as one call with all of them."""
    rng = np.random.default_rng(3)
    B, P, N = 2, 4, 8
    model = orc64.model(SMALL, small_w)
    cache = orc64.cache(SMALL, B, P + N)
    loop.prefill(orc64, model, cache, gen.make_prompts(B, 1, P, SMALL["vocab"], seed=10))
    parent = np.stack([random_tree(rng, N) for _ in range(B)])
    tokens = rng.integers(0, SMALL["vocab"], size=(B, N)).astype(np.int32)
    c1 = cache.copy()
    _, one = orc64.tree_forward(model, c1, tokens, parent)
    c2 = cache.copy()
    _, a = orc64.tree_forward(model, c2, tokens[:, :3], parent[:, :3])
    _, b = orc64.tree_forward(model, c2, tokens[:, 3:], parent, n_prev=3)
    two = np.concatenate([a.reshape(B, 3, -1), b.reshape(B, N - 3, -1)], axis=1)
    assert np.array_equal(one.reshape(B, N, -1), two)


def test_bad_trees_are_errors(orc32, small_w):
    from oracle.oracle import OracleError
    model = orc32.model(SMALL, small_w)
    cache = orc32.cache(SMALL, 1, 8)
    with pytest.raises(OracleError):
        orc32.tree_forward(model, cache, np.zeros((1, 3), np.int32), np.array([[-1, 1, 0]], np.int32))
    with pytest.raises(OracleError):  # capacity
        orc32.tree_forward(model, cache, np.zeros((1, 9), np.int32), loop.chain_parent(1, 9))
