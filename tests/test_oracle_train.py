"""Pins of the oracle's draft-training step (Sec. 4.2 "Draft Model Learning with Online Target Feedback"; Alg. 1, the
draft training phase), CPU only: the gradients against central finite differences of the oracle's own loss in fp64, the
loss and all gradients against the same forward written with torch library ops (embedding, linear, scaled-dot-product
attention, silu, smooth_l1_loss, log_softmax) and differentiated by autograd, and the optimiser step against
torch.optim.AdamW."""
import numpy as np
import pytest
import torch

MODEL = dict(name="train-pin", n_layers=1, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24, vocab=12,
             rms_eps=1e-6, rope_theta=10000.0, dtype="fp32")
SHAPES = lambda c: dict(fc=(c["d_model"], 2 * c["d_model"]),
                        wqkv=((c["n_q_heads"] + 2 * c["n_kv_heads"]) * c["head_dim"], c["d_model"]),
                        wo=(c["d_model"], c["n_q_heads"] * c["head_dim"]), w_gate=(c["d_ffn"], c["d_model"]),
                        w_up=(c["d_ffn"], c["d_model"]), w_down=(c["d_model"], c["d_ffn"]), norm_attn=(c["d_model"],),
                        norm_ffn=(c["d_model"],))


def make_case(seed, B=2, T=5):
    rng = np.random.default_rng(seed)
    c = MODEL
    w = {k: rng.standard_normal(s) * (0.4 if len(s) == 2 else 0.1) + (0.0 if len(s) == 2 else 1.0) for k, s in SHAPES(c).items()}
    embed = rng.standard_normal((c["vocab"], c["d_model"]))
    lm_head = rng.standard_normal((c["vocab"], c["d_model"])) * 0.7
    tokens = rng.integers(0, c["vocab"], size=(B, T)).astype(np.int32)
    feat_in = rng.standard_normal((B, T, c["d_model"]))
    feat_tgt = rng.standard_normal((B, T, c["d_model"])) * 1.5          # some |h - f| above 1: both branches of the smooth L1
    n_valid = np.array([T, max(T - 2, 1)][:B], dtype=np.int32)
    return w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid


def oracle_models(orc, w, embed, lm_head):
    target = orc.model(MODEL, dict(embed=embed, lm_head=lm_head, final_norm=np.ones(MODEL["d_model"]),
                                   layers=[{k: w[k] for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")}]))
    draft = orc.model(MODEL, dict(fc=w["fc"], layers=[{k: w[k] for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn",
                                                                           "norm_ffn")}]), embed_from=target)
    return draft


def torch_loss(w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid, w_ce):
    """The training loss from torch library ops (fp64); w: dict of tensors with requires_grad."""
    c = MODEL
    d, Hq, Hkv, hd = c["d_model"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"]
    B, T = tokens.shape
    E, LM = torch.as_tensor(embed), torch.as_tensor(lm_head)

    def rms(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + c["rms_eps"]) * g

    def rope(x):                                           # x [B, T, H, hd], position = index in the chain
        half = hd // 2
        inv = c["rope_theta"] ** (-2.0 * torch.arange(half, dtype=torch.float64) / hd)
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
        cos, sin = ang.cos()[None, :, None, :], ang.sin()[None, :, None, :]
        a, b = x[..., :half], x[..., half:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)

    x = torch.cat([torch.nn.functional.embedding(torch.as_tensor(tokens).long(), E), torch.as_tensor(feat_in)], dim=-1)
    h = torch.nn.functional.linear(x, w["fc"])
    qkv = torch.nn.functional.linear(rms(h, w["norm_attn"]), w["wqkv"])
    q = rope(qkv[..., :Hq * hd].reshape(B, T, Hq, hd))
    k = rope(qkv[..., Hq * hd:(Hq + Hkv) * hd].reshape(B, T, Hkv, hd))
    v = qkv[..., (Hq + Hkv) * hd:].reshape(B, T, Hkv, hd)
    k, v = k.repeat_interleave(Hq // Hkv, dim=2), v.repeat_interleave(Hq // Hkv, dim=2)
    att = torch.nn.functional.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2), is_causal=True)
    h = h + torch.nn.functional.linear(att.transpose(1, 2).reshape(B, T, Hq * hd), w["wo"])
    a = rms(h, w["norm_ffn"])
    h = h + torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(a, w["w_gate"])) *
                                       torch.nn.functional.linear(a, w["w_up"]), w["w_down"])
    ft = torch.as_tensor(feat_tgt)
    valid = torch.arange(T)[None, :] < torch.as_tensor(n_valid)[:, None]
    reg = torch.nn.functional.smooth_l1_loss(h, ft, reduction="none", beta=1.0).mean(-1)
    logq = torch.log_softmax(torch.nn.functional.linear(h, LM), dim=-1)
    p = torch.softmax(torch.nn.functional.linear(ft, LM), dim=-1)
    ce = -(p * logq).sum(-1)
    n = valid.sum()
    return (reg * valid).sum() / n, (ce * valid).sum() / n


@pytest.mark.parametrize("seed", [0, 1])
def test_draft_training_gradients_against_torch_autograd(orc64, seed):
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(seed)
    w_ce = 0.3
    loss, grads = orc64.draft_train(oracle_models(orc64, w, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
    tw = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()}
    reg, ce = torch_loss(tw, embed, lm_head, tokens, feat_in, feat_tgt, n_valid, w_ce)
    (reg + w_ce * ce).backward()
    assert abs(loss[0] - reg.item()) < 1e-12 and abs(loss[1] - ce.item()) < 1e-12
    for k in w:
        want = tw[k].grad.numpy()
        assert np.abs(grads[k] - want).max() <= 1e-10 * max(1.0, np.abs(want).max()), k
        assert np.abs(want).max() > 1e-6, k                     # every parameter really receives a gradient


def test_draft_training_gradients_against_finite_differences(orc64):
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(3)
    w_ce = 0.2

    def total(ww):
        l, _ = orc64.draft_train(oracle_models(orc64, ww, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
        return float(l[0]) + w_ce * float(l[1])
    _, grads = orc64.draft_train(oracle_models(orc64, w, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
    rng = np.random.default_rng(5)
    eps = 1e-6
    for k, g in grads.items():
        for _ in range(4):
            idx = tuple(int(rng.integers(0, s)) for s in g.shape)
            wp, wm = {n: a.copy() for n, a in w.items()}, {n: a.copy() for n, a in w.items()}
            wp[k][idx] += eps
            wm[k][idx] -= eps
            fd = (total(wp) - total(wm)) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd)), (k, idx, fd, g[idx])


def test_padding_behind_the_valid_entries_changes_nothing(orc64):
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(4, B=2, T=6)
    draft = oracle_models(orc64, w, embed, lm_head)
    n_valid = np.array([6, 3], np.int32)
    l0, g0 = orc64.draft_train(draft, tokens, feat_in, feat_tgt, n_valid)
    rng = np.random.default_rng(9)
    tokens2, fi2, ft2 = tokens.copy(), feat_in.copy(), feat_tgt.copy()
    tokens2[1, 3:] = rng.integers(0, MODEL["vocab"], size=3)
    fi2[1, 3:] = rng.standard_normal((3, MODEL["d_model"]))
    ft2[1, 3:] = rng.standard_normal((3, MODEL["d_model"]))
    l1, g1 = orc64.draft_train(draft, tokens2, fi2, ft2, n_valid)
    assert np.array_equal(l0, l1) and all(np.array_equal(g0[k], g1[k]) for k in g0)


def test_adamw_against_torch(orc64):
    rng = np.random.default_rng(0)
    p0 = rng.standard_normal(50)
    p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=1e-2, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.05)
    for step in range(1, 5):
        g = rng.standard_normal(50)
        orc64.adamw(p, g, m, v, 1e-2, 0.9, 0.95, 1e-8, 0.05, step)
        tp.grad = torch.tensor(g)
        opt.step()
        assert np.abs(p - tp.detach().numpy()).max() < 1e-13
