"""GPU parity of online draft learning (Sec. 4.2; Alg. 1, the draft training phase) against the CPU oracle, through the
C ABI: the training loss and the gradient of every draft parameter, the AdamW update, and a few whole steps."""
import numpy as np
import pytest
import torch

from synth import configs

pytestmark = pytest.mark.gpu

ODD = dict(name="odd", n_layers=1, d_model=72, n_q_heads=6, n_kv_heads=2, head_dim=12, d_ffn=100, vocab=260, rms_eps=1e-6,
           rope_theta=10000.0, dtype="fp32")
TINY1 = configs.draft_of(configs.TINY)
# grouped-query heads of 128 dims: the tiled attention kernels' other shape (two query heads per kv head, chains that end
# inside a 16-position tile and cross a 64-key tile)
GQA128 = dict(name="gqa128", n_layers=1, d_model=512, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=192, vocab=300, rms_eps=1e-6,
              rope_theta=10000.0, dtype="fp32")


@pytest.fixture(scope="module")
def fg():
    import paper_2509_21792_amd as m
    m.lib()
    assert torch.cuda.is_available()
    return m


@pytest.fixture(scope="module")
def orc():
    from oracle.oracle import Oracle
    return Oracle("f64")


def make_case(fg, cfg, B, T, n_valid, seed):
    rng = np.random.default_rng(seed)
    d, V = cfg["d_model"], cfg["vocab"]
    w = {}
    for k, s in fg.draft_param_shapes(cfg).items():
        w[k] = (rng.standard_normal(s) * (0.05 if len(s) == 2 else 0.05) + (0.0 if len(s) == 2 else 1.0)).astype(np.float32)
    embed = (rng.standard_normal((V, d)) * 0.5).astype(np.float32)
    lm_head = (rng.standard_normal((V, d)) * 0.2).astype(np.float32)
    tokens = rng.integers(0, V, size=(B, T)).astype(np.int32)
    feat_in = rng.standard_normal((B, T, d)).astype(np.float32)
    feat_tgt = (rng.standard_normal((B, T, d)) * 1.5).astype(np.float32)
    return w, embed, lm_head, tokens, feat_in, feat_tgt, np.asarray(n_valid, dtype=np.int32)


def oracle_draft(orc, cfg, w, embed, lm_head):
    layer = {k: w[k] for k in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")}
    target = orc.model(cfg, dict(embed=embed, lm_head=lm_head, final_norm=np.ones(cfg["d_model"]), layers=[layer]))
    return orc.model(cfg, dict(fc=w["fc"], layers=[layer]), embed_from=target)


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("name,cfg,B,T,n_valid", [("tiny", TINY1, 3, 37, [37, 20, 1]), ("odd", ODD, 2, 9, [9, 4]),
                                                  ("tiles", TINY1, 5, 130, [130, 129, 64, 2, 100]),
                                                  ("gqa128", GQA128, 2, 70, [70, 33])])
def test_training_loss_and_gradients_follow_the_oracle(fg, orc, name, cfg, B, T, n_valid):
    print(f"draft training gradients: {name}", flush=True)
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(fg, cfg, B, T, n_valid, 7)
    w_ce = 0.3
    o_loss, o_grad = orc.draft_train(oracle_draft(orc, cfg, w, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
    gw = {k: dev(v) for k, v in w.items()}
    loss, grad = fg.fg_draft_train_grad(cfg, dev(embed), dev(lm_head), gw, dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid), w_ce)
    torch.cuda.synchronize()
    assert np.abs(loss.cpu().numpy() - o_loss).max() <= 1e-5 * max(1.0, float(np.abs(o_loss).max()))
    for k in o_grad:
        got, want = grad[k].cpu().numpy().astype(np.float64), o_grad[k]
        assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max() + 1e-9, (k, np.abs(got - want).max(), np.abs(want).max())
    # a second call on the same inputs is bitwise the same (fixed summation orders, no atomics)
    loss2, grad2 = fg.fg_draft_train_grad(cfg, dev(embed), dev(lm_head), gw, dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid), w_ce)
    torch.cuda.synchronize()
    assert torch.equal(loss, loss2) and all(torch.equal(grad[k], grad2[k]) for k in grad)


def test_adamw_steps_follow_the_oracle(fg):
    from oracle.oracle import Oracle
    orc32 = Oracle("f32")
    cfg = ODD
    rng = np.random.default_rng(1)
    shapes = fg.draft_param_shapes(cfg)
    w = {k: rng.standard_normal(s).astype(np.float32) for k, s in shapes.items()}
    m = {k: np.zeros(s, np.float32) for k, s in shapes.items()}
    v = {k: np.zeros(s, np.float32) for k, s in shapes.items()}
    gw, gm, gv = ({k: dev(a) for k, a in x.items()} for x in (w, m, v))
    for step in range(1, 4):
        g = {k: rng.standard_normal(s).astype(np.float32) for k, s in shapes.items()}
        fg.fg_draft_adamw(cfg, gw, {k: dev(a) for k, a in g.items()}, gm, gv, lr=1e-2, step=step, beta1=0.9, beta2=0.95, eps=1e-8,
                          weight_decay=0.05)
        for k in shapes:
            orc32.adamw(w[k], g[k], m[k], v[k], 1e-2, 0.9, 0.95, 1e-8, 0.05, step)
    torch.cuda.synchronize()
    for k in shapes:
        assert np.abs(gw[k].cpu().numpy() - w[k]).max() <= 2e-6 * max(1.0, float(np.abs(w[k]).max())), k
        assert np.abs(gv[k].cpu().numpy() - v[k]).max() <= 1e-6 * max(1.0, float(np.abs(v[k]).max())), k


def test_training_steps_lower_the_loss_as_the_oracle_does(fg, orc):
    """Five whole steps (gradient + AdamW) on one batch: the GPU's loss trajectory follows the oracle's (fp64) and falls."""
    cfg = ODD
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(fg, cfg, 4, 12, [12, 12, 7, 3], 11)
    w_ce, lr = 0.1, 3e-3
    ow = {k: a.astype(np.float64) for k, a in w.items()}
    om = {k: np.zeros_like(a) for k, a in ow.items()}
    ov = {k: np.zeros_like(a) for k, a in ow.items()}
    gw = {k: dev(a) for k, a in w.items()}
    gm = {k: torch.zeros_like(t) for k, t in gw.items()}
    gv = {k: torch.zeros_like(t) for k, t in gw.items()}
    args = (dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid))
    e, l = dev(embed), dev(lm_head)
    first = None
    for step in range(1, 6):
        o_loss, o_grad = orc.draft_train(oracle_draft(orc, cfg, ow, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
        for k in ow:
            orc.adamw(ow[k], o_grad[k], om[k], ov[k], lr, 0.9, 0.999, 1e-8, 0.01, step)
        loss, grad = fg.fg_draft_train_grad(cfg, e, l, gw, *args, w_ce)
        fg.fg_draft_adamw(cfg, gw, grad, gm, gv, lr=lr, step=step)
        got = loss.cpu().numpy()
        total, o_total = got[0] + w_ce * got[1], o_loss[0] + w_ce * o_loss[1]
        assert abs(total - o_total) <= 1e-4 * o_total, (step, total, o_total)
        first = first if first is not None else total
    assert total < first


def test_online_learning_raises_the_accepted_length(fg):
    """The synthetic analogue of the paper's accepted-length-versus-training-steps figure (Sec. 4.2): a randomly
    initialised draft head is trained on the features and tokens the target's own greedy rollouts leave behind; the
    accepted length of speculative decoding on those rollouts' prompts rises well above its untrained value, and the
    emitted tokens stay those of plain decoding (speculation is lossless whatever the head predicts)."""
    from paper_2509_21792_amd import loop as gloop
    from synth import gen
    model = configs.TINY
    dcfg = configs.draft_of(model)
    tw = gen.make_weights(model, 3, device="cuda")
    dw = gen.make_weights(dcfg, 3, device="cuda", draft=True)
    gm = fg.Model(model, tw)
    B, P, n_new = 8, 24, 40
    prompts = torch.as_tensor(gen.make_prompts(B, 1, P, model["vocab"], 5)).cuda()
    prompts[1::2] = torch.as_tensor(np.random.default_rng(6).integers(0, model["vocab"], size=(B // 2, P)).astype(np.int32)).cuda()
    cap = P + n_new + 80
    slot = torch.arange(B, dtype=torch.int32, device="cuda")

    def rollout(gd):
        """(token lists, mean tokens emitted per verification over the speculative rounds) with draft head gd"""
        table, n_pages = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 1)
        dtable, dn = gen.make_page_table(np.zeros(B, np.int32), cap, 16, 2)
        kv, dkv = fg.KVCache(model, table, n_pages), fg.KVCache(dcfg, dtable, dn)
        ws_t, ws_d = gm.workspace(B * 64, cap), gd.workspace(B * 64, cap)
        first, st = gloop.prefill(gm, gd, kv, dkv, slot, prompts, ws_t, ws_d, max_seq_len=cap)
        outs, hist = gloop.generate(gm, gd, kv, dkv, slot, st, first.cpu().numpy(), np.full(B, n_new, np.int32), 48.0, ws_t, ws_d,
                                    max_seq_len=cap)
        spec = [h for h in hist if h["N"] > 1]
        return outs, sum(h["emitted"] for h in spec) / max(sum(h["B"] for h in spec), 1)

    trainer = gloop.DraftTrainer(dcfg, dw, tw, lr=2e-3, w_ce=0.1)
    outs0, tau0 = rollout(trainer.export(gm))
    # the cached supervision: the target's features over prompt + its own continuation, one pass per sequence
    seqs = torch.as_tensor(np.array([list(prompts[b].cpu().numpy()) + outs0[b] for b in range(B)], dtype=np.int32)).cuda()
    S = seqs.shape[1]
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), S + 16, 16, 3)
    kv = fg.KVCache(model, table, n_pages)
    ws = gm.workspace(B * 64, S + 16)
    feats = []
    for p0 in range(0, S, 64):
        n = min(64, S - p0)
        out = fg.fg_spec_verify(gm, kv, slot, seqs[:, p0:p0 + n].contiguous(), gloop.chain_parent(B, n, "cuda"), ws, max_seq_len=S + 16)
        ident = torch.arange(n, dtype=torch.int32, device="cuda").repeat(B, 1)
        fg.fg_kv_compact(kv, slot, torch.full((B,), n - 1, dtype=torch.int32, device="cuda"), ident)
        feats.append(out["feature"].view(B, n, -1).float())
    feature = torch.cat(feats, dim=1)
    tok, fin, ftg = gloop.training_chains(feature, seqs)
    n_valid = torch.full((B,), S - 1, dtype=torch.int32, device="cuda")
    losses = []
    for _ in range(60):
        losses.append(trainer.step(tok, fin, ftg, n_valid).cpu().numpy())
    # the regression term falls by far; the cross-entropy term falls towards its floor, the entropy of the target's own
    # (near-uniform, with random weights) next-token distribution
    assert losses[-1][0] < 0.2 * losses[0][0] and losses[-1][1] < losses[0][1]
    outs1, tau1 = rollout(trainer.export(gm))
    assert outs1 == outs0                      # lossless: the same tokens with either head
    print(f"accepted tokens per verification: {tau0:.2f} untrained -> {tau1:.2f} after 60 steps; "
          f"loss (reg, ce) {losses[0]} -> {losses[-1]}", flush=True)
    assert tau1 > tau0 + 0.5


def test_matrix_core_mode_follows_the_oracle_to_bf16_rounding(fg, orc):
    """compute="bf16": the step's matrix products on the matrix cores, operands rounded to bf16.  Against the fp64 oracle
    every gradient matrix agrees to about 1 % of its largest entry and points the same way (cosine above 0.999)."""
    cfg = TINY1
    B, T = 4, 64
    w, embed, lm_head, tokens, feat_in, feat_tgt, n_valid = make_case(fg, cfg, B, T, [64, 50, 64, 7], 13)
    w_ce = 0.3
    o_loss, o_grad = orc.draft_train(oracle_draft(orc, cfg, w, embed, lm_head), tokens, feat_in, feat_tgt, n_valid, w_ce)
    gw = {k: dev(v) for k, v in w.items()}
    loss, grad = fg.fg_draft_train_grad(cfg, dev(embed), dev(lm_head), gw, dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid), w_ce,
                                        compute="bf16")
    torch.cuda.synchronize()
    assert np.abs(loss.cpu().numpy() - o_loss).max() <= 2e-2 * float(np.abs(o_loss).max())
    for k in o_grad:
        got, want = grad[k].cpu().numpy().astype(np.float64).ravel(), o_grad[k].ravel()
        cos = float(got @ want / (np.linalg.norm(got) * np.linalg.norm(want)))
        assert cos > 0.999 and np.abs(got - want).max() <= 3e-2 * np.abs(want).max(), (k, cos, np.abs(got - want).max(), np.abs(want).max())
    # the frozen head packed ahead of time: bitwise the same step
    head = dev(lm_head)
    packed = fg.fg_draft_train_pack_head(cfg, head)
    loss2, grad2 = fg.fg_draft_train_grad(cfg, dev(embed), head, gw, dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid), w_ce,
                                          compute="bf16", head_packed=packed)
    torch.cuda.synchronize()
    assert torch.equal(loss, loss2) and all(torch.equal(grad[k], grad2[k]) for k in grad)
    with pytest.raises(fg.FgError):      # fp16 would flush the gradients
        fg.fg_draft_train_grad(cfg, dev(embed), dev(lm_head), gw, dev(tokens), dev(feat_in), dev(feat_tgt), dev(n_valid), w_ce, compute="fp16")
