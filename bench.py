#!/usr/bin/env python3
"""Benchmark of the speculative-verify hot path on one MI355X.

One "step" = one pass of the hot path over one batch: plan (host) -> L_draft draft steps + frontier updates +
rerank -> spec_verify -> spec_accept -> kv_compact -> accept lengths to the host.  Inputs (weights, paged KV cache, planted
draft trees) are resident in HBM before the timed region; the cache lengths are reset between steps so every step
sees the same ragged shape.  Prints ONE JSON line: the metric (accepted tokens/s of the whole round), the round /
verify / draft times, the step's fractions of the HBM and MFMA peaks, `roofline` for the dominant kernel (the gate/up
GEMM, timed with HIP events inside the timed region), the B = 8 points and `cpu_baseline` (the oracle on a sample).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM = 8.0e12          # B/s, MI355X HBM3E
PEAK_MFMA = 2516.6e12      # flop/s, dense bf16 / fp16 MFMA
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of that kernel at the
# benchmark's shape (bench.py --gemm gate_up --rows M), scaled by what the same counters read for the library's copy probe
# (FETCH_SIZE x 2.00, WRITE_SIZE x 1.00).  A recorded measurement, keyed by (workload, rows M); other workloads report null.
MEASURED_C_PEAK = 64       # knee of the 7B-class latency curve on the log2 batch axis (bench.py --sweep / --gen measure it afresh)
MEASURED_TRAFFIC = {("cfg4", 2048): 929.9e6 + 77.6e6,      # profiles/bench_cfg4_b256_n8_hbm_traffic_pmc.txt
                    ("b8", 8): 277.3e6 + 0.3e6}            # same file, rows "M=8"


def model_bytes_flops(model, M, lengths, N):
    """Algorithmic bytes and flops of one verify step (what the method itself must move / compute)."""
    d, Hq, Hkv, hd, F, V, nl = (model[k] for k in ("d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "n_layers"))
    per_layer = (Hq + 2 * Hkv) * hd * d + d * Hq * hd + 2 * F * d + d * F
    params = nl * per_layer + V * d
    kv_per_tok = 2 * Hkv * hd * 2 * nl
    sumL = int(np.sum(lengths))
    byts = 2 * params + M * d * 2 + sumL * kv_per_tok + M * kv_per_tok + M * d * 2 + M * 12
    gemm_flops = 2.0 * M * params
    attn_flops = 4.0 * Hq * hd * nl * float(np.sum((lengths + (N + 1) / 2.0) * N))
    return dict(params=params, bytes=float(byts), weight_bytes=2.0 * params, kv_bytes=float(sumL * kv_per_tok),
                flops=gemm_flops + attn_flops, gemm_flops=gemm_flops, attn_flops=attn_flops)


class Workload:
    """A model, a batch of ragged paged caches and a planted draft tree, all on the device."""

    def __init__(self, name, dtype, seed=0, B=None, N=None, n_layers=None, kv=None, verbose=False, with_draft=True):
        import torch
        import paper_2509_21792_amd as fg
        from synth import configs, gen
        self.fg, self.torch = fg, torch
        cfg = dict(configs.CONFIGS[name])
        model = configs.with_dtype(cfg["model"], dtype)
        if n_layers:
            model = configs.scaled(model, n_layers)
        self.cfg, self.model, self.name = cfg, model, name
        self.B = B or cfg["B"]
        self.N = N or cfg["N"]
        lo, hi = kv or (cfg["kv_lo"], cfg["kv_hi"])
        pd = configs.PLAN_DEFAULTS
        # the tree shape is what the concurrency rule gives for C_peak = B * N (Eq. 1-3)
        self.plan = fg.fg_plan(self.B, float(self.B * self.N), pd["alpha"], pd["K_max"], pd["L_max"], pd["N_cap"])
        Np, Kd, Ld = self.plan
        if cfg["tree"][0] in ("chain", "tree") and not N:
            self.spec = cfg["tree"]                      # the configuration pins its own shape
        else:
            assert Np == self.N, (self.plan, self.N)
            self.spec = ("tree", max(Kd, 1), max(Ld, 1), self.N)
        t0 = time.time()
        self.weights = gen.make_weights(model, seed, device="cuda")
        self.gm = fg.Model(model, self.weights)
        self.lengths = gen.make_kv_lengths(self.B, lo, hi, seed)
        self.lengths[0], self.lengths[-1] = lo, hi
        table, n_pages = gen.make_page_table(self.lengths, self.N + 1, 16, seed)
        self.kv = fg.KVCache(model, table, n_pages)
        for b in range(self.B):
            k, v = gen.make_prefix_kv(model, int(self.lengths[b]), seed, b, device="cuda")
            self.kv.write_prefix(b, k, v)
        self.len0 = self.kv.seq_len.clone()
        self.cap = int(self.lengths.max()) + self.N + 1
        self.slot = torch.arange(self.B, dtype=torch.int32, device="cuda")
        self.ws = self.gm.workspace(self.B * self.N, self.cap)
        self.parent, self.principal = gen.make_trees(self.spec, self.B, self.N, seed + 2)
        rng = np.random.default_rng(seed + 3)
        self.root = rng.integers(0, model["vocab"], size=self.B).astype(np.int32)
        nxt = self.greedy_continuation(self.principal.shape[1])
        tokens, self.hit = gen.plant_tokens(self.parent, self.principal, self.root, nxt, cfg["plant_p"] or 0.0,
                                            model["vocab"], seed + 4)
        self.tokens_d = torch.as_tensor(tokens).cuda()
        self.parent_d = torch.as_tensor(self.parent).cuda()
        self.max_seq_len = int(self.lengths.max()) + self.N
        # the draft head, its own 1-layer paged cache (synthetic prefix of the same lengths) and the pending
        # catch-up entries a previous round would have left (accept lengths drawn at the planted rate)
        self.K_draft, self.L_draft = Kd, Ld
        self.draft_ready = False
        if with_draft and Kd > 0 and Ld > 0:
            from paper_2509_21792_amd import loop as gloop
            self.gloop = gloop
            dcfg = configs.draft_of(model)
            self.gd = fg.Model(dcfg, gen.make_weights(dcfg, seed, device="cuda", draft=True), target=self.gm)
            dtable, dn = gen.make_page_table(self.lengths, Ld + 1 + (Ld - 1) * Kd + 1, 16, seed + 5)
            self.dkv = fg.KVCache(dcfg, dtable, dn)
            for b in range(self.B):
                k, v = gen.make_prefix_kv(dcfg, int(self.lengths[b]), seed + 6, b, device="cuda")
                self.dkv.write_prefix(b, k, v)
            self.dlen0 = self.dkv.seq_len.clone()
            Kin = Ld + 1
            self.d_max_len = int(self.lengths.max()) + Kin + (Ld - 1) * Kd
            self.ws_d = self.gd.workspace(self.B * max(Kin, Kd), self.d_max_len)
            td = torch.bfloat16 if dtype == "bf16" else torch.float16
            g = torch.Generator(device="cuda").manual_seed(seed + 7)
            catch_tok = torch.randint(0, model["vocab"], (self.B, Kin), generator=g, device="cuda", dtype=torch.int32)
            catch_feat = torch.randn((self.B, Kin, model["d_model"]), generator=g, device="cuda").to(td)
            last = torch.as_tensor(np.minimum(self.hit.cumprod(axis=1).sum(axis=1), Ld).astype(np.int32)).cuda()
            self.spec_state = gloop.SpecState(catch_tok, catch_feat, last)
            self.draft_ready = True
        torch.cuda.synchronize()
        if verbose:
            print(f"# workload {name} {dtype}: B={self.B} N={self.N} plan={self.plan} sumL={int(self.lengths.sum())} "
                  f"set-up {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    def greedy_continuation(self, depth):
        """The target's own next tokens after the root, by `depth` plain decode steps of the HIP path (set-up, untimed)."""
        fg, torch = self.fg, self.torch
        B = self.B
        out = np.zeros((B, depth), dtype=np.int32)
        cur = torch.as_tensor(self.root).cuda().view(B, 1)
        par = torch.full((B, 1), -1, dtype=torch.int32, device="cuda")
        zero = torch.zeros(B, dtype=torch.int32, device="cuda")
        path = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
        for l in range(depth):
            o = fg.fg_spec_verify(self.gm, self.kv, self.slot, cur, par, self.ws, want_feature=False)
            fg.fg_kv_compact(self.kv, self.slot, zero, path)
            cur = o["argmax"].view(B, 1).clone()
            out[:, l] = cur.view(-1).cpu().numpy()
        self.kv.seq_len.copy_(self.len0)
        return out

    def draft(self):
        """The drafting phase of a round: L_draft steps of the draft head, frontier updates and the rerank.  Its
        tree is computed and then set aside: the verify step reads the planted tree, as the workload prescribes."""
        fg = self.fg
        ct, cp, cs = self.gloop.draft_expand(self.gm, self.gd, self.dkv, self.slot, self.spec_state, self.K_draft,
                                             self.L_draft, self.ws_d, max_seq_len=self.d_max_len)
        tree = fg.fg_build_tree(ct, cp, cs, ct.shape[1], self.N)
        self.dkv.seq_len.copy_(self.dlen0)
        return tree

    def accept(self, o):
        """The acceptance rule the configuration prescribes: the greedy walk on the verify step's row arg-max, or
        rejection sampling over sibling sets on its logits (seeded uniforms and draft distributions)."""
        fg = self.fg
        if self.cfg["accept"] == "reject":
            if not hasattr(self, "draft_q"):
                torch = self.torch
                g = torch.Generator(device="cuda").manual_seed(1234)
                M, V = self.B * self.N, self.model["vocab"]
                self.draft_q = torch.softmax(torch.randn((M, V), generator=g, device="cuda"), dim=1)
                self.unif = torch.rand((self.B, self.N), generator=g, device="cuda")
                self.acc_ws = torch.empty(self.B * 2 * V * 4, dtype=torch.uint8, device="cuda")
            return fg.fg_spec_accept(self.tokens_d, self.parent_d, mode=fg.ACCEPT_REJECT, logits=o["logits"],
                                     vocab=self.model["vocab"], temperature=self.cfg.get("temperature", 1.0),
                                     draft_probs=self.draft_q, uniforms=self.unif, seed=99, workspace=self.acc_ws)
        return fg.fg_spec_accept(self.tokens_d, self.parent_d, row_argmax=o["argmax"])

    def verify(self):
        rej = self.cfg["accept"] == "reject"
        return self.fg.fg_spec_verify(self.gm, self.kv, self.slot, self.tokens_d, self.parent_d, self.ws, want_feature=True,
                                      want_logits=rej, want_argmax=not rej, max_seq_len=self.max_seq_len)

    def step(self):
        fg = self.fg
        fg.fg_plan(self.B, float(self.B * self.N))
        if self.draft_ready:
            self.draft()
        acc, path, otok, fin = self.accept(self.verify())
        fg.fg_kv_compact(self.kv, self.slot, acc, path)
        a = acc.cpu()                                  # host bookkeeping: accept lengths cross to the host
        self.kv.seq_len.copy_(self.len0)               # harness: same ragged shape for the next repetition
        return int(a.sum()) + self.B

    def device_round(self):
        """The device side of `step` (everything but the trip to the host), as one callable for a HIP graph."""
        if self.draft_ready:
            self.draft()
        acc, path, otok, fin = self.accept(self.verify())
        self.fg.fg_kv_compact(self.kv, self.slot, acc, path)
        self.kv.seq_len.copy_(self.len0)               # harness: same ragged shape for the next repetition
        return acc

    def step_graph(self):
        """`step` with the device side recorded once as a HIP graph and replayed (after an eager step has run)."""
        torch = self.torch
        if not hasattr(self, "_graph"):
            self._graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self._graph):
                self._graph_acc = self.device_round()
        self._graph.replay()
        return int(self._graph_acc.cpu().sum()) + self.B

    def verify_only(self):
        self.verify()


def time_steps(torch, fn, steps, warmup):
    """Mean seconds per call over exactly `steps` calls between two device synchronisations, and the last result."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    last = None
    for _ in range(steps):
        last = fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps, last


def time_each(torch, fn, steps, warmup):
    """Every call timed on its own between HIP events on the current stream (the appendix's protocol: warm-ups, then
    repetitions, each bracketed by events): (median, p10, p90, mean) in seconds."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = np.array([a.elapsed_time(b) for a, b in ev]) * 1e-3
    return float(np.median(t)), float(np.percentile(t, 10)), float(np.percentile(t, 90)), float(t.mean())


def spread(ts):
    return dict(median_ms=ts[0] * 1e3, p10_ms=ts[1] * 1e3, p90_ms=ts[2] * 1e3, mean_ms=ts[3] * 1e3)


def cpu_baseline(wl, n_seq=8, reps=3):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle.oracle import Oracle
    from synth import gen
    orc = Oracle("f32")
    model = wl.model
    om = orc.model(model, gen.weights_to_numpy(wl.weights))
    order = np.argsort(wl.lengths)
    pick = sorted(set([int(order[0]), int(order[-1])] + [int(order[i]) for i in np.linspace(0, wl.B - 1, n_seq).astype(int)]))[:max(n_seq, 2)]
    S, N = len(pick), wl.N
    cache = orc.cache(model, S, wl.cap)
    for j, b in enumerate(pick):
        L = int(wl.lengths[b])
        k, v = gen.make_prefix_kv(model, L, wl.cfg["seed"], b, device="cuda")
        cache.k[:, j, :L] = k.float().cpu().numpy()
        cache.v[:, j, :L] = v.float().cpu().numpy()
    cache.len[:] = wl.lengths[pick]
    parent, principal = wl.parent[pick], wl.principal[pick]
    # the oracle plants from its own continuation (no oracle input comes from the HIP path)
    cur = wl.root[pick].copy()
    nxt = np.zeros((S, principal.shape[1]), dtype=np.int32)
    for l in range(principal.shape[1]):
        _, lg = orc.tree_forward(om, cache, cur.reshape(S, 1), np.full((S, 1), -1, np.int32))
        cur, _ = orc.row_argmax(lg)
        nxt[:, l] = cur
        cache.len += 1
    cache.len[:] = wl.lengths[pick]
    tokens, _ = gen.plant_tokens(parent, principal, wl.root[pick], nxt, wl.cfg["plant_p"] or 0.0, model["vocab"], 99)
    t0 = time.perf_counter()
    emitted = 0
    for _ in range(reps):
        _, lg = orc.tree_forward(om, cache, tokens, parent)
        acc, path, out, fin, _, _ = orc.accept_greedy(tokens, parent, lg)
        orc.kv_compact(cache, model, acc, path)
        emitted = int(acc.sum()) + S
        cache.len[:] = wl.lengths[pick]
    dt = (time.perf_counter() - t0) / reps
    return dict(value=emitted / dt, unit="tokens/s", cores=orc.num_threads(), kind="oracle",
                sample=f"{S} of the {wl.B} sequences (shortest and longest cache included), N={N}, all {model['n_layers']} layers, "
                       f"verify+accept+compact, {reps} repetition(s), {dt * 1e3:.0f} ms per step",
                ms_per_step=dt * 1e3, sequences=S, sequence_steps_per_s=S / dt)


def gen_experiment(args):
    """--gen: the concurrency-aware generation loop end to end (Alg. 1) on a synthetic workload: B sequences with
    ragged response budgets decay to one; the tree shape is (a) the rule's (Eq. 1-3 with the measured C_peak),
    (b) plain decoding throughout, (c) one fixed shape tuned for a single sequence.  No trained draft head exists
    here, so the target's decisions along each reranked tree's first-child chain are set to agree with the draft at
    a fixed rate (token values then carry no meaning; every kernel runs at its real shape, the draft steps
    included).  Prints one JSON line."""
    import torch
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    from synth import configs, gen
    pd = configs.PLAN_DEFAULTS
    model = configs.with_dtype(configs.CONFIGS["cfg4"]["model"], args.dtype)
    if args.layers:
        model = configs.scaled(model, args.layers)
    B = args.B or 64
    seed, p_agree = 11, args.agree
    rng = np.random.default_rng(seed)
    lengths = rng.integers(256, 1025, size=B).astype(np.int32)
    budgets = np.clip(np.exp(rng.normal(np.log(args.mean_len), 0.45, size=B)), args.mean_len / 3, args.mean_len * 2.5).astype(np.int32)
    cap_extra = int(budgets.max()) + 64 + 16
    weights = gen.make_weights(model, seed, device="cuda")
    gm = fg.Model(model, weights)
    dcfg = configs.draft_of(model)
    gd = fg.Model(dcfg, gen.make_weights(dcfg, seed, device="cuda", draft=True), target=gm)
    table, n_pages = gen.make_page_table(lengths, cap_extra, 16, seed)
    kv = fg.KVCache(model, table, n_pages)
    dtable, dn = gen.make_page_table(lengths, cap_extra, 16, seed + 1)
    dkv = fg.KVCache(dcfg, dtable, dn)
    for b in range(B):
        k, v = gen.make_prefix_kv(model, int(lengths[b]), seed, b, device="cuda")
        kv.write_prefix(b, k, v)
        k, v = gen.make_prefix_kv(dcfg, int(lengths[b]), seed + 2, b, device="cuda")
        dkv.write_prefix(b, k, v)
    len0, dlen0 = kv.seq_len.clone(), dkv.seq_len.clone()
    cap = int(lengths.max()) + cap_extra
    rows_max = B * 64
    ws_t = gm.workspace(rows_max, cap)
    ws_d = gd.workspace(rows_max, cap)
    first = rng.integers(0, model["vocab"], size=B).astype(np.int32)
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda").manual_seed(seed)
    feat0 = torch.randn((B, 1, model["d_model"]), generator=g, device="cuda").to(td)

    # C_peak (appendix): latency against batch size at sequence length 1
    sizes = [1, 2, 4, 8, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512]
    ptab, pn = gen.make_page_table(np.zeros(max(sizes), np.int32), 16, 16, seed + 3)
    pkv = fg.KVCache(model, ptab, pn)
    c_peak, lat = gloop.measure_c_peak(gm, pkv, gm.workspace(max(sizes), 32), sizes)
    del pkv
    c_peak_linear = int(sizes[fg.fg_knee(sizes, lat, log2_axis=False)])     # the knee on the batch-size axis itself
    print(f"# C_peak = {c_peak} (knee on the log2 B axis; {c_peak_linear} on the B axis); latency ms by batch size: " +
          ", ".join(f"{b}:{t:.2f}" for b, t in zip(sizes, lat)), file=sys.stderr, flush=True)
    if args.c_peak:
        c_peak = args.c_peak

    prng = np.random.default_rng(seed + 5)

    def decide(tokens, parent, amax):
        """Synthetic acceptance: along the first-child chain of each tree the target agrees with the draft with
        probability p_agree per node (its decision at the node is set to the child's token) and otherwise picks a
        token no child carries.  With random weights the target's own choices are not stable across batch shapes
        in bf16, so planted tokens from a reference run would stop matching after the first flip."""
        par, tok = parent.cpu().numpy(), tokens.cpu().numpy()
        am = amax.cpu().numpy().reshape(par.shape).copy()
        for j in range(par.shape[0]):
            node = 0
            while True:
                kids = np.nonzero(par[j] == node)[0]
                if len(kids) == 0:
                    break
                if prng.random() < p_agree:
                    am[j, node] = tok[j, kids[0]]
                    node = int(kids[0])
                else:
                    miss = int(am[j, node])
                    while miss in tok[j, kids]:
                        miss = (miss + 1) % model["vocab"]
                    am[j, node] = miss
                    break
        return torch.as_tensor(am.reshape(-1)).to(amax.device)

    def run(plan, hook):
        kv.seq_len.copy_(len0)
        dkv.seq_len.copy_(dlen0)
        slot = torch.arange(B, dtype=torch.int32, device="cuda")
        st = gloop.SpecState(torch.as_tensor(first).cuda().view(B, 1).contiguous(), feat0.clone(),
                             torch.zeros(B, dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        outs, hist = gloop.generate(gm, gd, kv, dkv, slot, st, first, budgets, float(c_peak), ws_t, ws_d, alpha=pd["alpha"],
                                    K_max=pd["K_max"], L_max=pd["L_max"], N_cap=pd["N_cap"], max_seq_len=cap, plan=plan,
                                    decide=hook)
        torch.cuda.synchronize()
        return outs, hist, time.perf_counter() - t0

    res = {}
    total = int(budgets.sum()) - B
    for name, plan in (("plain", lambda b: (1, 0, 0)), ("rule", None), ("fixed", lambda b: fg.fg_plan(1, float(c_peak)))):
        outs, hist, t = run(plan, decide)
        spec = [h for h in hist if h["N"] > 1]
        shapes = []
        for h in hist:
            if not shapes or shapes[-1][1:] != (h["N"], h["K"], h["L"]):
                shapes.append((h["B"], h["N"], h["K"], h["L"]))
        res[name] = dict(seconds=t, tokens_per_s=total / t, rounds=len(hist),
                         tau=sum(h["emitted"] for h in hist) / max(sum(h["B"] for h in hist), 1),
                         tau_speculative_rounds=(sum(h["emitted"] for h in spec) / sum(h["B"] for h in spec)) if spec else None,
                         shapes_B_N_K_L=shapes[:24])
    out = {"metric": "generated tokens/s over a whole rollout with concurrency decay (Alg. 1)", "unit": "tokens/s",
           "value": res["rule"]["tokens_per_s"], "n_gpus": 1, "higher_is_better": True, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": f"{model['name']} {model['n_layers']} layers, {B} sequences, prefixes U[256,1024], response budgets "
                                  f"{int(budgets.min())}..{int(budgets.max())} (mean {budgets.mean():.0f}), planted agreement {p_agree}, greedy"},
           "c_peak": c_peak, "c_peak_knee_on_linear_axis": c_peak_linear, "c_peak_latency_ms": dict(zip(map(str, sizes), lat)),
           "runs": res,
           "speedup_rule_vs_plain": res["rule"]["tokens_per_s"] / res["plain"]["tokens_per_s"],
           "speedup_rule_vs_fixed": res["rule"]["tokens_per_s"] / res["fixed"]["tokens_per_s"]}
    print(json.dumps(out))


def gemm_kernel_bench(args):
    """--gemm NAME: one GEMM of the 7B-class layer at --rows rows, launched --reps times through the kernel-level entry
    point (the command the per-kernel rocprofv3 summaries under profiles/ are taken with).  The weights of --cycle
    different layers are used in turn so that, as in the step, they come from HBM and not from the last-level cache."""
    import torch
    import paper_2509_21792_amd as fg
    from synth import configs
    m = configs.Q7B
    d, F, V = m["d_model"], m["d_ffn"], m["vocab"]
    qkvd = (m["n_q_heads"] + 2 * m["n_kv_heads"]) * m["head_dim"]
    shapes = {"qkv": (qkvd, d, 0), "o": (d, d, 0), "o_residual": (d, d, 3), "gate_up": (2 * F, d, 1), "down": (d, F, 0),
              "down_residual": (d, F, 3), "lm_head": (V, d, 0), "lm_head_topk": (V, d, 4)}
    n_out, n_in, epi = shapes[args.gemm]
    M = args.rows
    code = fg.FG_BF16 if args.dtype == "bf16" else fg.FG_F16
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda").manual_seed(0)

    def rnd(*shape):
        return (torch.randn(*shape, generator=g, device="cuda") * 0.05).to(torch.bfloat16).to(td)
    n_w = 1 if n_out >= 100000 else args.cycle
    ws = []
    for _ in range(n_w):
        if epi == 1:
            ws.append(fg.fg_pack_weight(code, rnd(n_out // 2, n_in), rnd(n_out // 2, n_in)))
        else:
            ws.append(fg.fg_pack_weight(code, rnd(n_out, n_in)))
    x = rnd(M, n_in)
    h = torch.zeros((M, n_out), dtype=torch.float32, device="cuda") if epi == 3 else None
    it = [0]

    def f():
        w = ws[it[0] % n_w]
        it[0] += 1
        if epi == 4:
            fg.fg_lm_head_topk(code, x, w, V, 2)
        else:
            fg.fg_gemm(code, x, w, n_out, epilogue=epi, split_k=args.split, variant=args.variant, out=h)
    ts = time_each(torch, f, args.reps, 5)
    flops = 2.0 * M * n_out * n_in
    byts = 2.0 * n_out * n_in + 2.0 * M * n_in
    print(json.dumps({"metric": "one GEMM of the 7B-class layer (kernel-level entry point)", "n_gpus": 1, "dtype": args.dtype,
                      "data": "synthetic", "config": {"workload": f"{args.gemm} M={M} n_out={n_out} n_in={n_in} variant={args.variant} split={args.split}"},
                      "kernel": fg.fg_gemm_kernel_name(M, n_out, n_in, min(epi, 3)), "us": spread(ts), "TFLOPs": flops / ts[0] / 1e12,
                      "mfma_frac": flops / ts[0] / PEAK_MFMA, "weight_stream_GBps": byts / ts[0] / 1e9}))


def attention_kernel_bench(args):
    """--attention: the tree attention of one layer on the workload's paged cache (B, N, KV lengths of --workload),
    launched --reps times through the kernel-level entry point, layers taken in turn so that K/V come from HBM.  The
    in-round nodes' K/V cells hold whatever the cache fill left there: their values do not matter to the timing."""
    import torch
    import paper_2509_21792_amd as fg
    wl = Workload(args.workload, args.dtype, B=args.B or None, N=args.N or None, verbose=True, with_draft=False)
    m = wl.model
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda").manual_seed(0)
    q = torch.randn((wl.B * wl.N, m["n_q_heads"] * m["head_dim"]), generator=g, device="cuda").to(td)
    it = [0]

    def f():
        fg.fg_attention(wl.kv, it[0] % m["n_layers"], wl.slot, wl.parent_d, wl.B, wl.N, m["n_q_heads"], q, max_seq_len=wl.max_seq_len)
        it[0] += 1
    ts = time_each(torch, f, args.reps, 5)
    kv_bytes = float(wl.lengths.sum()) * 2 * m["n_kv_heads"] * m["head_dim"] * 2
    print(json.dumps({"metric": "tree attention of one layer (kernel-level entry point)", "n_gpus": 1, "dtype": args.dtype, "data": "synthetic",
                      "config": {"workload": f"{wl.name}: B={wl.B} N={wl.N}, KV lengths U[{int(wl.lengths.min())},{int(wl.lengths.max())}]"},
                      "us": spread(ts), "kv_bytes_per_layer": kv_bytes, "kv_GBps": kv_bytes / ts[0] / 1e9,
                      "hbm_frac": kv_bytes / ts[0] / PEAK_HBM}))


def train_bench(args):
    """--train: one step of online draft learning (Sec. 4.2) on the 7B-class draft head: loss + gradients of B chains of T
    cached (token, feature) entries and the AdamW update, fp32.  Tokens/s of training entries and the fraction of the fp32
    vector peak over the step's GEMM flops."""
    import torch
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    from synth import configs, gen
    model = configs.with_dtype(configs.Q7B, "fp32")
    dcfg = configs.draft_of(model)
    B, T = args.B or 8, args.T
    d, F, V = model["d_model"], model["d_ffn"], model["vocab"]
    g = torch.Generator(device="cuda").manual_seed(0)
    tw = {"embed": torch.randn((V, d), generator=g, device="cuda") * 0.02, "lm_head": torch.randn((V, d), generator=g, device="cuda") * 0.02}
    dw = gen.make_weights(dcfg, 0, device="cuda", draft=True)
    compute = "fp32" if args.train == "fp32" else "bf16"
    trainer = gloop.DraftTrainer(dcfg, dw, tw, compute=compute)
    tokens = torch.randint(0, V, (B, T), generator=g, device="cuda", dtype=torch.int32)
    fin = torch.randn((B, T, d), generator=g, device="cuda")
    ftg = torch.randn((B, T, d), generator=g, device="cuda")
    n_valid = torch.full((B,), T, dtype=torch.int32, device="cuda")
    def f():
        trainer.step(tokens, fin, ftg, n_valid)
    ts = time_each(torch, f, max(3, args.steps // 3), 1)
    qkvd = (model["n_q_heads"] + 2 * model["n_kv_heads"]) * model["head_dim"]
    hq = model["n_q_heads"] * model["head_dim"]
    p_fc, p_layer, p_lm = 2 * d * d, qkvd * d + hq * d + 3 * F * d, V * d
    M = B * T
    flops = 2.0 * M * (3 * (p_fc + p_layer) - p_fc + 3 * p_lm)
    peak = 157.3e12 if compute == "fp32" else PEAK_MFMA
    print(json.dumps({"metric": "draft training entries/s (online draft learning step: loss, gradients, AdamW)", "unit": "tokens/s",
                      "value": M / ts[0], "n_gpus": 1, "dtype": "f32" if compute == "fp32" else "bf16", "data": "synthetic",
                      "higher_is_better": True,
                      "config": {"workload": f"7B-class draft head (1 layer, d={d}, F={F}, vocab {V}), {B} chains of {T} entries, "
                                             f"matrix products in {compute}"},
                      "step": spread(ts), "step_flops": flops,
                      "roofline": {"bound": "alu" if compute == "fp32" else "mfma", "achieved": flops / ts[0] / 1e12, "peak": peak / 1e12,
                                   "unit": "TFLOP/s", "frac": flops / ts[0] / peak, "traffic": None,
                                   "kernel": "the step's GEMMs (whole-step flops over whole-step time: casts, packs, row-wise "
                                             "kernels and the optimiser included)"}}))


def ceilings(args):
    """--ceilings: what this GPU sustains for the two resources the path is bound by, next to the nominal peaks:
    a read-only stream and a plain copy over buffers far larger than the last-level cache, and a register-resident
    MFMA loop on every SIMD (short bursts and a sustained run, where the clock settles under the power limit)."""
    import torch
    import paper_2509_21792_amd as fg

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    nbytes = 4 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.random_(0, 255)
    dst = torch.empty(nbytes // 2, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    out = {"metric": "achievable ceilings (measured) next to the nominal peaks", "n_gpus": 1, "data": "synthetic",
           "config": {"workload": "ceiling probes: 4 GiB read stream, 2 GiB copy, register-resident MFMA loop"},
           "nominal": {"hbm_GBps": PEAK_HBM / 1e9, "mfma_16bit_TFLOPs": PEAK_MFMA / 1e12}}
    reads = {}
    for nt in (0, 1):
        for blocks in (1024, 2048, 4096, 8192, 16384):
            t = timed(lambda: fg.fg_probe_read(src, nt, blocks, sink), 5)
            reads[f"{'nontemporal' if nt else 'plain'}_{blocks}_blocks"] = nbytes / t / 1e9
    out["hbm_read_GBps"] = reads
    out["hbm_read_best_GBps"] = max(reads.values())
    paged = {}
    for blocks in (2048, 4096, 8192, 16384, 32768):
        t = timed(lambda: fg.fg_probe_read(src, 2, blocks, sink), 5)
        paged[f"{blocks}_blocks"] = nbytes / t / 1e9
    out["hbm_read_scattered_4KiB_pages_GBps"] = paged
    out["hbm_read_scattered_4KiB_pages_best_GBps"] = max(paged.values())
    # L2 -> L1: every block streams one 1 MiB region 256 times (it stays in L2, no 32 KiB L1 holds it)
    small = src[:1 << 20]
    l2 = {}
    for per_cu in (1, 2, 4):
        blocks = 256 * per_cu
        t = timed(lambda: fg.fg_probe_read(small, 3, blocks, sink), 3)
        l2[f"{per_cu}_blocks_per_cu"] = dict(aggregate_GBps=blocks * 256 * (1 << 20) / t / 1e9, per_cu_GBps=blocks * (1 << 20) / t / 1e9)
    out["l2_to_l1_stream"] = l2
    out["l2_to_l1_best_per_cu_GBps"] = max(v["per_cu_GBps"] for v in l2.values())
    # what one CU draws from HBM: at most one block per CU, each streaming its own slice with 4 ... 32 loads per lane in
    # flight (4 ... 32 KiB per wave); a launch with fewer blocks than CUs is bound by this times its block count
    one = {}
    for blocks in (64, 128, 198, 256):
        for mode, depth in ((4, 8), (5, 16), (6, 32)):
            used = nbytes // blocks // (4096 * depth) * (4096 * depth) * blocks
            t = timed(lambda: fg.fg_probe_read(src, mode, blocks, sink), 3)
            one[f"{blocks}_blocks_{depth}_in_flight"] = dict(aggregate_GBps=used / t / 1e9, per_block_GBps=used / t / 1e9 / blocks)
    out["hbm_read_one_block_per_cu"] = one
    copies = {}
    half = src[:nbytes // 2]
    for blocks in (2048, 4096, 8192, 16384):
        t = timed(lambda: fg.fg_probe_copy(half, dst, blocks), 5)
        copies[f"{blocks}_blocks"] = 2 * (nbytes // 2) / t / 1e9
    out["hbm_copy_GBps_read_plus_write"] = copies
    out["hbm_copy_best_GBps"] = max(copies.values())
    mf = {}
    flop_per_wave_iter = 16 * 2.0 * 32 * 32 * 16
    for name, code in (("bf16", fg.FG_BF16), ("fp16", fg.FG_F16)):
        for rnd in (1, 0):                      # hashed operands that toggle the buses like real data / constant ones
            for wps in (1, 2):                  # waves per SIMD: 256 CUs x 4 SIMDs x wps waves
                blocks = 256 * wps
                for label, iters, reps in (("burst_1ms", 4000 // wps, 3), ("sustained_200ms", 80000 // wps, 10)):
                    t = timed(lambda: fg.fg_probe_mfma(code, iters, rnd, blocks, sink), reps)
                    tf = blocks * 4 * iters * flop_per_wave_iter / t / 1e12
                    mf[f"{name}_{'random' if rnd else 'constant'}_operands_{wps}_waves_per_simd_{label}"] = dict(
                        TFLOPs=tf, implied_clock_GHz=tf / (PEAK_MFMA / 1e12) * 2.4, ms_per_launch=t * 1e3)
    out["mfma_loop"] = mf
    out["mfma_sustained_best_TFLOPs"] = max(v["TFLOPs"] for k, v in mf.items() if "sustained" in k and "random" in k)
    out["mfma_burst_best_TFLOPs"] = max(v["TFLOPs"] for k, v in mf.items() if "burst" in k and "random" in k)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--dtype", default="fp16", choices=["bf16", "fp16"],
                    help="activation type of the 16-bit path: fp16 (default: the mode that meets the stated 3e-2 / 0.05 parity bar "
                         "on all five configurations; weights and cache hold the same bf16-representable values) or bf16")
    ap.add_argument("--no-other-dtype", action="store_true", help="skip the round time of the other 16-bit mode")
    ap.add_argument("--B", type=int, default=0)
    ap.add_argument("--N", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-b8", action="store_true", help="skip the B = 8 point of the metric's range")
    ap.add_argument("--gen", action="store_true", help="the generation loop with concurrency decay instead of the step benchmark")
    ap.add_argument("--agree", type=float, default=0.7, help="--gen: planted per-node agreement rate")
    ap.add_argument("--mean-len", type=int, default=160, help="--gen: mean response budget")
    ap.add_argument("--c-peak", type=int, default=0, help="--gen, --sweep: use this C_peak instead of the measured knee")
    ap.add_argument("--prefill", type=int, default=0, metavar="P",
                    help="prefill B prompts of P tokens through chain verify steps of 64 positions (target + draft head)")
    ap.add_argument("--graph", action="store_true", help="also time the round with its device side replayed as a HIP graph")
    ap.add_argument("--sweep", action="store_true",
                    help="the metric's range: B = 8 ... 256 on the 7B-class target, each with the shape Eq. 1-3 give")
    ap.add_argument("--gemm", default="", choices=["", "qkv", "o", "o_residual", "gate_up", "down", "down_residual", "lm_head", "lm_head_topk"],
                    help="time one GEMM of the 7B-class layer through the kernel-level entry point and exit")
    ap.add_argument("--attention", action="store_true", help="time the tree attention of one layer on the workload's cache and exit")
    ap.add_argument("--rows", type=int, default=2048, help="--gemm: rows M")
    ap.add_argument("--reps", type=int, default=56, help="--gemm: timed launches")
    ap.add_argument("--variant", type=int, default=0, help="--gemm: 0 = the library's kernel choice, 1-14 force one (see fastgrpo.h)")
    ap.add_argument("--split", type=int, default=0, help="--gemm: k splits of the partial-sum epilogue (0 = the library's choice)")
    ap.add_argument("--cycle", type=int, default=8, help="--gemm: number of different weight matrices used in turn")
    ap.add_argument("--train", default="", choices=["", "bf16", "fp32"],
                    help="time one online draft learning step on the 7B-class draft head (matrix products on the matrix cores "
                         "in bf16, or exact fp32) and exit")
    ap.add_argument("--T", type=int, default=256, help="--train: entries per chain")
    ap.add_argument("--ceilings", action="store_true",
                    help="measure the achievable HBM stream rate and MFMA rate of this GPU (probe kernels) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every box of this build has one MI355X and the path shards by sequence "
              "with no collective, so --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2509_21792_amd as fg
    fg.lib()
    assert torch.cuda.is_available(), "no GPU: the HIP path has no CPU fallback"
    if args.attention:
        attention_kernel_bench(args)
        return
    if args.gemm:
        gemm_kernel_bench(args)
        return
    if args.train:
        train_bench(args)
        return
    if args.ceilings:
        ceilings(args)
        return
    if args.gen:
        gen_experiment(args)
        return
    if args.sweep:
        sweep(args)
        return
    if args.prefill:
        prefill_bench(args)
        return

    def measure(dtype, full):
        """The timed region for one arithmetic mode.  full: with stage timing, the B = 8 points and everything else the
        JSON line carries; otherwise the round time only (the other 16-bit mode, for the same line)."""
        wl = Workload(args.workload, dtype, B=args.B or None, N=args.N or None, n_layers=args.layers or None, verbose=True)
        model, M = wl.model, wl.B * wl.N
        if not full:
            t_step, emitted = time_steps(torch, wl.step, args.steps, args.warmup)
            return dict(ms_per_step=t_step * 1e3, value=emitted / t_step), wl
        acct = model_bytes_flops(model, M, wl.lengths.astype(np.float64), wl.N)
        from synth import configs as cfgs_
        pd_ = cfgs_.PLAN_DEFAULTS
        v_spread = time_each(torch, wl.verify_only, max(args.steps, 30), args.warmup)
        d_spread = time_each(torch, wl.draft, max(args.steps, 30), 2) if wl.draft_ready else None
        t_verify = v_spread[0]
        # the timed region: exactly `steps` whole rounds.  Inside it the dominant kernel's launches (the gate/up stage of the
        # target's verify step) are bracketed by HIP events on the launch stream, two per layer; the split over all stages
        # is taken in rounds of its own afterwards (nine events per layer stretch a round by about 1 %)
        for _ in range(args.warmup):
            wl.step()
        fg.fg_model_profile(wl.gm, True, max_marks=(args.steps + 1) * (model["n_layers"] * 2 + 4), only="gate_up")
        torch.cuda.synchronize()
        per_step = []
        t0 = time.perf_counter()
        emitted = 0
        for _ in range(args.steps):
            t1 = time.perf_counter()
            emitted = wl.step()          # ends with the accept lengths on the host: a step is complete when it returns
            per_step.append(time.perf_counter() - t1)
        torch.cuda.synchronize()
        t_step = (time.perf_counter() - t0) / args.steps
        stages = fg.fg_model_profile_read(wl.gm)
        fg.fg_model_profile(wl.gm, False)
        n_split = min(args.steps, 5)
        fg.fg_model_profile(wl.gm, True, max_marks=(n_split + 1) * (model["n_layers"] * 10 + 16))
        if wl.draft_ready:
            fg.fg_model_profile(wl.gd, True, max_marks=(n_split + 1) * 32 * (wl.L_draft + 1))
        for _ in range(n_split):
            wl.step()
        torch.cuda.synchronize()
        st_ms = {k: v[0] / n_split for k, v in fg.fg_model_profile_read(wl.gm).items() if v[1]}
        fg.fg_model_profile(wl.gm, False)
        draft_st_ms = None
        if wl.draft_ready:
            draft_st_ms = {k: v[0] / n_split for k, v in fg.fg_model_profile_read(wl.gd).items() if v[1]}
            fg.fg_model_profile(wl.gd, False)
        n_out, n_in = 2 * model["d_ffn"], model["d_model"]
        k_cnt = stages["gate_up"][1]
        assert k_cnt == args.steps * model["n_layers"], (k_cnt, args.steps)
        k_avg = stages["gate_up"][0] / k_cnt * 1e-3
        epi = 1 if "swiglu" not in st_ms else 0
        gemm_flops = 2.0 * M * n_out * n_in
        gemm_bytes = 2.0 * n_out * n_in + 2.0 * M * n_in + (2.0 * M * n_out / 2 if epi else 4.0 * M * n_out)
        compute_bound = gemm_flops / PEAK_MFMA > gemm_bytes / PEAK_HBM
        if compute_bound:
            roof = dict(bound="mfma", achieved=gemm_flops / k_avg / 1e12, peak=PEAK_MFMA / 1e12, unit="TFLOP/s")
        else:
            roof = dict(bound="hbm", achieved=gemm_bytes / k_avg / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s")
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["traffic"] = MEASURED_TRAFFIC.get((wl.name, M))
        roof["algorithmic"] = gemm_flops if compute_bound else gemm_bytes
        roof["algorithmic_bytes"] = gemm_bytes
        roof["kernel"] = (f"{fg.fg_gemm_kernel_name(M, n_out, n_in, epi)} (gate/up, M={M}, n_out={n_out}, n_in={n_in}, "
                          f"epilogue={'swiglu' if epi else 'fp32 split-K slabs'})")
        roof["launches"] = k_cnt
        roof["avg_us"] = k_avg * 1e6
        gemm_ms = sum(st_ms.get(k, 0.0) for k in ("qkv", "o", "gate_up", "down", "lm_head"))
        attn_ms = st_ms.get("attention", 0.0)
        ps = np.array(per_step)
        out = {
            "metric": "accepted tokens/s (7B-class speculative step: draft + rerank + verify + accept + compact)",
            "value": emitted / t_step,
            "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_step * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
            "config": {"workload": f"{wl.name}: {model['name']} {model['n_layers']} layers, B={wl.B}, N_verify={wl.N} "
                                   f"(K_draft={wl.plan[1]}, L_draft={wl.plan[2]} from Eq. 1-3), KV lengths U[{int(wl.lengths.min())},"
                                   f"{int(wl.lengths.max())}] in 16-token pages, planted agreement {wl.cfg['plant_p']}, "
                                   f"{'rejection sampling' if wl.cfg['accept'] == 'reject' else 'greedy'}"},
            "step_spread": dict(median_ms=float(np.median(ps)) * 1e3, p10_ms=float(np.percentile(ps, 10)) * 1e3,
                                p90_ms=float(np.percentile(ps, 90)) * 1e3),
            "verify_ms": t_verify * 1e3, "verify_spread": spread(v_spread),
            "draft_ms": d_spread[0] * 1e3 if d_spread else 0.0, "draft_spread": spread(d_spread) if d_spread else None,
            "tau": emitted / wl.B,
            "verify_tokens_per_s": emitted / t_verify, "verify_sequence_steps_per_s": wl.B / t_verify,
            "step_hbm_frac": acct["bytes"] / t_verify / PEAK_HBM, "step_mfma_frac": acct["flops"] / t_verify / PEAK_MFMA,
            "step_bytes": acct["bytes"], "step_flops": acct["flops"],
            # per launch group of the verify step, from the stage timing inside the timed region (ms per step)
            "verify_stage_ms": st_ms, "draft_stage_ms": draft_st_ms,
            "gemm_frac": acct["gemm_flops"] / (gemm_ms * 1e-3) / PEAK_MFMA if gemm_ms else None,
            "attn_frac": (acct["kv_bytes"] + M * 2.0 * model["n_q_heads"] * model["head_dim"] * 2 * model["n_layers"]) / (attn_ms * 1e-3) / PEAK_HBM if attn_ms else None,
            "gemm_ms": gemm_ms, "attn_ms": attn_ms,
            "roofline": roof,
            # the configuration pins N_verify (C_peak = B * N in Eq. 1); what Eq. 1-3 give this batch for the C_peak measured
            # on this chip and model (bench.py --sweep, profiles/sweep_7b_b8_to_b256_rule_shapes.txt) stands beside it
            "shape_for_measured_c_peak": dict(zip(("c_peak", "N_verify", "K_draft", "L_draft"),
                                                  (MEASURED_C_PEAK,) + tuple(fg.fg_plan(wl.B, float(MEASURED_C_PEAK), pd_["alpha"], pd_["K_max"],
                                                                                        pd_["L_max"], pd_["N_cap"])))),
        }
        if args.graph:
            t_graph, emitted_g = time_steps(torch, wl.step_graph, args.steps, args.warmup)
            assert emitted_g == emitted, (emitted_g, emitted)
            out["graph_ms_per_step"] = t_graph * 1e3
            out["graph_value"] = emitted_g / t_graph
        if not args.no_b8 and args.workload == "cfg4" and not args.B:
            # the low end of the metric's range on the same model: B = 8; N = 1, the configured chain and tree, and the shape
            # Eq. 1-3 give for the measured C_peak (64 -> N = 8)
            out["b8"] = [b8_point(wl, N, args) for N in (1, 6, 8, 24)]
        return out, wl

    other = "bf16" if args.dtype == "fp16" else "fp16"
    out, wl = measure(args.dtype, True)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    if not args.no_other_dtype:
        import gc
        del wl
        gc.collect()
        torch.cuda.empty_cache()
        o2, wl2 = measure(other, False)
        out["other_dtype"] = dict(dtype=other, **o2)
        del wl2
    print(json.dumps(out))


def sweep(args):
    """B = 8, 16, ..., 256 sequences with KV lengths U[256, 2048] on the 7B-class target, each batch with the tree
    shape the concurrency rule gives it (Eq. 1-3, C_peak = the measured knee unless --c-peak): whole-round and
    verify-step times, accepted tokens/s and the step's fractions of the HBM and MFMA peaks."""
    import gc
    import torch
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    from synth import configs, gen
    cfg = configs.CONFIGS["b8"]
    model = configs.with_dtype(cfg["model"], args.dtype)
    c_peak, lat, sizes = args.c_peak, None, [1, 2, 4, 8, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512]
    if not c_peak:
        gm = fg.Model(model, gen.make_weights(model, 0, device="cuda"))
        ptab, pn = gen.make_page_table(np.zeros(max(sizes), np.int32), 16, 16, 3)
        pkv = fg.KVCache(model, ptab, pn)
        c_peak, lat = gloop.measure_c_peak(gm, pkv, gm.workspace(max(sizes), 32), sizes)
        del gm, pkv
        gc.collect()
        torch.cuda.empty_cache()
    pd = configs.PLAN_DEFAULTS
    points = []
    for B in (8, 16, 32, 64, 128, 256):
        N, K, L = fg.fg_plan(B, float(c_peak), pd["alpha"], pd["K_max"], pd["L_max"], pd["N_cap"])
        wl = Workload("b8", args.dtype, B=B, N=N, verbose=True)
        t_verify, _ = time_steps(torch, wl.verify_only, max(3, args.steps // 2), args.warmup)
        t_step, emitted = time_steps(torch, wl.step, args.steps, args.warmup)
        # the same round with its device side replayed as a HIP graph (small batches are launch-bound in the drafting steps)
        t_graph, emitted_g = time_steps(torch, wl.step_graph, args.steps, args.warmup)
        acct = model_bytes_flops(wl.model, B * N, wl.lengths.astype(np.float64), N)
        points.append(dict(B=B, N=N, K_draft=K, L_draft=L, round_ms=t_step * 1e3, verify_ms=t_verify * 1e3,
                           accepted_tokens_per_s=emitted / t_step, tau=emitted / B,
                           graph_round_ms=t_graph * 1e3, graph_accepted_tokens_per_s=emitted_g / t_graph,
                           step_hbm_frac=acct["bytes"] / t_verify / PEAK_HBM, step_mfma_frac=acct["flops"] / t_verify / PEAK_MFMA))
        print(f"# B={B} N={N} K={K} L={L}: round {t_step * 1e3:.2f} ms ({t_graph * 1e3:.2f} replayed), verify {t_verify * 1e3:.2f} ms, "
              f"{emitted / t_step:.0f} tokens/s", file=sys.stderr, flush=True)
        del wl
        gc.collect()
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "accepted tokens/s and verify-step ms over B = 8 ... 256 with rule-chosen shapes",
                      "unit": "tokens/s", "n_gpus": 1, "dtype": args.dtype, "data": "synthetic",
                      "config": {"workload": f"{model['name']} {model['n_layers']} layers, KV lengths U[{cfg['kv_lo']},{cfg['kv_hi']}], "
                                             f"planted agreement {cfg['plant_p']}, greedy"},
                      "c_peak": c_peak, "c_peak_latency_ms": None if lat is None else {str(b): t for b, t in zip(sizes, lat)},
                      "points": points}))


def prefill_bench(args):
    """Prompts of P tokens for B sequences through the prefill of the generation loop: chain verify steps of 64
    positions per sequence (M = 64 B rows per step, the pipelined GEMM and the tree attention kernel with a chain
    mask), the draft head consuming its entries alongside.  Tokens/s over the whole prefill."""
    import torch
    import paper_2509_21792_amd as fg
    from paper_2509_21792_amd import loop as gloop
    from synth import configs, gen
    model = configs.with_dtype(configs.CONFIGS["cfg4"]["model"], args.dtype)
    B, P = args.B or 64, args.prefill
    gm = fg.Model(model, gen.make_weights(model, 0, device="cuda"))
    dcfg = configs.draft_of(model)
    gd = fg.Model(dcfg, gen.make_weights(dcfg, 0, device="cuda", draft=True), target=gm)
    table, n_pages = gen.make_page_table(np.zeros(B, np.int32), P + 80, 16, 1)
    dtable, dn = gen.make_page_table(np.zeros(B, np.int32), P + 80, 16, 2)
    kv, dkv = fg.KVCache(model, table, n_pages), fg.KVCache(dcfg, dtable, dn)
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws_t, ws_d = gm.workspace(B * 64, P + 80), gd.workspace(B * 64, P + 80)
    prompts = torch.randint(0, model["vocab"], (B, P), dtype=torch.int32, device="cuda",
                            generator=torch.Generator(device="cuda").manual_seed(3))

    def run():
        kv.seq_len.zero_()
        dkv.seq_len.zero_()
        gloop.prefill(gm, gd, kv, dkv, slot, prompts, ws_t, ws_d, max_seq_len=P + 64)
    t, _ = time_steps(torch, run, max(2, args.steps // 5), 1)
    acct = model_bytes_flops(model, B * P, np.zeros(1), 1)
    attn_flops = 4.0 * model["n_q_heads"] * model["head_dim"] * model["n_layers"] * B * P * (P + 1) / 2.0
    flops = acct["gemm_flops"] - 2.0 * B * P * model["vocab"] * model["d_model"] + attn_flops   # no LM head but for the last step
    print(json.dumps({"metric": "prefill tokens/s (chain verify steps of 64 positions, target + draft head)", "unit": "tokens/s",
                      "value": B * P / t, "n_gpus": 1, "dtype": args.dtype, "data": "synthetic",
                      "config": {"workload": f"{model['name']} {model['n_layers']} layers, {B} prompts of {P} tokens"},
                      "seconds": t, "mfma_frac": flops / t / PEAK_MFMA}))


def b8_point(wl, N, args):
    """B = 8 on the same weights: verify-step time and the HBM fraction of the memory-bound regime."""
    import torch
    fg = wl.fg
    from synth import configs, gen
    cfg = configs.CONFIGS["b8"]
    B = cfg["B"]
    lengths = gen.make_kv_lengths(B, cfg["kv_lo"], cfg["kv_hi"], 7)
    table, n_pages = gen.make_page_table(lengths, N + 1, 16, 7)
    kv = fg.KVCache(wl.model, table, n_pages)
    for b in range(B):
        k, v = gen.make_prefix_kv(wl.model, int(lengths[b]), 7, b, device="cuda")
        kv.write_prefix(b, k, v)
    spec = ("tree", 4, 5 if N > 8 else 4, N) if N > 6 else ("chain", N - 1)
    parent, _ = gen.make_trees(spec, B, N, 8)
    rng = np.random.default_rng(9)
    tokens = torch.as_tensor(rng.integers(0, wl.model["vocab"], size=(B, N)).astype(np.int32)).cuda()
    parent = torch.as_tensor(parent).cuda()
    slot = torch.arange(B, dtype=torch.int32, device="cuda")
    ws = wl.gm.workspace(B * N, int(lengths.max()) + N + 1)
    msl = int(lengths.max()) + N

    out_buf = {}

    def f():
        out_buf["o"] = fg.fg_spec_verify(wl.gm, kv, slot, tokens, parent, ws, want_feature=True, max_seq_len=msl)
    ts = time_each(torch, f, max(args.steps, 30), args.warmup)
    t = ts[0]
    # the same step recorded once as a HIP graph and replayed: at this size the step is ~260 short launches and the
    # gaps between them are a measurable share of it
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        f()
    tg = time_each(torch, graph.replay, max(args.steps, 30), args.warmup)
    # where the step's time goes (a separate pass: at this size the events between launches cost a few per cent)
    reps = 20
    fg.fg_model_profile(wl.gm, True, max_marks=(reps + 1) * (wl.model["n_layers"] * 10 + 16))
    for _ in range(reps):
        f()
    stage_us = {k: v[0] / reps * 1e3 for k, v in fg.fg_model_profile_read(wl.gm).items() if v[1]}
    fg.fg_model_profile(wl.gm, False)
    acct = model_bytes_flops(wl.model, B * N, lengths.astype(np.float64), N)
    return dict(B=B, N=N, verify_ms=t * 1e3, stage_us=stage_us, hbm_frac=acct["bytes"] / t / PEAK_HBM, mfma_frac=acct["flops"] / t / PEAK_MFMA,
                verify_spread=spread(ts), graph_verify_ms=tg[0] * 1e3, graph_hbm_frac=acct["bytes"] / tg[0] / PEAK_HBM,
                graph_verify_spread=spread(tg), bytes=acct["bytes"])


if __name__ == "__main__":
    main()
