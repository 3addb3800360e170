"""Seeded synthetic inputs shared by the oracle's tests and the HIP path's tests and benchmark.

Everything here is plain random-number generation and index bookkeeping: weights, prompts, KV prefixes,
page tables, tree shapes, planted draft tokens, uniforms and draft distributions.  None of the method's
arithmetic (no forward pass, no acceptance rule, no rerank) is in this module: where planting needs the
target's own next tokens they are handed in by the caller.
"""
import numpy as np
import torch


def _gen(seed, device="cpu"):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def _store(t, dtype):
    """16-bit workloads hold bf16-representable values (rounded once, here); fp32 workloads keep fp32.
    "fp16" keeps those bf16-rounded values in an fp16 container (exact down to 6e-5, subnormal below)."""
    if dtype == "bf16":
        return t.to(torch.bfloat16)
    if dtype == "fp16":
        return t.to(torch.bfloat16).to(torch.float16)
    return t


def make_weights(model, seed, device="cpu", draft=False):
    """N(0, 0.02) matrices, [out, in] row-major; RMSNorm gains 1 + N(0, 0.02).

    Returns {"embed", "lm_head", "final_norm", "layers": [{wqkv, wo, w_gate, w_up, w_down, norm_attn,
    norm_ffn}]}; a draft head has "fc" [d, 2d] and its single layer, and no embed / lm_head / final_norm
    (it uses the target's embedding and LM head).
    """
    d, Hq, Hkv, hd, F, V = (model[k] for k in ("d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab"))
    dt = model["dtype"]
    g = _gen(seed * 1000003 + (7 if draft else 1), device)

    def mat(o, i):
        return _store(torch.randn(o, i, generator=g, device=device, dtype=torch.float32) * 0.02, dt)

    def gain():
        return _store(1.0 + torch.randn(d, generator=g, device=device, dtype=torch.float32) * 0.02, dt)

    w = {}
    if draft:
        w["fc"] = mat(d, 2 * d)
    else:
        w["embed"] = mat(V, d)
        w["lm_head"] = mat(V, d)
        w["final_norm"] = gain()
    w["layers"] = []
    for _ in range(model["n_layers"]):
        w["layers"].append(dict(wqkv=mat((Hq + 2 * Hkv) * hd, d), wo=mat(d, Hq * hd), w_gate=mat(F, d),
                                w_up=mat(F, d), w_down=mat(d, F), norm_attn=gain(), norm_ffn=gain()))
    return w


def weights_to_numpy(w):
    """float32 numpy copies (for the CPU side)."""
    def cv(t):
        return t.detach().to("cpu", torch.float32).numpy()
    out = {k: cv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: cv(v) for k, v in lay.items()} for lay in w["layers"]]
    return out


def make_prompts(B, group, prompt_len, vocab, seed):
    """B // group distinct prompts of uniform-random token ids, each repeated `group` times (GRPO rollouts)."""
    rng = np.random.default_rng(seed + 11)
    n_prompts = max(1, B // group)
    p = rng.integers(0, vocab, size=(n_prompts, prompt_len), dtype=np.int64).astype(np.int32)
    return np.repeat(p, group, axis=0)[:B].copy()


def make_kv_lengths(B, lo, hi, seed):
    rng = np.random.default_rng(seed + 23)
    return rng.integers(lo, hi + 1, size=B, dtype=np.int64).astype(np.int32)


def make_prefix_kv(model, L, seed, b, device="cpu"):
    """Synthetic committed KV prefix of one sequence: k, v [n_layers, L, Hkv, hd], N(0,1); the values are taken
    as already rotated keys / values.  Seeded per sequence so any subset can be regenerated alone."""
    g = _gen(seed * 7919 + 104729 * (b + 1), device)
    shape = (model["n_layers"], int(L), model["n_kv_heads"], model["head_dim"])
    k = _store(torch.randn(shape, generator=g, device=device, dtype=torch.float32), model["dtype"])
    v = _store(torch.randn(shape, generator=g, device=device, dtype=torch.float32), model["dtype"])
    return k, v


def make_page_table(lengths, extra, page_size, seed, spare_pages=0):
    """Pages for lengths[b] + extra tokens per sequence, handed out in a shuffled (non-contiguous) order.
    Returns (page_table [B, max_pages] int32 with -1 padding, n_pages)."""
    rng = np.random.default_rng(seed + 37)
    need = [(int(L) + extra + page_size - 1) // page_size for L in lengths]
    n_pages = int(sum(need)) + spare_pages
    perm = rng.permutation(n_pages).astype(np.int32)
    table = np.full((len(lengths), max(need)), -1, dtype=np.int32)
    at = 0
    # interleave the hand-out so that a sequence's pages are scattered
    cursor = [0] * len(lengths)
    remaining = sum(need)
    while remaining:
        for b, n in enumerate(need):
            if cursor[b] < n:
                table[b, cursor[b]] = perm[at]
                at += 1
                cursor[b] += 1
                remaining -= 1
    return table, n_pages


def tree_shape(spec, N, rng):
    """parent [N] (parent[0] = -1, parent[i] < i, nodes ordered by depth) and the principal path's node
    indices [depth_p] for one sequence.  spec: ("chain", depth) | ("tree", top_k, depth, n_nodes)."""
    if N == 1:
        return np.array([-1], dtype=np.int32), np.zeros(0, dtype=np.int32)
    if spec[0] == "chain":
        par = np.arange(-1, N - 1, dtype=np.int32)
        return par, np.arange(1, N, dtype=np.int32)
    _, top_k, depth, _ = spec
    par, dep, nch = [-1], [0], [0]
    prev = 0
    dp = min(depth, N - 1)
    principal = []
    for _ in range(dp):
        par.append(prev); dep.append(dep[prev] + 1); nch.append(0); nch[prev] += 1
        prev = len(par) - 1
        principal.append(prev)
    while len(par) < N:
        cands = [i for i in range(len(par)) if dep[i] < depth and nch[i] < top_k]
        if not cands:
            raise ValueError("tree spec cannot hold N nodes")
        # shallower parents are likelier, as in a confidence-reranked draft tree
        wts = np.array([0.5 ** dep[i] for i in cands])
        u = cands[int(rng.choice(len(cands), p=wts / wts.sum()))]
        par.append(u); dep.append(dep[u] + 1); nch.append(0); nch[u] += 1
    order = sorted(range(N), key=lambda i: (dep[i], i))
    new = {old: n for n, old in enumerate(order)}
    parent = np.array([-1 if par[o] < 0 else new[par[o]] for o in order], dtype=np.int32)
    return parent, np.array([new[i] for i in principal], dtype=np.int32)


def make_trees(spec, B, N, seed):
    """Tree shapes for a batch: parent [B, N] int32, principal [B, depth_p] int32."""
    rng = np.random.default_rng(seed + 41)
    ps, prs = zip(*[tree_shape(spec, N, rng) for _ in range(B)])
    return np.stack(ps), np.stack(prs)


def plant_tokens(parent, principal, root_tokens, next_tokens, p, vocab, seed):
    """Draft tokens with agreement planted at rate p.

    next_tokens [B, depth_p]: the tokens the target itself emits along the principal path (handed in by the
    caller).  The principal node at depth l carries next_tokens[:, l-1] with probability p while all shallower
    principal nodes agreed; from the first miss on, and on every other node, tokens are uniform-random but
    distinct from their siblings and from the target's token at that point.
    """
    rng = np.random.default_rng(seed + 53)
    B, N = parent.shape
    tokens = np.zeros((B, N), dtype=np.int32)
    tokens[:, 0] = root_tokens
    hit = np.zeros((B, principal.shape[1]), dtype=bool)
    for b in range(B):
        used = {}  # parent -> set of tokens already among its children
        alive = True
        avoid = {}  # node -> token that must not appear among its children by accident
        for l, node in enumerate(principal[b]):
            u = int(parent[b, node])
            if alive:
                avoid[u] = int(next_tokens[b, l])
            if alive and rng.random() < p:
                tok = int(next_tokens[b, l]); hit[b, l] = True
            else:
                alive = False
                tok = None
            if tok is not None:
                tokens[b, node] = tok
                used.setdefault(u, set()).add(tok)
        pset = set(int(x) for x in principal[b][hit[b]])
        for i in range(1, N):
            if i in pset:
                continue
            u = int(parent[b, i])
            s = used.setdefault(u, set())
            while True:
                t = int(rng.integers(0, vocab))
                if t not in s and t != avoid.get(u, -1):
                    break
            tokens[b, i] = t
            s.add(t)
    return tokens, hit


def make_uniforms(B, N, seed):
    rng = np.random.default_rng(seed + 67)
    return rng.random((B, N), dtype=np.float32)


def make_draft_probs(M, vocab, seed, device="cpu"):
    """Draft distributions [M, vocab]: softmax of N(0,1) logits, fp32."""
    g = _gen(seed * 31 + 71, device)
    z = torch.randn(M, vocab, generator=g, device=device, dtype=torch.float32)
    return torch.softmax(z, dim=-1)
