"""ctypes front end of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.  It loads
oracle/liboracle_{f32,f64}.so (built from fg_oracle.c by oracle/build.py) and passes numpy arrays
through; all of the method's arithmetic is in the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_I32P = C.POINTER(C.c_int32)


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "act_round")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p), ("fc", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in
                ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


class OracleError(RuntimeError):
    pass


class Model:
    """Weights of a target (or a draft head) held in the oracle's precision."""

    def __init__(self, orc, cfg, weights, embed_from=None, act_round=None):
        """act_round: None for the oracle proper; "bf16" / "fp16" for its rounding twin (activations stored in 16 bits
        between the steps of a layer, exact arithmetic in between)."""
        self.cfg = dict(cfg)
        self.real = orc.real
        self.act_round = {None: 0, "bf16": 1, "fp16": 2}[act_round]
        conv = lambda a: np.ascontiguousarray(a, dtype=orc.real)
        self._keep = []
        self.c = _Cfg(cfg["n_layers"], cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                      cfg["d_ffn"], cfg["vocab"], self.act_round, cfg.get("rms_eps", 1e-6), cfg.get("rope_theta", 10000.0))
        w = _Weights()
        src = embed_from if embed_from is not None else None
        for name in ("embed", "lm_head", "final_norm", "fc"):
            arr = None
            if name in weights and weights[name] is not None:
                arr = conv(weights[name])
            elif src is not None and name in ("embed", "lm_head"):
                arr = getattr(src, "_" + name)
            setattr(self, "_" + name, arr)
            setattr(w, name, _ptr(arr))
        nl = cfg["n_layers"]
        for name in ("wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn"):
            arrs = [conv(weights["layers"][l][name]) for l in range(nl)]
            self._keep.append(arrs)
            tab = (C.c_void_p * nl)(*[a.ctypes.data for a in arrs])
            self._keep.append(tab)
            setattr(w, name, C.cast(tab, C.POINTER(C.c_void_p)))
        self.w = w


def _twin(self, act_round):
    """The same weights (shared, not copied) seen through the rounding twin (or, with None, the oracle proper)."""
    import copy
    t = copy.copy(self)
    t.act_round = {None: 0, "bf16": 1, "fp16": 2}[act_round]
    cfg = self.cfg
    t.c = _Cfg(cfg["n_layers"], cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"],
               t.act_round, cfg.get("rms_eps", 1e-6), cfg.get("rope_theta", 10000.0))
    return t


Model.twin = _twin


class KVCache:
    """Contiguous per-sequence cache [n_layers][B][cap][Hkv][hd] and lengths [B]."""

    def __init__(self, orc, cfg, B, cap):
        """B = number of cache slots."""
        shape = (cfg["n_layers"], B, cap, cfg["n_kv_heads"], cfg["head_dim"])
        self.k = np.zeros(shape, dtype=orc.real)
        self.v = np.zeros(shape, dtype=orc.real)
        self.len = np.zeros(B, dtype=np.int32)
        self.cap = cap
        self.B = B

    def copy(self):
        o = object.__new__(KVCache)
        o.k, o.v, o.len, o.cap, o.B = self.k.copy(), self.v.copy(), self.len.copy(), self.cap, self.B
        return o


class Oracle:
    def __init__(self, kind="f32"):
        path = _build.lib_path(kind)
        if not os.path.exists(path):
            _build.build()
        self.lib = C.CDLL(path)
        self.kind = kind
        self.real = np.float32 if kind == "f32" else np.float64
        assert self.lib.orc_sizeof_real() == np.dtype(self.real).itemsize
        self.lib.orc_uniform01.restype = C.c_double
        self.lib.orc_uniform01.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]

    def num_threads(self):
        return int(self.lib.orc_num_threads())

    def _check(self, rc, what):
        if rc != 0:
            raise OracleError(f"{what} failed with code {rc}")

    # -- Eq. 1-3 ---------------------------------------------------------------------------------
    def plan(self, B_cur, C_peak, alpha=0.5, K_max=4, L_max=6, N_cap=64):
        N, K, L = C.c_int32(), C.c_int32(), C.c_int32()
        rc = self.lib.orc_plan(C.c_int32(B_cur), C.c_double(C_peak), C.c_double(alpha), C.c_int32(K_max),
                               C.c_int32(L_max), C.c_int32(N_cap), C.byref(N), C.byref(K), C.byref(L))
        self._check(rc, "orc_plan")
        return N.value, K.value, L.value

    def knee(self, x, y):
        """Index of the knee of the curve y(x) (appendix, measurement of C_peak)."""
        x = np.ascontiguousarray(x, dtype=np.float64)
        y = np.ascontiguousarray(y, dtype=np.float64)
        k = C.c_int64()
        self._check(self.lib.orc_knee(_ptr(x), _ptr(y), C.c_int64(len(x)), C.byref(k)), "orc_knee")
        return k.value

    # -- forward ---------------------------------------------------------------------------------
    def model(self, cfg, weights, embed_from=None, act_round=None):
        return Model(self, cfg, weights, embed_from, act_round)

    def round_act(self, x, kind):
        """x rounded to the nearest bf16 / fp16 value, ties to even (what the rounding twin applies)."""
        x = np.array(x, dtype=self.real)
        self._check(self.lib.orc_round_act(_ptr(x), C.c_int64(x.size), C.c_int32({"bf16": 1, "fp16": 2}[kind])), "orc_round_act")
        return x

    def cache(self, cfg, B, cap):
        return KVCache(self, cfg, B, cap)

    def tree_forward(self, model, cache, tokens, parent, feat_in=None, n_prev=0, is_draft=False, want_logits=True,
                     slot=None):
        """slot [B]: cache slot of each row of the call (identity if None)."""
        slot = None if slot is None else _i32(slot)
        tokens = _i32(tokens)
        parent = _i32(parent)
        B, N_new = tokens.shape
        assert parent.shape == (B, n_prev + N_new), (parent.shape, B, n_prev, N_new)
        d, V = model.cfg["d_model"], model.cfg["vocab"]
        hidden = np.empty((B * N_new, d), dtype=self.real)
        logits = np.empty((B * N_new, V), dtype=self.real) if want_logits else None
        if is_draft:
            feat_in = np.ascontiguousarray(feat_in, dtype=self.real)
            assert feat_in.shape == (B, N_new, d)
        rc = self.lib.orc_tree_forward(C.byref(model.c), C.byref(model.w), C.c_int32(int(is_draft)), C.c_int32(B),
                                       C.c_int32(n_prev), C.c_int32(N_new), _ptr(tokens), _ptr(feat_in),
                                       _ptr(parent), _ptr(cache.k), _ptr(cache.v), C.c_int64(cache.cap),
                                       C.c_int32(cache.B), _ptr(slot), _ptr(cache.len), _ptr(hidden),
                                       _ptr(logits))
        self._check(rc, "orc_tree_forward")
        return hidden, logits

    def rope_head(self, v, pos, theta=10000.0):
        v = np.array(v, dtype=self.real)
        self.lib.orc_rope_head(_ptr(v), C.c_int32(v.shape[0]), C.c_int64(pos), C.c_double(theta))
        return v

    # -- random numbers --------------------------------------------------------------------------
    def uniform01(self, seed, row, v):
        return self.lib.orc_uniform01(seed, row, v)

    def gumbel_scores(self, logits, T, seed, row0=0):
        logits = np.ascontiguousarray(logits, dtype=self.real)
        M, V = logits.shape
        out = np.empty_like(logits)
        rc = self.lib.orc_gumbel_scores(_ptr(logits), C.c_int64(M), C.c_int64(V), C.c_double(T), C.c_uint64(seed),
                                        C.c_int64(row0), _ptr(out))
        self._check(rc, "orc_gumbel_scores")
        return out

    def row_argmax(self, scores):
        scores = np.ascontiguousarray(scores, dtype=self.real)
        M, V = scores.shape
        idx = np.empty(M, dtype=np.int32)
        margin = np.empty(M, dtype=self.real)
        self._check(self.lib.orc_row_argmax(_ptr(scores), C.c_int64(M), C.c_int64(V), _ptr(idx), _ptr(margin)),
                    "orc_row_argmax")
        return idx, margin

    # -- acceptance ------------------------------------------------------------------------------
    def walk(self, tokens, parent, target_tok, eos_id=-1):
        tokens, parent, target_tok = _i32(tokens), _i32(parent), _i32(target_tok)
        B, N = tokens.shape
        acc = np.empty(B, dtype=np.int32)
        path = np.empty((B, N), dtype=np.int32)
        out = np.empty((B, N), dtype=np.int32)
        fin = np.empty(B, dtype=np.int32)
        rc = self.lib.orc_walk(C.c_int32(B), C.c_int32(N), _ptr(tokens), _ptr(parent), _ptr(target_tok),
                               C.c_int32(eos_id), _ptr(acc), _ptr(path), _ptr(out), _ptr(fin))
        self._check(rc, "orc_walk")
        return acc, path, out, fin

    def accept_greedy(self, tokens, parent, logits, eos_id=-1):
        """Greedy acceptance (temperature 0): target token = argmax of the node's logits."""
        B, N = np.shape(tokens)
        tt, margin = self.row_argmax(logits)
        acc, path, out, fin = self.walk(tokens, parent, tt.reshape(B, N), eos_id)
        return acc, path, out, fin, tt.reshape(B, N), margin.reshape(B, N)

    def accept_sample_match(self, tokens, parent, logits, T, seed, row0=0, eos_id=-1):
        """Strict token match at temperature T: target token = one Gumbel-max sample per node."""
        B, N = np.shape(tokens)
        tt, margin = self.row_argmax(self.gumbel_scores(logits, T, seed, row0))
        acc, path, out, fin = self.walk(tokens, parent, tt.reshape(B, N), eos_id)
        return acc, path, out, fin, tt.reshape(B, N), margin.reshape(B, N)

    def accept_reject(self, tokens, parent, logits, draft_probs, unif, T, seed, row0=0, eos_id=-1):
        tokens, parent = _i32(tokens), _i32(parent)
        B, N = tokens.shape
        logits = np.ascontiguousarray(logits, dtype=self.real)
        draft_probs = np.ascontiguousarray(draft_probs, dtype=self.real)
        unif = np.ascontiguousarray(unif, dtype=self.real)
        V = logits.shape[-1]
        assert logits.size == B * N * V and draft_probs.size == B * N * V and unif.shape == (B, N)
        acc = np.empty(B, dtype=np.int32)
        path = np.empty((B, N), dtype=np.int32)
        out = np.empty((B, N), dtype=np.int32)
        fin = np.empty(B, dtype=np.int32)
        bm = np.empty(B, dtype=self.real)
        gap = np.empty(B, dtype=self.real)
        rc = self.lib.orc_accept_reject(C.c_int32(B), C.c_int32(N), C.c_int32(V), _ptr(tokens), _ptr(parent),
                                        _ptr(logits), _ptr(draft_probs), _ptr(unif), C.c_double(T),
                                        C.c_uint64(seed), C.c_int64(row0), C.c_int32(eos_id), _ptr(acc), _ptr(path),
                                        _ptr(out), _ptr(fin), _ptr(bm), _ptr(gap))
        self._check(rc, "orc_accept_reject")
        return acc, path, out, fin, bm, gap

    def kv_compact(self, cache, cfg, accept_len, path, slot=None):
        slot = None if slot is None else _i32(slot)
        accept_len, path = _i32(accept_len), _i32(path)
        B, N = path.shape
        rc = self.lib.orc_kv_compact(C.c_int32(cfg["n_layers"]), C.c_int32(B), C.c_int32(N),
                                     C.c_int32(cfg["n_kv_heads"]), C.c_int32(cfg["head_dim"]), _ptr(cache.k),
                                     _ptr(cache.v), C.c_int64(cache.cap), C.c_int32(cache.B), _ptr(slot),
                                     _ptr(cache.len), _ptr(accept_len), _ptr(path))
        self._check(rc, "orc_kv_compact")

    # -- draft side ------------------------------------------------------------------------------
    def topk_logp(self, logits, K):
        logits = np.ascontiguousarray(logits, dtype=self.real)
        M, V = logits.shape
        tok = np.empty((M, K), dtype=np.int32)
        logp = np.empty((M, K), dtype=self.real)
        self._check(self.lib.orc_topk_logp(_ptr(logits), C.c_int64(M), C.c_int64(V), C.c_int32(K), _ptr(tok),
                                           _ptr(logp)), "orc_topk_logp")
        return tok, logp

    def topk_index(self, scores, K):
        scores = np.ascontiguousarray(scores, dtype=np.float32)
        B, Cn = scores.shape
        idx = np.empty((B, K), dtype=np.int32)
        self._check(self.lib.orc_topk_index(_ptr(scores), C.c_int32(B), C.c_int32(Cn), C.c_int32(K), _ptr(idx)),
                    "orc_topk_index")
        return idx

    def build_tree(self, cand_tok, cand_parent, cand_score, N):
        cand_tok, cand_parent = _i32(cand_tok), _i32(cand_parent)
        cand_score = np.ascontiguousarray(cand_score, dtype=np.float32)
        B, Cn = cand_tok.shape
        tokens = np.empty((B, N), dtype=np.int32)
        parent = np.empty((B, N), dtype=np.int32)
        sel = np.empty((B, N), dtype=np.int32)
        rc = self.lib.orc_build_tree(_ptr(cand_tok), _ptr(cand_parent), _ptr(cand_score), C.c_int32(B),
                                     C.c_int32(Cn), C.c_int32(N), _ptr(tokens), _ptr(parent), _ptr(sel))
        self._check(rc, "orc_build_tree")
        return tokens, parent, sel

    # -- online draft learning -------------------------------------------------------------------
    def draft_train(self, draft, tokens, feat_in, feat_tgt, n_valid, w_ce=0.1):
        """Loss terms and gradients of every draft parameter (see orc_draft_train).  Returns (loss [2], grads dict)."""
        cfg = draft.cfg
        tokens = _i32(tokens)
        B, T = tokens.shape
        d, F = cfg["d_model"], cfg["d_ffn"]
        qkvd = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
        hq = cfg["n_q_heads"] * cfg["head_dim"]
        feat_in = np.ascontiguousarray(feat_in, dtype=self.real)
        feat_tgt = np.ascontiguousarray(feat_tgt, dtype=self.real)
        n_valid = _i32(n_valid)
        loss = np.zeros(2, dtype=self.real)
        shapes = dict(fc=(d, 2 * d), wqkv=(qkvd, d), wo=(d, hq), w_gate=(F, d), w_up=(F, d), w_down=(d, F), norm_attn=(d,), norm_ffn=(d,))
        g = {k: np.zeros(s, dtype=self.real) for k, s in shapes.items()}
        rc = self.lib.orc_draft_train(C.byref(draft.c), C.byref(draft.w), C.c_int32(B), C.c_int32(T), _ptr(tokens), _ptr(feat_in),
                                      _ptr(feat_tgt), _ptr(n_valid), C.c_double(w_ce), _ptr(loss), _ptr(g["fc"]), _ptr(g["wqkv"]),
                                      _ptr(g["wo"]), _ptr(g["w_gate"]), _ptr(g["w_up"]), _ptr(g["w_down"]), _ptr(g["norm_attn"]),
                                      _ptr(g["norm_ffn"]))
        self._check(rc, "orc_draft_train")
        return loss, g

    def adamw(self, p, g, m, v, lr, b1, b2, eps, wd, step):
        """In place on p, m, v (arrays of the oracle's real type)."""
        assert p.dtype == self.real and m.dtype == self.real and v.dtype == self.real
        g = np.ascontiguousarray(g, dtype=self.real)
        rc = self.lib.orc_adamw(_ptr(p), _ptr(g), _ptr(m), _ptr(v), C.c_int64(p.size), C.c_double(lr), C.c_double(b1),
                                C.c_double(b2), C.c_double(eps), C.c_double(wd), C.c_int32(step))
        self._check(rc, "orc_adamw")
