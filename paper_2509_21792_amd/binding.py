"""Thin ctypes binding of libfastgrpo.so: the same entry points as include/fastgrpo.h, taking torch tensors.

Argument marshalling only.  torch is used for device memory and the current HIP stream; every step of the
hot path runs in the library's kernels.  There is no CPU fallback: without the built library (or without a
GPU for the compute calls) this module raises.
"""
import ctypes as C
import os

import numpy as np
import torch

FG_F32, FG_BF16, FG_F16 = 0, 1, 2
FG_MAX_NODES = 64
ACCEPT_GREEDY, ACCEPT_SAMPLE_MATCH, ACCEPT_REJECT = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastgrpo.so")

EXPORTS = ["fg_last_error", "fg_plan", "fg_packed_bytes", "fg_pack_weight", "fg_model_create", "fg_model_destroy",
           "fg_workspace_bytes", "fg_workspace_bytes_for", "fg_step_workspace_bytes", "fg_spec_verify", "fg_spec_accept", "fg_kv_compact", "fg_draft_step",
           "fg_draft_frontier", "fg_build_tree", "fg_gemm", "fg_attention", "fg_attention_workspace_bytes",
           "fg_topk_logp", "fg_lm_head_topk", "fg_lm_head_topk_workspace_bytes", "fg_knee", "fg_select_rows", "fg_model_profile",
           "fg_model_profile_read", "fg_gemm_kernel_name", "fg_spec_accept_static", "fg_draft_train_workspace_bytes", "fg_draft_train_grad", "fg_draft_train_head_bytes", "fg_draft_train_pack_head", "fg_draft_adamw", "fg_probe_read", "fg_probe_copy", "fg_probe_mfma"]
STATIC_SCRATCH_BYTES = 4 << 20


class FgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libfastgrpo error {code}: {msg}")
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                         "dtype", "max_pos")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p), ("fc", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_ffn")]


class KvCacheC(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("page_table", C.c_void_p), ("seq_len", C.c_void_p),
                ("status", C.c_void_p)] + \
               [(n, C.c_int32) for n in ("n_layers", "n_kv_heads", "head_dim", "dtype", "page_size", "max_pages_per_seq",
                                         "n_pages", "n_slots")]


class DraftParamsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("fc", "wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")]


class TreeC(C.Structure):
    _fields_ = [("slot", C.c_void_p), ("tokens", C.c_void_p), ("parent", C.c_void_p)] + \
               [(n, C.c_int32) for n in ("B", "N", "n_prev", "max_seq_len")]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -c 'import __graft_entry__ as g; g.build()')."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (__graft_entry__.build()); there is no fallback")
        L = C.CDLL(LIB_PATH)
        L.fg_last_error.restype = C.c_char_p
        L.fg_packed_bytes.restype = C.c_int64
        L.fg_packed_bytes.argtypes = [C.c_int32, C.c_int64, C.c_int64]
        L.fg_workspace_bytes.restype = C.c_int64
        L.fg_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.fg_workspace_bytes_for.restype = C.c_int64
        L.fg_workspace_bytes_for.argtypes = [C.POINTER(ModelCfg), C.c_int32, C.c_int32, C.c_int32]
        L.fg_step_workspace_bytes.restype = C.c_int64
        L.fg_step_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.fg_attention_workspace_bytes.restype = C.c_int64
        L.fg_attention_workspace_bytes.argtypes = [C.c_int32] * 6
        L.fg_plan.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_int32, C.c_int32] + [C.POINTER(C.c_int32)] * 3
        L.fg_pack_weight.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]
        L.fg_model_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(Weights), C.POINTER(C.c_void_p)]
        L.fg_model_destroy.argtypes = [C.c_void_p]
        L.fg_spec_verify.argtypes = [C.c_void_p, C.POINTER(KvCacheC), C.POINTER(TreeC), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_spec_accept.argtypes = [C.POINTER(TreeC), C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p,
                                     C.c_void_p, C.c_uint64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_spec_accept_static.argtypes = L.fg_spec_accept.argtypes[:15] + [C.c_void_p]
        L.fg_probe_read.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.fg_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
        L.fg_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.fg_draft_train_workspace_bytes.restype = C.c_int64
        L.fg_draft_train_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int32, C.c_int32]
        L.fg_draft_train_grad.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p, C.POINTER(DraftParamsC), C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.POINTER(DraftParamsC), C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_draft_train_head_bytes.restype = C.c_int64
        L.fg_draft_train_head_bytes.argtypes = [C.POINTER(ModelCfg)]
        L.fg_draft_train_pack_head.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_draft_adamw.argtypes = [C.POINTER(ModelCfg), C.POINTER(DraftParamsC), C.POINTER(DraftParamsC), C.POINTER(DraftParamsC),
                                     C.POINTER(DraftParamsC)] + [C.c_float] * 5 + [C.c_int32, C.c_void_p]
        L.fg_kv_compact.argtypes = [C.POINTER(KvCacheC), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.fg_draft_step.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(KvCacheC), C.POINTER(TreeC), C.c_void_p, C.c_void_p,
                                    C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_draft_frontier.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32] + [C.c_void_p] * 4 + \
                                       [C.c_int32, C.c_int32] + \
                                       [C.c_void_p] * 8 + [C.c_int32, C.c_void_p, C.c_void_p]
        L.fg_knee.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        L.fg_select_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.fg_topk_logp.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.fg_lm_head_topk_workspace_bytes.restype = C.c_int64
        L.fg_lm_head_topk_workspace_bytes.argtypes = [C.c_int32] * 3
        L.fg_lm_head_topk.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.fg_build_tree.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.fg_gemm.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                              C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_void_p]
        L.fg_gemm_kernel_name.restype = C.c_char_p
        L.fg_gemm_kernel_name.argtypes = [C.c_int32] * 4
        L.fg_model_profile.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.fg_model_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        L.fg_attention.argtypes = [C.POINTER(KvCacheC), C.c_int32, C.POINTER(TreeC), C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int64, C.c_void_p]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise FgError(rc, lib().fg_last_error().decode())


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _tdtype(dtype):
    return {FG_F32: torch.float32, FG_BF16: torch.bfloat16, FG_F16: torch.float16}[dtype]


def dtype_code(name):
    return {"fp32": FG_F32, "bf16": FG_BF16, "fp16": FG_F16}[name]


def _code_of(t):
    return {torch.float32: FG_F32, torch.bfloat16: FG_BF16, torch.float16: FG_F16}[t.dtype]


# ---- host-only ---------------------------------------------------------------------------------------------
def fg_plan(B_cur, C_peak, alpha=0.5, K_max=4, L_max=6, N_cap=64):
    N, K, Lr = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().fg_plan(B_cur, C_peak, alpha, K_max, L_max, N_cap, C.byref(N), C.byref(K), C.byref(Lr)))
    return N.value, K.value, Lr.value


def model_cfg_struct(cfg, max_pos=8192):
    return ModelCfg(cfg["n_layers"], cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ffn"],
                    cfg["vocab"], dtype_code(cfg["dtype"]), max_pos, cfg.get("rms_eps", 1e-6), cfg.get("rope_theta", 10000.0))


def fg_workspace_bytes_for(cfg, is_draft, max_rows, max_seq_len):
    """Host only: the workspace that suffices for every call of at most max_rows rows (see fastgrpo.h)."""
    c = model_cfg_struct(cfg)
    return lib().fg_workspace_bytes_for(C.byref(c), int(is_draft), max_rows, max_seq_len)


def fg_step_workspace_bytes(cfg, is_draft, B, N, max_seq_len, with_logits=True):
    """Host only: what one call of shape (B, N) carves from its workspace."""
    c = model_cfg_struct(cfg)
    return lib().fg_step_workspace_bytes(C.byref(c), int(is_draft), B, N, max_seq_len, int(with_logits))


# ---- weights and model ---------------------------------------------------------------------------------------
def fg_pack_weight(dtype, src, src2=None):
    """src [n_out, n_in] (and optionally src2 of the same shape, interleaved in blocks of 32 rows) -> packed tensor."""
    src = src.contiguous()
    n_out, n_in = src.shape
    total = n_out * (2 if src2 is not None else 1)
    if src2 is not None:
        src2 = src2.contiguous()
        assert src2.shape == src.shape
    dst = torch.empty(total * n_in, dtype=_tdtype(dtype), device=src.device)
    assert lib().fg_packed_bytes(dtype, total, n_in) == dst.numel() * dst.element_size()
    _check(lib().fg_pack_weight(dtype, _p(src), _p(src2), _p(dst), n_out, n_in, _stream()))
    return dst


class Model:
    """A target model or a draft head on the device.  `weights` is the dict layout of synth.gen.make_weights with
    torch tensors on the device; a draft head passes target=<Model> to share its embedding and LM head."""

    def __init__(self, cfg, weights, target=None, max_pos=8192):
        self.cfg = dict(cfg)
        self.dtype = dtype_code(cfg["dtype"])
        td = _tdtype(self.dtype)
        dev = weights["layers"][0]["wqkv"].device
        cast = lambda t: t.to(device=dev, dtype=td).contiguous()
        self.keep = []

        def packed(a, b=None):
            t = fg_pack_weight(self.dtype, cast(a), None if b is None else cast(b))
            self.keep.append(t)
            return t

        w = Weights()
        if target is None:
            self.embed = cast(weights["embed"])
            self.lm_head = packed(weights["lm_head"])
            self.final_norm = cast(weights["final_norm"])
            self.fc = None
        else:
            self.embed, self.lm_head, self.final_norm = target.embed, target.lm_head, None
            self.fc = packed(weights["fc"])
        w.embed, w.lm_head = self.embed.data_ptr(), self.lm_head.data_ptr()
        w.final_norm = None if self.final_norm is None else self.final_norm.data_ptr()
        w.fc = None if self.fc is None else self.fc.data_ptr()
        nl = cfg["n_layers"]
        per = {k: [] for k in ("wqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_ffn")}
        for lay in weights["layers"]:
            per["wqkv"].append(packed(lay["wqkv"]))
            per["wo"].append(packed(lay["wo"]))
            per["w_gate_up"].append(packed(lay["w_gate"], lay["w_up"]))
            per["w_down"].append(packed(lay["w_down"]))
            for k in ("norm_attn", "norm_ffn"):
                t = cast(lay[k])
                self.keep.append(t)
                per[k].append(t)
        self._tabs = []
        for k, lst in per.items():
            tab = (C.c_void_p * nl)(*[t.data_ptr() for t in lst])
            self._tabs.append(tab)
            setattr(w, k, C.cast(tab, C.POINTER(C.c_void_p)))
        c = model_cfg_struct(cfg, max_pos)
        self.max_pos = max_pos
        h = C.c_void_p()
        torch.cuda.current_stream().synchronize()
        _check(lib().fg_model_create(C.byref(c), C.byref(w), C.byref(h)))
        self.handle = h

    def workspace(self, max_rows, max_seq_len):
        n = lib().fg_workspace_bytes(self.handle, max_rows, max_seq_len)
        if n <= 0:
            raise FgError(-1, "fg_workspace_bytes failed")
        return torch.empty(n, dtype=torch.uint8, device=self.embed.device)

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                lib().fg_model_destroy(self.handle)
                self.handle = None
        except Exception:
            pass


class KVCache:
    """Paged cache on the device.  page_table: int32 [n_slots, max_pages] (numpy or tensor)."""

    def __init__(self, cfg, page_table, n_pages, device="cuda", page_size=16):
        self.cfg = dict(cfg)
        self.dtype = dtype_code(cfg["dtype"])
        td = _tdtype(self.dtype)
        nl, Hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
        self.page_table = torch.as_tensor(np.asarray(page_table), dtype=torch.int32).to(device).contiguous()
        self.n_slots, self.max_pages = self.page_table.shape
        self.n_pages, self.page_size = n_pages, page_size
        self.k_pool = torch.zeros((nl, n_pages, Hkv, page_size, hd), dtype=td, device=device)
        self.v_pool = torch.zeros((nl, n_pages, Hkv, hd, page_size), dtype=td, device=device)
        self.seq_len = torch.zeros(self.n_slots, dtype=torch.int32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.c = KvCacheC(self.k_pool.data_ptr(), self.v_pool.data_ptr(), self.page_table.data_ptr(), self.seq_len.data_ptr(),
                          self.status.data_ptr(), nl, Hkv, hd, self.dtype, page_size, self.max_pages, n_pages, self.n_slots)

    @property
    def capacity(self):
        return self.max_pages * self.page_size

    def check(self):
        """Raise if a call since the last check ran past a page table or the RoPE table (reads the status word: one
        small device-to-host copy)."""
        flags = int(self.status.item())
        if flags:
            self.status.zero_()
            what = [n for bit, n in ((1, "a sequence ran past its page table (nothing was appended or committed for it)"),
                                     (2, "a position beyond the RoPE table was clamped")) if flags & bit]
            raise FgError(-3, "; ".join(what))

    def _where(self, slot, L):
        t = torch.arange(L, device=self.k_pool.device)
        pages = self.page_table[slot, (t // self.page_size)].long()
        return pages, (t % self.page_size)

    def _k_offsets(self):
        """[page_size, hd] element offsets of (token, dim) inside one (page, kv head) block of k_pool: MFMA operand
        order for 16-bit caches with head_dim % 32 == 0, token-major otherwise (see fastgrpo.h)."""
        hd, dev = self.cfg["head_dim"], self.k_pool.device
        t = torch.arange(self.page_size, device=dev)[:, None]
        e = torch.arange(hd, device=dev)[None, :]
        if self.dtype in (FG_BF16, FG_F16) and hd % 32 == 0 and self.page_size == 16:
            q = hd // 4
            g, r = e // q, e % q
            return (((r // 8) * 4 + g) * 16 + t) * 8 + r % 8
        return t * hd + e

    def write_prefix(self, slot, k, v):
        """Set-up helper: k, v [n_layers, L, Hkv, hd] become positions 0..L-1 of `slot`; seq_len[slot] = L."""
        L = k.shape[1]
        pages, off = self._where(slot, L)
        nl, n_pages, Hkv = self.k_pool.shape[:3]
        flat = self.k_pool.view(nl, n_pages, Hkv, -1)
        # index tensors [L, 1] and [L, hd] around a slice: the result is laid out [L, hd, n_layers, Hkv]
        flat[:, pages[:, None], :, self._k_offsets()[off]] = k.to(self.k_pool.dtype).permute(1, 3, 0, 2)
        self.v_pool[:, pages, :, :, off] = v.to(self.v_pool.dtype).permute(1, 0, 2, 3)
        self.seq_len[slot] = L

    def read(self, slot, L):
        """Test helper: positions 0..L-1 of `slot` as contiguous k, v [n_layers, L, Hkv, hd]."""
        pages, off = self._where(slot, L)
        nl, n_pages, Hkv = self.k_pool.shape[:3]
        flat = self.k_pool.view(nl, n_pages, Hkv, -1)
        k = flat[:, pages[:, None], :, self._k_offsets()[off]].permute(2, 0, 3, 1).contiguous()
        v = self.v_pool[:, pages, :, :, off].permute(1, 0, 2, 3).contiguous()
        return k, v


def _tree(slot, tokens, parent, B, N, n_prev, max_seq_len):
    return TreeC(None if slot is None else slot.data_ptr(), None if tokens is None else tokens.data_ptr(),
                 None if parent is None else parent.data_ptr(), B, N, n_prev, max_seq_len)


def _dev_i32(x, device):
    if isinstance(x, torch.Tensor):
        return x.to(device=device, dtype=torch.int32).contiguous()
    return torch.as_tensor(np.ascontiguousarray(x, dtype=np.int32)).to(device)


# ---- the hot path -----------------------------------------------------------------------------------------
def fg_spec_verify(model, kv, slot, tokens, parent, workspace, n_prev=0, max_seq_len=0, want_logits=False,
                   want_feature=True, want_argmax=True, want_top2=False):
    dev = kv.k_pool.device
    slot, tokens, parent = _dev_i32(slot, dev), _dev_i32(tokens, dev), _dev_i32(parent, dev)
    B, N = tokens.shape
    M, d, V = B * N, model.cfg["d_model"], model.cfg["vocab"]
    out = {}
    out["logits"] = torch.empty((M, V), dtype=torch.float32, device=dev) if want_logits else None
    out["feature"] = torch.empty((M, d), dtype=_tdtype(model.dtype), device=dev) if want_feature else None
    out["argmax"] = torch.empty(M, dtype=torch.int32, device=dev) if want_argmax else None
    out["top2"] = torch.empty((M, 2), dtype=torch.float32, device=dev) if want_top2 else None
    tree = _tree(slot, tokens, parent, B, N, n_prev, max_seq_len)
    _check(lib().fg_spec_verify(model.handle, C.byref(kv.c), C.byref(tree), _p(out["logits"]), _p(out["feature"]),
                                _p(out["argmax"]), _p(out["top2"]), _p(workspace), workspace.numel(), _stream()))
    out["_keep"] = (slot, tokens, parent)
    return out


def fg_spec_accept(tokens, parent, mode=ACCEPT_GREEDY, logits=None, row_argmax=None, vocab=0, temperature=1.0,
                   draft_probs=None, uniforms=None, seed=0, row0=0, eos_id=-1, workspace=None):
    dev = tokens.device if isinstance(tokens, torch.Tensor) else (logits if logits is not None else row_argmax).device
    tokens, parent = _dev_i32(tokens, dev), _dev_i32(parent, dev)
    B, N = tokens.shape
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, N), dtype=torch.int32, device=dev)
    out = torch.empty((B, N), dtype=torch.int32, device=dev)
    fin = torch.empty(B, dtype=torch.int32, device=dev)
    if workspace is None:
        need = B * N * 4 if mode != ACCEPT_REJECT else B * 2 * max(vocab, 1) * 4
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    tree = _tree(None, tokens, parent, B, N, 0, 0)
    _check(lib().fg_spec_accept(C.byref(tree), mode, _p(logits), _p(row_argmax), vocab, temperature, _p(draft_probs),
                                _p(uniforms), seed, row0, eos_id, _p(acc), _p(path), _p(out), _p(fin), _p(workspace),
                                workspace.numel(), _stream()))
    return acc, path, out, fin


def fg_spec_accept_static(tokens, parent, mode=ACCEPT_GREEDY, logits=None, row_argmax=None, vocab=0, temperature=1.0,
                          draft_probs=None, uniforms=None, seed=0, row0=0, eos_id=-1, out=None):
    """fg_spec_accept on the library's static scratch.  `out` = (accept_len, path, out_tokens, finished) tensors to
    write into (a caller that may not allocate passes them); allocated here otherwise."""
    dev = tokens.device
    B, N = tokens.shape
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev),
               torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev))
    acc, path, otok, fin = out
    tree = _tree(None, tokens, parent, B, N, 0, 0)
    _check(lib().fg_spec_accept_static(C.byref(tree), mode, _p(logits), _p(row_argmax), vocab, temperature, _p(draft_probs),
                                       _p(uniforms), seed, row0, eos_id, _p(acc), _p(path), _p(otok), _p(fin), _stream()))
    return acc, path, otok, fin


def fg_kv_compact(kv, slot, accept_len, path, feature_in=None, d_model=0):
    dev = kv.k_pool.device
    slot = _dev_i32(slot, dev)
    B, N = path.shape
    fout = None
    fdt = kv.dtype
    if feature_in is not None:
        fout = torch.empty((B, N, d_model), dtype=feature_in.dtype, device=dev)
        fdt = _code_of(feature_in)
    _check(lib().fg_kv_compact(C.byref(kv.c), _p(slot), _p(accept_len), _p(path), B, N, _p(feature_in), _p(fout), d_model,
                               fdt, _stream()))
    return fout


def fg_draft_step(target, draft, draft_kv, slot, tokens, parent, in_feature, workspace, K_draft, n_prev=0, feat_index=None,
                  n_commit=None, commit_bias=0, max_seq_len=0, want_children=True, expand_row=None):
    """expand_row [B]: decode only that node of each sequence; the child lists are then [B, 1, K_draft]."""
    dev = draft_kv.k_pool.device
    slot, tokens, parent = _dev_i32(slot, dev), _dev_i32(tokens, dev), _dev_i32(parent, dev)
    B, N = tokens.shape
    d = draft.cfg["d_model"]
    in_feature = in_feature.contiguous()
    assert in_feature.dim() == 3 and in_feature.shape[0] == B and in_feature.shape[2] == d
    assert in_feature.dtype == _tdtype(draft.dtype)
    feat_rows = in_feature.shape[1]
    if feat_index is not None:
        feat_index = _dev_i32(feat_index, dev)
    rows = N if expand_row is None else 1
    if expand_row is not None:
        expand_row = _dev_i32(expand_row, dev)
    ctok = torch.empty((B, rows, K_draft), dtype=torch.int32, device=dev) if want_children else None
    clogp = torch.empty((B, rows, K_draft), dtype=torch.float32, device=dev) if want_children else None
    ofeat = torch.empty((B, N, d), dtype=_tdtype(draft.dtype), device=dev)
    if n_commit is not None:
        n_commit = _dev_i32(n_commit, dev)
    tree = _tree(slot, tokens, parent, B, N, n_prev, max_seq_len)
    _check(lib().fg_draft_step(target.handle, draft.handle, C.byref(draft_kv.c), C.byref(tree), _p(in_feature), _p(feat_index),
                               feat_rows, _p(n_commit), commit_bias, K_draft, _p(expand_row), _p(ctok), _p(clogp), _p(ofeat), _p(workspace),
                               workspace.numel(), _stream()))
    return ctok, clogp, ofeat


def fg_draft_frontier(child_tok, child_logp, n_cand, cand_tok, cand_parent, cand_score, node_cand=None, node_score=None,
                      node_pick=None, node_tok=None, parent_prev=None):
    """Returns (next_tok, next_cand, next_score, next_src, parent_next); parent_prev [B, n] is the round's in-round
    parent list so far (None / empty before the first step)."""
    B, child_rows, K = child_tok.shape
    K_in = child_rows if node_tok is None else node_tok.shape[1]
    dev = child_tok.device
    nt = torch.empty((B, K), dtype=torch.int32, device=dev)
    nc = torch.empty((B, K), dtype=torch.int32, device=dev)
    ns = torch.empty((B, K), dtype=torch.float32, device=dev)
    nsrc = torch.empty((B, K), dtype=torch.int32, device=dev)
    npp = 0 if parent_prev is None else parent_prev.shape[1]
    pnext = torch.empty((B, npp + K), dtype=torch.int32, device=dev)
    _check(lib().fg_draft_frontier(B, K_in, K, _p(child_tok), _p(child_logp), child_rows, _p(node_cand), _p(node_score), _p(node_pick),
                                   _p(node_tok), n_cand, cand_tok.shape[1], _p(cand_tok), _p(cand_parent), _p(cand_score), _p(nt),
                                   _p(nc), _p(ns), _p(nsrc), _p(parent_prev) if npp else None, npp, _p(pnext), _stream()))
    return nt, nc, ns, nsrc, pnext


def fg_build_tree(cand_tok, cand_parent, cand_score, n_cand, N):
    B, stride = cand_tok.shape
    dev = cand_tok.device
    tokens = torch.empty((B, N), dtype=torch.int32, device=dev)
    parent = torch.empty((B, N), dtype=torch.int32, device=dev)
    sel = torch.empty((B, N), dtype=torch.int32, device=dev)
    _check(lib().fg_build_tree(_p(cand_tok), _p(cand_parent), _p(cand_score), B, n_cand, stride, N, _p(tokens), _p(parent),
                               _p(sel), _stream()))
    return tokens, parent, sel


def fg_topk_logp(logits, K):
    M, V = logits.shape
    tok = torch.empty((M, K), dtype=torch.int32, device=logits.device)
    logp = torch.empty((M, K), dtype=torch.float32, device=logits.device)
    _check(lib().fg_topk_logp(_p(logits), M, V, K, _p(tok), _p(logp), _stream()))
    return tok, logp


def fg_lm_head_topk(dtype, x, lm_head_packed, vocab, K):
    """Top-K tokens and log-probabilities of x . lm_head^T with the selection in the GEMM's epilogue."""
    x = x.contiguous()
    M, d = x.shape
    tok = torch.empty((M, K), dtype=torch.int32, device=x.device)
    logp = torch.empty((M, K), dtype=torch.float32, device=x.device)
    ws = torch.empty(max(lib().fg_lm_head_topk_workspace_bytes(M, vocab, K), 256), dtype=torch.uint8, device=x.device)
    _check(lib().fg_lm_head_topk(dtype, _p(x), _p(lm_head_packed), M, vocab, d, K, _p(tok), _p(logp), _p(ws), ws.numel(), _stream()))
    return tok, logp


def fg_knee(x, y, log2_axis=False):
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.float64)
    k = C.c_int32()
    _check(lib().fg_knee(x.ctypes.data_as(C.c_void_p), y.ctypes.data_as(C.c_void_p), len(x), int(log2_axis), C.byref(k)))
    return k.value


def fg_select_rows(src, index):
    """src [n_src, ...] contiguous device tensor, index int32 [n] on the device -> src[index] ([n, ...])."""
    assert src.is_contiguous()
    n_src = src.shape[0]
    row_bytes = src[0].numel() * src.element_size() if n_src else 0
    dst = torch.empty((index.shape[0],) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    _check(lib().fg_select_rows(_p(src), row_bytes, n_src, _p(index), index.shape[0], _p(dst), _stream()))
    return dst


# ---- online draft learning -------------------------------------------------------------------------------------------
PARAM_NAMES = ("fc", "wqkv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")


def draft_param_shapes(cfg):
    d, F = cfg["d_model"], cfg["d_ffn"]
    hq = cfg["n_q_heads"] * cfg["head_dim"]
    qkvd = (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    return dict(fc=(d, 2 * d), wqkv=(qkvd, d), wo=(d, hq), w_gate=(F, d), w_up=(F, d), w_down=(d, F), norm_attn=(d,), norm_ffn=(d,))


def _params_struct(p):
    for n in PARAM_NAMES:
        assert p[n].dtype == torch.float32 and p[n].is_contiguous() and p[n].is_cuda, n
    return DraftParamsC(*[p[n].data_ptr() for n in PARAM_NAMES])


def fg_draft_train_workspace_bytes(cfg, B, T, compute="fp32"):
    c = model_cfg_struct(dict(cfg, dtype=compute))
    return lib().fg_draft_train_workspace_bytes(C.byref(c), B, T)


def fg_draft_train_pack_head(cfg, lm_head):
    """The frozen LM head (fp32 [vocab, d] on the device) rounded to bf16 and packed once for the matrix-core training
    step; pass the returned buffer as head_packed to fg_draft_train_grad while lm_head stays the same."""
    c = model_cfg_struct(dict(cfg, dtype="bf16"))
    assert lm_head.dtype == torch.float32 and lm_head.is_contiguous()
    buf = torch.empty(lib().fg_draft_train_head_bytes(C.byref(c)), dtype=torch.uint8, device=lm_head.device)
    _check(lib().fg_draft_train_pack_head(C.byref(c), _p(lm_head), _p(buf), buf.numel(), _stream()))
    return buf


def fg_draft_train_grad(cfg, embed, lm_head, w, tokens, feat_in, feat_tgt, n_valid, w_ce=0.1, grad=None, workspace=None,
                        compute="fp32", head_packed=None):
    """Loss terms (device tensor [2]) and gradients (dict of fp32 tensors shaped like `w`) of the draft head's training
    loss; embed / lm_head: the target's, fp32 row-major on the device.  compute: "fp32" (exact) or "bf16" (the step's
    matrix products on the matrix cores; head_packed: fg_draft_train_pack_head(cfg, lm_head), optional)."""
    dev = tokens.device
    B, T = tokens.shape
    c = model_cfg_struct(dict(cfg, dtype=compute))
    if grad is None:
        grad = {n: torch.empty(s, dtype=torch.float32, device=dev) for n, s in draft_param_shapes(cfg).items()}
    if workspace is None:
        workspace = torch.empty(lib().fg_draft_train_workspace_bytes(C.byref(c), B, T), dtype=torch.uint8, device=dev)
    loss = torch.empty(2, dtype=torch.float32, device=dev)
    ws, gs = _params_struct(w), _params_struct(grad)
    for t in (embed, lm_head, feat_in, feat_tgt):
        assert t.dtype == torch.float32 and t.is_contiguous()
    _check(lib().fg_draft_train_grad(C.byref(c), _p(embed), _p(lm_head), C.byref(ws), _p(_dev_i32(tokens, dev)), _p(feat_in), _p(feat_tgt),
                                     _p(_dev_i32(n_valid, dev)), B, T, w_ce, C.byref(gs), _p(loss),
                                     _p(head_packed) if head_packed is not None else None, _p(workspace), workspace.numel(), _stream()))
    return loss, grad


def fg_draft_adamw(cfg, w, grad, m, v, lr, step, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    c = model_cfg_struct(dict(cfg, dtype="fp32"))
    ws, gs, ms, vs = (_params_struct(x) for x in (w, grad, m, v))
    _check(lib().fg_draft_adamw(C.byref(c), C.byref(ws), C.byref(gs), C.byref(ms), C.byref(vs), lr, beta1, beta2, eps, weight_decay,
                                step, _stream()))


# ---- stage timing ------------------------------------------------------------------------------------------------
STAGES = ["prep", "norm", "qkv", "rope", "attention", "o", "gate_up", "swiglu", "down", "lm_head", "select", "fc"]


def fg_model_profile(model, enable, max_marks=1 << 16, only=None):
    """enable: off / every stage; only="gate_up" (a name from STAGES): bracket that stage alone."""
    code = int(bool(enable)) if only is None or not enable else 2 + STAGES.index(only)
    _check(lib().fg_model_profile(model.handle, code, max_marks))


def fg_model_profile_read(model):
    """{stage: (milliseconds, launches)} since the last read."""
    n = len(STAGES)
    ms, cnt = (C.c_double * n)(), (C.c_int32 * n)()
    _check(lib().fg_model_profile_read(model.handle, ms, cnt))
    return {STAGES[i]: (ms[i], cnt[i]) for i in range(n)}


def fg_gemm_kernel_name(M, n_out, n_in, epilogue=0):
    return lib().fg_gemm_kernel_name(M, n_out, n_in, epilogue).decode()


# ---- ceiling probes ---------------------------------------------------------------------------------------------
def fg_probe_read(src, nontemporal, blocks, sink):
    _check(lib().fg_probe_read(_p(src), src.numel() * src.element_size(), int(nontemporal), blocks, _p(sink), _stream()))


def fg_probe_copy(src, dst, blocks):
    _check(lib().fg_probe_copy(_p(src), _p(dst), src.numel() * src.element_size(), blocks, _stream()))


def fg_probe_mfma(dtype, iters, random_operands, blocks, sink):
    _check(lib().fg_probe_mfma(dtype, iters, int(random_operands), blocks, _p(sink), _stream()))


# ---- kernel-level ---------------------------------------------------------------------------------------------
def fg_gemm(dtype, x, w_packed, n_out, epilogue=0, split_k=0, variant=0, out=None):
    """epilogue 0: returns (slabs [split, M, n_out] fp32, split): the caller adds the slabs.  1: (silu(gate) * up, 1).
    3: `out` fp32 [M, n_out] is updated in place and returned."""
    x = x.contiguous()
    M, n_in = x.shape
    used = C.c_int32(1)
    if epilogue == 0:
        smax = 16 if split_k == 0 else split_k
        out = torch.empty((smax, M, n_out), dtype=torch.float32, device=x.device)
    elif epilogue == 1:
        out = torch.empty((M, n_out // 2), dtype=x.dtype, device=x.device)
    else:
        assert out is not None and out.dtype == torch.float32 and out.shape == (M, n_out) and out.is_contiguous()
    _check(lib().fg_gemm(dtype, _p(x), _p(w_packed), _p(out), M, n_out, n_in, epilogue, split_k, C.byref(used), variant, _stream()))
    if epilogue == 0:
        return out[:used.value], used.value
    return out, 1


def fg_attention(kv, layer, slot, parent, B, N, n_q_heads, q, n_prev=0, max_seq_len=0):
    dev = kv.k_pool.device
    slot, parent = _dev_i32(slot, dev), _dev_i32(parent, dev)
    hd = kv.cfg["head_dim"]
    cap = kv.max_pages * kv.page_size
    ws = torch.empty(lib().fg_attention_workspace_bytes(B, N, n_q_heads, kv.cfg["n_kv_heads"], hd, max_seq_len or cap), dtype=torch.uint8, device=dev)
    out = torch.empty_like(q)
    tree = _tree(slot, None, parent, B, N, n_prev, max_seq_len)
    _check(lib().fg_attention(C.byref(kv.c), layer, C.byref(tree), n_q_heads, _p(q), _p(out), _p(ws), ws.numel(), _stream()))
    return out
