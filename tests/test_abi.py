"""CPU-side checks of the boundary: the library loads, exports what include/fastgrpo.h declares, and its host-only
logic (the concurrency rule, argument validation) behaves.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fastgrpo.h")


@pytest.fixture(scope="module")
def L():
    from paper_2509_21792_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.lib()


def declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fg_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared()
    assert "fg_spec_verify" in names and "fg_spec_accept" in names and "fg_kv_compact" in names and "fg_draft_step" in names
    for n in names:
        assert hasattr(L, n), n
    from paper_2509_21792_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_plan_matches_the_worked_table(L):
    from paper_2509_21792_amd import fg_plan
    for line in open(os.path.join(ROOT, "tests", "golden", "plan_table.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        f = line.split()
        got = fg_plan(int(f[0]), float(f[1]), float(f[2]), int(f[3]), int(f[4]), int(f[5]))
        assert got == (int(f[6]), int(f[7]), int(f[8])), line


def test_plan_agrees_with_oracle_on_a_sweep(L, orc32):
    from paper_2509_21792_amd import fg_plan
    for B in list(range(1, 70)) + [96, 128, 255, 256, 257, 512, 1000]:
        for Cp in (1.0, 7.5, 64.0, 100.0, 256.0, 315.0, 512.0, 1024.0, 2048.0, 4096.0):
            for alpha in (0.25, 0.5, 1.0, 3.0):
                assert fg_plan(B, Cp, alpha) == orc32.plan(B, Cp, alpha), (B, Cp, alpha)


def test_bad_arguments_are_errors_not_crashes(L):
    from paper_2509_21792_amd import FgError, fg_plan
    for args in [(0, 256.0), (4, 0.0), (4, 256.0, 0.0), (4, 256.0, 0.5, -1), (4, 256.0, 0.5, 4, 6, 65)]:
        with pytest.raises(FgError):
            fg_plan(*args)
    assert L.fg_spec_verify(None, None, None, None, None, None, None, None, 0, None) == -1
    assert b"NULL" in L.fg_last_error()
    assert L.fg_model_create(None, None, None) == -1
    assert L.fg_pack_weight(1, None, None, None, 32, 64, None) == -1
    assert L.fg_kv_compact(None, None, None, None, 1, 1, None, None, 0, 0, None) == -1
    assert L.fg_build_tree(None, None, None, 1, 4, 4, 8, None, None, None, None) == -1     # N > n_cand
    assert L.fg_draft_frontier(1, 9, 8, None, None, 9, *([None] * 4), 0, 100, *([None] * 8), 0, None, None, None) == -1   # K_in * K > 64
    assert L.fg_workspace_bytes(None, 8, 8) == 0
    assert L.fg_packed_bytes(1, 64, 128) == 64 * 128 * 2 and L.fg_packed_bytes(0, 64, 128) == 64 * 128 * 4


def test_knee_agrees_with_the_oracle_on_random_curves(L, orc32):
    """Host arithmetic of the library against the oracle's independent implementation (appendix, C_peak knee)."""
    import numpy as np
    from paper_2509_21792_amd import binding
    rng = np.random.default_rng(0)
    for t in range(300):
        n = int(rng.integers(3, 70))
        x = np.cumsum(rng.integers(1, 5, size=n)).astype(float)
        y = np.sort(rng.random(n)) * rng.random() * 10 if t % 2 else rng.random(n)
        assert binding.fg_knee(x, y) == orc32.knee(x, y)
    flat_then_up = [3.0] * 10 + [3.0 + 0.5 * i for i in range(1, 20)]
    assert binding.fg_knee(list(range(1, 30)), flat_then_up) == 9
    # the log2 axis is the library's own arithmetic: the same as handing it log2(x)
    xs = [1, 2, 4, 8, 16, 32, 64, 128, 256, 512]
    ys = [3.0, 3.0, 3.05, 3.1, 3.1, 3.3, 3.9, 5.1, 6.8, 9.2]
    assert binding.fg_knee(xs, ys, log2_axis=True) == binding.fg_knee(np.log2(xs), ys) == orc32.knee(np.log2(xs), ys)
    assert binding.fg_knee(xs, ys) == orc32.knee(xs, ys)
    with pytest.raises(binding.FgError):
        binding.fg_knee([1, 2], [1.0, 2.0])
    with pytest.raises(binding.FgError):
        binding.fg_knee([1, 1, 2], [1.0, 2.0, 3.0])


def test_kv_cache_helper_follows_the_documented_k_layout():
    """The Python cache helper plants and reads K through the page layouts the header documents: MFMA operand order
    for 16-bit caches with head_dim % 32 == 0, token-major otherwise.  Runs on CPU tensors (no kernel involved)."""
    import numpy as np
    import torch
    import paper_2509_21792_amd.binding as bd
    for dtype, hd in (("bf16", 128), ("fp16", 64), ("fp32", 16), ("bf16", 48)):
        cfg = dict(n_layers=2, n_kv_heads=3, head_dim=hd, dtype=dtype)
        pt = np.array([[3, 1, 4], [0, 2, 5]], np.int32)
        kv = bd.KVCache(cfg, pt, 6, device="cpu")
        L = 37
        g = torch.Generator().manual_seed(hd)
        k = torch.randn(2, L, 3, hd, generator=g).to(kv.k_pool.dtype)
        v = torch.randn(2, L, 3, hd, generator=g).to(kv.k_pool.dtype)
        kv.write_prefix(1, k, v)
        k2, v2 = kv.read(1, L)
        assert torch.equal(k2, k) and torch.equal(v2, v), (dtype, hd)
        flat = kv.k_pool.view(2, 6, 3, -1)
        for (l, t, h, e) in ((1, 20, 2, hd - 1), (0, 5, 0, 9), (1, 36, 1, hd // 2 + 3)):
            page, tt = pt[1, t // 16], t % 16
            if dtype != "fp32" and hd % 32 == 0:
                q = hd // 4
                grp, r = e // q, e % q
                off = (((r // 8) * 4 + grp) * 16 + tt) * 8 + r % 8
            else:
                off = tt * hd + e
            assert flat[l, page, h, off] == k[l, t, h, e], (dtype, hd, l, t, h, e)
        assert kv.v_pool[1, pt[1, 1], 2, 7, 4] == v[1, 20, 2, 7]


@pytest.mark.parametrize("model_name,max_rows,cap", [("7b", 160, 4096), ("7b", 640, 4096), ("1.5b", 640, 2048), ("7b", 1408, 2100)])
def test_workspace_bound_covers_every_call_shape(model_name, max_rows, cap):
    """fg_workspace_bytes_for(max_rows) must cover what any single call with B * N <= max_rows carves (host only): the
    attention part depends on how keys are cut into chunks, which is monotone neither in B nor in N (Eq. 1 produces
    N = 3, 5, 10, 44 ... as readily as powers of two)."""
    from synth import configs
    import paper_2509_21792_amd as fg
    cfg = configs.Q7B if model_name == "7b" else configs.Q1P5B
    for is_draft in (False, True):
        bound = fg.binding.fg_workspace_bytes_for(cfg, is_draft, max_rows, cap)
        assert bound > 0
        worst = 0
        for N in range(1, 65):
            for B in sorted(set([1, 2, 3, max_rows // N // 2, max_rows // N - 1, max_rows // N])):
                if B < 1 or B * N > max_rows:
                    continue
                need = fg.binding.fg_step_workspace_bytes(cfg, is_draft, B, N, cap, with_logits=True)
                assert 0 < need <= bound, (is_draft, B, N, need, bound)
                worst = max(worst, need)
        assert worst > 0.5 * bound          # the bound is not absurdly loose either
    # the shapes named as failing before the bound took every (B, N) into account
    for B, N in ((32, 5), (16, 3), (32, 44), (64, 10)):
        if B * N <= max_rows:
            assert fg.binding.fg_step_workspace_bytes(cfg, False, B, N, cap) <= fg.binding.fg_workspace_bytes_for(cfg, False, B * N, cap)


@pytest.mark.parametrize("M,n_out,n_in,epilogue,kernel", [
    # 7B-class gate/up with SwiGLU: decode kernel, few-row kernel, then the pipelined kernel from 32 rows on
    (8, 37888, 3584, 1, "gemm_mfma_decode_kernel"), (16, 37888, 3584, 1, "gemm_mfma_decode_kernel"),
    (24, 37888, 3584, 1, "gemm_mfma_skinny_kernel"), (32, 37888, 3584, 1, "gemm_mfma_big_kernel"),
    (128, 37888, 3584, 1, "gemm_mfma_big_kernel"), (2048, 37888, 3584, 1, "gemm_mfma_big_kernel"),
    # 1.5B-class gate/up: too few blocks for the pipelined kernel up to 64 rows
    (48, 17920, 1536, 1, "gemm_mfma_skinny_kernel"), (64, 17920, 1536, 1, "gemm_mfma_skinny_kernel"),
    (96, 17920, 1536, 1, "gemm_mfma_big_kernel"),
    # narrow outputs: few-row up to 64 rows, up to 128 for short contractions
    (8, 3584, 18944, 0, "gemm_mfma_skinny_kernel"), (64, 3584, 18944, 0, "gemm_mfma_skinny_kernel"),
    (96, 3584, 18944, 0, "gemm_mfma_big_kernel"), (96, 4608, 3584, 0, "gemm_mfma_skinny_kernel"),
    (128, 3584, 3584, 0, "gemm_mfma_skinny_kernel"), (144, 4608, 3584, 0, "gemm_mfma_big_kernel"),
    # LM head: few-row, streaming at 33 - 64 rows, pipelined above
    (8, 152064, 3584, 0, "gemm_mfma_skinny_kernel"), (32, 152064, 3584, 0, "gemm_mfma_skinny_kernel"),
    (48, 152064, 3584, 0, "gemm_mfma_kernel"), (64, 152064, 3584, 0, "gemm_mfma_kernel"),
    (96, 152064, 3584, 0, "gemm_mfma_big_kernel"),
    # fused epilogues exist in the pipelined kernel only
    (2048, 3584, 18944, 3, "gemm_mfma_big_kernel"),
])
def test_gemm_kernel_choice_at_the_measured_shapes(L, M, n_out, n_in, epilogue, kernel):
    """fg_gemm_kernel_name (host-only): the kernel the library picks at the row counts where its measurements put the
    switch points, for the 7B-class and 1.5B-class matrices -- a guard against an edit of one threshold moving another."""
    L.fg_gemm_kernel_name.restype = C.c_char_p
    L.fg_gemm_kernel_name.argtypes = [C.c_int32] * 4
    assert L.fg_gemm_kernel_name(M, n_out, n_in, epilogue).decode() == kernel
