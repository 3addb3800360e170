"""Kernel-level checks on the GPU (through the C ABI): the packed bf16 MFMA GEMM and the tree attention kernels
against their plain definitions evaluated with torch library routines in fp64 on the CPU.  The step-level parity
against the oracle is in test_gpu_verify.py; these narrow a failure down to one kernel."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fg():
    import paper_2509_21792_amd as m
    m.lib()
    assert torch.cuda.is_available()
    return m


def bf16_randn(shape, gen, scale=1.0, dt=torch.bfloat16):
    return (torch.randn(shape, generator=gen, dtype=torch.float32) * scale).to(torch.bfloat16).to(dt)


CODES = {"bf16": 1, "fp16": 2}
TD = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}


def gemm_sum(fg, code, x, wp, N, **kw):
    """x . W^T through fg_gemm's partial-sum epilogue: the k-split slabs added in slab order (what the library's
    consumer kernels do); returns (sum [M, N] fp32, number of slabs)."""
    slabs, used = fg.fg_gemm(code, x, wp, N, epilogue=0, **kw)
    out = slabs[0].clone()
    for s in range(1, used):
        out += slabs[s]
    return out, used


@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (8, 4608, 3584), (48, 3584, 3584), (40, 96, 128), (130, 1024, 704 - 64),
                                   (192, 3584, 18944), (256, 512, 256), (257, 544, 192), (700, 4608, 1536)])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_gemm_16bit_partial_epilogue(fg, M, N, K, dtype):
    print(f"gemm {dtype} M={M} N={N} K={K}", flush=True)
    code = CODES[dtype]
    g = torch.Generator().manual_seed(M * 7 + N)
    x, w = bf16_randn((M, K), g, dt=TD[dtype]), bf16_randn((N, K), g, 0.05, dt=TD[dtype])
    ref = x.double() @ w.double().T
    wp = fg.fg_pack_weight(code, w.cuda())
    for split in (0, 1, 3):
        out, used = gemm_sum(fg, code, x.cuda(), wp, N, split_k=split)
        torch.cuda.synchronize()
        err = (out.double().cpu() - ref).abs().max().item()
        scale = ref.abs().max().item()
        assert err <= 2e-5 * scale + 1e-4, (split, used, err, scale)
    # run twice: split-K slabs are summed in a fixed order, so results are bitwise repeatable
    a, _ = gemm_sum(fg, code, x.cuda(), wp, N)
    b, _ = gemm_sum(fg, code, x.cuda(), wp, N)
    assert torch.equal(a, b)


@pytest.mark.parametrize("chunks", [1, 2, 3, 4, 5, 6, 7, 8, 11, 12, 13, 19])
def test_gemm_16bit_many_rows_every_k_tail(fg, chunks):
    """More than 256 rows takes the pipelined kernel, whose main loop handles six 64-wide k chunks per trip: every
    tail length, a ragged last row block and a ragged last column band."""
    M, N, K = 300, 288, 64 * chunks
    print(f"gemm many rows chunks={chunks}", flush=True)
    g = torch.Generator().manual_seed(chunks)
    for dtype in ("bf16", "fp16"):
        x, w = bf16_randn((M, K), g, dt=TD[dtype]), bf16_randn((N, K), g, 0.05, dt=TD[dtype])
        ref = x.double() @ w.double().T
        wp = fg.fg_pack_weight(CODES[dtype], w.cuda())
        out, used = gemm_sum(fg, CODES[dtype], x.cuda(), wp, N, split_k=1)
        torch.cuda.synchronize()
        err = (out.double().cpu() - ref).abs().max().item()
        assert used == 1 and err <= 2e-5 * ref.abs().max().item() + 1e-4, (dtype, err)


@pytest.mark.parametrize("chunks", [1, 2, 3, 4, 5, 7, 8, 9, 13, 18])
def test_gemm_16bit_few_rows_every_k_tail(fg, chunks):
    """Up to 128 rows (narrow outputs) takes the few-row kernel (k split inside the block, rounds of four 64-wide k
    chunks): every tail length of the last round, one to four row tiles with ragged ends, two row blocks, an odd number of column bands, requested
    splits that leave the last split short or empty, and the fused SwiGLU epilogue."""
    K = 64 * chunks
    print(f"gemm few rows chunks={chunks}", flush=True)
    g = torch.Generator().manual_seed(100 + chunks)
    for dtype, M in (("bf16", 1), ("fp16", 31), ("bf16", 33), ("fp16", 64), ("bf16", 65), ("fp16", 96), ("bf16", 127),
                     ("fp16", 129), ("bf16", 200), ("fp16", 256)):   # two row blocks (short k)
        N = 96 + 64 * (M % 3)          # 3, 5 or 7 bands of 32 columns
        x, w = bf16_randn((M, K), g, dt=TD[dtype]), bf16_randn((N, K), g, 0.05, dt=TD[dtype])
        ref = x.double() @ w.double().T
        wp = fg.fg_pack_weight(CODES[dtype], w.cuda())
        for split in (0, 1, 2, 3, 5):
            out, used = gemm_sum(fg, CODES[dtype], x.cuda(), wp, N, split_k=split)
            torch.cuda.synchronize()
            err = (out.double().cpu() - ref).abs().max().item()
            assert err <= 2e-5 * ref.abs().max().item() + 1e-4, (dtype, M, split, used, err)
        F = 64
        wg, wu = bf16_randn((F, K), g, 0.05, dt=TD[dtype]), bf16_randn((F, K), g, 0.05, dt=TD[dtype])
        act = torch.nn.functional.silu(x.double() @ wg.double().T) * (x.double() @ wu.double().T)
        wp2 = fg.fg_pack_weight(CODES[dtype], wg.cuda(), wu.cuda())
        out, _ = fg.fg_gemm(CODES[dtype], x.cuda(), wp2, 2 * F, epilogue=1)
        torch.cuda.synchronize()
        err = (out.double().cpu() - act).abs()
        assert (err <= 2 ** -8 * act.abs() + 1e-3).all(), (dtype, M, err.max().item())


@pytest.mark.parametrize("M,F,K", [(8, 704, 256), (33, 1024, 128), (200, 18944, 3584), (300, 2048, 512), (1000, 1024, 256)])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_gemm_16bit_swiglu_epilogue(fg, M, F, K, dtype):
    print(f"swiglu gemm {dtype} M={M} F={F} K={K}", flush=True)
    g = torch.Generator().manual_seed(M + F)
    dt = TD[dtype]
    x, wg, wu = bf16_randn((M, K), g, dt=dt), bf16_randn((F, K), g, 0.05, dt=dt), bf16_randn((F, K), g, 0.05, dt=dt)
    gate, up = x.double() @ wg.double().T, x.double() @ wu.double().T
    ref = torch.nn.functional.silu(gate) * up
    wp = fg.fg_pack_weight(CODES[dtype], wg.cuda(), wu.cuda())
    out, _ = fg.fg_gemm(CODES[dtype], x.cuda(), wp, 2 * F, epilogue=1)
    torch.cuda.synchronize()
    err = (out.double().cpu() - ref).abs()
    assert (err <= 2 ** -8 * ref.abs() + 1e-3).all(), err.max().item()


@pytest.mark.parametrize("variant", [3, 4, 5, 7, 8, 9, 10, 11, 12, 13, 14])
@pytest.mark.parametrize("chunks", [1, 2, 3, 4, 5, 6, 7, 13, 27])
def test_gemm_16bit_pipelined_block_heights_and_residual_epilogue(fg, variant, chunks):
    """The pipelined kernel with 256-, 128- and 160-row blocks of 256 columns (3, 4, 5), of 192 columns (9, 7, 8), 128-row blocks
    of 128 columns (10) 192-row blocks of 256 / 192 columns (11, 12) and 224-row blocks (13, 14), where the waves without columns only stage X, forced through fg_gemm's variant: partial-sum slabs with and without a k split,
    SwiGLU, and (256-column blocks) the residual epilogue (out += x . W^T in place), on ragged row blocks and a ragged
    last column band; the chunk counts run through every tail length of the main loop and of the staging wave's."""
    print(f"pipelined variant {variant} chunks={chunks}", flush=True)
    K = 64 * chunks
    g = torch.Generator().manual_seed(17 * variant + chunks)
    for dtype, M, N in (("bf16", 300, 288), ("fp16", 129, 544), ("bf16", 1100, 256), ("fp16", 640, 96)):
        code, dt = CODES[dtype], TD[dtype]
        x, w = bf16_randn((M, K), g, dt=dt), bf16_randn((N, K), g, 0.05, dt=dt)
        ref = x.double() @ w.double().T
        wp = fg.fg_pack_weight(code, w.cuda())
        for split in (1, 2):
            out, used = gemm_sum(fg, code, x.cuda(), wp, N, split_k=split, variant=variant)
            torch.cuda.synchronize()
            err = (out.double().cpu() - ref).abs().max().item()
            assert err <= 2e-5 * ref.abs().max().item() + 1e-4, (dtype, M, N, split, used, err)
        h0 = torch.randn((M, N), generator=g, dtype=torch.float32)
        h = h0.clone().cuda()
        if variant >= 7:   # these block shapes have the partial-sum and SwiGLU epilogues only
            with pytest.raises(fg.FgError):
                fg.fg_gemm(code, x.cuda(), wp, N, epilogue=3, variant=variant, out=h)
        else:
            fg.fg_gemm(code, x.cuda(), wp, N, epilogue=3, variant=variant, out=h)
            torch.cuda.synchronize()
            err = (h.double().cpu() - (h0.double() + ref)).abs().max().item()
            assert err <= 2e-5 * ref.abs().max().item() + 1e-4, (dtype, M, N, "residual", err)
        F = 64 if N % 64 else N // 2
        wg, wu = bf16_randn((F, K), g, 0.05, dt=dt), bf16_randn((F, K), g, 0.05, dt=dt)
        act = torch.nn.functional.silu(x.double() @ wg.double().T) * (x.double() @ wu.double().T)
        wp2 = fg.fg_pack_weight(code, wg.cuda(), wu.cuda())
        out, _ = fg.fg_gemm(code, x.cuda(), wp2, 2 * F, epilogue=1, variant=variant)
        torch.cuda.synchronize()
        err = (out.double().cpu() - act).abs()
        assert (err <= 2 ** -8 * act.abs() + 1e-3).all(), (dtype, M, err.max().item())


def test_gemm_residual_epilogue_is_the_library_choice_for_many_rows(fg):
    """At 1024 rows and more the O / down projections add into the residual stream in their own epilogue."""
    M, N, K = 1024, 512, 320
    g = torch.Generator().manual_seed(5)
    x, w = bf16_randn((M, K), g), bf16_randn((N, K), g, 0.05)
    wp = fg.fg_pack_weight(fg.FG_BF16, w.cuda())
    h0 = torch.randn((M, N), generator=g, dtype=torch.float32)
    h = h0.clone().cuda()
    fg.fg_gemm(fg.FG_BF16, x.cuda(), wp, N, epilogue=3, out=h)
    torch.cuda.synchronize()
    ref = h0.double() + x.double() @ w.double().T
    assert (h.double().cpu() - ref).abs().max().item() <= 1e-4 + 2e-5 * ref.abs().max().item()
    assert fg.fg_gemm_kernel_name(M, N, K, 3) == "gemm_mfma_big_kernel"
    with pytest.raises(fg.FgError):
        fg.fg_gemm(fg.FG_BF16, x.cuda(), wp, N, epilogue=3, variant=2, out=h)


def test_gemm_f32(fg):
    g = torch.Generator().manual_seed(1)
    x, w = torch.randn((37, 704), generator=g), torch.randn((1024, 704), generator=g) * 0.05
    wp = fg.fg_pack_weight(fg.FG_F32, w.cuda())
    out, _ = gemm_sum(fg, fg.FG_F32, x.cuda(), wp, 1024)
    torch.cuda.synchronize()
    ref = x.double() @ w.double().T
    assert (out.double().cpu() - ref).abs().max().item() < 1e-4


def test_gemm_rejects_unsupported_shapes(fg):
    x = torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((64, 100), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fg.FgError):
        fg.fg_pack_weight(fg.FG_BF16, w)
    with pytest.raises(fg.FgError):
        fg.fg_gemm(fg.FG_BF16, x, w, 64)


def ref_attention(q, k, v, L, parent, n_prev, Hq, Hkv, hd):
    """q [N_new, Hq, hd], k / v [L + n_tot, Hkv, hd] of one sequence, fp64 torch; explicit boolean mask."""
    n_tot = parent.shape[0]
    N_new = n_tot - n_prev
    mask = torch.zeros((N_new, L + n_tot), dtype=torch.bool)
    mask[:, :L] = True
    for j in range(N_new):
        u = n_prev + j
        while u >= 0:
            mask[j, L + u] = True
            u = int(parent[u])
    kk = k.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    vv = v.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    o = torch.nn.functional.scaled_dot_product_attention(q.permute(1, 0, 2), kk, vv, attn_mask=mask[None])
    return o.permute(1, 0, 2)


@pytest.mark.parametrize("dtype,Hq,Hkv,hd,B,N,n_prev,lens", [
    ("fp32", 4, 4, 64, 3, 5, 0, (0, 7, 40)),
    ("bf16", 12, 2, 128, 4, 6, 0, (512, 100, 17, 31)),
    ("bf16", 28, 4, 128, 5, 24, 0, (256, 1000, 33, 2048, 15)),
    ("bf16", 28, 4, 128, 3, 8, 0, (1024, 4096, 1500)),
    ("fp16", 28, 4, 128, 3, 8, 0, (1024, 4096, 1500)),
    ("fp16", 28, 4, 128, 4, 24, 0, (640, 33, 2048, 15)),
    ("fp16", 12, 2, 128, 3, 6, 2, (512, 100, 17)),
    ("bf16", 8, 4, 64, 3, 5, 0, (70, 300, 5)),
    ("bf16", 28, 4, 128, 3, 32, 0, (300, 3072, 16)),
    ("bf16", 28, 4, 128, 2, 4, 8, (77, 640)),
    ("bf16", 28, 4, 128, 9, 1, 0, (1, 16, 17, 255, 256, 257, 1023, 2000, 0)),
    ("bf16", 28, 4, 128, 2, 64, 0, (128, 50)),
    # batches large enough for the four-tiles-per-wave plan (1024 (sequence, kv head, wave) triples): one wave and three
    ("fp16", 28, 4, 128, 256, 8, 0, (40, 17, 64, 100) * 64),
    ("bf16", 28, 4, 128, 96, 24, 0, (20, 50, 33) * 32),
])
def test_tree_attention(fg, dtype, Hq, Hkv, hd, B, N, n_prev, lens):
    from synth import gen
    print(f"attention {dtype} Hq={Hq} Hkv={Hkv} hd={hd} B={B} N={N} n_prev={n_prev} lens={lens}", flush=True)
    cfg = dict(n_layers=2, n_kv_heads=Hkv, head_dim=hd, dtype=dtype)
    n_tot = n_prev + N
    rng = np.random.default_rng(N + B)
    table, n_pages = gen.make_page_table(np.array(lens), n_tot, 16, seed=3, spare_pages=2)
    kv = fg.KVCache(cfg, table, n_pages)
    td = TD[dtype]
    g = torch.Generator().manual_seed(5)
    parent = np.stack([np.array([-1] + [int(rng.integers(-1, i)) for i in range(1, n_tot)], dtype=np.int32) for _ in range(B)])
    ks, vs = [], []
    for b in range(B):
        k = torch.randn((2, lens[b] + n_tot, Hkv, hd), generator=g).to(torch.bfloat16 if td != torch.float32 else td).to(td)
        v = torch.randn((2, lens[b] + n_tot, Hkv, hd), generator=g).to(torch.bfloat16 if td != torch.float32 else td).to(td)
        kv.write_prefix(b, k.cuda(), v.cuda())
        ks.append(k); vs.append(v)
    kv.seq_len.copy_(torch.tensor(lens, dtype=torch.int32))
    q = (torch.randn((B * N, Hq * hd), generator=g) * 1.5).to(td)
    layer = 1
    out = fg.fg_attention(kv, layer, np.arange(B, dtype=np.int32), parent, B, N, Hq, q.cuda(), n_prev=n_prev)
    torch.cuda.synchronize()
    out = out.double().cpu().view(B, N, Hq, hd)
    for b in range(B):
        ref = ref_attention(q.double().view(B, N, Hq, hd)[b], ks[b][layer].double(), vs[b][layer].double(), lens[b],
                            parent[b], n_prev, Hq, Hkv, hd)
        err = (out[b] - ref).abs().max().item()
        tol = {"fp32": 1e-5, "bf16": 2.5e-2, "fp16": 4e-3}[dtype]
        assert err < tol, (b, err)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("M,V,K", [(129, 16384, 4), (300, 16480, 1), (1030, 16640, 8), (520, 33024, 2), (70, 33024, 3)])
def test_lm_head_with_the_selection_in_its_epilogue(fg, dtype, M, V, K):
    """fg_lm_head_topk (per-block top-K / log-sum-exp partials in the GEMM epilogue + merge, no [M, V] tensor) against the
    two-kernel path on the same accumulators (fg_gemm slabs, then the oracle's definition of top-K / log-softmax on
    them): token ids bit-exact, including exact ties between duplicated vocabulary rows (the lower id must win, within a
    block and across blocks) and a vocabulary that ends inside a 256-token block; log-probabilities to fp32 rounding."""
    from oracle.oracle import Oracle
    print(f"lm head top-k {dtype} M={M} V={V} K={K}", flush=True)
    code, dt, d = CODES[dtype], TD[dtype], 192
    g = torch.Generator().manual_seed(M + V + K)
    x, w = bf16_randn((M, d), g, dt=dt), bf16_randn((V, d), g, 0.3, dt=dt)
    # duplicated rows: exact ties inside one block, across blocks, and at the very end of the vocabulary
    w[7] = w[3]; w[300] = w[3]; w[V - 1] = w[V - 200]; w[9000] = w[8999]; w[9001] = w[8999]
    # a dominant direction so that the duplicated rows are among the winners of some rows
    x[::3] = (w[3].float() * 4).to(dt); x[1::3] = (w[V - 200].float() * 4).to(dt); x[2::7] = (w[8999].float() * 4).to(dt)
    wp = fg.fg_pack_weight(code, w.cuda())
    tok, logp = fg.fg_lm_head_topk(code, x.cuda(), wp, V, K)
    slabs, used = fg.fg_gemm(code, x.cuda(), wp, V, epilogue=0, split_k=1)
    torch.cuda.synchronize()
    assert used == 1
    logits = slabs[0].cpu().numpy()
    o_tok, o_logp = Oracle("f32").topk_logp(logits, K)
    assert np.array_equal(tok.cpu().numpy(), o_tok)
    # log p = logit - logsumexp: both near the largest logit (tens, with the planted direction), each good to a few ulp
    assert np.abs(logp.cpu().numpy() - o_logp).max() <= 1e-5 + 1e-6 * float(np.abs(logits).max())
    # the ties were really there: some row has the duplicated tokens next to each other in rank order
    if K >= 2:
        assert any({3, 7} <= set(r) or {V - 200, V - 1} <= set(r) or {8999, 9000} <= set(r) for r in o_tok.tolist())
    # the library's own one-pass kernel on the same logits agrees too
    t2, l2 = fg.fg_topk_logp(slabs[0], K)
    assert torch.equal(t2, tok)


@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (5, 64, 192), (8, 3584, 3584), (13, 96, 640), (16, 3584, 18944), (9, 160, 384), (8, 37888, 3584),
                                   (15, 16384 + 32, 256)])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_decode_gemm_partial_sums_and_swiglu(fg, M, N, K, dtype):
    """The decode-shape kernel (at most 16 rows, forced through fg_gemm's variant 6) against a double-precision product
    of the same operands: partial-sum slabs with the library's k split, none, and one that leaves empty splits; SwiGLU
    (ragged band groups included); bitwise repeatable."""
    print(f"decode gemm {dtype} M={M} N={N} K={K}", flush=True)
    code, dt = CODES[dtype], TD[dtype]
    g = torch.Generator().manual_seed(M * 11 + N + K)
    x, w = bf16_randn((M, K), g, dt=dt), bf16_randn((N, K), g, 0.05, dt=dt)
    ref = x.double() @ w.double().T
    scale = ref.abs().max().item()
    wp = fg.fg_pack_weight(code, w.cuda())
    for split in (0, 1, 3, 16):
        out, used = gemm_sum(fg, code, x.cuda(), wp, N, split_k=split, variant=6)
        torch.cuda.synchronize()
        assert (out.double().cpu() - ref).abs().max().item() <= 2e-5 * scale + 1e-4, (split, used)
    a, _ = gemm_sum(fg, code, x.cuda(), wp, N, variant=6)
    b, _ = gemm_sum(fg, code, x.cuda(), wp, N, variant=6)
    assert torch.equal(a, b)
    if N % 64 == 0:
        F = N // 2
        wg, wu = w[:F], w[F:]
        wp2 = fg.fg_pack_weight(code, wg.cuda(), wu.cuda())
        refs = torch.nn.functional.silu(x.double() @ wg.double().T) * (x.double() @ wu.double().T)
        act, _ = fg.fg_gemm(code, x.cuda(), wp2, N, epilogue=1, variant=6)
        torch.cuda.synchronize()
        err = (act.double().cpu() - refs).abs()
        assert (err <= 2 ** -8 * refs.abs() + 1e-3).all(), err.max().item()


def test_decode_gemm_rejects_shapes_it_does_not_take(fg):
    x = torch.zeros((17, 128), dtype=torch.bfloat16, device="cuda")
    w = fg.fg_pack_weight(1, torch.zeros((32, 128), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(fg.FgError):
        fg.fg_gemm(1, x, w, 32, variant=6)                       # 17 rows
    h = torch.zeros((8, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(fg.FgError):
        fg.fg_gemm(1, x[:8], w, 32, epilogue=3, out=h, variant=6)  # no residual epilogue


def test_ceiling_probes_run_and_reject_bad_shapes(fg):
    """The measurement probes of bench.py --ceilings (no part of the method): every read pattern, the copy and the MFMA loop
    launch on small buffers, the copy copies, and shapes a pattern cannot take are errors, not launches."""
    src = torch.randint(0, 255, (8 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    sink = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    for mode in range(7):
        fg.fg_probe_read(src, mode, 64, sink)
    fg.fg_probe_copy(src, dst, 64)
    fg.fg_probe_mfma(fg.FG_BF16, 4, True, 8, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(fg.FgError):
        fg.fg_probe_read(src[:4096], 6, 64, sink)      # 64 slices of 32 loads per lane do not fit 4 KiB
    with pytest.raises(fg.FgError):
        fg.fg_probe_read(src[:3 << 20], 3, 64, sink)    # the L2-resident pattern wants a power-of-two size
    with pytest.raises(fg.FgError):
        fg.fg_probe_read(src, 7, 64, sink)
