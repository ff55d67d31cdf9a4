"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Tolerances: fp32 mode 1e-4 relative (rel-L2 per tensor), bf16 mode 2e-2 relative on
gradients and loss; kernel-level cases are tighter where the arithmetic allows."""
import json
import math
import os

import numpy as np
import pytest
import torch

import l2l_synth as S
import paper_2002_05645_amd as P
from paper_2002_05645_amd import binding as B
from paper_2002_05645_amd.trainer import L2LTrainer, pack, unpack
from oracle import l2l_oracle as O
from gpu_util import to_dev, to_host, rounded, pinned

pytestmark = pytest.mark.gpu

# fp16 carries 11 significand bits against bf16's 8: its bar is 8x tighter
TOL = {"fp32": 1e-4, "bf16": 2e-2, "fp16": 2.5e-3}
DT = {"fp32": P.L2L_F32, "bf16": P.L2L_BF16, "fp16": P.L2L_FP16}
OUT16 = {"fp32": 2e-6, "bf16": 3e-3, "fp16": 4e-4}      # one rounding of a 16-bit (or no rounding of an fp32) output
# Largest single error over a tensor, in units of the tensor's largest entry (oracle's max_rel).  fp32: a handful of
# fp32 roundings of sums of a few thousand terms.  16-bit modes: activations and activation gradients pass through a
# dozen roundings to the format inside a layer (unit roundoff 2^-8 = 3.9e-3 for bf16, 2^-11 = 4.9e-4 for fp16) and the
# single worst of up to 10^7 entries sits several standard deviations out.  Measured worst cases over this file:
# fp32 1.7e-6, bf16 1.6e-2 (the BERT-Base step through 12 layers), fp16 1.6e-3; the bounds leave a factor of 2.5 or more.
MAXTOL = {"fp32": 2e-5, "bf16": 4e-2, "fp16": 5e-3}
ULP = {"bf16": 2.0 ** -7, "fp16": 2.0 ** -10}           # spacing of the format relative to the value, at most: half of it per rounding


@pytest.fixture(scope="module")
def ctx():
    cfg = P.make_config(64, 2, 128, 16, 2, 2, "bf16", 1e-5, 0)
    c = P.Context(cfg)
    yield c
    c.close()


# ------------------------------------------------------------------------------------- GEMM kernel
def _gemm_case(ctx, dtype, impl, a_kc, b_kc, M, N, K, bias=False, resid=False, gelu=False, accumulate=False,
               out_f32=False, alpha=1.0, seed=0, pad=3):
    rng = np.random.default_rng(seed)
    A = rng.normal(size=(M, K)).astype(np.float32)
    Bm = rng.normal(size=(K, N)).astype(np.float32)
    lda = ((K if a_kc else M) + 7) // 8 * 8 + 8
    ldb = ((K if b_kc else N) + 7) // 8 * 8 + 8
    ldc = N + pad   # pad 3: rows not 16-byte aligned (element-wise epilogue); pad 8: the vector epilogue
    Ah = np.zeros((M, lda) if a_kc else (K, lda), np.float32)
    Bh = np.zeros((N, ldb) if b_kc else (K, ldb), np.float32)
    if a_kc:
        Ah[:, :K] = A
    else:
        Ah[:, :M] = A.T
    if b_kc:
        Bh[:, :K] = Bm.T
    else:
        Bh[:, :N] = Bm
    f32out = out_f32 or dtype == "fp32"
    C0 = rng.normal(size=(M, ldc)).astype(np.float32)
    Cd = torch.from_numpy(C0).cuda() if f32out else to_dev(C0, dtype)
    C0v = to_host(Cd)
    bias_h = rng.normal(size=N).astype(np.float32) if bias else None
    res_h = rng.normal(size=(M, ldc)).astype(np.float32) if resid else None
    Ad, Bd = to_dev(Ah, dtype), to_dev(Bh, dtype)
    bd = to_dev(bias_h, dtype) if bias else None
    rd = to_dev(res_h, dtype) if resid else None
    ctx.op_gemm(DT[dtype], f32out, a_kc, b_kc, M, N, K, Ad, lda, Bd, ldb, Cd, ldc, alpha, bd, rd, gelu, accumulate,
                impl)
    torch.cuda.synchronize()
    ref = alpha * (rounded(A, dtype) @ rounded(Bm, dtype))
    if bias:
        ref = ref + rounded(bias_h, dtype)
    if gelu:
        ref = O.gelu(ref)
    if resid:
        ref = ref + rounded(res_h, dtype)[:, :N]
    if accumulate:
        ref = ref + C0v[:, :N]
    got = to_host(Cd)
    assert np.array_equal(got[:, N:], C0v[:, N:]), "wrote outside the N columns"
    return O.rel_l2(got[:, :N], ref)


@pytest.mark.parametrize("a_kc,b_kc", [(1, 0), (1, 1), (0, 0), (0, 1)])
@pytest.mark.parametrize("dtype,impl", [("fp32", 1), ("bf16", 1), ("bf16", 2), ("fp16", 1), ("fp16", 2)])
def test_gemm_layouts_ragged(ctx, dtype, impl, a_kc, b_kc):
    for (M, N, K) in [(200, 136, 96), (128, 128, 32), (1, 8, 8), (300, 72, 264), (130, 258, 40)]:
        err = _gemm_case(ctx, dtype, impl, a_kc, b_kc, M, N, K, out_f32=True, seed=M + N)
        assert err < 2e-6, (M, N, K, err)
        err = _gemm_case(ctx, dtype, impl, a_kc, b_kc, M, N, K, bias=True, resid=True, seed=M)
        assert err < OUT16[dtype], (M, N, K, err)


@pytest.mark.parametrize("dtype,impl", [("fp32", 1), ("bf16", 1), ("bf16", 2), ("fp16", 1), ("fp16", 2)])
def test_gemm_epilogues(ctx, dtype, impl):
    lim = OUT16[dtype]
    assert _gemm_case(ctx, dtype, impl, 1, 0, 256, 192, 128, bias=True, gelu=True, alpha=0.1) < lim
    assert _gemm_case(ctx, dtype, impl, 0, 0, 192, 256, 520, accumulate=True, out_f32=True) < 2e-6
    assert _gemm_case(ctx, dtype, impl, 1, 1, 264, 136, 64, alpha=0.125, out_f32=True) < 2e-6
    # ragged K (not a multiple of 8) on the strided-K layout
    assert _gemm_case(ctx, dtype, impl, 0, 0, 136, 72, 613, accumulate=True, out_f32=True) < 2e-6


def test_gemm_large_tile_sweep(ctx):
    # several tiles in every direction plus tails, MFMA kernel
    assert _gemm_case(ctx, "bf16", 2, 1, 0, 1000, 520, 264, bias=True, out_f32=True) < 2e-6
    assert _gemm_case(ctx, "bf16", 2, 1, 1, 520, 1000, 136, out_f32=True) < 2e-6
    assert _gemm_case(ctx, "bf16", 2, 0, 0, 520, 392, 1000, out_f32=True) < 2e-6
    assert _gemm_case(ctx, "fp16", 2, 1, 1, 520, 1000, 136, bias=True) < OUT16["fp16"]
    assert _gemm_case(ctx, "fp16", 2, 0, 0, 520, 392, 1000, out_f32=True) < 2e-6


@pytest.mark.parametrize("variant", range(9))
def test_gemm_every_tile_variant(ctx, variant):
    # each compiled tile shape of the MFMA kernel, forced: ragged edges, all three layouts, both output types
    impl = 100 + variant
    assert _gemm_case(ctx, "bf16", impl, 1, 0, 600, 520, 264, bias=True, out_f32=True) < 2e-6
    assert _gemm_case(ctx, "bf16", impl, 1, 1, 520, 776, 136, bias=True, resid=True, alpha=0.5, pad=8) < OUT16["bf16"]
    assert _gemm_case(ctx, "bf16", impl, 0, 0, 520, 392, 1000, accumulate=True, out_f32=True, pad=8) < 2e-6
    assert _gemm_case(ctx, "fp16", impl, 1, 0, 264, 520, 200, bias=True, gelu=True, pad=8) < OUT16["fp16"]
    with pytest.raises(P.L2LError):
        x = torch.zeros(64, 64, device="cuda", dtype=torch.bfloat16)
        ctx.op_gemm(P.L2L_BF16, False, 1, 0, 64, 64, 64, x, 64, x, 64, x, 64, impl=100 + 9)   # one past the last variant


@pytest.mark.parametrize("workspace_mb", [0, 64])
def test_gemm_split_k_through_workspace_and_with_atomics(monkeypatch, workspace_mb):
    # an accumulating fp32 GEMM with few tiles and a long K is split over K; the splits either store partial tiles in a
    # workspace that one kernel adds up (contexts size it from their layer shapes; forced here), or add with atomics
    if workspace_mb:
        monkeypatch.setenv("L2L_SPLIT_WS_MB", str(workspace_mb))
    else:
        monkeypatch.setenv("L2L_SPLIT_ATOMICS", "1")
    c = P.Context(P.make_config(64, 2, 128, 16, 2, 2, "bf16", 1e-5, 0))
    try:
        for dtype in ("bf16", "fp16"):
            assert _gemm_case(c, dtype, 0, 0, 0, 256, 512, 4096, accumulate=True, out_f32=True, pad=8) < 2e-6    # 2 tiles, 8 splits
            assert _gemm_case(c, dtype, 0, 0, 0, 264, 520, 4200, accumulate=True, out_f32=True, pad=8) < 2e-6    # ragged everywhere
            assert _gemm_case(c, dtype, 0, 1, 1, 256, 256, 4096 + 64, accumulate=True, out_f32=True, pad=8) < 2e-6    # K-contiguous operands
            assert _gemm_case(c, dtype, 0, 0, 0, 200, 136, 8192, accumulate=True, out_f32=True, pad=3) < 2e-6    # rows not 16-byte aligned
    finally:
        c.close()


# every epilogue the 256 x 256 direct-to-LDS kernel has a compiled-in instantiation for (flags as the library numbers
# them: bias 1, GELU 2, GELU' 4, residual 8, column sums 32, keep gelu' 64, times aux 128), by the l2l_op_gemm_ex
# arguments that select it; 4, 36 and 32 go to the instantiation that reads its flags at run time
EPILOGUES = {0: dict(), 1: dict(bias=True), 9: dict(bias=True, resid=True), 3: dict(bias=True, gelu=True),
             67: dict(bias=True, gelu=True, keepgrad=True), 128: dict(mulaux=True), 160: dict(mulaux=True, colsum=True), 8: dict(resid=True),
             4: dict(gelugrad=True), 36: dict(gelugrad=True, colsum=True), 32: dict(colsum=True)}


def _gemm_ex_case(ctx, dtype, M, N, K, bias=False, resid=False, gelu=False, gelugrad=False, colsum=False, a_kc=1, b_kc=1,
                  out_f32=False, accumulate=False, seed=0, keepgrad=False, mulaux=False):
    """One l2l_op_gemm_ex launch (library's choice of kernel) checked ELEMENT BY ELEMENT against
    epilogue(rounded(A) @ rounded(B)) in fp64.  Bounds per element: an fp32 output may differ by the fp32
    accumulation error (2e-6 of the row-times-column magnitude); a 16-bit output additionally by one rounding to the
    format (half a unit in the last place, ULP / 2 relative).  The 16-bit epilogues evaluate Phi(u) and gelu'(u) by
    polynomials with absolute errors below 4e-5 and 2e-4 (pinned on the CPU), which enter as 5e-5 |u| and 2.5e-4 |acc|."""
    rng = np.random.default_rng(seed)
    A = rng.normal(size=(M, K)).astype(np.float32)
    Bm = (rng.normal(size=(K, N)) / math.sqrt(K)).astype(np.float32)
    ldr, ldaux, ldc = N + 8, N + 16, N + 24
    Ad = to_dev(A if a_kc else np.ascontiguousarray(A.T), dtype)
    Bd = to_dev(np.ascontiguousarray(Bm.T) if b_kc else Bm, dtype)
    lda, ldb = (K if a_kc else M), (K if b_kc else N)
    Ar, Br = rounded(A, dtype), rounded(Bm, dtype)
    acc = Ar @ Br
    scale = np.abs(Ar) @ np.abs(Br)                         # magnitude of the sum of products, per output
    tol = 2e-6 * scale
    ref = acc.copy()
    kw = dict(epi=0)
    if bias:
        bh = rng.normal(size=N).astype(np.float32)
        kw["bias"] = to_dev(bh, dtype)
        ref = ref + rounded(bh, dtype)
    if gelu:
        u = ref.copy()
        ref = O.gelu(u)
        tol = tol + 5e-5 * np.abs(u)
        aux_out = to_dev(np.full((M, ldaux), 7.0, np.float32), dtype)
        kw.update(epi=kw["epi"] | B.EPI_GELU | (B.EPI_KEEPGRAD if keepgrad else 0), aux_out=aux_out, ldaux=ldaux)
    if gelugrad:
        auxh = (rng.normal(size=(M, ldaux)) * 1.5).astype(np.float32)
        kw.update(epi=kw["epi"] | B.EPI_GELUGRAD, aux=to_dev(auxh, dtype), ldaux=ldaux)
        ref = ref * O.gelu_grad(rounded(auxh, dtype)[:, :N])
        tol = tol + 2.5e-4 * np.abs(acc)
    if mulaux:
        auxh = rng.normal(size=(M, ldaux)).astype(np.float32)
        kw.update(epi=kw["epi"] | B.EPI_MULAUX, aux=to_dev(auxh, dtype), ldaux=ldaux)
        fac = rounded(auxh, dtype)[:, :N]
        ref = ref * fac
        tol = tol * np.abs(fac)
    if resid:
        rh = rng.normal(size=(M, ldr)).astype(np.float32)
        kw.update(resid=to_dev(rh, dtype), ldr=ldr)
        ref = ref + rounded(rh, dtype)[:, :N]
    f32out = out_f32 or dtype == "fp32"
    C0 = rng.normal(size=(M, ldc)).astype(np.float32)
    Cd = torch.from_numpy(C0).cuda() if f32out else to_dev(C0, dtype)
    C0v = to_host(Cd)
    if accumulate:
        kw["epi"] |= B.EPI_ACCUM
        ref = ref + C0v[:, :N]
    cs_rows = (M + 63) // 64
    if colsum:
        csd = torch.full((cs_rows + 1, N), 12345.0, device="cuda")      # one canary row behind what may be written
        kw.update(epi=kw["epi"] | B.EPI_COLSUM, colsum=csd, colsum_rows=cs_rows)
    used = ctx.op_gemm_ex(DT[dtype], f32out, a_kc, b_kc, M, N, K, Ad, lda, Bd, ldb, Cd, ldc, 1.0, impl=0, **kw)
    torch.cuda.synchronize()
    got = to_host(Cd)
    assert np.array_equal(got[:, N:], C0v[:, N:]), "wrote outside the N columns"
    # (fp16 results below 2^-14 are subnormal: their spacing is 2^-24 whatever their size)
    out_tol = tol if f32out else tol + 0.5 * ULP[dtype] * 1.001 * np.abs(ref) + (2.0 ** -25 if dtype == "fp16" else 0.0)
    excess = np.abs(got[:, :N] - ref) - out_tol
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (f"element {worst}: got {got[worst]}, want {ref[worst]} +- {out_tol[worst]}; "
                                f"{int((excess > 0).sum())} of {excess.size} out of bounds")
    if gelu:       # what was kept: one rounding of the pre-activation u, or of gelu'(u) (Phi's polynomial: 4e-5)
        au = to_host(aux_out)
        assert np.all(au[:, N:] == 7.0)
        kept = O.gelu_grad(u) if keepgrad else u
        slack = 2e-6 * scale * (1.2 if keepgrad else 1.0) + (5e-5 if keepgrad else 0.0)      # (|gelu''| <= 1.13)
        assert np.all(np.abs(au[:, :N] - kept) <= slack + 0.5 * ULP[dtype] * 1.001 * np.abs(kept))
    if colsum:     # partial sums of the values before their rounding to the output format; rows beyond `used` untouched
        assert 0 < used <= cs_rows
        cs = to_host(csd)
        assert np.all(cs[used:] == 12345.0), "column-sum rows beyond the reported count were written"
        col_tol = tol.sum(axis=0) + 1e-6 * np.abs(ref).sum(axis=0)
        assert np.all(np.abs(cs[:used].sum(axis=0) - ref.sum(axis=0)) <= col_tol)
    return O.rel_l2(got[:, :N], ref), O.max_rel(got[:, :N], ref)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("epi", sorted(EPILOGUES))
def test_gemm_every_compiled_epilogue_elementwise(ctx, dtype, epi):
    # 256 x 256 tiles with 16-bit output and both operands K-contiguous: the instantiations with the epilogue flags
    # compiled in (flag sets 0, 1, 9, 3, 67, 128, 160, 8) and, for 4, 36 and 32, the one that reads them at run time; two
    # tile rows and columns with ragged edges, K with a tail
    errs = _gemm_ex_case(ctx, dtype, 392, 520, 264, seed=epi, **EPILOGUES[epi])
    _report(f"gemm_ex[{dtype}-epi{epi}]", {"C": errs[0], "max:C": errs[1]})


@pytest.mark.parametrize("K", [136, 1032])
@pytest.mark.parametrize("epi", [9, 67, 160])
def test_gemm_resident_tile_walk_elementwise(ctx, K, epi):
    # 19 x 18 = 342 tiles of 256 x 256, more than the chip has compute units: workgroups stay resident and walk the tile
    # order, fetching the next tile's first k-tile under the epilogue of the current one; ragged M, N and K.  K = 136
    # leaves that prefetch as most of a tile's loads, K = 1032 is the layer's depth plus a tail
    errs = _gemm_ex_case(ctx, "bf16", 4616, 4360, K, seed=K + epi, **EPILOGUES[epi])
    _report(f"gemm_resident[K{K}-epi{epi}]", {"C": errs[0], "max:C": errs[1]})


def test_gemm_resident_tile_walk_other_layouts_elementwise(ctx):
    # the same walk for the dW layout (both operands K-strided, fp32 accumulate into C: 342 tiles, no K split) and for
    # fp16 operands
    _gemm_ex_case(ctx, "bf16", 4616, 4360, 520, a_kc=0, b_kc=0, out_f32=True, accumulate=True, seed=5)
    _gemm_ex_case(ctx, "fp16", 4616, 4360, 264, seed=6, **EPILOGUES[9])
    _gemm_ex_case(ctx, "bf16", 4616, 4360, 264, a_kc=1, b_kc=0, out_f32=True, seed=7)


def test_gemm_column_sums_row_count_at_wave_tile_edges(ctx):
    # M = 64 and M = 320 leave wave tiles of the 128- and 256-row block tiles entirely past M: they must not write a
    # row of partial sums (the buffer has ceil(M / 64) rows and a canary row behind them)
    for M, N in [(64, 264), (320, 136), (448, 520), (72, 128)]:
        _gemm_ex_case(ctx, "bf16", M, N, 264, mulaux=True, colsum=True, seed=M)
        _gemm_ex_case(ctx, "bf16", M, N, 264, colsum=True, seed=M + 1)


def test_gemm_ex_rejects_bad_arguments(ctx):
    x = torch.zeros(256, 256, device="cuda", dtype=torch.bfloat16)
    f = torch.zeros(256, 256, device="cuda")
    kw = dict(in_dtype=P.L2L_BF16, out_f32=False, a_kc=1, b_kc=1, M=256, N=256, K=256, A=x, lda=256, B=x, ldb=256, Cm=x, ldc=256)
    for bad in (dict(epi=B.EPI_GELUGRAD),                                  # no pre-activation
                dict(epi=B.EPI_GELU | B.EPI_GELUGRAD, aux=x, ldaux=256),   # both at once
                dict(epi=64),                                              # unknown flag
                dict(epi=B.EPI_ACCUM),                                     # accumulate into a 16-bit output
                dict(resid=x, ldr=8),                                      # residual stride below N
                dict(epi=B.EPI_COLSUM),                                    # no buffer
                dict(epi=B.EPI_COLSUM, colsum=f, colsum_rows=1),           # too few rows
                dict(epi=B.EPI_COLSUM, colsum=f, colsum_rows=8, impl=1)):  # the plain kernel has no column sums
        with pytest.raises(P.L2LError) as e:
            ctx.op_gemm_ex(**{**kw, **bad})
        assert e.value.code == P.L2L_E_ARG, bad


def test_gemm_rejects_bad_arguments(ctx):
    x = torch.zeros(64, 64, device="cuda")
    with pytest.raises(P.L2LError) as e:
        ctx.op_gemm(P.L2L_BF16, False, 1, 0, 8, 8, 8, x, 8, x, 8, x, 8, accumulate=True)
    assert e.value.code == P.L2L_E_ARG
    with pytest.raises(P.L2LError):
        ctx.op_gemm(P.L2L_F32, True, 1, 0, 8, 8, 8, None, 8, x, 8, x, 8)
    with pytest.raises(P.L2LError):
        ctx.op_gemm(P.L2L_BF16, True, 1, 0, 8, 8, 8, x, 7, x, 8, x, 8, impl=2)     # lda not a multiple of 8


# ------------------------------------------------------------------------------------- LayerNorm kernel
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("rows,n", [(1, 8), (37, 1024), (5, 200), (130, 6144)])
def test_layernorm(ctx, dtype, rows, n):
    rng = np.random.default_rng(rows)
    x = (rng.normal(size=(rows, n)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.normal(size=n)).astype(np.float32)
    b = (0.1 * rng.normal(size=n)).astype(np.float32)
    xd, gd, bd = to_dev(x, dtype), to_dev(g, dtype), to_dev(b, dtype)
    yd = torch.empty_like(xd)
    mean = torch.empty(rows, device="cuda")
    rstd = torch.empty(rows, device="cuda")
    ctx.op_layernorm(DT[dtype], rows, n, xd, gd, bd, 1e-12, yd, mean, rstd)
    torch.cuda.synchronize()
    ref, (xhat, rs) = O.layer_norm_fwd(rounded(x, dtype), rounded(g, dtype), rounded(b, dtype), 1e-12)
    assert O.rel_l2(to_host(yd), ref) < OUT16[dtype]
    assert O.rel_l2(to_host(rstd), rs[:, 0]) < 1e-5
    assert O.rel_l2(to_host(mean), rounded(x, dtype).mean(-1)) < 1e-5


# ------------------------------------------------------------------------------------- one layer, all micro-batches
def _layer_case(w: S.Workload, group=0, x_scale=1.0, check_fwd_only=False, dy_scale=1.0, stats=False):
    """stats: l2l_layer_fwd_stats / l2l_layer_bwd_stats (LayerNorm 2's 1 / sigma kept, FFN2 not recomputed) instead of
    l2l_layer_fwd / l2l_layer_bwd"""
    dtype = w.dtype
    cfg = P.make_config(w.hidden, w.heads, w.ffn, w.seq, w.ubatch, w.num_ubatches, dtype, 1e-12, 0, group)
    c = P.Context(cfg)
    try:
        lay = P.layer_layout(cfg)
        total = P.lib().l2l_layer_packed_elems(cfg)
        p32 = S.layer_params(w, 0)
        _progress("parameters drawn")
        flat = pack(lay, total, p32)
        host = pinned(O.bf16_bits(flat).view(np.int16) if dtype == "bf16" else O.fp16_bits(flat).view(np.int16) if dtype == "fp16" else flat)
        pr = {k: rounded(v, dtype) for k, v in p32.items()}
        X = S.activations(w) * x_scale
        dY = S.output_grads(w) * dy_scale
        Xd, dYd = to_dev(X, dtype), to_dev(dY, dtype)
        Yd = torch.empty_like(Xd)
        c.param_stage(0, host, 0)
        if stats:
            rstd = torch.full((w.num_ubatches * w.ubatch * w.seq,), float("nan"), device="cuda")
            c.layer_fwd_stats(0, 0, Xd, Yd, rstd)
        else:
            c.layer_fwd(0, 0, Xd, Yd)
        c.sync()
        _progress("device forward done")
        Xr, dYr = rounded(X, dtype), rounded(dY, dtype)
        Yref = O.layer_l2l_fwd(Xr, pr, w.heads, 1e-12)
        _progress("oracle forward done")
        errs = {}
        _both(errs, "Y", to_host(Yd), Yref)
        if not check_fwd_only:
            if stats:
                c.layer_bwd_stats(0, 0, Xd, Yd, rstd, dYd)
            else:
                c.layer_bwd(0, 0, Xd, dYd)
            gh = torch.empty(total, dtype=torch.float32).pin_memory()
            c.grad_drain(0, gh)
            c.drain_wait(0)
            c.sync()
            _progress("device backward done")
            dXref, gref = O.layer_l2l_bwd(Xr, dYr, pr, w.heads, 1e-12)
            _progress("oracle backward done")
            _both(errs, "dX", to_host(dYd), dXref)
            got = unpack(lay, S.layer_shapes(w), gh.numpy())
            for k in gref:
                _both(errs, "d" + k, got[k], gref[k])
            # The QKV bias gradient part by part: its K part is zero in exact arithmetic (every row of dS sums to zero;
            # the oracle's is rounding noise, the fused attention path writes zeros) and would drown in the norm of the
            # whole vector; the Q and V parts come from different kernels on that path.
            H = w.hidden
            gq, gk, gv = (got["bqkv"][i * H:(i + 1) * H] for i in range(3))
            rq, rk, rv = (gref["bqkv"][i * H:(i + 1) * H] for i in range(3))
            scale = np.abs(gref["bqkv"]).max()
            assert np.abs(rk).max() <= 1e-9 * scale
            errs["part:dbqkv[Q]"] = O.rel_l2(gq, rq)
            errs["part:dbqkv[V]"] = O.rel_l2(gv, rv)
            errs["max:dbqkv[K]"] = float(np.abs(gk).max() / scale)
            # padding of the gradient block stays zero
            mask = np.ones(total, bool)
            for off, n in lay.values():
                mask[off:off + n] = False
            assert not gh.numpy()[mask].any()
        return errs
    finally:
        c.close()


def _report_dir():
    """where the cases leave their error figures and progress lines: the folder named by L2L_TEST_REPORT_DIR, if any"""
    d = os.environ.get("L2L_TEST_REPORT_DIR", "")
    return d if d and os.path.isdir(d) else None


def _report(case, errs):
    """every parity case leaves its error figures in parity_errors.jsonl of the report folder"""
    d = _report_dir()
    if d:
        with open(os.path.join(d, "parity_errors.jsonl"), "a") as f:
            f.write(json.dumps({"case": case, **{k: float(v) for k, v in errs.items()}}) + "\n")


def _progress(msg):
    """long cases say where they are (a line in progress.log of the report folder), so that a quiet minute is not taken for a hang"""
    d = _report_dir()
    if d:
        with open(os.path.join(d, "progress.log"), "a") as f:
            f.write(f"{os.environ.get('PYTEST_CURRENT_TEST', '?').split(' ')[0]}: {msg}\n")


def _assert_errs(errs, tol, max_tol=None):
    """errs: {tensor: rel-L2} and {"max:" + tensor: max |got - ref| / max |ref|}.  rel-L2 is held to `tol` (the north
    star's bar); the largest single error to `max_tol` (default MAXTOL of the same precision), so that a few wrong
    rows or a dropped tile, which a norm over a large tensor averages away, fail on their own."""
    if max_tol is None:
        max_tol = {v: MAXTOL[k] for k, v in TOL.items()}.get(tol, 4 * tol)
    case = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    _report(case, errs)
    # ("part:" entries: a slice of a tensor on its own, which may be small beside the rest of it and then carries a larger
    # share of the rounding; held to ten times the bar, which a slice computed wrongly still misses by far)
    bad = {k: v for k, v in errs.items() if not (v < (max_tol if k.startswith("max:") else 10 * tol if k.startswith("part:") else tol))}
    assert not bad, f"over tolerance {tol} (max-error {max_tol}): {bad}; all: {errs}"


def _both(errs, name, got, ref):
    errs[name] = O.rel_l2(got, ref)
    errs["max:" + name] = O.max_rel(got, ref)


def test_layer_tiny_fp32():
    w = S.WORKLOADS[0]
    _assert_errs(_layer_case(w), TOL["fp32"])


def test_layer_tiny_fp32_ungrouped_equals_grouped():
    w = S.WORKLOADS[0]
    _assert_errs(_layer_case(w, group=1), TOL["fp32"])
    _assert_errs(_layer_case(w.scaled(num_ubatches=3), group=2), TOL["fp32"])     # ragged last group


def test_layer_ragged_bf16():
    # nothing is a multiple of a tile: H=96 (3 heads of 32), F=200, S=24, ub=3, U=3 in groups of 2
    w = S.Workload("ragged", 1, 96, 3, 200, 24, 50, 3, 3, "bf16", 1.0, 77)
    _assert_errs(_layer_case(w, group=2), TOL["bf16"])
    w32 = w.scaled(dtype="fp32")
    _assert_errs(_layer_case(w32, group=2), TOL["fp32"])


def test_layer_fp16():
    # the paper's device precision (Section 2.3): same kernels on IEEE half; ragged and tile-sized shapes
    w = S.Workload("ragged16", 1, 96, 3, 200, 24, 50, 3, 3, "fp16", 1.0, 177)
    _assert_errs(_layer_case(w, group=2), TOL["fp16"])
    w = S.WORKLOADS[1].scaled(num_ubatches=2, ubatch=4, dtype="fp16")
    _assert_errs(_layer_case(w), TOL["fp16"])


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_layer_with_kept_layernorm_statistics(dtype):
    # l2l_layer_fwd_stats / l2l_layer_bwd_stats: the backward pass takes LayerNorm 2's xhat from the stashed output and
    # the kept 1 / sigma and does not recompute FFN2; same oracle, same bars as the plain pair
    w = S.Workload("ragged-stats", 1, 96, 3, 200, 24, 50, 3, 3, dtype, 1.0, 277)
    _assert_errs(_layer_case(w, group=2, stats=True), TOL[dtype])
    w = S.Workload("fused-stats", 1, 128, 2, 256, 64, 50, 3, 2, dtype, 1.0, 278)
    _assert_errs(_layer_case(w, stats=True), TOL[dtype])
    if dtype != "fp32":
        w = S.Workload("long-stats", 1, 128, 2, 256, 256, 50, 2, 3, dtype, 1.0, 279)      # chunked attention, ragged last group
        _assert_errs(_layer_case(w, group=2, stats=True, **(dict(dy_scale=256.0) if dtype == "fp16" else {})), TOL[dtype])


def test_layer_with_kept_statistics_wide_rows_recomputes_in_full():
    # H = 2304 > 2048: LayerNorm backward has no one-pass form there, l2l_layer_bwd_stats recomputes like l2l_layer_bwd
    w = S.Workload("wide-stats", 1, 2304, 36, 256, 32, 50, 2, 2, "bf16", 1.0, 280)
    _assert_errs(_layer_case(w, stats=True), TOL["bf16"])


@pytest.mark.slow
def test_layer_bert_large_full_shape_bf16_kept_statistics():
    _assert_errs(_layer_case(S.WORKLOADS[2], stats=True), TOL["bf16"])


def test_layer_single_sequence_single_ubatch():
    w = S.Workload("one", 1, 64, 1, 64, 8, 50, 1, 1, "bf16", 1.0, 78)
    _assert_errs(_layer_case(w), TOL["bf16"])


def test_layer_bert_base_shape_bf16():
    w = S.WORKLOADS[1].scaled(num_ubatches=2, ubatch=4)          # real widths, fewer rows: oracle in seconds
    _assert_errs(_layer_case(w), TOL["bf16"])


@pytest.mark.slow
def test_layer_bert_large_full_shape_bf16():
    # the benchmark's launch configuration: U = 8 micro-batches of 32 sequences, S = 128
    w = S.WORKLOADS[2]
    _assert_errs(_layer_case(w), TOL["bf16"])


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("seq", [32, 64, 96, 128])
def test_layer_fused_attention_sequence_lengths(seq, dtype):
    # head width 64 and S a multiple of 32 up to 128: the fused attention kernels (forward and backward)
    w = S.Workload("fused", 1, 128, 2, 256, seq, 50, 3, 2, dtype, 1.0, 79 + seq)
    _assert_errs(_layer_case(w), TOL[dtype])


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("seq", [160, 256, 320, 384, 512])
def test_layer_chunked_attention_long_sequences(seq, dtype):
    # head width 64 and S a multiple of 32 beyond 128: the chunked attention kernels (running softmax statistics in
    # the forward pass; dQ and dK / dV kernels that rebuild P from the stored log-sum-exp in the backward pass);
    # 160 and 320 end in a short chunk of 32 and 64 rows
    w = S.Workload("long", 1, 128, 2, 256, seq, 50, 2, 3, dtype, 1.0, 300 + seq)
    # fp16: with attention weights near 1 / S the score gradients of the synthetic dY fall into fp16's subnormals on
    # any path (the batched-GEMM one included), which is what the loss scale of Section 2.3's FP16 mode is for: the
    # incoming gradient carries a factor 256 here, as it would from a scaled loss
    kw = dict(dy_scale=256.0) if dtype == "fp16" else {}
    _assert_errs(_layer_case(w, **kw), TOL[dtype])
    _assert_errs(_layer_case(w, group=2, **kw), TOL[dtype])     # ragged last group


@pytest.mark.parametrize("seq", [160, 512])
def test_layer_chunked_attention_fp16_unscaled_gradient(seq):
    # The same fp16 cases WITHOUT the factor on dY: upstream gradients of size 1e-3 times attention weights of size
    # 1 / S put the score gradients at 1e-5 .. 1e-6, where half precision keeps 3 to 7 bits (subnormal spacing 6e-8).
    # The forward pass is unaffected and held to the fp16 bar; the gradients are held to 8e-3, about three times
    # that bar (the bf16 bar is 2e-2), which is what is left of them there.  With a loss scale (the mode Section 2.3's
    # FP16 is run in) the case above applies.
    w = S.Workload("long", 1, 128, 2, 256, seq, 50, 2, 3, "fp16", 1.0, 300 + seq)
    errs = _layer_case(w)
    _assert_errs({k: v for k, v in errs.items() if k.endswith("Y")}, TOL["fp16"])
    _assert_errs({k: v for k, v in errs.items() if not k.endswith("Y")}, 8e-3, 8e-3)     # measured: 3.1e-3 at S = 512


def test_layer_rows_below_one_wave_tile_bf16():
    # 64 rows per launch with F >= 3 H: the GELU' GEMM (M = 64: 128 x 128 tiles of 64-row wave tiles) leaves its
    # bias-gradient partial sums in a buffer of ceil(64 / 64) = 1 row; the wave tile past M must not write a second one
    # (it would land in the LayerNorm statistics behind the buffer)
    w = S.Workload("m64", 1, 128, 2, 512, 32, 50, 2, 1, "bf16", 1.0, 641)
    _assert_errs(_layer_case(w), TOL["bf16"])
    w = S.Workload("m320", 1, 128, 2, 512, 32, 50, 10, 1, "bf16", 1.0, 642)      # 320 rows: 256 x 128 tiles, 3 dead wave tiles
    _assert_errs(_layer_case(w), TOL["bf16"])


@pytest.mark.slow
def test_layer_deep_wide_full_width_bf16():
    # the deep-wide workload's layer at its real widths (H = 6144, 48 heads, F = 24576: 453 M parameters), one
    # micro-batch of 8 sequences: GEMMs with K and N of 6144, 18432 and 24576, dW GEMMs of 6144 x 24576 outputs
    # (2304 tiles), LayerNorm in its two-kernel form
    w = S.WORKLOADS[4].scaled(num_ubatches=1)
    _assert_errs(_layer_case(w), TOL["bf16"])


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_layer_unfused_attention_path_still_matches(monkeypatch, dtype):
    # the batched-GEMM attention path (used for other head widths / sequence lengths), forced at a fused shape
    monkeypatch.setenv("L2L_NO_FUSED_ATTENTION", "1")
    w = S.Workload("unfused", 1, 128, 2, 256, 64, 50, 3, 2, dtype, 1.0, 80)
    _assert_errs(_layer_case(w), TOL[dtype])


@pytest.mark.parametrize("hidden,heads", [(1536, 24), (2304, 36), (6144, 48)])
def test_layer_wide_hidden_bf16(hidden, heads):
    # LayerNorm backward with its column sums in one pass takes up to 2048 columns (four column chunks per lane at
    # 1536); wider rows (2304; 6144 is the deep-wide workload's width) go through the separate dx and column-sum kernels
    w = S.Workload("wide", 1, hidden, heads, 256, 32, 50, 2, 2, "bf16", 1.0, 90 + heads)
    _assert_errs(_layer_case(w), TOL["bf16"])


def test_layer_seq512_bf16():
    w = S.WORKLOADS[3].scaled(num_ubatches=2, ubatch=1)
    _assert_errs(_layer_case(w), TOL["bf16"])


# ------------------------------------------------------------------------------------- whole step
def _step_case(w: S.Workload, stash="device", group=0, lr=1e-4, eager=False, **trainer_kw):
    dtype = w.dtype
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab,
                    ubatch=w.ubatch, num_ubatches=w.num_ubatches, dtype=dtype, lr=lr, stash=stash, ubatch_group=group,
                    eps_threads=8, eager=eager, **trainer_kw)
    try:
        assert tr.eps.is_pinned()
        emb = S.embed_params(w)
        layers = [S.layer_params(w, l) for l in range(w.layers)]
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        tokd, labd = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
        e_r = {k: rounded(v, dtype) for k, v in emb.items()}
        l_r = [{k: rounded(v, dtype) for k, v in p.items()} for p in layers]
        loss_ref, gemb_ref, gl_ref = O.run_l2l(e_r, l_r, tok, lab, w.heads, 1e-12)
        loss = tr.step(tokd, labd)
        errs = {"loss": abs(loss - loss_ref) / abs(loss_ref)}
        ge, gl = tr.grads()
        for k in gemb_ref:
            _both(errs, "emb.d" + k, ge[k], gemb_ref[k])
        for l in range(w.layers):
            for k in gl_ref[l]:
                _both(errs, f"l{l}.d{k}", gl[l][k], gl_ref[l][k])
        # optimizer: the EPS's fp32 master after one Adam step, from ITS OWN gradients, against the oracle's Adam
        me, ml = tr.master_params()
        for k in emb:
            wref, _, _ = O.adam_step(emb[k].astype(np.float64), ge[k].astype(np.float64), 0.0, 0.0, 1, lr=lr)
            errs["adam.emb." + k] = O.rel_l2(me[k] - emb[k], wref - emb[k]) if np.any(ge[k]) else 0.0
        for k in layers[0]:
            wref, _, _ = O.adam_step(layers[0][k].astype(np.float64), gl[0][k].astype(np.float64), 0.0, 0.0, 1, lr=lr)
            errs["adam.l0." + k] = O.rel_l2(ml[0][k] - layers[0][k], wref - layers[0][k])
        return errs, loss, loss_ref
    finally:
        tr.close()


def test_step_tiny_fp32_matches_oracle():
    w = S.WORKLOADS[0]
    errs, loss, loss_ref = _step_case(w)
    adam = {k: v for k, v in errs.items() if k.startswith("adam.")}
    rest = {k: v for k, v in errs.items() if not k.startswith("adam.")}
    _assert_errs(rest, TOL["fp32"])
    _assert_errs(adam, 1e-3)      # w - w0 is a difference of fp32 numbers of size 1: ~1e-7 / 1e-4
    # random init: logits are ~N(0, H * 0.02^2), so the loss sits at ln V + H * 0.02^2 / 2
    assert abs(loss_ref - (math.log(w.vocab) + w.hidden * 0.02 ** 2 / 2)) < 0.03


def test_step_tiny_fp32_eager_eps():
    errs, _, _ = _step_case(S.WORKLOADS[0], eager=True)
    adam = {k: v for k, v in errs.items() if k.startswith("adam.")}
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["fp32"])
    _assert_errs(adam, 1e-3)


def test_three_training_steps_match_oracle_fp32():
    # the whole loop, three times: stage -> forward -> head -> backward -> drain -> EPS Adam -> ship -> stage ...
    w = S.WORKLOADS[0]
    lr = 1e-3
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype="fp32", lr=lr, eager=True, eps_threads=4)
    try:
        emb = {k: v.astype(np.float64) for k, v in S.embed_params(w).items()}
        layers = [{k: v.astype(np.float64) for k, v in S.layer_params(w, l).items()} for l in range(w.layers)]
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        tokd, labd = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
        blocks = [emb] + layers
        m = [{k: np.zeros_like(v) for k, v in b.items()} for b in blocks]
        v2 = [{k: np.zeros_like(v) for k, v in b.items()} for b in blocks]
        for t in range(1, 4):
            loss = tr.step(tokd, labd)
            loss_ref, gemb, gl = O.run_l2l(emb, layers, tok, lab, w.heads, 1e-12)
            assert abs(loss - loss_ref) / abs(loss_ref) < 1e-4, (t, loss, loss_ref)
            for b, g, mm, vv in zip(blocks, [gemb] + gl, m, v2):
                for k in b:
                    b[k], mm[k], vv[k] = O.adam_step(b[k], g[k], mm[k], vv[k], t, lr=lr)
        me, ml = tr.master_params()
        ref0 = {k: v.astype(np.float64) for k, v in S.embed_params(w).items()}
        for k in emb:       # compare the accumulated update, not the weights (which are dominated by their initial value)
            if np.any(emb[k] != ref0[k]):
                assert O.rel_l2(me[k] - ref0[k], emb[k] - ref0[k]) < 2e-3, k
        l0 = S.layer_params(w, 0)
        for k in layers[0]:
            assert O.rel_l2(ml[0][k] - l0[k], layers[0][k] - l0[k]) < 2e-3, k
    finally:
        tr.close()


@pytest.mark.parametrize("eager", [False, True])
def test_two_lamb_steps_match_oracle_fp32(eager):
    # LAMB on the host EPS, tensor by tensor, matrices decayed and vectors not; tail loop and eager per-layer update
    w = S.WORKLOADS[0]
    lr, wd = 2e-3, 0.01
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype="fp32", lr=lr, eps_a=1e-6, eager=eager, eps_threads=4,
                    optimizer="lamb", weight_decay=wd)
    try:
        emb = {k: v.astype(np.float64) for k, v in S.embed_params(w).items()}
        layers = [{k: v.astype(np.float64) for k, v in S.layer_params(w, l).items()} for l in range(w.layers)]
        start = [dict(b) for b in [emb] + layers]
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        tokd, labd = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
        blocks = [emb] + layers
        m = [{k: np.zeros_like(v) for k, v in b.items()} for b in blocks]
        v2 = [{k: np.zeros_like(v) for k, v in b.items()} for b in blocks]
        for t in range(1, 3):
            loss = tr.step(tokd, labd)
            loss_ref, gemb, gl = O.run_l2l(emb, layers, tok, lab, w.heads, 1e-12)
            assert abs(loss - loss_ref) / abs(loss_ref) < 1e-4, (t, loss, loss_ref)
            for b, g, mm, vv in zip(blocks, [gemb] + gl, m, v2):
                for k in b:
                    b[k], mm[k], vv[k] = O.lamb_step(b[k], g[k], mm[k], vv[k], t, lr=lr, eps_a=1e-6,
                                                     weight_decay=wd if b[k].ndim == 2 else 0.0)
        me, ml = tr.master_params()
        for got, ref, s0 in zip([me] + ml, blocks, start):
            for k in ref:
                if np.any(ref[k] != s0[k]):
                    assert O.rel_l2(got[k] - s0[k], ref[k] - s0[k]) < 2e-3, k
    finally:
        tr.close()


@pytest.mark.parametrize("keep_ln_stats", [True, False])
def test_step_tiny_fp32_host_stash(keep_ln_stats):
    # three transit slots with kept LayerNorm statistics (a layer's backward reads its input and its output), two without
    errs, _, _ = _step_case(S.WORKLOADS[0].scaled(layers=5), stash="host", keep_ln_stats=keep_ln_stats)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["fp32"])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_step_without_kept_layernorm_statistics(dtype):
    # the literal recompute of Section 2.1 (l2l_layer_fwd / l2l_layer_bwd): every step test above runs the pair that
    # keeps LayerNorm 2's statistics, this one the plain pair
    errs, _, _ = _step_case(S.WORKLOADS[0].scaled(dtype=dtype), keep_ln_stats=False)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL[dtype])


def test_step_falls_back_to_full_recompute_where_a_layernorm_gain_is_tiny():
    # xhat = (y - be2) / g2 needs |g2| away from zero: the driver checks the master weights per layer and runs the
    # plain backward where they are not
    w = S.WORKLOADS[0]
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype="fp32", eps_threads=4)
    try:
        emb = S.embed_params(w)
        layers = [S.layer_params(w, l) for l in range(w.layers)]
        layers[1]["g2"][5] = 1e-6
        layers[1]["g2"][9] = 0.0
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        loss = tr.step(torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda())
        assert tr._stats_ok == [True, False]
        loss_ref, gemb, gl = O.run_l2l(emb, layers, tok, lab, w.heads, 1e-12)
        assert abs(loss - loss_ref) / abs(loss_ref) < 1e-4
        ge, glayers = tr.grads()
        errs = {}
        for k in gemb:
            _both(errs, "emb." + k, ge[k], gemb[k])
        for l in range(w.layers):
            for k in gl[l]:
                _both(errs, f"l{l}.{k}", glayers[l][k], gl[l][k])
        _assert_errs(errs, TOL["fp32"])
    finally:
        tr.close()


@pytest.mark.parametrize("head_rows,label_prob", [(5, 1.0), (64, 1.0), (64, 0.3)])
def test_step_head_in_several_passes(monkeypatch, head_rows, label_prob):
    # the head takes the labelled rows of the mini-batch head_rows at a time: full passes, a ragged last
    # one, and (label_prob < 1) passes past the labelled count that must do nothing
    monkeypatch.setenv("L2L_HEAD_ROWS", str(head_rows))
    errs, _, _ = _step_case(S.WORKLOADS[0].scaled(label_prob=label_prob))
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["fp32"])


def test_step_with_a_micro_batch_without_labels():
    # one of the four micro-batches carries no label at all: its rows must contribute nothing to the loss and to
    # the head's gradients, and the normalisation is by the labelled count of the whole mini-batch
    w = S.WORKLOADS[0]
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype="fp32", eps_threads=4)
    try:
        emb = S.embed_params(w)
        layers = [S.layer_params(w, l) for l in range(w.layers)]
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        lab = lab.copy()
        lab[2] = -1
        lab[0, 1, 5:] = -1                                   # and a ragged count elsewhere
        tr.device_pipeline(torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda())
        loss = tr.finish()
        loss_ref, gemb, gl = O.run_l2l({k: v.astype(np.float64) for k, v in emb.items()},
                                       [{k: v.astype(np.float64) for k, v in p.items()} for p in layers], tok, lab, w.heads, 1e-12)
        assert abs(loss - loss_ref) / abs(loss_ref) < 1e-4
        ge, glayers = tr.grads()
        errs = {"emb." + k: O.rel_l2(ge[k], gemb[k]) for k in gemb}
        errs.update({f"l{l}.{k}": O.rel_l2(glayers[l][k], gl[l][k]) for l in range(w.layers) for k in gl[l]})
        _assert_errs(errs, TOL["fp32"])
    finally:
        tr.close()


# ------------------------------------------------------------------------------------- sequence-classification head
@pytest.mark.parametrize("dtype,classes,label_prob,eager", [("fp32", 2, 1.0, False), ("fp32", 5, 0.6, True), ("bf16", 3, 1.0, False),
                                                            ("fp16", 2, 0.8, False)])
def test_step_with_sequence_classification_head(dtype, classes, label_prob, eager):
    # the paper's fine-tuning task head (one label per sequence) in place of the LM head: loss, every gradient of the
    # embedding, the layers and the head, and the head's Adam update, against the oracle's Algorithm 2 with that head
    w = S.WORKLOADS[0].scaled(dtype=dtype)
    lr = 1e-4
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype=dtype, lr=lr, eps_threads=4, eager=eager, num_classes=classes)
    try:
        emb, layers, cls = S.embed_params(w), [S.layer_params(w, l) for l in range(w.layers)], S.cls_params(w, classes)
        tr.load_params(emb, layers, cls)
        tok, _ = S.tokens_and_labels(w)
        lab = S.seq_labels(w, classes, label_prob)
        assert (lab < 0).any() == (label_prob < 1.0)
        rd = lambda d: {k: rounded(v, dtype) for k, v in d.items()}
        loss_ref, gemb, gl, gcls = O.run_l2l_cls(rd(emb), [rd(p) for p in layers], rd(cls), tok, lab, w.heads, 1e-12)
        loss = tr.step(torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda())
        errs = {"loss": abs(loss - loss_ref) / abs(loss_ref)}
        ge, glayers = tr.grads()
        gc = tr.cls_grads()
        errs.update({"cls.d" + k: O.rel_l2(gc[k], gcls[k]) for k in gcls})
        errs.update({"emb.d" + k: O.rel_l2(ge[k], gemb[k]) for k in gemb if gemb[k].any()})
        errs.update({f"l{l}.d{k}": O.rel_l2(glayers[l][k], gl[l][k]) for l in range(w.layers) for k in gl[l]})
        _assert_errs(errs, TOL[dtype])
        assert not ge["bv"].any()                                  # the LM head took no part
        cm = tr.cls_master()
        for k in cls:
            wref, _, _ = O.adam_step(cls[k].astype(np.float64), gc[k].astype(np.float64), 0.0, 0.0, 1, lr=lr)
            assert O.rel_l2(cm[k] - cls[k], wref - cls[k]) < 2e-3, k
    finally:
        tr.close()


# ------------------------------------------------------------------------------------- fp16 with loss scaling
@pytest.mark.parametrize("eager", [False, True])
def test_step_fp16_with_loss_scale(eager):
    # Section 2.3's device precision: IEEE half with the loss gradient scaled by 2^15 and the scale divided out on the host
    w = S.WORKLOADS[0].scaled(dtype="fp16")
    errs, loss, loss_ref = _step_case(w, eager=eager)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["fp16"])
    _assert_errs({k: v for k, v in errs.items() if k.startswith("adam.")}, 2e-3)


def test_fp16_without_loss_scale_loses_the_small_gradients():
    # the loss gradient per logit is ~1/(N V) ~ 1e-6, in half precision's subnormal range: without scaling the
    # gradients come out several times less accurate than with it (why Section 2.3 scales the loss)
    w = S.WORKLOADS[0].scaled(dtype="fp16")
    scaled, _, _ = _step_case(w)
    unscaled, _, _ = _step_case(w, loss_scale=1.0)
    grads = [k for k in scaled if not k.startswith("adam.") and not k.startswith("max:") and k != "loss"]
    assert max(unscaled[k] for k in grads) > 4 * max(scaled[k] for k in grads)


def test_fp16_overflow_skips_the_step_and_halves_the_scale():
    w = S.WORKLOADS[0].scaled(dtype="fp16")
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype="fp16", eps_threads=4, loss_scale=2.0 ** 40, scale_growth_interval=2)
    try:
        tr.load_params(S.embed_params(w), [S.layer_params(w, l) for l in range(w.layers)])
        tok, lab = S.tokens_and_labels(w)
        tokd, labd = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
        before = tr.eps.master(1).copy()
        loss = tr.step(tokd, labd)                          # 2^40 / N overflows half precision: step skipped
        assert math.isfinite(loss)                          # the loss itself is not scaled
        assert tr.t == 0 and tr.scaler.skipped == 1 and tr.scaler.scale == 2.0 ** 39
        assert np.array_equal(tr.eps.master(1), before)
        assert not tr.eps.moment(1, 0).any()
        tr.scaler.scale = 2.0 ** 12                          # a workable scale: the next steps go through and grow it
        tr.ctx.set_loss_scale(tr.scaler.scale)
        tr.step(tokd, labd)
        tr.step(tokd, labd)
        assert tr.t == 2 and tr.scaler.scale == 2.0 ** 13
        assert not np.array_equal(tr.eps.master(1), before)
        assert np.isfinite(tr.eps.master(1)).all()
    finally:
        tr.close()


def test_step_bf16_small_depth():
    # BERT-Base widths, 3 layers, fewer rows; 15% random labels
    w = S.WORKLOADS[1].scaled(layers=3, ubatch=2, num_ubatches=3, vocab=3000)
    errs, loss, loss_ref = _step_case(w, group=2)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["bf16"])


@pytest.mark.parametrize("stash", ["device", "host"])
def test_step_bf16_long_sequences(stash):
    # S = 256: the chunked attention kernels inside whole steps (two layers, so that a layer's row statistics from the
    # recompute pass are overwritten by the next layer's before its backward kernels run), device and host stash
    w = S.Workload("long-step", 2, 128, 2, 256, 256, 500, 2, 3, "bf16", 0.15, 901)
    errs, loss, loss_ref = _step_case(w, stash=stash, group=2)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["bf16"])


def test_step_bf16_wide_hidden():
    # H = 3584: the embedding backward kernel turns each row through LDS (5 H floats, more than the 64 KB a kernel gets
    # without asking), LayerNorm backward takes its two-kernel form (H > 2048)
    w = S.Workload("wide-step", 1, 3584, 56, 256, 32, 50, 2, 2, "bf16", 1.0, 555)
    errs, loss, loss_ref = _step_case(w)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["bf16"])


@pytest.mark.slow
def test_step_bert_base_bf16_full():
    w = S.WORKLOADS[1]
    errs, loss, loss_ref = _step_case(w)
    _assert_errs({k: v for k, v in errs.items() if not k.startswith("adam.")}, TOL["bf16"])
    assert abs(loss_ref - (math.log(w.vocab) + w.hidden * 0.02 ** 2 / 2)) < 0.03


@pytest.mark.parametrize("compute,grad_dtype,eager", [("fp32", "bf16", False), ("fp32", "fp16", True), ("bf16", "bf16", True), ("fp16", "fp16", False)])
def test_step_with_16_bit_gradient_drains(compute, grad_dtype, eager):
    # l2l_set_drain_dtype: the fp32 accumulators are rounded on the device, cross the host link in 16 bits and are
    # widened on the host; the optimizer then sees the rounded gradients
    w = S.WORKLOADS[0].scaled(dtype=compute)
    kw = dict(loss_scale=256.0) if compute == "fp16" else {}
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype=compute, lr=1e-3, eager=eager, eps_threads=4, grad_dtype=grad_dtype, **kw)
    try:
        emb, layers = S.embed_params(w), [S.layer_params(w, l) for l in range(w.layers)]
        tr.load_params(emb, layers)
        tok, lab = S.tokens_and_labels(w)
        loss = tr.step(torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda())
        e64 = {k: rounded(v, compute).astype(np.float64) for k, v in emb.items()}
        l64 = [{k: rounded(v, compute).astype(np.float64) for k, v in l.items()} for l in layers]
        loss_ref, gemb, gl = O.run_l2l(e64, l64, tok, lab, w.heads, 1e-12)
        assert abs(loss - loss_ref) / abs(loss_ref) < (1e-4 if compute == "fp32" else 2e-2)
        ge, gls = tr.grads()
        scale = tr.scaler.scale
        for name, got, ref in [("emb", ge, gemb)] + [(f"layer{i}", g, r) for i, (g, r) in enumerate(zip(gls, gl))]:
            for k in ref:
                # what landed (before the host's unscaling) is representable in the 16-bit format
                raw = (got[k].astype(np.float64) * scale).astype(np.float32)
                assert np.array_equal(rounded(raw, grad_dtype).astype(np.float32), raw), (name, k)
                if np.abs(ref[k]).max() > 0:
                    tol = 4e-3 if compute == "fp32" else TOL[compute]      # one 16-bit rounding on top of the fp32 path
                    assert O.rel_l2(got[k], ref[k]) < tol, (name, k, O.rel_l2(got[k], ref[k]))
        # and the block landed in 16 bits: the landing buffer holds the same values
        if grad_dtype == "bf16":
            landed = (tr.eps.grad16(1).astype(np.uint32) << 16).view(np.float32)
        else:
            landed = tr.eps.grad16(1).view(np.float16).astype(np.float32)
        assert np.array_equal(landed.astype(np.float64) / scale, tr.eps.grad(1).astype(np.float64))
    finally:
        tr.close()


def test_embedding_block_staged_and_drained_in_pieces():
    # l2l_embed_stage_part / l2l_embed_grad_drain_part: same bytes as the one-piece calls, pieces in order only
    w = S.WORKLOADS[0]
    cfg = P.make_config(w.hidden, w.heads, w.ffn, w.seq, w.ubatch, w.num_ubatches, "fp32", 1e-12, w.vocab)
    n = P.lib().l2l_embed_packed_elems(cfg)
    lay = P.embed_layout(cfg)
    host = pinned(pack(lay, n, S.embed_params(w)).astype(np.float32))
    tok, lab = S.tokens_and_labels(w)
    tokd, labd = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
    shape = (w.num_ubatches, w.ubatch, w.seq, w.hidden)
    pieces = [(0, 1000), (1000, 7), (1007, n - 1007)]
    outs, grads = [], []
    for in_pieces in (False, True):
        c = P.Context(cfg)
        try:
            x, dy = torch.zeros(shape, device="cuda"), torch.zeros(shape, device="cuda")
            loss = torch.zeros(1, device="cuda")
            if in_pieces:
                with pytest.raises(P.L2LError) as e:
                    c.embed_stage_part(host, n - 5, 6)
                assert e.value.code == P.L2L_E_ARG
                for first, count in reversed(pieces):       # any order: the caller only has to cover the block
                    c.embed_stage_part(host, first, count)
            else:
                c.embed_stage(host)
            c.embed_fwd(tokd, x)
            c.head_loss(x, labd, dy, loss)
            c.embed_bwd(tokd, dy)
            g = torch.zeros(n, dtype=torch.float32).pin_memory()
            if in_pieces:
                with pytest.raises(P.L2LError) as e:
                    c.embed_grad_drain_part(g, 1000, 7)      # must start at element 0
                assert e.value.code == P.L2L_E_ARG
                c.embed_grad_drain_part(g, *pieces[0])
                with pytest.raises(P.L2LError) as e:
                    c.embed_grad_drain(g)                    # a drain in pieces is under way
                assert e.value.code == P.L2L_E_STATE
                with pytest.raises(P.L2LError) as e:
                    c.embed_grad_drain_part(g, 1007, 5)      # gap
                assert e.value.code == P.L2L_E_ARG
                c.embed_grad_drain_part(g, *pieces[1])
                c.embed_grad_drain_part(g, *pieces[2])
                with pytest.raises(P.L2LError) as e:
                    c.embed_grad_drain_part(g, 0, 10)        # nothing left to drain
                assert e.value.code == P.L2L_E_STATE
            else:
                c.embed_grad_drain(g)
            c.embed_drain_wait()
            c.sync()
            outs.append(x.cpu().numpy())
            grads.append(g.numpy().copy())
            c.embed_fwd(tokd, x)                             # the accumulator was released: the next step may start
            c.sync()
        finally:
            c.close()
    assert np.array_equal(outs[0], outs[1])
    assert O.rel_l2(grads[1], grads[0]) < 1e-6               # (fp32 atomics: the order of the additions is not fixed)
    assert np.abs(grads[0]).max() > 0


def test_row_copies_move_every_byte_in_both_directions():
    # l2l_memcpy_rows_async: rows of 64 KiB plus a plain copy of the remainder; sizes below, at and across the row size
    stream = torch.cuda.Stream()
    rng = np.random.default_rng(3)
    for n in (1, 1000, 65536, 65536 * 3 + 123, 5 * 1024 * 1024 + 8):
        src = torch.from_numpy(rng.integers(0, 256, size=n, dtype=np.uint8)).pin_memory()
        dev = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
        back = torch.zeros(n + 64, dtype=torch.uint8).pin_memory()
        torch.cuda.synchronize()
        B.memcpy_rows_async(dev, src, n, False, stream.cuda_stream)
        B.memcpy_rows_async(back, dev, n, True, stream.cuda_stream)
        stream.synchronize()
        assert torch.equal(dev[:n].cpu(), src) and not dev[n:].any(), n
        assert torch.equal(back[:n], src) and not back[n:].any(), n
    B.memcpy_rows_async(dev, src, 0, False, stream.cuda_stream)          # nothing to move: no error
    with pytest.raises(P.L2LError):
        B.memcpy_rows_async(None, src, 8, False, stream.cuda_stream)


# ------------------------------------------------------------------------------------- call-order errors
def test_call_order_errors():
    cfg = P.make_config(64, 2, 128, 16, 2, 2, "fp32", 1e-5, 0)
    c = P.Context(cfg)
    x = torch.zeros(2, 2, 16, 64, device="cuda")
    y = torch.zeros_like(x)
    try:
        with pytest.raises(P.L2LError) as e:
            c.layer_fwd(0, 0, x, y)                       # never staged
        assert e.value.code == P.L2L_E_STATE
        with pytest.raises(P.L2LError) as e:
            c.layer_fwd(0, 2, x, y)
        assert e.value.code == P.L2L_E_ARG
        with pytest.raises(P.L2LError) as e:
            c.grad_drain(0, pinned(np.zeros(4, np.float32)))
        assert e.value.code == P.L2L_E_STATE
        with pytest.raises(P.L2LError) as e:
            c.embed_fwd(x, y)                             # vocab = 0
        assert e.value.code == P.L2L_E_STATE
        n = P.lib().l2l_layer_packed_elems(cfg)
        host = pinned(np.zeros(n, np.float32))
        c.param_stage(3, host, 1)
        with pytest.raises(P.L2LError) as e:
            c.layer_fwd(2, 1, x, y)                       # slot holds another layer
        assert e.value.code == P.L2L_E_STATE
        with pytest.raises(P.L2LError):
            c.layer_fwd(3, 1, None, y)
        c.layer_bwd(3, 1, x, y)
        c.param_stage(4, host, 0)
        c.layer_bwd(4, 0, x, y)
        with pytest.raises(P.L2LError) as e:
            c.layer_bwd(3, 1, x, y)                       # both accumulators hold un-drained gradients
        assert e.value.code == P.L2L_E_STATE
        g = torch.empty(n, dtype=torch.float32).pin_memory()
        c.grad_drain(3, g)
        c.drain_wait(3)
        c.layer_bwd(3, 1, x, y)
        c.sync()
    finally:
        c.close()
