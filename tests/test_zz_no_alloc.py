"""GPU test of the entry point that allocates nothing (l2l_op_gemm_accum_noalloc) against the existing entry point
it is a variant of (l2l_op_gemm with an fp32 output and accumulate), through the C ABI, on two calls in a row, the
second with a smaller input (the file name sorts behind the other test files, so pytest collects it last)."""
import numpy as np
import pytest
import torch

import paper_2002_05645_amd as P
from paper_2002_05645_amd import binding as B
from oracle import l2l_oracle as O
from gpu_util import to_dev, to_host, rounded

pytestmark = pytest.mark.gpu


def _operands(M, N, K, a_kc, b_kc, dtype, seed):
    rng = np.random.default_rng(seed)
    A = rng.normal(size=(M, K)).astype(np.float32)
    Bm = (rng.normal(size=(K, N)) / np.sqrt(K)).astype(np.float32)
    C0 = rng.normal(size=(M, N + 8)).astype(np.float32)
    Ad = to_dev(A if a_kc else np.ascontiguousarray(A.T), dtype)
    Bd = to_dev(np.ascontiguousarray(Bm.T) if b_kc else Bm, dtype)
    ref = rounded(A, dtype) @ rounded(Bm, dtype) + C0[:, :N].astype(np.float64)
    return Ad, Bd, C0, ref, (K if a_kc else M), (K if b_kc else N)


def test_noalloc_gemm_matches_context_gemm_on_two_calls_in_a_row(monkeypatch):
    monkeypatch.setenv("L2L_SPLIT_WS_MB", "64")     # the context's own K-split workspace: room for the same split factors
    ctx = P.Context(P.make_config(64, 2, 128, 16, 2, 2, "bf16", 1e-5, 0))
    stream = torch.cuda.Stream()
    try:
        assert P.lib().l2l_noalloc_scratch_bytes() == 32 << 20
        # (1) 8 tiles x 16 K-splits: 16 x 512 x 1024 floats fill the scratch array exactly; dW layout (both operands K-strided)
        # (2) smaller and ragged everywhere, K-contiguous operands, fp16: its partial results land over the first call's
        # (3) many tiles, no split: the scratch array is not used at all
        cases = [(512, 1024, 8192, 0, 0, "bf16"), (264, 520, 4200 - 8, 1, 1, "fp16"), (1024, 2048, 512, 0, 0, "bf16")]
        # two rounds over the cases: the first use of a kernel makes the runtime load its code object, which takes
        # device memory; in the second round nothing is left to load and device memory must not move at all
        for i, (M, N, K, a_kc, b_kc, dtype) in enumerate(cases + cases):
            Ad, Bd, C0, ref, lda, ldb = _operands(M, N, K, a_kc, b_kc, dtype, seed=100 + i)
            c_ctx = torch.from_numpy(C0).cuda()
            c_new = torch.from_numpy(C0).cuda()
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            ctx.op_gemm(B.DTYPES[dtype], True, a_kc, b_kc, M, N, K, Ad, lda, Bd, ldb, c_ctx, N + 8, accumulate=True)
            stream.wait_stream(torch.cuda.current_stream())
            B.op_gemm_accum_noalloc(stream.cuda_stream, B.DTYPES[dtype], a_kc, b_kc, M, N, K, Ad, lda, Bd, ldb, c_new, N + 8)
            torch.cuda.synchronize()
            if i >= len(cases):
                assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed"
            got_ctx, got_new = to_host(c_ctx), to_host(c_new)
            assert np.array_equal(got_new[:, N:], C0[:, N:].astype(np.float64)), "wrote outside the N columns"
            assert O.rel_l2(got_new[:, :N], got_ctx[:, :N]) < 2e-6 and O.max_rel(got_new[:, :N], got_ctx[:, :N]) < 1e-5, (M, N, K)
            assert O.rel_l2(got_new[:, :N], ref) < 2e-6 and O.max_rel(got_new[:, :N], ref) < 1e-5, (M, N, K)
    finally:
        ctx.close()


def test_noalloc_gemm_rejects_what_it_cannot_hold_or_address():
    M, N, K = 2048, 4096, 8192      # 128 tiles x 2 K-splits: 2 x 2048 x 4096 floats = 64 MiB, twice the scratch array
    A = torch.zeros(K, M, device="cuda", dtype=torch.bfloat16)
    Bm = torch.zeros(K, N, device="cuda", dtype=torch.bfloat16)
    Cm = torch.zeros(M, N, device="cuda")
    with pytest.raises(P.L2LError) as e:
        B.op_gemm_accum_noalloc(0, P.L2L_BF16, 0, 0, M, N, K, A, M, Bm, N, Cm, N)
    assert e.value.code == P.L2L_E_ARG and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert not Cm.any()                                              # nothing ran
    for bad in (dict(in_dtype=P.L2L_F32), dict(A=None), dict(lda=M + 1), dict(ldc=N - 8), dict(M=-1)):
        kw = dict(stream=0, in_dtype=P.L2L_BF16, a_kc=0, b_kc=0, M=M, N=N, K=K, A=A, lda=M, B=Bm, ldb=N, Cm=Cm, ldc=N)
        kw.update(bad)
        with pytest.raises(P.L2LError) as e:
            B.op_gemm_accum_noalloc(**kw)
        assert e.value.code == P.L2L_E_ARG, bad
    B.op_gemm_accum_noalloc(0, P.L2L_BF16, 0, 0, 0, N, K, A, M, Bm, N, Cm, N)      # empty: nothing to do, no error
