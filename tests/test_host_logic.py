"""CPU-only tests: the C-ABI library loads and exports what the header declares; packed layouts;
config checking; the host EPS (Adam, bf16 shipping copy) against the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2002_05645_amd as P
from paper_2002_05645_amd import binding as B
from oracle import l2l_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "l2l.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b((?:l2l|eps)_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) > 40
    lib = C.CDLL(P.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.EXPORTS), set(names) ^ set(B.EXPORTS)


def test_layout_and_counts():
    cfg = P.make_config(1024, 16, 4096, 128, 32, 8, "bf16", 1e-12, 30522)
    L = P.lib()
    assert L.l2l_layer_param_count(cfg) == O.layer_param_count(1024, 4096) == 12596224
    lay = P.layer_layout(cfg)
    assert list(lay) == list(O.LAYER_KEYS)
    end = 0
    for k, (off, n) in lay.items():
        assert off % 128 == 0 and off >= end
        end = off + n
    assert L.l2l_layer_packed_elems(cfg) >= end
    assert L.l2l_layer_param_bytes(cfg) == 2 * L.l2l_layer_packed_elems(cfg)
    assert L.l2l_layer_grad_bytes(cfg) == 4 * L.l2l_layer_packed_elems(cfg)
    assert sum(n for _, n in lay.values()) == 12596224
    el = P.embed_layout(cfg)
    assert list(el) == list(O.EMBED_KEYS)
    assert el["E"][1] == 30522 * 1024 and el["bv"][1] == 30522
    # ragged sizes get padded sub-blocks
    cfg2 = P.make_config(72, 3, 200, 24, 3, 3, "fp32", 1e-5, 50)
    lay2 = P.layer_layout(cfg2)
    assert all(off % 128 == 0 for off, _ in lay2.values())
    assert L.l2l_layer_param_bytes(cfg2) == 4 * L.l2l_layer_packed_elems(cfg2)


@pytest.mark.parametrize("bad", [dict(hidden=100), dict(heads=3), dict(ffn=130), dict(seq=12), dict(dtype=7),
                                 dict(vocab=31), dict(ubatch=0), dict(num_ubatches=0), dict(ubatch_group=9),
                                 dict(ln_eps=-1.0)])
def test_config_check_rejects(bad):
    kw = dict(hidden=128, heads=2, ffn=512, seq=64, ubatch=4, num_ubatches=4, dtype=0, ln_eps=1e-12, vocab=1000,
              ubatch_group=0)
    assert P.lib().l2l_config_check(B.l2l_config(**kw)) == P.L2L_OK
    kw.update(bad)
    cfg = B.l2l_config(**kw)
    assert P.lib().l2l_config_check(cfg) == P.L2L_E_ARG
    assert P.lib().l2l_layer_packed_elems(cfg) == 0
    assert P.lib().l2l_layer_tensor_offset(cfg, 0) == -1


def test_null_arguments_are_errors_not_crashes():
    L = P.lib()
    assert L.l2l_config_check(None) == P.L2L_E_ARG
    assert L.l2l_param_stage(None, 0, None, 0) == P.L2L_E_ARG
    assert L.l2l_layer_fwd(None, 0, 0, None, None) == P.L2L_E_ARG
    assert L.l2l_layer_bwd(None, 0, 0, None, None) == P.L2L_E_ARG
    assert L.l2l_grad_drain(None, 0, None) == P.L2L_E_ARG
    assert L.l2l_drain_wait(None, 0) == P.L2L_E_ARG
    assert L.l2l_sync(None) == P.L2L_E_ARG
    assert L.l2l_destroy(None) == P.L2L_E_ARG
    assert L.l2l_layer_tensor_name(99) is None
    assert L.eps_destroy(None) == P.L2L_E_ARG
    assert L.eps_adam_step(None, 0, 0, 1, 1e-4, 0.9, 0.999, 1e-8) == P.L2L_E_ARG
    out = C.c_void_p()
    assert L.eps_create(0, None, 1, 1, C.byref(out)) == P.L2L_E_ARG
    assert L.l2l_create(None, None, None, C.byref(out)) == P.L2L_E_ARG


def test_eps_bf16_ship_is_round_to_nearest_even_bit_exact():
    n = 1 << 18
    rng = np.random.default_rng(0)
    w = (rng.normal(size=n) * np.exp(rng.normal(size=n) * 4)).astype(np.float32)
    w[:8] = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0x00000001, 0x80000000, 0x7F800000],
                     np.uint32).view(np.float32)
    e = P.EPS([n], "bf16", 4)
    e.master(0)[:] = w
    e.refresh_ship()
    assert np.array_equal(e.ship(0), O.bf16_bits(w))
    e.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_eps_widens_16_bit_gradients(dtype):
    # gradients that crossed the host link in 16 bits are widened into the fp32 buffers the optimizer reads
    n = 100003
    rng = np.random.default_rng(5)
    e = P.EPS([9, n], dtype, 3)
    with pytest.raises(P.L2LError):
        e.grad_widen(0, 1, dtype)                      # landing buffers not enabled yet
    e.enable_grad16()
    e.enable_grad16()                                  # idempotent
    vals = (rng.normal(size=n) * 10.0 ** rng.integers(-8, 4, size=n)).astype(np.float32)
    if dtype == "bf16":
        bits = O.bf16_bits(vals)
        want = (bits.astype(np.uint32) << 16).view(np.float32)
    else:
        vals[:7] = [np.inf, -np.inf, 65504.0, 6e-8, -0.0, 1e-9, 70000.0]      # inf, max, subnormal, zero, underflow, overflow
        with np.errstate(over="ignore"):
            h = vals.astype(np.float16)
        bits, want = h.view(np.uint16), h.astype(np.float32)
    e.grad16(1)[:] = bits
    e.grad(1)[:] = -1.0
    e.grad_widen_range(1, 10, 50000, dtype)
    assert np.array_equal(e.grad(1)[10:50010], want[10:50010]) and np.all(e.grad(1)[:10] == -1.0) and np.all(e.grad(1)[50010:] == -1.0)
    e.grad_widen(0, 1, dtype)
    assert np.array_equal(e.grad(1), want) and np.all(e.grad(0) == 0)
    for bad in [(1, -1, 5), (1, 0, 0), (1, n - 3, 4), (2, 0, 1)]:
        with pytest.raises(P.L2LError):
            e.grad_widen_range(bad[0], bad[1], bad[2], dtype)
    with pytest.raises(P.L2LError):
        e.grad_widen(0, 1, "fp32")
    e.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_eps_adam_from_16_bit_gradients_equals_widen_then_adam(dtype):
    n = 70001
    rng = np.random.default_rng(6)
    a, b = P.EPS([n], "bf16", 3), P.EPS([n], "bf16", 2)
    for e in (a, b):
        e.enable_grad16()
        e.master(0)[:] = np.linspace(-1, 1, n, dtype=np.float32)
    for t in range(1, 4):
        g = (rng.normal(size=n) * 1e-2).astype(np.float32)
        bits = O.bf16_bits(g) if dtype == "bf16" else g.astype(np.float16).view(np.uint16)
        a.grad16(0)[:] = bits
        b.grad16(0)[:] = bits
        b.grad(0)[:] = 7.0                                   # the fused step must not look at the fp32 buffer
        a.grad_widen(0, 0, dtype)
        a.adam_step(0, 0, t, lr=1e-3)
        b.adam_step_range16(0, 0, 30000, t, dtype, lr=1e-3)
        b.adam_step_range16(0, 30000, n - 30000, t, dtype, lr=1e-3)
        assert np.array_equal(a.master(0), b.master(0)) and np.array_equal(a.ship(0), b.ship(0))
        assert np.array_equal(a.moment(0, 0), b.moment(0, 0)) and np.array_equal(a.moment(0, 1), b.moment(0, 1))
        assert np.all(b.grad(0) == 7.0)
    with pytest.raises(P.L2LError):
        b.adam_step_range16(0, 0, n, 1, "fp32")
    c = P.EPS([n], "bf16", 1)
    with pytest.raises(P.L2LError):
        c.adam_step_range16(0, 0, n, 1, dtype)               # no 16-bit landing buffers
    for e in (a, b, c):
        e.close()


def test_eps_adam_in_pieces_equals_the_whole_block():
    # the ranged step (the embedding block is updated piece by piece as its gradients land) is the same arithmetic
    n = 200000
    rng = np.random.default_rng(3)
    w0 = rng.normal(size=n).astype(np.float32)
    a, b = P.EPS([n], "bf16", 3), P.EPS([5, n], "bf16", 4)
    a.master(0)[:] = w0
    b.master(1)[:] = w0
    pieces = [(0, 70000), (70000, 1), (70001, 129999)]
    for t in range(1, 3):
        g = rng.normal(size=n).astype(np.float32)
        a.grad(0)[:] = g
        b.grad(1)[:] = g
        a.adam_step(0, 0, t, lr=1e-3)
        for first, count in pieces:
            b.adam_step_range(1, first, count, t, lr=1e-3)
        assert np.array_equal(a.master(0), b.master(1))
        assert np.array_equal(a.moment(0, 0), b.moment(1, 0)) and np.array_equal(a.moment(0, 1), b.moment(1, 1))
        assert np.array_equal(a.ship(0), b.ship(1))
    assert np.all(b.master(0) == 0)
    for bad in [(1, -1, 5), (1, 0, 0), (1, n - 3, 4), (2, 0, 1)]:
        with pytest.raises(P.L2LError):
            b.adam_step_range(bad[0], bad[1], bad[2], 1)
    a.close()
    b.close()


def test_eps_grad_unscale_of_a_piece():
    # the ranged form touches its elements only, and reports a non-finite value only if it lies inside them
    n = 100000
    e = P.EPS([7, n], "fp16", 3)
    g0 = np.random.default_rng(5).normal(size=n).astype(np.float32)
    e.grad(1)[:] = g0
    assert e.grad_unscale_range(1, 1000, 70000, 0.25) is False
    want = g0.copy()
    want[1000:71000] *= np.float32(0.25)
    assert np.array_equal(e.grad(1), want)
    e.grad(1)[80000] = np.inf
    assert e.grad_unscale_range(1, 0, 80000, 1.0) is False
    assert e.grad_unscale_range(1, 79999, 2, 1.0) is True
    e.grad(1)[80000] = np.nan
    assert e.grad_unscale_range(1, 80000, n - 80000, 0.5) is True
    for bad in [(1, -1, 5), (1, 0, 0), (1, n - 3, 4), (2, 0, 1)]:
        with pytest.raises(P.L2LError):
            e.grad_unscale_range(bad[0], bad[1], bad[2], 1.0)
    e.close()


@pytest.mark.parametrize("threads", [1, 5])
def test_eps_adam_matches_oracle(threads):
    n = 300001
    rng = np.random.default_rng(1)
    w0 = rng.normal(size=n).astype(np.float32)
    e = P.EPS([7, n], "bf16", threads)
    e.master(1)[:] = w0
    w, m, v = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 4):
        g = (rng.normal(size=n) * 10.0 ** rng.integers(-6, 1, size=n)).astype(np.float32)
        g[::17] = 0
        e.grad(1)[:] = g
        e.adam_step(1, 1, t, lr=1e-3)
        w, m, v = O.adam_step(w, g.astype(np.float64), m, v, t, lr=1e-3)
        np.testing.assert_allclose(e.master(1), w, rtol=2e-6, atol=1e-9)
        np.testing.assert_allclose(e.moment(1, 0), m, rtol=1e-5, atol=1e-7)      # fp32 cancellation when m crosses zero
        np.testing.assert_allclose(e.moment(1, 1), v, rtol=1e-5, atol=1e-30)
        assert np.array_equal(e.ship(1), O.bf16_bits(e.master(1)))
    assert np.all(e.master(0) == 0)          # untouched block
    # first step of Adam moves every weight with a non-zero gradient by about lr
    e2 = P.EPS([n], "fp32", threads)
    e2.master(0)[:] = w0
    g = rng.normal(size=n).astype(np.float32)
    e2.grad(0)[:] = g
    e2.adam_step(0, 0, 1, lr=1e-3)
    np.testing.assert_allclose(e2.master(0) - w0, -1e-3 * g / (np.abs(g) + 1e-8), atol=5e-7)
    assert np.array_equal(e2.ship(0), e2.master(0))
    e.close()
    e2.close()


def test_cls_head_layout():
    cfg = P.make_config(768, 12, 3072, 128, 4, 2, "bf16", 1e-12, 0)
    lay = P.cls_layout(cfg, 3)
    assert list(lay) == ["Wp", "bp", "Wc", "bc"]
    assert [n for _, n in lay.values()] == [768 * 768, 768, 768 * 3, 3]
    end = 0
    for off, n in lay.values():
        assert off % 128 == 0 and off >= end
        end = off + n
    assert P.lib().l2l_cls_packed_elems(cfg, 3) == (end + 127) // 128 * 128
    assert P.lib().l2l_cls_packed_elems(cfg, 1) == 0                     # at least two classes
    assert P.lib().l2l_cls_tensor_offset(cfg, 3, 4) == -1
    assert P.lib().l2l_cls_stage(None, None, 2) == P.L2L_E_ARG


def test_eps_fp16_ship_and_grad_unscale():
    n = 1 << 17
    rng = np.random.default_rng(9)
    w = (rng.normal(size=n) * np.exp(rng.normal(size=n) * 6)).astype(np.float32)     # from subnormal halves to overflow
    w[:4] = [65504.0, 65520.0, 2.0 ** -25, -(1.0 + 2.0 ** -11)]
    e = P.EPS([n], "fp16", 3)
    e.master(0)[:] = w
    e.refresh_ship()
    assert np.array_equal(e.ship(0), O.fp16_bits(w))                                # IEEE half, ties to even, bit for bit
    g = rng.normal(size=n).astype(np.float32) * 1024.0
    e.grad(0)[:] = g
    assert e.grad_unscale(0, 0, 1.0 / 1024.0) is False
    assert np.array_equal(e.grad(0), g / np.float32(1024.0))                        # a power of two divides out exactly
    for bad in (np.inf, -np.inf, np.nan):
        e.grad(0)[n // 2] = bad
        assert e.grad_unscale(0, 0, 0.5) is True
        e.grad(0)[n // 2] = 0.0
    assert e.grad_unscale(0, 0, 1.0) is False
    e.close()


def test_loss_scaler_policy():
    from paper_2002_05645_amd.trainer import LossScaler
    s = LossScaler(scale=1024.0, growth_interval=3)
    assert [s.update(False), s.update(False)] == [True, True] and s.scale == 1024.0
    assert s.update(True) is False and s.scale == 512.0 and s.skipped == 1      # overflow: skip, halve, restart the count
    assert [s.update(False) for _ in range(3)] == [True] * 3 and s.scale == 1024.0
    assert s.update(False) and s.scale == 1024.0
    floor = LossScaler(scale=1.0, growth_interval=1, min_scale=1.0)
    assert floor.update(True) is False and floor.scale == 1.0                       # never below the floor
    fixed = LossScaler(scale=64.0, growth_interval=1, static=True)
    assert fixed.update(False) and fixed.update(True) is False and fixed.scale == 64.0


@pytest.mark.parametrize("threads", [1, 5])
def test_eps_lamb_matches_oracle_per_tensor(threads):
    # three tensors of different size inside one block, with padding between them that must stay untouched
    n = 200000
    segs = [(0, 70001), (70016, 70016 + 999), (80000, 200000)]
    mask = [1.0, 0.0, 1.0]
    rng = np.random.default_rng(3)
    w0 = rng.normal(size=n).astype(np.float32)
    e = P.EPS([n, n], "bf16", threads)
    e.master(0)[:] = w0
    e.master(1)[:] = w0
    e.refresh_ship()
    w = w0.astype(np.float64)
    m, v = np.zeros(n), np.zeros(n)
    hp = dict(lr=2e-3, beta1=0.9, beta2=0.999, eps_a=1e-6, weight_decay=0.01)
    for t in range(1, 4):
        g = (rng.normal(size=n) * 10.0 ** rng.integers(-4, 1, size=n)).astype(np.float32)
        e.grad(1)[:] = g
        e.lamb_step(1, 1, t, segs, decay_mask=mask, **hp)
        for (a, b), dm in zip(segs, mask):
            w[a:b], m[a:b], v[a:b] = O.lamb_step(w[a:b], g[a:b].astype(np.float64), m[a:b], v[a:b], t, lr=hp["lr"],
                                                 eps_a=hp["eps_a"], weight_decay=hp["weight_decay"] * dm)
        np.testing.assert_allclose(e.master(1), w, rtol=3e-6, atol=1e-8)
        np.testing.assert_allclose(e.moment(1, 1), v, rtol=1e-5, atol=1e-30)
        assert np.array_equal(e.ship(1), O.bf16_bits(e.master(1)))
    pad = np.ones(n, bool)
    for a, b in segs:
        pad[a:b] = False
    assert np.array_equal(e.master(1)[pad], w0[pad])          # outside every tensor: untouched
    assert np.array_equal(e.master(0), w0)                    # other block untouched
    # without decay a step moves each tensor by lr * ||w||
    e.master(0)[:] = w0
    e.grad(0)[:] = rng.normal(size=n).astype(np.float32)
    e.lamb_step(0, 0, 1, segs, lr=1e-2, weight_decay=0.0)
    for a, b in segs:
        np.testing.assert_allclose(np.linalg.norm(e.master(0)[a:b].astype(np.float64) - w0[a:b]),
                                   1e-2 * np.linalg.norm(w0[a:b].astype(np.float64)), rtol=1e-4)
    # malformed segment lists are rejected
    for bad in ([(10, 5)], [(0, 100), (50, 200)], [(0, n + 1)]):
        with pytest.raises(P.L2LError) as ex:
            e.lamb_step(0, 0, 1, bad)
        assert ex.value.code == P.L2L_E_ARG
    e.close()


# ------------------------------------------------------------------ polynomial GELU of the bf16 epilogues
def _fast_form(name, a):
    """Evaluates, in fp32 and in the kernel's order, the odd polynomial `name` of csrc/common.h on clamped u / a."""
    import re
    src = open(os.path.join(os.path.dirname(B.__file__), "csrc", "common.h")).read()
    body = src[src.index("float " + name):]
    body = body[:body.index("return")]
    c = [np.float32(x) for x in re.findall(r"(-?\d\.\d+e[+-]\d+)f", body)]
    assert len(c) >= 8

    def f(u):
        s = (np.clip(u, -a, a).astype(np.float32) * np.float32(1.0 / a)).astype(np.float32)
        t = (s * s).astype(np.float32)
        p = np.full_like(t, c[0])
        for k in c[1:]:
            p = (p * t + k).astype(np.float32)
        return (p * s + np.float32(0.5)).astype(np.float32)
    return f


def test_fast_gelu_polynomials_match_exact_functions():
    # the bf16 GEMM epilogues use polynomial forms of Phi and gelu'; their error must stay far below the
    # bf16 rounding step (2^-8 relative) of the values they produce
    u = np.linspace(-20.0, 20.0, 800001).astype(np.float32)
    u64 = u.astype(np.float64)
    gelu = u * _fast_form("gelu_fast_f", 4.0)(u)
    dgelu = _fast_form("gelu_grad_fast_f", 4.5)(u)
    assert np.abs(gelu - O.gelu(u64)).max() < 2e-4
    assert np.abs(dgelu - O.gelu_grad(u64)).max() < 3e-4
    big = np.abs(u) > 6                                              # tails: the limits, to fp32 rounding
    assert np.abs(gelu[big] - np.maximum(u[big], 0)).max() <= 1e-6 * 20
    assert np.abs(dgelu[big] - (u[big] > 0)).max() <= 1e-5


def test_gelu_gradient_from_phi_and_the_density_matches_the_exact_function():
    # the recompute pass's FFN1 epilogue forms gelu'(u) = Phi(u) + u phi(u) from the polynomial Phi and an exponential
    # (csrc/common.h, gelu_and_grad_fast_f): the same arithmetic in fp32 here, against the exact derivative
    u = np.linspace(-20.0, 20.0, 800001).astype(np.float32)
    cdf = _fast_form("gelu_fast_f", 4.0)(u)
    arg = np.maximum((u * u).astype(np.float32) * np.float32(-0.72134752044448170), np.float32(-126.0)).astype(np.float32)
    dens = np.exp2(arg).astype(np.float32)
    grad = ((u * dens).astype(np.float32) * np.float32(0.39894228040143268) + cdf).astype(np.float32)
    assert np.abs(grad - O.gelu_grad(u.astype(np.float64))).max() < 6e-5
    big = np.abs(u) > 6
    assert np.abs(grad[big] - (u[big] > 0)).max() <= 1e-6


@pytest.mark.parametrize("kind", ["address,undefined", "thread"])
def test_eps_under_sanitizers_with_two_calling_threads(kind, tmp_path):
    # csrc/eps.cpp built for the host alone under ASan + UBSan and under TSan, driven by two threads that call into one
    # store at the same time (the trainer's eager-update thread and its main thread): no finding, and the same
    # results as the same calls made in sequence
    import subprocess
    from paper_2002_05645_amd import build as bld
    exe = bld.build_host_sanitized(kind, os.path.join(ROOT, "tests", "host", "eps_threads_driver.cpp"), str(tmp_path / "eps_threads"))
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "eps threads driver: ok" in r.stdout
    assert "Sanitizer" not in r.stderr, r.stderr
