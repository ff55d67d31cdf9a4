"""Pins for the CPU oracle: everything here is fixed by mathematics or by values the paper prints,
never by the oracle's own output."""
import math
import os

import numpy as np
import pytest

from oracle import l2l_oracle as O

RNG = np.random.default_rng(7)
EPS = 1e-5


def tiny_model(H=8, A=2, F=16, S=4, V=11, L=2, rng=RNG):
    def n(*s):
        return rng.normal(0, 0.3, s)
    layers = []
    for _ in range(L):
        layers.append({"Wqkv": n(H, 3 * H), "bqkv": n(3 * H), "Wo": n(H, H), "bo": n(H),
                       "g1": 1 + n(H), "be1": n(H), "W1": n(H, F), "b1": n(F),
                       "W2": n(F, H), "b2": n(H), "g2": 1 + n(H), "be2": n(H)})
    emb = {"E": n(V, H), "P": n(S, H), "ge": 1 + n(H), "be": n(H), "bv": n(V)}
    return emb, layers


def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = v.strip()
    return out


# ----------------------------------------------------------------------------- closed forms
def test_gelu_closed_forms():
    u = np.linspace(-6, 6, 241)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert O.gelu_grad(np.array([0.0]))[0] == 0.5
    np.testing.assert_allclose(O.gelu(u) - O.gelu(-u), u, atol=1e-14)
    ref = np.array([0.5 * x * (1 + math.erf(x / math.sqrt(2))) for x in u])
    np.testing.assert_allclose(O.gelu(u), ref, atol=1e-15)
    h = 1e-6
    np.testing.assert_allclose(O.gelu_grad(u), (O.gelu(u + h) - O.gelu(u - h)) / (2 * h), atol=1e-9)
    # differs from the tanh approximation (guards against using the wrong form)
    tanh_form = 0.5 * u * (1 + np.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u ** 3)))
    assert np.abs(O.gelu(u) - tanh_form).max() > 1e-4


def test_softmax_closed_forms():
    s = RNG.normal(size=(3, 5, 7))
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-15)
    np.testing.assert_allclose(O.softmax_rows(s + 1000.0), p, atol=1e-13)
    np.testing.assert_allclose(O.softmax_rows(np.zeros((2, 4))), 0.25)


def test_layernorm_closed_forms():
    H = 16
    r = RNG.normal(size=(5, H)) * 3 + 1
    y, (xhat, rstd) = O.layer_norm_fwd(r, np.ones(H), np.zeros(H), 1e-12)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-14)
    var = r.var(axis=-1)
    np.testing.assert_allclose(y.var(axis=-1), var / (var + 1e-12), rtol=1e-12)
    y2, _ = O.layer_norm_fwd(r * 7.5, np.ones(H), np.zeros(H), 0.0)
    y0, _ = O.layer_norm_fwd(r, np.ones(H), np.zeros(H), 0.0)
    np.testing.assert_allclose(y2, y0, atol=1e-12)
    g, b = RNG.normal(size=H), RNG.normal(size=H)
    yg, _ = O.layer_norm_fwd(r, g, b, 1e-12)
    np.testing.assert_allclose(yg, y * g + b, atol=1e-13)
    dy = RNG.normal(size=(5, H))
    dr, dg, db = O.layer_norm_bwd(dy, (xhat, rstd), g)
    np.testing.assert_allclose(dr.sum(-1), 0, atol=1e-13)
    np.testing.assert_allclose((dr * xhat).sum(-1), 0, atol=1e-11)    # exact only as eps/var -> 0
    np.testing.assert_allclose(db, dy.sum(0), atol=1e-14)


def test_attention_uniform_when_q_zero():
    H, A, S = 8, 2, 5
    emb, (p, _) = tiny_model(H=H, A=A, S=S)
    p = dict(p)
    p["Wqkv"] = p["Wqkv"].copy()
    p["bqkv"] = p["bqkv"].copy()
    p["Wqkv"][:, :H] = 0
    p["bqkv"][:H] = 0
    X = RNG.normal(size=(2, S, H))
    _, c = O.encoder_layer_fwd(X, p, A, EPS)
    np.testing.assert_allclose(c["P"], 1.0 / S, atol=1e-15)
    v = X @ p["Wqkv"][:, 2 * H:] + p["bqkv"][2 * H:]
    np.testing.assert_allclose(c["C"], np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape), atol=1e-14)


def test_layer_reduces_to_double_layernorm():
    H, A, S = 8, 2, 4
    _, (p, _) = tiny_model(H=H, A=A, S=S)
    p = {k: v.copy() for k, v in p.items()}
    for k in ("Wo", "bo", "W1", "b1", "W2", "b2"):
        p[k][...] = 0
    X = RNG.normal(size=(3, S, H))
    Y, _ = O.encoder_layer_fwd(X, p, A, EPS)

    def ln(r, g, b):
        mu = r.mean(-1, keepdims=True)
        return g * (r - mu) / np.sqrt(r.var(-1, keepdims=True) + EPS) + b
    np.testing.assert_allclose(Y, ln(ln(X, p["g1"], p["be1"]), p["g2"], p["be2"]), atol=1e-13)


def test_layer_single_head_single_token_is_gemm_chain():
    # A = 1, S = 1: softmax over one key is 1, so attention is X Wv Wo -- checked by plain loops
    H, F = 6, 10
    _, (p, _) = tiny_model(H=H, A=1, F=F, S=1)
    X = RNG.normal(size=(4, 1, H))
    _, c = O.encoder_layer_fwd(X, p, 1, EPS)
    Wv, bv = p["Wqkv"][:, 2 * H:], p["bqkv"][2 * H:]
    for b in range(4):
        v = [sum(X[b, 0, i] * Wv[i, j] for i in range(H)) + bv[j] for j in range(H)]
        np.testing.assert_allclose(c["C"][b, 0], v, atol=1e-14)
        r1 = [X[b, 0, j] + sum(v[i] * p["Wo"][i, j] for i in range(H)) + p["bo"][j] for j in range(H)]
        r1 = np.array(r1)
        y1 = p["g1"] * (r1 - r1.mean()) / math.sqrt(r1.var() + EPS) + p["be1"]
        np.testing.assert_allclose(c["Y1"][b, 0], y1, atol=1e-13)


def test_head_layout_matches_per_head_loops():
    # brute force attention for one sequence with explicit head slicing of the fused QKV output
    H, A, S = 8, 2, 3
    d = H // A
    _, (p, _) = tiny_model(H=H, A=A, S=S)
    X = RNG.normal(size=(1, S, H))
    _, c = O.encoder_layer_fwd(X, p, A, EPS)
    qkv = X[0] @ p["Wqkv"] + p["bqkv"]
    for h in range(A):
        q = qkv[:, h * d:(h + 1) * d]
        k = qkv[:, H + h * d:H + (h + 1) * d]
        v = qkv[:, 2 * H + h * d:2 * H + (h + 1) * d]
        for s in range(S):
            w = np.array([math.exp(sum(q[s, j] * k[t, j] for j in range(d)) / math.sqrt(d)) for t in range(S)])
            w /= w.sum()
            np.testing.assert_allclose(c["C"][0, s, h * d:(h + 1) * d], w @ v, atol=1e-14)


def test_cross_entropy_closed_forms():
    emb, _ = tiny_model(V=11)
    emb = {k: v.copy() for k, v in emb.items()}
    emb["E"][...] = 0
    emb["bv"][...] = 0
    x = RNG.normal(size=(2, 4, 8))
    lab = RNG.integers(0, 11, size=(2, 4))
    lab[0, 1] = -1
    loss, dx, g = O.head_loss(x, lab, emb, int((lab >= 0).sum()))
    assert abs(loss - math.log(11)) < 1e-14
    emb2, _ = tiny_model(V=11)
    loss, dx, g = O.head_loss(x, lab, emb2, 7)
    assert np.all(dx[0, 1] == 0)
    assert abs(g["bv"].sum()) < 1e-14           # rows of dz sum to zero


def test_paper_sizes():
    g = golden()
    H, F, S = int(g["bert_large_hidden"]), int(g["bert_large_ffn"]), int(g["bert_large_max_seq"])
    assert O.boundary_activation_bytes(S, H, 2) == int(g["boundary_activation_bytes_per_sample"])
    L = int(g["bert_large_layers"])
    total = L * O.layer_param_count(H, F) + 30522 * H + 512 * H
    assert abs(total / 1e6 - float(g["bert_large_params_millions"])) < 20     # "350M" to the paper's rounding
    assert O.layer_param_count(H, F) == 12596224
    for n_layers, bill in zip(map(int, g["table5_layers"].split()), map(float, g["table5_params_billions"].split())):
        assert abs(n_layers * O.layer_param_count(H, F) / 1e9 - bill) < 0.06 * bill + 0.01


def test_timing_model():
    g = golden()
    u = int(g["overhead_example_u"])
    assert O.transfer_overhead(u, 1.0, 1.0, training=False) <= float(g["overhead_example_bound"]) + 1e-15
    assert O.transfer_overhead(u, 1.0, 1.0, training=True) < float(g["overhead_example_bound"])
    assert O.total_time_ms(24, 1, 2.0, 3.0) == 24 * (4 * 2.0 + 2 * 3.0)        # Eq. 1 is Eq. 4 at u = 1
    assert O.total_time_ms(24, 4, 2.0, 3.0) == 24 * (16 * 2.0 + 2 * 3.0)
    assert abs(O.throughput_training(24, 4, 64, 2.0, 3.0) - 1000 * 256 / (24 * 38.0)) < 1e-9
    assert O.throughput_forward(24, 4, 64, 2.0, 0.0) == pytest.approx(1000 * 64 / (24 * 2.0))


# ----------------------------------------------------------------------------- finite differences
def _loss_of(emb, layers, tok, lab, A):
    n_lab = int((lab >= 0).sum())
    x, _ = O.embed_fwd(tok, emb, EPS)
    for p in layers:
        x, _ = O.encoder_layer_fwd(x, p, A, EPS)
    return O.head_loss(x, lab, emb, n_lab)[0]


def test_all_gradients_by_finite_differences():
    H, A, F, S, V, L = 8, 2, 16, 4, 11, 2
    rng = np.random.default_rng(3)
    emb, layers = tiny_model(H, A, F, S, V, L, rng)
    tok = rng.integers(0, V, size=(2, S))
    lab = rng.integers(0, V, size=(2, S))
    lab[1, 2] = -1
    loss, gemb, glayers = O.run_conventional(emb, layers, tok[None], lab[None], A, EPS)
    assert abs(loss - _loss_of(emb, layers, tok, lab, A)) < 1e-13
    h = 1e-5
    groups = [("emb", emb, gemb)] + [(f"layer{l}", layers[l], glayers[l]) for l in range(L)]
    for gname, params, grads in groups:
        for k, w in params.items():
            num = np.zeros_like(w)
            it = np.nditer(w, flags=["multi_index"])
            for _ in it:
                i = it.multi_index
                old = w[i]
                w[i] = old + h
                lp = _loss_of(emb, layers, tok, lab, A)
                w[i] = old - h
                lm = _loss_of(emb, layers, tok, lab, A)
                w[i] = old
                num[i] = (lp - lm) / (2 * h)
            err = np.linalg.norm(num - grads[k]) / max(np.linalg.norm(num), 1e-30)
            assert err < 2e-7, (gname, k, err)


def test_qkv_bias_gradient_parts_have_closed_forms():
    # d loss / d (bias of K) = 0: a bias on the keys moves all scores of a query alike, which softmax does not see;
    # d loss / d (bias of V) = colsum(dC) = colsum(dR1) Wo^T = dbo Wo^T: every row of P sums to one.  Neither is how the
    # oracle computes them (it sums dK and dV over the tokens).
    H, A, F, S = 8, 2, 16, 6
    rng = np.random.default_rng(11)
    _, layers = tiny_model(H, A, F, S, 11, 1, rng)
    p = layers[0]
    X = rng.normal(0, 1, (2, 3, S, H))
    dY = rng.normal(0, 1, (2, 3, S, H))
    _, g = O.layer_l2l_bwd(X, dY, p, A, EPS)
    bq, bk, bv = (g["bqkv"][i * H:(i + 1) * H] for i in range(3))
    assert np.abs(bk).max() < 1e-13 * np.abs(bq).max()
    assert np.allclose(bv, g["bo"] @ p["Wo"].T, rtol=1e-12, atol=1e-14)
    assert np.abs(bq).max() > 1e-3 and np.abs(bv).max() > 1e-3   # (the other two parts are not trivially zero)


def test_layer_input_gradient_by_finite_differences():
    H, A, F, S = 8, 2, 16, 4
    rng = np.random.default_rng(5)
    _, (p, _) = tiny_model(H, A, F, S, rng=rng)
    X = rng.normal(size=(2, S, H))
    Wt = rng.normal(size=(2, S, H))
    Y, c = O.encoder_layer_fwd(X, p, A, EPS)
    dX, _ = O.encoder_layer_bwd(Wt, c, p, A)
    num = np.zeros_like(X)
    h = 1e-6
    for i in np.ndindex(*X.shape):
        old = X[i]
        X[i] = old + h
        lp = (O.encoder_layer_fwd(X, p, A, EPS)[0] * Wt).sum()
        X[i] = old - h
        lm = (O.encoder_layer_fwd(X, p, A, EPS)[0] * Wt).sum()
        X[i] = old
        num[i] = (lp - lm) / (2 * h)
    assert np.linalg.norm(num - dX) / np.linalg.norm(num) < 1e-7


# ----------------------------------------------------------------------------- the L2L invariant
@pytest.mark.parametrize("U", [1, 2, 4, 8])
def test_l2l_equals_conventional_equals_concatenated(U):
    H, A, F, S, V, L = 16, 4, 32, 6, 23, 3
    rng = np.random.default_rng(11)
    emb, layers = tiny_model(H, A, F, S, V, L, rng)
    B = 8
    tok = rng.integers(0, V, size=(B, S))
    lab = np.where(rng.random((B, S)) < 0.4, rng.integers(0, V, size=(B, S)), -1)
    ref = O.run_conventional(emb, layers, tok[None], lab[None], A, EPS)          # one concatenated minibatch
    tu, lu = tok.reshape(U, B // U, S), lab.reshape(U, B // U, S)
    for res in (O.run_conventional(emb, layers, tu, lu, A, EPS), O.run_l2l(emb, layers, tu, lu, A, EPS)):
        assert abs(res[0] - ref[0]) < 1e-12
        for k in ref[1]:
            np.testing.assert_allclose(res[1][k], ref[1][k], atol=1e-12)
        for a, b in zip(res[2], ref[2]):
            for k in b:
                np.testing.assert_allclose(a[k], b[k], atol=1e-12)


def test_layer_l2l_helpers_match_drivers():
    H, A, F, S = 8, 2, 16, 4
    rng = np.random.default_rng(13)
    _, (p, _) = tiny_model(H, A, F, S, rng=rng)
    X = rng.normal(size=(3, 2, S, H))
    dY = rng.normal(size=(3, 2, S, H))
    Y = O.layer_l2l_fwd(X, p, A, EPS)
    Yc, c = O.encoder_layer_fwd(X.reshape(6, S, H), p, A, EPS)
    np.testing.assert_allclose(Y.reshape(6, S, H), Yc, atol=1e-14)
    dX, g = O.layer_l2l_bwd(X, dY, p, A, EPS)
    dXc, gc = O.encoder_layer_bwd(dY.reshape(6, S, H), c, p, A)
    np.testing.assert_allclose(dX.reshape(6, S, H), dXc, atol=1e-13)
    for k in gc:
        np.testing.assert_allclose(g[k], gc[k], atol=1e-12)


# ----------------------------------------------------------------------------- Adam and bf16
def test_adam_closed_forms():
    g = np.array([0.3, -2.0, 0.0, 1e-3])
    w = np.array([1.0, 2.0, 3.0, 4.0])
    z = np.zeros(4)
    lr, e = 1e-4, 1e-8
    w1, m1, v1 = O.adam_step(w, g, z, z, 1, lr=lr, eps_a=e)
    np.testing.assert_allclose(w1 - w, -lr * g / (np.abs(g) + e), rtol=1e-9, atol=1e-15)
    assert w1[2] == w[2]
    w2, m2, v2 = O.adam_step(w1, g, m1, v1, 2, lr=lr, eps_a=e)
    np.testing.assert_allclose(np.abs(w2 - w1)[[0, 1, 3]], lr, rtol=1e-4)
    np.testing.assert_allclose(m2, (1 - 0.9 ** 2) * g, rtol=1e-12)
    np.testing.assert_allclose(v2, (1 - 0.999 ** 2) * g * g, rtol=1e-12)


def test_lamb_closed_forms_and_invariants():
    rng = np.random.default_rng(7)
    n = 257
    w = rng.normal(size=n)
    g = rng.normal(size=n)
    z = np.zeros(n)
    lr = 2e-3
    # first step, no decay, eps -> 0: r = sign(g), ||u|| = sqrt(n), so w' = w - lr ||w|| sign(g) / sqrt(n)
    w1, m1, v1 = O.lamb_step(w, g, z, z, 1, lr=lr, eps_a=1e-30, weight_decay=0.0)
    np.testing.assert_allclose(w1, w - lr * np.linalg.norm(w) * np.sign(g) / np.sqrt(n), rtol=1e-12, atol=1e-15)
    # the moments are Adam's
    _, ma, va = O.adam_step(w, g, z, z, 1)
    np.testing.assert_array_equal(m1, ma)
    np.testing.assert_array_equal(v1, va)
    # without decay every step moves the tensor by exactly lr ||w||, whatever the gradient's scale
    for scale in (1e-3, 1.0, 1e3):
        w2, _, _ = O.lamb_step(w1, scale * rng.normal(size=n), m1, v1, 2, lr=lr, eps_a=1e-30)
        np.testing.assert_allclose(np.linalg.norm(w2 - w1), lr * np.linalg.norm(w1), rtol=1e-10)
    # scaling the whole gradient history leaves the update unchanged (eps -> 0)
    wa, _, _ = O.lamb_step(w, g, z, z, 1, lr=lr, eps_a=1e-30, weight_decay=0.01)
    wb, _, _ = O.lamb_step(w, 50.0 * g, z, z, 1, lr=lr, eps_a=1e-30, weight_decay=0.01)
    np.testing.assert_allclose(wa, wb, rtol=1e-12)
    # a zero tensor has trust ratio 1: the step is Adam's
    wz, _, _ = O.lamb_step(z, g, z, z, 1, lr=lr, eps_a=1e-8)
    wad, _, _ = O.adam_step(z, g, z, z, 1, lr=lr, eps_a=1e-8)
    np.testing.assert_allclose(wz, wad, rtol=1e-14)
    # zero gradient and no decay: nothing moves
    w0, m0, v0 = O.lamb_step(w, z, z, z, 1, lr=lr)
    np.testing.assert_array_equal(w0, w)
    # decay alone (zero gradient): u = lambda w, trust = 1 / lambda, so w' = (1 - lr) w
    wd, _, _ = O.lamb_step(w, z, z, z, 1, lr=lr, weight_decay=0.1)
    np.testing.assert_allclose(wd, (1 - lr) * w, rtol=1e-12)


def test_bf16_exhaustive_round_trip_and_ties():
    bits = np.arange(65536, dtype=np.uint16)
    f = O.bf16_to_f32(bits)
    finite = np.isfinite(f)
    assert np.array_equal(O.bf16_bits(f[finite]), bits[finite])
    assert np.all(np.isnan(O.bf16_to_f32(O.bf16_bits(f[np.isnan(f)]))))
    # midpoints between neighbouring bf16 values go to the even pattern
    def f32(u):
        return np.array([u], np.uint32).view(np.float32)
    assert O.bf16_bits(f32(0x3F808000))[0] == 0x3F80      # 1 + 2^-8 : tie, lower is even
    assert O.bf16_bits(f32(0x3F818000))[0] == 0x3F82      # tie, upper is even
    assert O.bf16_bits(f32(0x3F808001))[0] == 0x3F81      # just above the tie
    assert O.bf16_bits(f32(0x3F807FFF))[0] == 0x3F80
    assert O.bf16_bits(f32(0x7F7FFFFF))[0] == 0x7F80      # rounds up to infinity
    x = np.random.default_rng(0).normal(size=1000).astype(np.float32)
    r = O.bf16_round(x)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_fp16_exhaustive_round_trip_ties_and_range():
    bits = np.arange(65536, dtype=np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(f)
    assert np.array_equal(O.fp16_bits(f[finite]), bits[finite])
    # layout: 1 sign, 5 exponent (bias 15), 10 fraction bits
    assert O.fp16_bits(np.float32(1.0)) == 0x3C00
    assert O.fp16_bits(np.float32(-2.0)) == 0xC000
    assert O.fp16_bits(np.float32(65504.0)) == 0x7BFF                # largest finite
    assert O.fp16_bits(np.float32(2.0 ** -14)) == 0x0400             # smallest normal
    assert O.fp16_bits(np.float32(2.0 ** -24)) == 0x0001             # smallest subnormal
    # ties go to the even pattern; just above a tie goes up
    assert O.fp16_bits(np.float32(1.0 + 2.0 ** -11)) == 0x3C00
    assert O.fp16_bits(np.float32(1.0 + 3 * 2.0 ** -11)) == 0x3C02
    assert O.fp16_bits(np.float32(1.0 + 2.0 ** -11 + 2.0 ** -20)) == 0x3C01
    assert O.fp16_bits(np.float32(2.0 ** -25)) == 0x0000             # tie between 0 and the smallest subnormal
    assert O.fp16_bits(np.float32(3 * 2.0 ** -25)) == 0x0002
    # overflow: 65520 is the tie between 65504 and 2^16 and rounds to infinity
    assert O.fp16_bits(np.float32(65519.0)) == 0x7BFF
    assert O.fp16_bits(np.float32(65520.0)) == 0x7C00
    assert np.isinf(O.fp16_round(np.float32(1e6)))
    x = np.float32(0.1)
    assert abs(float(O.fp16_round(x)) - 0.1) <= 0.1 * 2.0 ** -11


# ----------------------------------------------------------------------------- sequence-classification head
def _cls_params(H, C, rng):
    return {"Wp": rng.normal(size=(H, H)) * 0.3, "bp": rng.normal(size=H) * 0.1,
            "Wc": rng.normal(size=(H, C)) * 0.3, "bc": rng.normal(size=C) * 0.1}


def test_cls_head_gradients_by_finite_differences_and_closed_forms():
    H, S, C, n = 6, 3, 4, 5
    rng = np.random.default_rng(11)
    c = _cls_params(H, C, rng)
    x = rng.normal(size=(n, S, H))
    lab = np.array([1, -1, 3, 0, 2])
    N = 7                                                   # labelled count of a larger minibatch
    loss, dx, g = O.cls_head_loss(x, lab, c, N)
    f = lambda: O.cls_head_loss(x, lab, c, N)[0]
    h = 1e-6
    for name, arr, grad in [("x", x, dx)] + [(k, c[k], g[k]) for k in c]:
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h
            lp = f()
            arr[i] = old - h
            lm = f()
            arr[i] = old
            num[i] = (lp - lm) / (2 * h)
        assert np.linalg.norm(num - grad) / max(np.linalg.norm(num), 1e-30) < 1e-7, name
    # only the first token of a labelled sequence receives a gradient
    assert not dx[:, 1:, :].any() and not dx[1].any() and dx[0, 0].any()
    # the gradient of bc sums to zero (softmax rows minus one-hot rows), and shifting bc leaves the loss alone
    assert abs(g["bc"].sum()) < 1e-15
    c2 = dict(c, bc=c["bc"] + 3.7)
    assert abs(O.cls_head_loss(x, lab, c2, N)[0] - loss) < 1e-12
    # a zero classifier predicts uniformly: loss = (labelled here / N) ln C
    c0 = dict(c, Wc=np.zeros((H, C)), bc=np.zeros(C))
    assert abs(O.cls_head_loss(x, lab, c0, N)[0] - 4 / N * np.log(C)) < 1e-14
    # no labelled sequence: nothing
    l0, dx0, g0 = O.cls_head_loss(x, np.full(n, -1), c, N)
    assert l0 == 0.0 and not dx0.any() and not any(v.any() for v in g0.values())


def test_l2l_with_cls_head_equals_one_concatenated_minibatch():
    H, A, F, S, V, L, C = 8, 2, 16, 4, 11, 2, 3
    rng = np.random.default_rng(12)
    emb, layers = tiny_model(H, A, F, S, V, L, rng)
    cls = _cls_params(H, C, rng)
    tok = rng.integers(0, V, size=(3, 2, S))                 # U = 3 micro-batches of 2 sequences
    lab = np.array([[0, 2], [-1, 1], [2, 2]])
    loss, gemb, gl, gcls = O.run_l2l_cls(emb, layers, cls, tok, lab, A, EPS)
    loss1, gemb1, gl1, gcls1 = O.run_l2l_cls(emb, layers, cls, tok.reshape(1, 6, S), lab.reshape(1, 6), A, EPS)
    assert abs(loss - loss1) < 1e-13
    for a, b in [(gemb, gemb1), (gcls, gcls1)] + list(zip(gl, gl1)):
        for k in a:
            assert np.allclose(a[k], b[k], rtol=1e-11, atol=1e-14), k
    assert not gemb["bv"].any()                               # the LM head is not in this graph


def test_error_measures_on_hand_values():
    # rel_l2 and max_rel are what every parity comparison rests on: values worked out by hand
    b = np.array([3.0, 4.0, 0.0, 0.0])                      # ||b|| = 5, max |b| = 4
    a = np.array([3.0, 4.0, 0.0, 1.0])                      # one entry off by 1
    assert O.rel_l2(a, b) == pytest.approx(1.0 / 5.0, rel=1e-15)
    assert O.max_rel(a, b) == pytest.approx(1.0 / 4.0, rel=1e-15)
    assert O.rel_l2(b, b) == 0.0 and O.max_rel(b, b) == 0.0
    assert O.rel_l2(2 * b, b) == pytest.approx(1.0) and O.max_rel(2 * b, b) == pytest.approx(1.0)
    assert O.rel_l2(-b, b) == pytest.approx(2.0)            # a sign flip is an error of 2, not 0
    # the measures are not symmetric: the second argument is the reference
    assert O.rel_l2(b, 2 * b) == pytest.approx(0.5) and O.max_rel(b, 2 * b) == pytest.approx(0.5)
    # zero reference: the absolute size of what was got
    assert O.rel_l2(a, np.zeros(4)) == pytest.approx(np.sqrt(26.0)) and O.max_rel(a, np.zeros(4)) == 4.0
    # shapes are flattened, dtypes widened
    assert O.rel_l2(a.reshape(2, 2).astype(np.float32), b.reshape(2, 2)) == pytest.approx(0.2)
    # what rel_l2 averages away max_rel keeps: 8 wrong rows of 32768 (each entry off by the typical size)
    rng = np.random.default_rng(0)
    ref = rng.normal(size=(32768, 16))
    got = ref.copy()
    got[:8] = 0.0
    assert O.rel_l2(got, ref) < 2e-2 < 0.2 < O.max_rel(got, ref)
    assert np.isnan(O.rel_l2(np.array([np.nan, 1.0]), np.array([1.0, 1.0])))      # a NaN never passes a "< tol" test


def test_layer_forward_against_nested_scalar_loops():
    # the whole encoder layer, every stage with non-zero weights (FFN included), written out element by element with
    # Python scalars and math.erf / math.exp: pins qkv split, head layout, softmax axis, both residuals, both
    # LayerNorms, GELU placement and every matrix orientation of encoder_layer_fwd and its cache
    import math
    n, S, H, A, F = 2, 3, 4, 2, 6
    d = H // A
    rng = np.random.default_rng(42)
    p = {"Wqkv": rng.normal(size=(H, 3 * H)) * 0.5, "bqkv": rng.normal(size=3 * H) * 0.3, "Wo": rng.normal(size=(H, H)) * 0.5,
         "bo": rng.normal(size=H) * 0.3, "g1": 1 + 0.2 * rng.normal(size=H), "be1": 0.2 * rng.normal(size=H),
         "W1": rng.normal(size=(H, F)) * 0.7, "b1": rng.normal(size=F) * 0.3, "W2": rng.normal(size=(F, H)) * 0.7,
         "b2": rng.normal(size=H) * 0.3, "g2": 1 + 0.2 * rng.normal(size=H), "be2": 0.2 * rng.normal(size=H)}
    X = rng.normal(size=(n, S, H))
    eps = 1e-5
    Y, cache = O.encoder_layer_fwd(X, p, A, eps)

    def ln(row, g, b):
        mu = sum(row) / len(row)
        var = sum((v - mu) ** 2 for v in row) / len(row)
        return [g[j] * (row[j] - mu) / math.sqrt(var + eps) + b[j] for j in range(len(row))]

    for q in range(n):
        qkv = [[sum(X[q, s, i] * p["Wqkv"][i, j] for i in range(H)) + p["bqkv"][j] for j in range(3 * H)] for s in range(S)]
        ctx = [[0.0] * H for _ in range(S)]
        for h in range(A):
            for s in range(S):
                sc = [sum(qkv[s][h * d + e] * qkv[t][H + h * d + e] for e in range(d)) / math.sqrt(d) for t in range(S)]
                m = max(sc)
                ex = [math.exp(v - m) for v in sc]
                den = sum(ex)
                for e in range(d):
                    ctx[s][h * d + e] = sum(ex[t] / den * qkv[t][2 * H + h * d + e] for t in range(S))
        for s in range(S):
            r1 = [X[q, s, j] + sum(ctx[s][i] * p["Wo"][i, j] for i in range(H)) + p["bo"][j] for j in range(H)]
            y1 = ln(r1, p["g1"], p["be1"])
            u1 = [sum(y1[i] * p["W1"][i, f] for i in range(H)) + p["b1"][f] for f in range(F)]
            ga = [0.5 * u * (1.0 + math.erf(u / math.sqrt(2.0))) for u in u1]
            r2 = [y1[j] + sum(ga[f] * p["W2"][f, j] for f in range(F)) + p["b2"][j] for j in range(H)]
            y = ln(r2, p["g2"], p["be2"])
            assert np.allclose(cache["Y1"][q, s], y1, rtol=1e-12, atol=1e-13)
            assert np.allclose(cache["U1"][q, s], u1, rtol=1e-12, atol=1e-13)
            assert np.allclose(cache["G"][q, s], ga, rtol=1e-12, atol=1e-13)
            assert np.allclose(cache["C"][q, s], ctx[s], rtol=1e-12, atol=1e-13)
            assert np.allclose(Y[q, s], y, rtol=1e-12, atol=1e-13)

