"""GPU check of the paper's transfer-overhead cost model (Section 2.2.1, Eq. 4, in the reading that keeps the factor N
in every formula): with transfers and compute serialised a step takes N (4 u C + 2 X) plus what does not depend on the
depth N; with the double-buffered prefetch it approaches N (max(u C, X_fwd) + max(3 u C, X_bwd)).  C and X are
measured on their own (a layer's forward and backward-with-recompute over all micro-batches; a parameter stage; a
gradient drain) and compared with the per-layer cost of whole steps, taken as the difference between a 6-layer and a
2-layer model so that embedding and head drop out."""
import time

import numpy as np
import pytest
import torch

import l2l_synth as S
from paper_2002_05645_amd.trainer import L2LTrainer

pytestmark = pytest.mark.gpu


def _trainer(w, layers, **kw):
    tr = L2LTrainer(layers=layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab, ubatch=w.ubatch,
                    num_ubatches=w.num_ubatches, dtype=w.dtype, eps_threads=8, **kw)
    p0 = S.layer_params(w, 0)
    tr.load_params(S.embed_params(w), [p0] * layers)
    return tr


def _step_ms(tr, tok, lab, reps=5):
    best = 1e30
    for _ in range(reps + 1):                   # (the first repetition warms up)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tr.device_pipeline(tok, lab)
        tr.finish()
        best = min(best, 1e3 * (time.perf_counter() - t0))
    return best


def _event_ms(stream, fn, reps=5):
    best = 1e30
    for _ in range(reps + 1):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(stream)
        fn()
        b.record(stream)
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b))
    return best


def test_serialised_and_overlapped_steps_follow_the_cost_model():
    # BERT-Large widths with few rows per layer visit (U = 2 micro-batches of 8 sequences), so that a layer's transfer
    # time X is of the size of its compute time u C -- the regime the model is about
    w = S.WORKLOADS[2].scaled(ubatch=8, num_ubatches=2)
    tok, lab = S.tokens_and_labels(w)
    tok, lab = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()
    per_layer = {}
    for mode, kw in (("serial", dict(serialize=True)), ("overlap", dict())):
        t = {}
        for L in (2, 6):
            tr = _trainer(w, L, **kw)
            try:
                t[L] = _step_ms(tr, tok, lab)
                if mode == "serial" and L == 2:
                    # the pieces, each on its own with the other stream idle
                    c, e = tr.ctx, tr.eps
                    x, y, dy = tr.stash[0], tr.stash[1], tr.dy
                    rs = tr.rstd2[0]
                    c.param_stage(0, e.ship_ptr(1), 0)
                    c.sync()
                    uC_f = _event_ms(tr.compute, lambda: c.layer_fwd_stats(0, 0, x, y, rs))

                    def bwd():
                        c.layer_bwd_stats(0, 0, x, y, rs, dy)
                    def bwd_and_drain():
                        bwd()
                        c.grad_drain(0, tr._land_ptr(1))
                    bwd_and_drain()
                    c.sync()
                    uC_b = 1e30
                    for _ in range(5):
                        uC_b = min(uC_b, _event_ms(tr.compute, bwd, reps=0))
                        c.grad_drain(0, tr._land_ptr(1))
                        c.sync()
                    X_s = _event_ms(tr.copy, lambda: c.param_stage(0, e.ship_ptr(1), 0))
                    X_d = 1e30
                    for _ in range(5):
                        bwd()
                        c.sync()
                        X_d = min(X_d, _event_ms(tr.copy, lambda: c.grad_drain(0, tr._land_ptr(1)), reps=0))
            finally:
                tr.close()
        per_layer[mode] = (t[6] - t[2]) / 4.0
    model_serial = uC_f + uC_b + 2 * X_s + X_d                  # N (4 u C + 2 X) per layer: 4 u C = forward + backward-with-recompute
    model_overlap = max(uC_f, X_s) + max(uC_b, X_s + X_d)
    msg = (f"per layer: serialised {per_layer['serial']:.3f} ms (model {model_serial:.3f}), overlapped {per_layer['overlap']:.3f} ms "
           f"(model {model_overlap:.3f}); u C forward {uC_f:.3f}, backward with recompute {uC_b:.3f}, stage {X_s:.3f}, drain {X_d:.3f}")
    print(msg)
    import os
    d = os.environ.get("L2L_TEST_REPORT_DIR", "")
    if d and os.path.isdir(d):
        with open(os.path.join(d, "timing_model.txt"), "a") as f:
            f.write(msg + "\n")
    assert abs(per_layer["serial"] - model_serial) <= 0.15 * model_serial, msg
    assert per_layer["overlap"] <= 1.15 * model_overlap, msg
    assert per_layer["overlap"] < per_layer["serial"], msg
