"""Benchmark of the L2L hot path on one MI355X: train samples/s of the BERT-Large-shaped workload
(24 layers, hidden 1024, 16 heads, FFN 4096, seq 128, vocab 30522; device batch 256 = 8 micro-batches
of 32; bf16 with fp32 accumulation; host EPS Adam), synthetic data, random-init weights.

One step = embedding -> 24 x (param stage, layer forward over all micro-batches) -> head + loss ->
24 x (param stage, layer backward with recompute, grad drain) -> embedding backward -> host Adam.
Prints one JSON line: metric, value (samples/s over the timed steps), unit, n_gpus, steps, warmup, ms_per_step, dtype,
data, config (workload and how the step went: device pipeline, exposed host optimizer time, overlap fractions, kernel
time by class, peak device bytes), roofline (the layer GEMMs against the dense bf16 MFMA peak, from HIP events around
every GEMM launch in a second set of steps) and cpu_baseline (the CPU oracle on a bounded sample of the workload)."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
# HBM bytes per layer-GEMM launch of the headline workload, from counters collected offline (see roofline.traffic_source)
HBM_TRAFFIC_PER_LAUNCH = 553.9e6


def cpu_baseline(w):
    """The CPU oracle, untuned, on a bounded sample of the same workload: one encoder layer's forward plus
    backward-with-recompute over micro-batches of the minibatch until about 10 s have passed (at least one),
    scaled to all micro-batches and layers."""
    import numpy as np
    import l2l_synth as S
    from oracle import l2l_oracle as O
    p = {k: O.bf16_round(v).astype(np.float64) for k, v in S.layer_params(w, 0).items()}
    X = S.activations(w).astype(np.float64)
    dY = S.output_grads(w).astype(np.float64)
    done, t0 = 0, time.perf_counter()
    while done < w.num_ubatches and (done == 0 or time.perf_counter() - t0 < 10.0):
        O.layer_l2l_fwd(X[done:done + 1], p, w.heads, 1e-12)
        O.layer_l2l_bwd(X[done:done + 1], dY[done:done + 1], p, w.heads, 1e-12)
        done += 1
    dt = time.perf_counter() - t0
    step_s = dt / done * w.num_ubatches * w.layers
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": w.num_ubatches * w.ubatch / step_s, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 encoder layer, forward + backward-with-recompute, {done} of {w.num_ubatches} micro-batches of "
                      f"{w.ubatch} sequences ({dt:.1f} s), scaled to {w.num_ubatches} micro-batches x {w.layers} layers; "
                      "embedding, head and Adam not included"}


def write_gemm_table(path, rows, w, steps, out):
    """The layer GEMMs of the instrumented steps by launch shape, as a markdown table."""
    H, F = w.hidden, w.ffn
    role = {(3 * H, H, 1): "QKV", (H, H, 9): "out-proj (+ residual)", (F, H, 3): "FFN1 (+ GELU)", (H, F, 9): "FFN2 (+ residual)",
            (F, H, 67): "FFN1 (+ GELU, keeps gelu')", (F, H, 128): "dU1 = dR2 W2^T * gelu'", (F, H, 160): "dU1 = dR2 W2^T * gelu' (+ db1 partial sums)",
            (F, H, 4): "dU1 = dR2 W2^T * gelu'", (F, H, 36): "dU1 = dR2 W2^T * gelu' (+ db1 partial sums)",
            (H, F, 8): "dY1 = dR2 + dU1 W1^T", (H, H, 0): "dC = dR1 Wo^T", (H, 3 * H, 8): "dX = dR1 + dQKV Wqkv^T"}
    lines = ["| GEMM | pass | M | N | K | layout (A, B) | launches / step | us / launch | TFLOP/s | of 2.5 PFLOP/s |", "|---|---|---|---|---|---|---|---|---|---|"]
    passes = ("forward", "recompute", "backward", "")
    tot_ms = tot_fl = 0.0
    for r in rows:
        if not r["launches"]:
            continue
        name = role.get((r["N"], r["K"], r["epi"]), "")
        if r["epi"] == 16:
            name = {(H, 3 * H): "dWqkv += X^T dQKV", (H, H): "dWo += C^T dR1", (H, F): "dW1 += Y1^T dU1", (F, H): "dW2 += G^T dR2"}.get((r["M"], r["N"]), "dW")
        fl = 2.0 * r["M"] * r["N"] * r["K"] * r["launches"]
        tf = fl / (r["ms"] * 1e-3) / 1e12
        tot_ms += r["ms"]
        tot_fl += fl
        lay = ("K-contiguous" if r["a_kc"] else "K-strided") + ", " + ("K-contiguous" if r["b_kc"] else "K-strided")
        lines.append(f"| {name} | {passes[r['pass']]} | {r['M']} | {r['N']} | {r['K']} | {lay} | {r['launches'] / steps:g} | {1e3 * r['ms'] / r['launches']:.1f} | {tf:.0f} | {tf / PEAK_BF16_TFLOPS:.3f} |")
    lines.append(f"| all | | | | | | {sum(r['launches'] for r in rows) / steps:g} | | {tot_fl / (tot_ms * 1e-3) / 1e12:.0f} | {tot_fl / (tot_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS:.3f} |")
    with open(path, "w") as f:
        f.write(f"Layer GEMMs by launch shape: HIP events around every GEMM launch on the compute stream, {steps} steps, no tracer attached.\n")
        f.write(f"Workload: {out['config']['workload']}; {out['ms_per_step']:.1f} ms per un-instrumented step.\n\n")
        f.write("\n".join(lines) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload index (2 = BERT-Large, the headline)")
    ap.add_argument("--group", type=int, default=0, help="micro-batches per kernel launch (0 = library default)")
    ap.add_argument("--stash", default="device", choices=["device", "host"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override depth (memory-vs-depth sweeps)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size dispatch for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--tail-adam", action="store_true",
                    help="run the host Adam after all gradients arrived instead of eagerly per layer during backward")
    ap.add_argument("--ubatches", type=int, default=0, help="override U, the number of micro-batches (sweeps of the paper's Tables 3 and 4)")
    ap.add_argument("--dtype", default="", choices=["", "bf16", "fp16", "fp32"],
                    help="override the workload's device dtype (fp16: the paper's CMP precision, with dynamic loss scaling)")
    ap.add_argument("--classes", type=int, default=0,
                    help="> 0: the sequence-classification head with this many classes (one synthetic label per sequence) instead of the LM head")
    ap.add_argument("--optimizer", default="adam", choices=["adam", "lamb"],
                    help="host optimizer (lamb: per-tensor trust ratio, learning rate 1e-3, weight decay 0.01 on matrices)")
    ap.add_argument("--no-ln-stats", action="store_true",
                    help="recompute the whole layer forward in the backward pass (l2l_layer_fwd / l2l_layer_bwd) instead of keeping "
                         "LayerNorm 2's row statistics and skipping the FFN2 product of the recompute")
    ap.add_argument("--stash-copy", default="rows", choices=["rows", "plain"],
                    help="host-stash mode: how the stash moves (rows: l2l_memcpy_rows_async, DMA engines; plain: torch copy_)")
    ap.add_argument("--serialize", action="store_true",
                    help="run every stage and drain alone, with the compute stream waiting for it (the execution Section 2.2.1's "
                         "cost model describes); a measuring switch: under a tracer it keeps kernels and copies apart")
    ap.add_argument("--gemm-table", default="", metavar="FILE",
                    help="write the layer GEMMs by launch shape (HIP-event durations of the instrumented steps: launches, "
                         "microseconds per launch, TFLOP/s) to FILE as a markdown table")
    ap.add_argument("--grad-dtype", default="fp32", choices=["fp32", "bf16", "fp16"],
                    help="format of the gradient drains over the host link (fp32 = the headline; 16-bit: rounded on the device, half the bytes)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    import l2l_synth as S
    from paper_2002_05645_amd.trainer import L2LTrainer

    w = S.WORKLOADS[a.config]
    full_depth = w.layers
    if a.config == 4 and not a.layers:
        # 453 M parameters per layer: fp32 master, two Adam moments, the shipping copy and the gradient landing buffer
        # are 18 bytes per parameter of host memory, 8.2 GB per layer, 390 GB at the workload's 48 layers: more than
        # a process may hold on these boxes.  The device side does not depend on depth (one resident layer, one
        # prefetch buffer), so the workload runs at a reduced depth that is said in config.workload.
        a.layers = 6
    if a.layers:
        w = w.scaled(layers=a.layers)
    if a.ubatches:
        w = w.scaled(num_ubatches=a.ubatches)
    if a.dtype:
        w = w.scaled(dtype=a.dtype)
    tr = L2LTrainer(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, vocab=w.vocab,
                    ubatch=w.ubatch, num_ubatches=w.num_ubatches, dtype=w.dtype, ubatch_group=a.group, stash=a.stash,
                    eager=not a.tail_adam, optimizer=a.optimizer, num_classes=a.classes, grad_dtype=a.grad_dtype, keep_ln_stats=not a.no_ln_stats, serialize=a.serialize, stash_copy=a.stash_copy,
                    **(dict(lr=1e-3, eps_a=1e-6, weight_decay=0.01) if a.optimizer == "lamb" else {}))
    if a.config == 4:
        # drawing 453 M normals per layer from the counter-based generator takes a minute per layer: layer 0 is drawn,
        # the others get each of its tensors rotated by a layer-dependent offset (same distribution, own memory)
        import numpy as np
        l0 = S.layer_params(w, 0)
        layer_list = [l0] + [{k: np.roll(v.reshape(-1), 7919 * l).reshape(v.shape) for k, v in l0.items()} for l in range(1, w.layers)]
    else:
        layer_list = [S.layer_params(w, l) for l in range(w.layers)]
    tr.load_params(S.embed_params(w), layer_list, S.cls_params(w, a.classes) if a.classes else None)
    del layer_list
    tok, lab = S.tokens_and_labels(w)
    if a.classes:
        lab = S.seq_labels(w, a.classes)
    tok, lab = torch.from_numpy(tok).cuda(), torch.from_numpy(lab).cuda()

    loss0 = None
    losses = []
    for _ in range(a.warmup):
        loss = tr.step(tok, lab)
        losses.append(loss)
        loss0 = loss if loss0 is None else loss0
    torch.cuda.synchronize()

    def run_steps(n):
        dev_s = adam_s = 0.0
        t0 = time.perf_counter()
        for _ in range(n):
            t1 = time.perf_counter()
            tr.device_pipeline(tok, lab)
            loss = tr.finish()
            t2 = time.perf_counter()
            tr.optimizer_step()
            t3 = time.perf_counter()
            dev_s += t2 - t1
            adam_s += t3 - t2
            losses.append(loss)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, dev_s, adam_s

    # timed region: K full steps, nothing instrumented
    torch.cuda.synchronize()
    total_s, dev_s, adam_s = run_steps(a.steps)
    loss = losses[-1]
    # the same K steps again with every layer-GEMM launch bracketed by HIP events on the compute stream
    # (the brackets cost a few percent of step time, which is why they stay out of the region above)
    tr.ctx.profile(2)
    prof_total_s, _, _ = run_steps(a.steps)
    prof = tr.ctx.profile_read()
    gemm_rows = tr.ctx.profile_gemm_table()
    tr.ctx.profile(0)
    # a few more steps with every kernel and every copy-stream operation bracketed: how much of the step has
    # a kernel running, and how much of the copy stream's work (stages, drains) runs under those kernels
    n_ov = min(3, a.steps)
    tr.ctx.profile(1)
    run_steps(n_ov)
    ov = tr.ctx.profile_overlap(merge_gap_ms=0.05)   # kernel-to-kernel launch gaps (<= 50 us) count as busy
    classes = tr.ctx.profile_read()
    tr.ctx.profile(0)
    kernel_ms = sum(v["ms"] for k, v in classes.items() if k != "copy") / n_ov

    samples = w.num_ubatches * w.ubatch
    ms_step = 1e3 * total_s / a.steps
    g = prof["gemm"]
    achieved = g["flops"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
    peak_mem = torch.cuda.max_memory_allocated() + tr.ctx.device_bytes()
    out = {
        # the headline workload carries the baseline's metric name; sweeps and the other workloads say what they are
        "metric": "train samples/sec, BERT-Large L2L batch 256" if (w.name == "bert-large" and samples == 256 and not a.serialize)
                  else f"train samples/sec, {w.name} L2L batch {samples}",
        "value": samples * a.steps / total_s,
        "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": {"bf16": "bf16", "fp16": "f16", "fp32": "f32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": f"{w.name}: L={w.layers} H={w.hidden} A={w.heads} F={w.ffn} S={w.seq} V={w.vocab} "
                               f"U={w.num_ubatches} x ub={w.ubatch}"
                               + (f" (reduced depth: {w.layers} of the workload's {full_depth} layers)" if w.layers < full_depth else ""),
                   "stash": a.stash, "ubatch_group": tr.ctx.cfg.ubatch_group,
                   "device_pipeline_samples_per_s": samples * a.steps / dev_s, "device_pipeline_ms": 1e3 * dev_s / a.steps,
                   "host_adam_exposed_ms": 1e3 * adam_s / a.steps, "eps": "tail" if a.tail_adam else "eager", "ln2_statistics_kept": bool(tr.keep_ln_stats), "transfers": "serialised" if a.serialize else "overlapped", "optimizer": a.optimizer, "head": f"classification, {a.classes} classes" if a.classes else "tied LM head", "loss_first": loss0, "loss_last": loss, "losses": [round(x, 4) for x in losses],
                   "peak_device_bytes": int(peak_mem), "ctx_device_bytes": int(tr.ctx.device_bytes()),
                   "instrumented_ms_per_step": 1e3 * prof_total_s / a.steps,
                   # sum of kernel durations over the un-instrumented device-pipeline time; and the fraction of the
                   # copy stream's busy time during which a compute kernel was running
                   "compute_busy_frac": kernel_ms / (1e3 * dev_s / a.steps),
                   "hidden_transfer_frac": ov["copy_hidden_ms"] / ov["copy_busy_ms"] if ov["copy_busy_ms"] > 0 else None,
                   # the brackets slow the host's enqueue, so the instrumented steps have idle gaps the timed steps do not
                   # have; in the timed steps at most (device pipeline - kernel time) of the copy work can be exposed:
                   "hidden_transfer_frac_timed_steps_at_least": max(0.0, 1.0 - max(0.0, 1e3 * dev_s / a.steps - kernel_ms)
                                                                    / (ov["copy_busy_ms"] / n_ov)) if ov["copy_busy_ms"] > 0 else None,
                   "copy_stream_busy_ms": ov["copy_busy_ms"] / n_ov,
                   # bytes moved by stages and drains per second of copy-stream busy time (beside the kernels)
                   "host_link_GBps_while_busy": classes["copy"]["bytes"] / (classes["copy"]["ms"] * 1e-3) / 1e9 if classes["copy"]["ms"] > 0 else None,
                   "host_link_bytes_per_step": classes["copy"]["bytes"] / n_ov,
                   "kernel_ms_by_class": {k: round(v["ms"] / n_ov, 3) for k, v in classes.items()}},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS,
                     # HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (profiles/bench_bert_large_gemm_hbm_traffic.md);
                     # measured on the headline workload only
                     "traffic": HBM_TRAFFIC_PER_LAUNCH if (a.config == 2 and not a.layers and not a.group and not a.ubatches and not a.dtype and not a.classes and a.grad_dtype == "fp32") else None,
                     "traffic_source": "offline: two rocprofv3 --pmc runs of this command (FETCH_SIZE, WRITE_SIZE), profiles/bench_bert_large_gemm_hbm_traffic.md; not measured in this run",
                     "kernel": "gemm_mfma_dlds_kernel / gemm_mfma_kernel: the layer's dense GEMMs (QKV, out-proj, FFN1, FFN2; forward, recompute, dX, dW)",
                     "gemm_ms_per_step": g["ms"] / a.steps, "launches_per_step": g["launches"] / a.steps,
                     "avg_launch_us": 1e3 * g["ms"] / max(g["launches"], 1),
                     "flops_per_launch": g["flops"] / max(g["launches"], 1)},
    }
    if a.gemm_table:
        write_gemm_table(a.gemm_table, gemm_rows, w, a.steps, out)
    if a.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    tr.close()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
