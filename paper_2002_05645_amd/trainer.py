"""Step driver of L2L relay execution (Algorithm 2) above the C ABI.

PyTorch supplies device memory and the two streams; every arithmetic step runs inside libl2l.so.
The host EPS (block 0 = embedding/head block, block 1 + l = encoder layer l) keeps fp32 master
weights and Adam state, ships the configured dtype, and receives fp32 gradients (Section 2.1, 2.3).
"""
from __future__ import annotations

import queue
import threading

import numpy as np
import torch

from . import binding as B


def pack(layout, total, tensors) -> np.ndarray:
    """dict of arrays -> flat fp32 packed block (padding zero)."""
    flat = np.zeros(total, np.float32)
    for k, (off, n) in layout.items():
        a = np.asarray(tensors[k], np.float32).reshape(-1)
        assert a.size == n, (k, a.size, n)
        flat[off:off + n] = a
    return flat


def unpack(layout, shapes, flat) -> dict:
    return {k: np.array(flat[off:off + n]).reshape(shapes[k]) for k, (off, n) in layout.items()}


class LossScaler:
    """Dynamic loss scale of mixed-precision training (Section 2.3 leaves the policy open; this is the usual one):
    an overflow (a non-finite gradient) skips the update and halves the scale; `growth_interval` consecutive good
    steps double it.  static=True keeps the scale fixed and only reports overflows."""

    def __init__(self, scale=2.0 ** 15, growth_interval=1000, static=False, min_scale=1.0, max_scale=2.0 ** 24):
        self.scale, self.growth_interval, self.static = float(scale), int(growth_interval), bool(static)
        self.min_scale, self.max_scale = float(min_scale), float(max_scale)
        self.good_steps = 0
        self.skipped = 0

    def update(self, overflow: bool) -> bool:
        """Call once per step with whether the gradients overflowed; returns whether to apply the update."""
        if overflow:
            self.skipped += 1
            self.good_steps = 0
            if not self.static:
                self.scale = max(self.min_scale, self.scale / 2.0)
            return False
        self.good_steps += 1
        if not self.static and self.good_steps >= self.growth_interval:
            self.scale = min(self.max_scale, self.scale * 2.0)
            self.good_steps = 0
        return True


class L2LTrainer:
    def __init__(self, *, layers, hidden, heads, ffn, seq, vocab, ubatch, num_ubatches, dtype="bf16",
                 ln_eps=1e-12, lr=1e-4, beta1=0.9, beta2=0.999, eps_a=1e-8, ubatch_group=0,
                 eps_threads=0, stash="device", device="cuda:0", eager=False, optimizer="adam", weight_decay=0.0,
                 copy_cus=0, run_ahead=2, loss_scale=None, dynamic_loss_scale=True, scale_growth_interval=1000,
                 num_classes=0, tail_parts=8, grad_dtype="fp32", keep_ln_stats=True, serialize=False, stash_copy="rows"):
        assert stash in ("device", "host")
        assert optimizer in ("adam", "lamb")
        self.optimizer = optimizer
        # Backward: the host enqueues at most this many layers ahead of the device (0: no limit).  Measured on
        # this runtime: gradient drains that are queued far ahead of their turn are carried out by a copy path
        # that moves 12.5 GB/s instead of 20 .. 54 GB/s, which makes deep models copy-bound.
        self.run_ahead = int(run_ahead)
        # serialize: every stage and drain runs alone, with the compute stream idle, and the compute stream waits for
        # it -- the execution that Section 2.2.1's cost model N (4 u C + 2 X) describes (no overlap of transfers and
        # compute).  A measuring switch: results are the same, only the streams are joined around each transfer.
        self.serialize = bool(serialize)
        # stash traffic of the host-stash mode: "rows" = l2l_memcpy_rows_async (a DMA engine in both directions),
        # "plain" = torch's copy_ (device to host by the runtime's copy kernel)
        assert stash_copy in ("rows", "plain")
        self.stash_copy = stash_copy
        self.L, self.H, self.S, self.V = layers, hidden, seq, vocab
        self.U, self.ub = num_ubatches, ubatch
        self.dtype = dtype
        self.hp = dict(lr=lr, beta1=beta1, beta2=beta2, eps_a=eps_a)
        self.stash_mode = stash
        self.device = torch.device(device)
        self.cfg = B.make_config(hidden, heads, ffn, seq, ubatch, num_ubatches, dtype, ln_eps, vocab, ubatch_group)
        if B.lib().l2l_config_check(self.cfg) != B.L2L_OK:
            raise ValueError("unsupported L2L configuration")
        self.layer_layout = B.layer_layout(self.cfg)
        self.embed_layout = B.embed_layout(self.cfg)
        self.layer_elems = B.lib().l2l_layer_packed_elems(self.cfg)
        self.embed_elems = B.lib().l2l_embed_packed_elems(self.cfg)
        # num_classes > 0: the sequence-classification head (one class label per sequence) replaces the tied LM head;
        # its parameters are one more EPS block, after the layers'
        self.num_classes = int(num_classes)
        blocks = [self.embed_elems] + [self.layer_elems] * layers
        if self.num_classes:
            self.cls_layout = B.cls_layout(self.cfg, self.num_classes)
            self.cls_elems = B.lib().l2l_cls_packed_elems(self.cfg, self.num_classes)
            blocks.append(self.cls_elems)
        self.eps = B.EPS(blocks, dtype, eps_threads)
        if optimizer == "lamb":
            # LAMB (Table 1's optimizer) works tensor by tensor: the tensors of a block, in packing order, with
            # biases and LayerNorm parameters (everything that is not a matrix) exempt from weight decay
            self.hp["weight_decay"] = weight_decay
            def segs(layout, shapes):
                names = sorted(layout, key=lambda k: layout[k][0])
                return ([(layout[k][0], layout[k][0] + layout[k][1]) for k in names],
                        [1.0 if len(shapes[k]) == 2 else 0.0 for k in names])
            self._segs = {True: segs(self.embed_layout, self.embed_shapes()), False: segs(self.layer_layout, self.layer_shapes())}
            if self.num_classes:
                self._segs["cls"] = segs(self.cls_layout, self.cls_shapes())
        torch.cuda.set_device(self.device)
        self.compute = torch.cuda.Stream(device=self.device)
        self._copy_handle = None
        if copy_cus > 0:
            # the runtime's copy kernels (stages, drains, stash traffic) confined to copy_cus of every 32 CUs
            self._copy_handle = B.stream_create_cu_masked(copy_cus)
            self.copy = torch.cuda.ExternalStream(self._copy_handle, device=self.device)
        else:
            self.copy = torch.cuda.Stream(device=self.device)
        self.ctx = B.Context(self.cfg, self.compute.cuda_stream, self.copy.cuda_stream)
        tdt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[dtype]
        # Loss scaling: on by default for fp16 (2^15, dynamic), off otherwise.  The eager per-layer update commits a
        # layer before the rest of the step's gradients are known, so it cannot skip a step: there the scale is static
        # and an overflow raises.
        if loss_scale is None:
            loss_scale = 2.0 ** 15 if dtype == "fp16" else 1.0
        self.scaler = LossScaler(loss_scale, scale_growth_interval, static=eager or not dynamic_loss_scale or loss_scale == 1.0)
        self.ctx.set_loss_scale(self.scaler.scale)
        # Gradients accumulate in fp32 on the device; grad_dtype is the format in which they cross the host link
        # (Section 2.3 sends 16-bit values): "fp32", or "bf16" / "fp16" = rounded on the device, half the drain
        # traffic, widened into the EPS's fp32 gradient buffers before the optimizer reads them.
        assert grad_dtype in ("fp32", "bf16", "fp16")
        self.grad_dtype = grad_dtype
        if grad_dtype != "fp32":
            self.eps.enable_grad16()
            self.ctx.set_drain_dtype(grad_dtype)
        # plain Adam on unscaled gradients reads the 16-bit landing buffer directly; LAMB and the loss-scale check work
        # on the fp32 gradient buffers, which are filled from it first
        self._adam_from16 = grad_dtype != "fp32" and optimizer == "adam" and self.scaler.scale == 1.0 and self.scaler.static
        shape = (num_ubatches, ubatch, seq, hidden)
        # keep_ln_stats: the forward pass keeps LayerNorm 2's 1 / sigma per token (4 bytes against the stash's 2 H), and
        # the backward pass takes that LayerNorm's normalised input back out of the stashed layer output instead of
        # recomputing the FFN2 product (l2l_layer_fwd_stats / l2l_layer_bwd_stats).  Only where the library has the
        # one-pass LayerNorm backward (H <= 2048); per layer only while no |g2| is small (see _stats_ok).
        self.keep_ln_stats = bool(keep_ln_stats) and hidden % 8 == 0 and hidden <= 2048
        # host stash: transit slots on the device; with keep_ln_stats the backward pass of layer l reads the inputs of
        # layers l and l + 1 while layer l - 1's is on its way in, hence three
        self.nslot = (3 if self.keep_ln_stats else 2) if stash == "host" else layers + 1
        self.stash = [torch.empty(shape, dtype=tdt, device=self.device) for _ in range(self.nslot)]
        if self.keep_ln_stats:
            self.rstd2 = torch.empty((layers, num_ubatches * ubatch * seq), dtype=torch.float32, device=self.device)
        self._stats_ok = [False] * layers
        if stash == "host":
            self.host_stash = [torch.empty(shape, dtype=tdt, pin_memory=True) for _ in range(layers + 1)]
            self.stash_stream = torch.cuda.Stream(device=self.device)
            self.stash_ev = [torch.cuda.Event() for _ in range(self.nslot)]
            self.stash_free = [torch.cuda.Event() for _ in range(self.nslot)]
        self.dy = torch.empty(shape, dtype=tdt, device=self.device)
        self.loss_dev = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.t = 0
        # eager EPS (Section 2.1 "reduces ... eagerly", Section 4.1): a host thread runs Adam on a block as
        # soon as its gradients have landed, while the device is still busy with the layers below it
        self.eager = eager
        self._landed = [torch.cuda.Event() for _ in range(layers + 2)]
        self._bwd_done = [torch.cuda.Event() for _ in range(layers)]
        self._fwd_done = [torch.cuda.Event() for _ in range(layers)]
        self._work = queue.Queue()
        self._worker_error = None
        self._worker = None
        # The embedding block is the last to be updated in a step and the first needed in the next, so its drain, its
        # Adam and its next stage are exposed.  With eager Adam they run as a pipeline over `tail_parts` pieces of the
        # block: piece k is updated while piece k + 1 is still on its way to the host, and shipped back while piece
        # k + 1 is being updated.  (LAMB needs whole tensors for its norms and keeps the one-piece path.  A loss scale is
        # static in eager mode, so its unscale-and-check runs piece by piece as well.)
        self._parts = []
        self._prestaged = False
        if eager and optimizer == "adam" and tail_parts > 1:
            step = -(-self.embed_elems // tail_parts)
            step = -(-step // 256) * 256     # (whole kilobytes of fp32)
            self._parts = [(a, min(step, self.embed_elems - a)) for a in range(0, self.embed_elems, step)]
            self._part_landed = [torch.cuda.Event() for _ in self._parts]
            self._part_done = [threading.Event() for _ in self._parts]
        if eager:
            self._worker = threading.Thread(target=self._eager_loop, daemon=True)
            self._worker.start()

    # ---- parameters -------------------------------------------------------------------------------
    def load_params(self, emb: dict, layers: list, cls: dict = None):
        self._prestaged = False
        self.eps.master(0)[:] = pack(self.embed_layout, self.embed_elems, emb)
        for l, p in enumerate(layers):
            self.eps.master(1 + l)[:] = pack(self.layer_layout, self.layer_elems, p)
        if self.num_classes:
            self.eps.master(1 + self.L)[:] = pack(self.cls_layout, self.cls_elems, cls)
        self.eps.refresh_ship()

    def cls_shapes(self):
        return {"Wp": (self.H, self.H), "bp": (self.H,), "Wc": (self.H, self.num_classes), "bc": (self.num_classes,)}

    def cls_grads(self):
        if self._adam_from16:
            self.eps.grad_widen(1 + self.L, 1 + self.L, self.grad_dtype)
        return unpack(self.cls_layout, self.cls_shapes(), self.eps.grad(1 + self.L))

    def cls_master(self):
        return unpack(self.cls_layout, self.cls_shapes(), self.eps.master(1 + self.L))

    def layer_shapes(self):
        H, F = self.cfg.hidden, self.cfg.ffn
        return {"Wqkv": (H, 3 * H), "bqkv": (3 * H,), "Wo": (H, H), "bo": (H,), "g1": (H,), "be1": (H,),
                "W1": (H, F), "b1": (F,), "W2": (F, H), "b2": (H,), "g2": (H,), "be2": (H,)}

    def embed_shapes(self):
        return {"E": (self.V, self.H), "P": (self.S, self.H), "ge": (self.H,), "be": (self.H,), "bv": (self.V,)}

    def grads(self):
        """(embedding-block grads, per-layer grads) as dicts, from the EPS landing buffers."""
        if self._adam_from16:                 # the optimizer read the 16-bit buffers; widen them for the caller
            self.eps.grad_widen(0, self._last_block(), self.grad_dtype)
        ge = unpack(self.embed_layout, self.embed_shapes(), self.eps.grad(0))
        gl = [unpack(self.layer_layout, self.layer_shapes(), self.eps.grad(1 + l)) for l in range(self.L)]
        return ge, gl

    def master_params(self):
        e = unpack(self.embed_layout, self.embed_shapes(), self.eps.master(0))
        ls = [unpack(self.layer_layout, self.layer_shapes(), self.eps.master(1 + l)) for l in range(self.L)]
        return e, ls

    # ---- one step -----------------------------------------------------------------------------------
    def _land_ptr(self, block):
        """where a block's drain writes: the fp32 gradient buffer, or the 16-bit landing buffer"""
        return self.eps.grad_ptr(block) if self.grad_dtype == "fp32" else self.eps.grad16_ptr(block)

    def _stash_slot(self, l):
        return self.stash[l % self.nslot]

    def _stage(self, layer, block, slot):
        if self.serialize:
            self.copy.wait_stream(self.compute)
        self.ctx.param_stage(layer, self.eps.ship_ptr(block), slot)
        if self.serialize:
            self.compute.wait_stream(self.copy)

    def _drain(self, layer, block):
        if self.serialize:
            self.copy.wait_stream(self.compute)
        self.ctx.grad_drain(layer, self._land_ptr(block))
        if self.serialize:
            self.compute.wait_stream(self.copy)

    def _check_ln_gains(self):
        """per layer: whether xhat = (y - be2) / g2 is safe to take from the stashed output (from the master weights)"""
        if not self.keep_ln_stats:
            return
        o_g, n = self.layer_layout["g2"]
        o_b, _ = self.layer_layout["be2"]
        for l in range(self.L):
            m = self.eps.master(1 + l)
            g, b = np.abs(m[o_g:o_g + n]), np.abs(m[o_b:o_b + n])
            self._stats_ok[l] = bool(g.min() >= 1.0 / 64.0 and (b <= 8.0 * g).all())

    def device_pipeline(self, tokens: torch.Tensor, labels: torch.Tensor):
        """Stage -> forward over layers -> head -> backward over layers -> drain.  Asynchronous:
        call finish() (or read the loss) to wait.  tokens / labels: int32 device tensors [U, ub, S]."""
        c, e, L = self.ctx, self.eps, self.L
        host_mode = self.stash_mode == "host"
        self._check_ln_gains()
        if self._prestaged:          # the previous step's optimizer shipped the block (and layer 0) already
            self._prestaged = False
        else:
            c.embed_stage(e.ship_ptr(0))
            c.param_stage(0, e.ship_ptr(1), 0)
        c.embed_fwd(tokens, self._stash_slot(0))
        if host_mode:
            self._offload(0)
        for l in range(L):
            if l + 1 < L:
                self._stage(l + 1, 2 + l, (l + 1) % 2)
            if host_mode:
                self.compute.wait_event(self.stash_free[(l + 1) % self.nslot])
                if self.run_ahead and l >= self.run_ahead:     # the stash offloads are device-to-host copies too
                    self._fwd_done[l - self.run_ahead].synchronize()
            if self.keep_ln_stats:
                c.layer_fwd_stats(l, l % 2, self._stash_slot(l), self._stash_slot(l + 1), self.rstd2[l])
            else:
                c.layer_fwd(l, l % 2, self._stash_slot(l), self._stash_slot(l + 1))
            if host_mode:
                self._fwd_done[l].record(self.compute)
                self._offload(l + 1)
        if self.num_classes:                 # labels: int32 [U, ub], one class per sequence
            c.cls_stage(e.ship_ptr(1 + L), self.num_classes)
            c.cls_head_loss(self._stash_slot(L), labels, self.dy, self.loss_dev)
            c.cls_grad_drain(self._land_ptr(1 + L))
            self._after_drain(1 + L)
        else:
            c.head_loss(self._stash_slot(L), labels, self.dy, self.loss_dev)
        if host_mode:
            # the head is the consumer of the transit slot that holds layer L - 1's output: the reload of
            # layer L - 2's input into that slot must wait for it
            self.stash_free[L % self.nslot].record(self.compute)
        for l in reversed(range(L)):
            if l - 1 >= 0:
                self._stage(l - 1, l, (l - 1) % 2)
            if host_mode and l < L - 1:      # (layer L - 1's input is still in its slot from the forward pass)
                self._reload(l)
            if self.run_ahead and l + self.run_ahead < L:
                self._bwd_done[l + self.run_ahead].synchronize()
            if self._stats_ok[l]:
                c.layer_bwd_stats(l, l % 2, self._stash_slot(l), self._stash_slot(l + 1), self.rstd2[l], self.dy)
            else:
                c.layer_bwd(l, l % 2, self._stash_slot(l), self.dy)
            self._bwd_done[l].record(self.compute)
            if host_mode:
                if self.keep_ln_stats:
                    # three slots: layer l + 1's input, read above as layer l's output, is done with; layer l's own
                    # input stays for layer l - 1's backward
                    self.stash_free[(l + 1) % self.nslot].record(self.compute)
                    if l == 0:
                        self.stash_free[0].record(self.compute)
                else:
                    self.stash_free[l % self.nslot].record(self.compute)
            self._drain(l, 1 + l)
            self._after_drain(1 + l)
        c.embed_bwd(tokens, self.dy)
        if self._parts:
            for k, (first, count) in enumerate(self._parts):
                c.embed_grad_drain_part(self._land_ptr(0), first, count)
                self._part_landed[k].record(self.copy)
                self._part_done[k].clear()
                self._work.put(("part", k, self.t + 1))
        else:
            c.embed_grad_drain(self._land_ptr(0))
            self._after_drain(0)

    def _eps_update(self, first, last, t, unscale=True):
        if self._adam_from16:
            for b in range(first, last + 1):
                self.eps.adam_step_range16(b, 0, self.eps.elems[b], t, self.grad_dtype, **self.hp)
            return
        if self.grad_dtype != "fp32" and unscale:       # (the tail loop has widened already, before its overflow check)
            self.eps.grad_widen(first, last, self.grad_dtype)
        if unscale and self.scaler.scale != 1.0:
            if self.eps.grad_unscale(first, last, 1.0 / self.scaler.scale):
                raise FloatingPointError(f"gradient overflow in blocks {first}..{last} at loss scale {self.scaler.scale}")
        if self.optimizer == "adam":
            self.eps.adam_step(first, last, t, **self.hp)
            return
        if first == 0:                        # the embedding block has its own tensors
            seg, mask = self._segs[True]
            self.eps.lamb_step(0, 0, t, seg, decay_mask=mask, **self.hp)
            first = 1
        if self.num_classes and last == self.L + 1:      # the classification head's block has its own tensors too
            seg, mask = self._segs["cls"]
            self.eps.lamb_step(last, last, t, seg, decay_mask=mask, **self.hp)
            last -= 1
        if first <= last:
            seg, mask = self._segs[False]
            self.eps.lamb_step(first, last, t, seg, decay_mask=mask, **self.hp)

    def _last_block(self):
        return self.L + 1 if self.num_classes else self.L

    def _after_drain(self, block):
        if self.eager:
            self._landed[block].record(self.copy)
            self._work.put((block, self.t + 1))

    def _eager_loop(self):
        while True:
            item = self._work.get()
            if item is None:
                return
            try:
                if item[0] == "part":     # one piece of the embedding block
                    _, k, t = item
                    first, count = self._parts[k]
                    self._part_landed[k].synchronize()
                    if self._adam_from16:
                        self.eps.adam_step_range16(0, first, count, t, self.grad_dtype, **self.hp)
                    else:
                        if self.grad_dtype != "fp32":
                            self.eps.grad_widen_range(0, first, count, self.grad_dtype)
                        if self.scaler.scale != 1.0 and self.eps.grad_unscale_range(0, first, count, 1.0 / self.scaler.scale):
                            raise FloatingPointError(f"gradient overflow in the embedding block at loss scale {self.scaler.scale}")
                        self.eps.adam_step_range(0, first, count, t, **self.hp)
                else:
                    block, t = item
                    self._landed[block].synchronize()
                    self._eps_update(block, block, t)
            except Exception as ex:       # surfaced by optimizer_step
                self._worker_error = ex
            finally:
                if item[0] == "part":
                    self._part_done[item[1]].set()
                self._work.task_done()

    def _offload(self, l):
        """device stash slot -> pinned host after the producing kernels, on a stream of its own: the stash traffic
        then runs beside the parameter stages and gradient drains of the copy stream (the host link is full duplex)."""
        k = l % self.nslot
        ev = self.stash_ev[k]
        ev.record(self.compute)
        self.stash_stream.wait_event(ev)
        with torch.cuda.stream(self.stash_stream):
            if self.stash_copy == "rows":
                B.memcpy_rows_async(self.host_stash[l], self.stash[k], self.stash[k].numel() * self.stash[k].element_size(), True,
                                    self.stash_stream.cuda_stream)
            else:
                self.host_stash[l].copy_(self.stash[k], non_blocking=True)
            self.stash_free[k].record(self.stash_stream)

    def _reload(self, l):
        """pinned host -> device stash slot before layer l's backward (layer L's input is not needed)."""
        k = l % self.nslot
        self.stash_stream.wait_event(self.stash_free[k])
        with torch.cuda.stream(self.stash_stream):
            if self.stash_copy == "rows":
                B.memcpy_rows_async(self.stash[k], self.host_stash[l], self.stash[k].numel() * self.stash[k].element_size(), False,
                                    self.stash_stream.cuda_stream)
            else:
                self.stash[k].copy_(self.host_stash[l], non_blocking=True)
            ev = self.stash_ev[k]
            ev.record(self.stash_stream)
        self.compute.wait_event(ev)

    def finish(self) -> float:
        self.ctx.sync()
        if self.stash_mode == "host":
            self.stash_stream.synchronize()
        return float(self.loss_dev.item())

    def optimizer_step(self):
        """EPS Adam over every block, after all gradients have landed (Algorithm 2's tail loop)."""
        if self.eager:
            if self._parts:               # ship each piece of the embedding block back as soon as it is updated
                for k, (first, count) in enumerate(self._parts):
                    self._part_done[k].wait()
                    if self._worker_error is None:
                        if k == 0:        # the worker takes blocks in order: layer 0's update is complete as well
                            self.ctx.param_stage(0, self.eps.ship_ptr(1), 0)
                        self.ctx.embed_stage_part(self.eps.ship_ptr(0), first, count)
                self._prestaged = self._worker_error is None
            self._work.join()             # every block was queued by device_pipeline; wait for the stragglers
            if self._worker_error is not None:
                # Blocks that were updated before the failure keep their update (an eager update cannot be taken
                # back) while t is not advanced: after an overflow the caller lowers loss_scale and reloads the
                # parameters, or goes on knowing that those blocks are one step ahead.
                err, self._worker_error = self._worker_error, None
                self._prestaged = False
                raise err
            self.t += 1
            return
        if self.grad_dtype != "fp32" and not self._adam_from16:
            self.eps.grad_widen(0, self._last_block(), self.grad_dtype)
        if self.scaler.scale != 1.0:
            overflow = self.eps.grad_unscale(0, self._last_block(), 1.0 / self.scaler.scale)
            if self.scaler.static and overflow:
                raise FloatingPointError(f"gradient overflow at loss scale {self.scaler.scale}")
            apply = self.scaler.update(overflow)
            self.ctx.set_loss_scale(self.scaler.scale)
            if not apply:
                return                    # step skipped: weights, moments and t unchanged
        self.t += 1
        self._eps_update(0, self._last_block(), self.t, unscale=False)

    def step(self, tokens, labels) -> float:
        self.device_pipeline(tokens, labels)
        loss = self.finish()
        self.optimizer_step()
        return loss

    def close(self):
        if self._worker is not None:
            self._work.put(None)
            self._worker.join()
            self._worker = None
        self.ctx.close()
        self.eps.close()
        if self._copy_handle is not None:
            torch.cuda.synchronize(self.device)
            B.stream_destroy(self._copy_handle)
            self._copy_handle = None
