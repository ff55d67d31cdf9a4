"""Seeded synthetic inputs for the L2L relay-execution workloads.

This module only draws numbers: token ids, labels, and N(0, sigma) parameter
values, from a counter-based generator (splitmix64 finaliser over a per-tensor
stream id and an element counter).  It contains none of the method's
arithmetic -- no layer math, no rounding to reduced precision, no optimizer --
so that the CPU oracle's tests and the GPU path's tests can both draw the very
same inputs from it without sharing any code of the method itself.

Workloads stand in for the paper's GLUE fine-tuning runs of BERT-Large
(Section 3.1, Table 1): same tensor shapes, random token ids, random labels.
"""
from __future__ import annotations

import dataclasses
import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def raw_u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit draws; element i depends only on (seed, stream, offset + i)."""
    with np.errstate(over="ignore"):
        base = _mix(np.uint64(seed) * _GOLDEN + np.uint64(stream))
        ctr = np.arange(offset, offset + n, dtype=np.uint64)
        return _mix(base + (ctr + np.uint64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """float64 uniforms in [0, 1) with 53 random bits."""
    return (raw_u64(seed, stream, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(seed: int, stream: int, n: int) -> np.ndarray:
    """float64 standard normals by Box-Muller on counter pairs (2i, 2i+1)."""
    u = uniform01(seed, stream, 2 * n)
    u1 = 1.0 - u[0::2]          # (0, 1]
    u2 = u[1::2]
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def integers(seed: int, stream: int, n: int, high: int) -> np.ndarray:
    """int64 draws in [0, high)."""
    return (raw_u64(seed, stream, n) % np.uint64(high)).astype(np.int64)


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one synthetic L2L training workload."""
    name: str
    layers: int      # L
    hidden: int      # H
    heads: int       # A
    ffn: int         # F
    seq: int         # S
    vocab: int       # V
    ubatch: int      # ub, sequences per micro-batch
    num_ubatches: int  # U
    dtype: str       # "fp32" | "bf16"
    label_prob: float  # probability that a position carries a label
    seed: int

    @property
    def tokens_per_ubatch(self) -> int:
        return self.ubatch * self.seq

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five named workloads (index = configuration number).
WORKLOADS = [
    Workload("tiny", 2, 128, 2, 512, 64, 1000, 4, 4, "fp32", 1.0, 1234),
    Workload("bert-base", 12, 768, 12, 3072, 128, 30522, 16, 8, "bf16", 0.15, 1235),
    Workload("bert-large", 24, 1024, 16, 4096, 128, 30522, 32, 8, "bf16", 0.15, 1236),
    Workload("bert-large-s512", 24, 1024, 16, 4096, 512, 30522, 4, 16, "bf16", 0.15, 1237),
    Workload("deep-wide", 48, 6144, 48, 24576, 128, 30522, 8, 8, "bf16", 0.15, 1238),
]

# stream ids: one per tensor kind; layer tensors add 64 * (layer + 1)
_ST_TOKENS, _ST_LABEL_MASK, _ST_LABEL_VAL = 1, 2, 3
_ST_EMB = {"E": 10, "P": 11, "ge": 12, "be": 13, "bv": 14}
_ST_LAYER = {"Wqkv": 0, "bqkv": 1, "Wo": 2, "bo": 3, "g1": 4, "be1": 5,
             "W1": 6, "b1": 7, "W2": 8, "b2": 9, "g2": 10, "be2": 11}
_ST_ACT, _ST_DY = 40, 41

LAYER_TENSORS = tuple(_ST_LAYER)          # packed order of an encoder layer's parameters
EMBED_TENSORS = ("E", "P", "ge", "be", "bv")


def layer_shapes(w: Workload) -> dict:
    H, F = w.hidden, w.ffn
    return {"Wqkv": (H, 3 * H), "bqkv": (3 * H,), "Wo": (H, H), "bo": (H,),
            "g1": (H,), "be1": (H,), "W1": (H, F), "b1": (F,),
            "W2": (F, H), "b2": (H,), "g2": (H,), "be2": (H,)}


def embed_shapes(w: Workload) -> dict:
    return {"E": (w.vocab, w.hidden), "P": (w.seq, w.hidden),
            "ge": (w.hidden,), "be": (w.hidden,), "bv": (w.vocab,)}


def _param(seed, stream, shape, name, sigma):
    n = int(np.prod(shape))
    x = normal(seed, stream, n) * sigma
    if name in ("g1", "g2", "ge"):      # LayerNorm gains are centred on one
        x = 1.0 + x
    return x.reshape(shape).astype(np.float32)


def layer_params(w: Workload, layer: int, sigma: float = 0.02) -> dict:
    """fp32 parameters of encoder layer `layer`: every tensor N(0, sigma), gains 1 + N(0, sigma)."""
    shp = layer_shapes(w)
    return {k: _param(w.seed, 64 * (layer + 1) + s, shp[k], k, sigma) for k, s in _ST_LAYER.items()}


def embed_params(w: Workload, sigma: float = 0.02) -> dict:
    """fp32 parameters of the embedding / tied-head block."""
    shp = embed_shapes(w)
    return {k: _param(w.seed, s, shp[k], k, sigma) for k, s in _ST_EMB.items()}


def tokens_and_labels(w: Workload):
    """int32 arrays [U, ub, S]: token ids uniform in [0, V); label uniform in [0, V) with
    probability label_prob per position, else -1 (ignored).  Position 0 is forced to carry a
    label if the draw left the whole minibatch unlabelled."""
    n = w.num_ubatches * w.ubatch * w.seq
    tok = integers(w.seed, _ST_TOKENS, n, w.vocab)
    lab = integers(w.seed, _ST_LABEL_VAL, n, w.vocab)
    if w.label_prob < 1.0:
        keep = uniform01(w.seed, _ST_LABEL_MASK, n) < w.label_prob
        if not keep.any():
            keep[0] = True
        lab = np.where(keep, lab, -1)
    shape = (w.num_ubatches, w.ubatch, w.seq)
    return tok.reshape(shape).astype(np.int32), lab.reshape(shape).astype(np.int32)


_ST_CLS = {"Wp": 20, "bp": 21, "Wc": 22, "bc": 23}
_ST_SEQ_LABEL, _ST_SEQ_MASK = 24, 25
CLS_TENSORS = tuple(_ST_CLS)              # packed order of the sequence-classification head


def cls_shapes(w: Workload, num_classes: int) -> dict:
    H = w.hidden
    return {"Wp": (H, H), "bp": (H,), "Wc": (H, num_classes), "bc": (num_classes,)}


def cls_params(w: Workload, num_classes: int, sigma: float = 0.02) -> dict:
    """fp32 parameters of the sequence-classification head (pooler and classifier), N(0, sigma)."""
    shp = cls_shapes(w, num_classes)
    return {k: _param(w.seed, s, shp[k], k, sigma) for k, s in _ST_CLS.items()}


def seq_labels(w: Workload, num_classes: int, label_prob: float = 1.0) -> np.ndarray:
    """int32 [U, ub]: one class per sequence, uniform in [0, num_classes); with probability 1 - label_prob a
    sequence carries no label (-1); sequence 0 is forced to carry one if the draw left none."""
    n = w.num_ubatches * w.ubatch
    lab = integers(w.seed, _ST_SEQ_LABEL, n, num_classes)
    if label_prob < 1.0:
        keep = uniform01(w.seed, _ST_SEQ_MASK, n) < label_prob
        if not keep.any():
            keep[0] = True
        lab = np.where(keep, lab, -1)
    return lab.reshape(w.num_ubatches, w.ubatch).astype(np.int32)


def activations(w: Workload, stream_offset: int = 0) -> np.ndarray:
    """fp32 N(0,1) layer-boundary activations [U, ub, S, H] for single-layer parity runs."""
    shape = (w.num_ubatches, w.ubatch, w.seq, w.hidden)
    return normal(w.seed, _ST_ACT + 1000 * stream_offset, int(np.prod(shape))).reshape(shape).astype(np.float32)


def output_grads(w: Workload, scale: float = 1e-3) -> np.ndarray:
    """fp32 N(0, scale) upstream gradients dL/dY [U, ub, S, H] for single-layer parity runs."""
    shape = (w.num_ubatches, w.ubatch, w.seq, w.hidden)
    return (normal(w.seed, _ST_DY, int(np.prod(shape))) * scale).reshape(shape).astype(np.float32)
