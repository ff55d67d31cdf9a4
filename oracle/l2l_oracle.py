"""CPU oracle for L2L relay execution -- TEST INFRASTRUCTURE, not product code.

A plain, slow, fp64 NumPy statement of what the L2L hot path computes: the
gradients of the minibatch loss of an L-layer post-LayerNorm transformer
encoder with respect to every parameter, obtained either in the conventional
order (Algorithm 1: micro-batch outer loop, whole model inside) or in the L2L
order (Algorithm 2: layer outer loop, all micro-batches inside, only layer
boundary activations stashed, the layer forward recomputed in the backward
pass, Section 2.1), followed by the host optimizer step of the eager
param-server (Section 2.1, Section 2.3).

The method is exact -- a loop inversion plus recomputation (Section 2.2) -- so
the oracle is the plain definition.  The paper never writes the encoder-layer
equations (it inherits BERT's); the readings taken here are: post-LN encoder,
GELU in its exact erf form, biased variance in LayerNorm, no dropout, no
attention mask, loss normalised by the number of labelled positions in the
whole minibatch, Adam with bias correction and no weight decay.

Nothing here is imported, linked or called by the product path; the product
shares no code with this file.  Only tests, the smoke check and the
cpu-baseline leg of the benchmark may import it.

Pins (tests/test_oracle_*.py): central finite differences for every backward
formula, Algorithm 1 == Algorithm 2 == one concatenated minibatch, closed
forms for softmax / LayerNorm / GELU / cross-entropy / both heads / Adam / LAMB (plus LAMB's
step-length and scale invariances), exhaustive bf16 and fp16 round trips with hand-built ties, the two error measures on hand values, the whole layer forward against nested scalar loops.  Unpinned: end-to-end task accuracy against the paper's Table 7
(needs the GLUE data and pretrained weights) -- parity unpinned.
"""
from __future__ import annotations

import math
import numpy as np
from scipy.special import erf as _erf

F64 = np.float64

LAYER_KEYS = ("Wqkv", "bqkv", "Wo", "bo", "g1", "be1", "W1", "b1", "W2", "b2", "g2", "be2")
EMBED_KEYS = ("E", "P", "ge", "be", "bv")


# --------------------------------------------------------------------------- sizes
def layer_param_count(H: int, F: int) -> int:
    """Parameters of one encoder layer: 4 H^2 + 2 H F weights, 9 H + F vector entries."""
    return 4 * H * H + 2 * H * F + 9 * H + F


def boundary_activation_bytes(S: int, H: int, bytes_per_elem: int = 2) -> int:
    """Size of one sample's layer-boundary activation (Section 1: 1 MB for BERT-Large in FP16)."""
    return S * H * bytes_per_elem


# --------------------------------------------------------------------------- elementwise pieces
def gelu(u):
    """GELU, exact form: u * Phi(u)."""
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def gelu_grad(u):
    """d gelu / du = Phi(u) + u * phi(u)."""
    return 0.5 * (1.0 + _erf(u / math.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)


def softmax_rows(s):
    """Softmax over the last axis."""
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def layer_norm_fwd(r, gamma, beta, eps):
    """LN(r) = gamma * (r - mean) / sqrt(var_biased + eps) + beta over the last axis."""
    mu = r.mean(axis=-1, keepdims=True)
    var = ((r - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (r - mu) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def layer_norm_bwd(dy, cache, gamma):
    """Returns (dr, dgamma, dbeta) for y = LN(r)."""
    xhat, rstd = cache
    g = dy * gamma
    dr = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dr, (dy * xhat).sum(axis=red), dy.sum(axis=red)


# --------------------------------------------------------------------------- encoder layer
def encoder_layer_fwd(X, p, heads, eps):
    """One post-LN encoder layer.  X: [n_seq, S, H] -> (Y [n_seq, S, H], cache).

    Q,K,V = X Wqkv + bqkv split three ways then into heads of width d;
    P_h = softmax_rows(Q_h K_h^T / sqrt(d)); C = concat_h(P_h V_h);
    Y1 = LN(X + C Wo + bo); G = gelu(Y1 W1 + b1); Y = LN(Y1 + G W2 + b2).
    """
    X = np.asarray(X, F64)
    n, S, H = X.shape
    A = heads
    d = H // A
    qkv = X @ p["Wqkv"] + p["bqkv"]                       # [n,S,3H]
    q, k, v = (qkv[..., i * H:(i + 1) * H].reshape(n, S, A, d).transpose(0, 2, 1, 3) for i in range(3))
    sc = (q @ k.transpose(0, 1, 3, 2)) / math.sqrt(d)     # [n,A,S,S]
    P = softmax_rows(sc)
    C = (P @ v).transpose(0, 2, 1, 3).reshape(n, S, H)
    R1 = X + C @ p["Wo"] + p["bo"]
    Y1, ln1 = layer_norm_fwd(R1, p["g1"], p["be1"], eps)
    U1 = Y1 @ p["W1"] + p["b1"]
    G = gelu(U1)
    R2 = Y1 + G @ p["W2"] + p["b2"]
    Y, ln2 = layer_norm_fwd(R2, p["g2"], p["be2"], eps)
    cache = dict(X=X, q=q, k=k, v=v, P=P, C=C, ln1=ln1, Y1=Y1, U1=U1, G=G, ln2=ln2)
    return Y, cache


def encoder_layer_bwd(dY, cache, p, heads):
    """Backward of encoder_layer_fwd.  Returns (dX, grads dict keyed like p)."""
    dY = np.asarray(dY, F64)
    c = cache
    n, S, H = dY.shape
    A = heads
    d = H // A
    T = n * S
    g = {}
    dR2, g["g2"], g["be2"] = layer_norm_bwd(dY, c["ln2"], p["g2"])
    dR2f = dR2.reshape(T, H)
    g["W2"] = c["G"].reshape(T, -1).T @ dR2f
    g["b2"] = dR2f.sum(axis=0)
    dG = dR2 @ p["W2"].T
    dU1 = dG * gelu_grad(c["U1"])
    dU1f = dU1.reshape(T, -1)
    g["W1"] = c["Y1"].reshape(T, H).T @ dU1f
    g["b1"] = dU1f.sum(axis=0)
    dY1 = dR2 + dU1 @ p["W1"].T
    dR1, g["g1"], g["be1"] = layer_norm_bwd(dY1, c["ln1"], p["g1"])
    dR1f = dR1.reshape(T, H)
    g["Wo"] = c["C"].reshape(T, H).T @ dR1f
    g["bo"] = dR1f.sum(axis=0)
    dC = (dR1 @ p["Wo"].T).reshape(n, S, A, d).transpose(0, 2, 1, 3)     # [n,A,S,d]
    P = c["P"]
    dV = P.transpose(0, 1, 3, 2) @ dC
    dP = dC @ c["v"].transpose(0, 1, 3, 2)
    dSc = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dQ = (dSc @ c["k"]) / math.sqrt(d)
    dK = (dSc.transpose(0, 1, 3, 2) @ c["q"]) / math.sqrt(d)
    dqkv = np.concatenate([t.transpose(0, 2, 1, 3).reshape(n, S, H) for t in (dQ, dK, dV)], axis=-1)
    dqkvf = dqkv.reshape(T, 3 * H)
    g["Wqkv"] = c["X"].reshape(T, H).T @ dqkvf
    g["bqkv"] = dqkvf.sum(axis=0)
    dX = dR1 + dqkv @ p["Wqkv"].T
    return dX, g


# --------------------------------------------------------------------------- embedding and head
def embed_fwd(tokens, e, eps):
    """x0[b,s] = LN_e(E[tok[b,s]] + Ppos[s]).  tokens: int [n,S]."""
    r = e["E"][tokens] + e["P"][None, :tokens.shape[1], :]
    y, ln = layer_norm_fwd(r.astype(F64), e["ge"], e["be"], eps)
    return y, ln


def embed_bwd(dy, tokens, ln, e):
    """Returns grads {E, P, ge, be} of the embedding block (E part only from the lookup)."""
    dr, dge, dbe = layer_norm_bwd(dy, ln, e["ge"])
    dE = np.zeros_like(e["E"], dtype=F64)
    np.add.at(dE, tokens.reshape(-1), dr.reshape(-1, dr.shape[-1]))
    dP = np.zeros_like(e["P"], dtype=F64)
    dP[:tokens.shape[1]] = dr.sum(axis=0)
    return {"E": dE, "P": dP, "ge": dge, "be": dbe}


def head_loss(xL, labels, e, n_lab_total):
    """Tied LM head + cross-entropy over labelled positions (label >= 0).

    z = x E^T + bv ; contribution to the loss = -(1/N) sum_t log softmax(z_t)[label_t], with N
    the labelled count of the WHOLE minibatch, so that micro-batch contributions simply add.
    Returns (loss_contribution, d xL, {E, bv} grads).
    """
    n, S, H = xL.shape
    xf = xL.reshape(-1, H)
    lab = labels.reshape(-1)
    idx = np.nonzero(lab >= 0)[0]
    dx = np.zeros_like(xf)
    dE = np.zeros_like(e["E"], dtype=F64)
    dbv = np.zeros_like(e["bv"], dtype=F64)
    if idx.size == 0:
        return 0.0, dx.reshape(n, S, H), {"E": dE, "bv": dbv}
    z = xf[idx] @ e["E"].T + e["bv"]
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    loss = float((lse - z[np.arange(idx.size), lab[idx]]).sum() / n_lab_total)
    dz = np.exp(z - lse[:, None])
    dz[np.arange(idx.size), lab[idx]] -= 1.0
    dz /= n_lab_total
    dx[idx] = dz @ e["E"]
    dE += dz.T @ xf[idx]
    dbv += dz.sum(axis=0)
    return loss, dx.reshape(n, S, H), {"E": dE, "bv": dbv}


def cls_head_loss(xL, seq_labels, c, n_lab_total):
    """Sequence-classification head (the GLUE task head of the fine-tuning runs of Sections 3.1 and 3.5, Table 7; the paper does not
    write it out: this is the usual BERT one): pooled = tanh(x_[first token] Wp + bp), z = pooled Wc + bc,
    loss contribution = -(1/N) sum_q log softmax(z_q)[label_q] over the sequences with label >= 0, N being
    the labelled count of the WHOLE minibatch.  xL: [n, S, H]; seq_labels: [n].
    Returns (loss_contribution, d xL, {Wp, bp, Wc, bc} grads)."""
    n, S, H = xL.shape
    lab = np.asarray(seq_labels).reshape(-1)
    dx = np.zeros_like(xL)
    g = {k: np.zeros_like(v, dtype=F64) for k, v in c.items()}
    idx = np.nonzero(lab >= 0)[0]
    if idx.size == 0:
        return 0.0, dx, g
    x0 = xL[idx, 0, :]
    pooled = np.tanh(x0 @ c["Wp"] + c["bp"])
    z = pooled @ c["Wc"] + c["bc"]
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    loss = float((lse - z[np.arange(idx.size), lab[idx]]).sum() / n_lab_total)
    dz = np.exp(z - lse[:, None])
    dz[np.arange(idx.size), lab[idx]] -= 1.0
    dz /= n_lab_total
    g["Wc"] += pooled.T @ dz
    g["bc"] += dz.sum(axis=0)
    du = (dz @ c["Wc"].T) * (1.0 - pooled * pooled)
    g["Wp"] += x0.T @ du
    g["bp"] += du.sum(axis=0)
    dx[idx, 0, :] = du @ c["Wp"].T
    return loss, dx, g


# --------------------------------------------------------------------------- whole-model drivers
def _to64(d):
    return {k: np.asarray(v, F64) for k, v in d.items()}


def _zeros_like_params(emb, layers):
    return ({k: np.zeros_like(v) for k, v in emb.items()},
            [{k: np.zeros_like(v) for k, v in p.items()} for p in layers])


def _acc(dst, src):
    for k, v in src.items():
        dst[k] += v


def model_fwd_bwd(emb, layers, tokens, labels, heads, eps, n_lab_total):
    """Whole model on one batch [n,S] with every layer's cache alive (conventional execution).
    Returns (loss contribution, embedding-block grads, per-layer grads)."""
    x, ln_e = embed_fwd(tokens, emb, eps)
    caches = []
    for p in layers:
        x, c = encoder_layer_fwd(x, p, heads, eps)
        caches.append(c)
    loss, dx, gh = head_loss(x, labels, emb, n_lab_total)
    glayers = [None] * len(layers)
    for l in reversed(range(len(layers))):
        dx, glayers[l] = encoder_layer_bwd(dx, caches[l], layers[l], heads)
    ge = embed_bwd(dx, tokens, ln_e, emb)
    ge["E"] = ge["E"] + gh["E"]
    ge["bv"] = gh["bv"]
    return loss, ge, glayers


def run_conventional(emb, layers, tokens, labels, heads, eps):
    """Algorithm 1 (baseline with accumulated gradients): for each micro-batch run the whole
    model forward and backward and add its gradients.  tokens/labels: int [U, ub, S]."""
    emb, layers = _to64(emb), [_to64(p) for p in layers]
    n_lab = int((labels >= 0).sum())
    gemb, glayers = _zeros_like_params(emb, layers)
    loss = 0.0
    for u in range(tokens.shape[0]):
        l_u, ge, gl = model_fwd_bwd(emb, layers, tokens[u], labels[u], heads, eps, n_lab)
        loss += l_u
        _acc(gemb, ge)
        for a, b in zip(glayers, gl):
            _acc(a, b)
    return loss, gemb, glayers


def run_l2l(emb, layers, tokens, labels, heads, eps, return_stash=False):
    """Algorithm 2 (L2L): layer loop outside, micro-batch loop inside.  Forward keeps only each
    layer's boundary output per micro-batch (the stash); backward walks layers in reverse,
    recomputes the layer forward from the stash for each micro-batch, back-propagates, and
    accumulates that layer's parameter gradient over micro-batches (Section 2.1)."""
    emb, layers = _to64(emb), [_to64(p) for p in layers]
    U = tokens.shape[0]
    L = len(layers)
    n_lab = int((labels >= 0).sum())
    gemb, glayers = _zeros_like_params(emb, layers)
    stash = [[None] * U for _ in range(L + 1)]
    ln_e = [None] * U
    for u in range(U):                                   # first resident "layer": the embedding
        stash[0][u], ln_e[u] = embed_fwd(tokens[u], emb, eps)
    for l in range(L):                                   # relay: one encoder layer resident at a time
        for u in range(U):
            stash[l + 1][u], _ = encoder_layer_fwd(stash[l][u], layers[l], heads, eps)
    loss = 0.0
    g = [None] * U                                       # boundary gradient per micro-batch
    for u in range(U):                                   # last resident "layer": head, fwd+bwd adjacent
        l_u, g[u], gh = head_loss(stash[L][u], labels[u], emb, n_lab)
        loss += l_u
        _acc(gemb, gh)
    for l in reversed(range(L)):
        for u in range(U):
            _, cache = encoder_layer_fwd(stash[l][u], layers[l], heads, eps)   # recompute
            g[u], gl = encoder_layer_bwd(g[u], cache, layers[l], heads)
            _acc(glayers[l], gl)
    for u in range(U):
        _acc(gemb, embed_bwd(g[u], tokens[u], ln_e[u], emb))
    if return_stash:
        return loss, gemb, glayers, stash
    return loss, gemb, glayers


def run_l2l_cls(emb, layers, cls, tokens, seq_labels, heads, eps):
    """Algorithm 2 with the sequence-classification head in place of the LM head: as run_l2l, but the last
    resident "layer" is cls_head_loss over each micro-batch's sequences.  seq_labels: [U, ub].
    Returns (loss, embedding grads, per-layer grads, head grads)."""
    emb, layers, cls = _to64(emb), [_to64(p) for p in layers], _to64(cls)
    U = tokens.shape[0]
    L = len(layers)
    n_lab = int((np.asarray(seq_labels) >= 0).sum())
    gemb, glayers = _zeros_like_params(emb, layers)
    gcls = {k: np.zeros_like(v) for k, v in cls.items()}
    x = [None] * U
    ln_e = [None] * U
    stash = [[None] * U for _ in range(L + 1)]
    for u in range(U):
        stash[0][u], ln_e[u] = embed_fwd(tokens[u], emb, eps)
    for l in range(L):
        for u in range(U):
            stash[l + 1][u], _ = encoder_layer_fwd(stash[l][u], layers[l], heads, eps)
    loss = 0.0
    g = [None] * U
    for u in range(U):
        l_u, g[u], gh = cls_head_loss(stash[L][u], seq_labels[u], cls, n_lab)
        loss += l_u
        _acc(gcls, gh)
    for l in reversed(range(L)):
        for u in range(U):
            _, cache = encoder_layer_fwd(stash[l][u], layers[l], heads, eps)
            g[u], gl = encoder_layer_bwd(g[u], cache, layers[l], heads)
            _acc(glayers[l], gl)
    for u in range(U):
        _acc(gemb, embed_bwd(g[u], tokens[u], ln_e[u], emb))
    return loss, gemb, glayers, gcls


def layer_l2l_fwd(X, p, heads, eps):
    """Forward of one resident layer over all micro-batches.  X: [U, ub, S, H]."""
    p = _to64(p)
    return np.stack([encoder_layer_fwd(X[u], p, heads, eps)[0] for u in range(X.shape[0])])


def layer_l2l_bwd(X, dY, p, heads, eps):
    """Backward of one resident layer over all micro-batches with recompute from the stash X.
    Returns (dX [U,ub,S,H], parameter grads accumulated over micro-batches)."""
    p = _to64(p)
    acc = {k: np.zeros_like(v) for k, v in p.items()}
    dX = np.empty(X.shape, F64)
    for u in range(X.shape[0]):
        _, cache = encoder_layer_fwd(X[u], p, heads, eps)
        dX[u], gl = encoder_layer_bwd(dY[u], cache, p, heads)
        _acc(acc, gl)
    return dX, acc


# --------------------------------------------------------------------------- EPS: optimizer and shipping copy
def adam_step(w, g, m, v, t, lr=1e-4, beta1=0.9, beta2=0.999, eps_a=1e-8):
    """One bias-corrected Adam update (no weight decay).  Returns (w, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return w - lr * mhat / (np.sqrt(vhat) + eps_a), m, v


def lamb_step(w, g, m, v, t, lr=1e-3, beta1=0.9, beta2=0.999, eps_a=1e-6, weight_decay=0.0):
    """One LAMB update of ONE parameter tensor (the optimizer Table 1 names; the update rule is the one of
    the LAMB publication the paper cites, with bias correction and the identity scaling function):
        m, v as in Adam;  r = mhat / (sqrt(vhat) + eps);  u = r + weight_decay * w;
        trust = ||w|| / ||u|| (1 where either norm is zero);  w <- w - lr * trust * u.
    The norms are over the whole tensor, which is why the host EPS, holding each layer's tensors whole,
    can apply it layer by layer.  Returns (w, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    u = mhat / (np.sqrt(vhat) + eps_a) + weight_decay * w
    wn = float(np.sqrt(np.sum(np.square(w, dtype=np.float64))))
    un = float(np.sqrt(np.sum(np.square(u, dtype=np.float64))))
    trust = wn / un if (wn > 0.0 and un > 0.0) else 1.0
    return w - lr * trust * u, m, v


def bf16_bits(x):
    """Round float32 values to bfloat16 (nearest, ties to even); returns the uint16 patterns.
    NaNs are quieted, infinities kept."""
    x = np.asarray(x, np.float32)
    b = x.view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = ((b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, ((b >> np.uint64(16)) | np.uint64(0x40)).astype(np.uint16), r)
    return r


def bf16_to_f32(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def fp16_bits(x):
    """Round float32 values to IEEE half precision (nearest, ties to even, overflow to infinity, gradual
    underflow); returns the uint16 patterns.  The FP16 of the paper's cross mixed precision (Section 2.3)."""
    with np.errstate(over="ignore"):
        return np.asarray(x, np.float32).astype(np.float16).view(np.uint16)


def fp16_round(x):
    """float32 -> nearest half-precision value, returned as float32."""
    x = np.asarray(x, np.float32)
    return fp16_bits(x).view(np.float16).astype(np.float32).reshape(x.shape)


def bf16_round(x):
    """float32 -> nearest bfloat16 value, returned as float32 (the CMP shipping precision,
    Section 2.3, with bf16 in place of the paper's FP16)."""
    x = np.asarray(x, np.float32)
    return bf16_to_f32(bf16_bits(x)).reshape(x.shape)


# --------------------------------------------------------------------------- timing model (Section 2.2.1)
def total_time_ms(N, u, C, X):
    """Eq. 4: N (u C + X) forward plus N (3 u C + X) backward-with-recompute, no overlap."""
    return N * (u * C + X) + N * (3 * u * C + X)


def throughput_forward(N, u, ub, C, X):
    """Forward samples/s; the reading of Eq. 5 consistent with the text before it."""
    return 1000.0 * u * ub / (N * (u * C + X))


def throughput_training(N, u, ub, C, X):
    """Training samples/s from Eq. 4 (Eq. 6 with the factor N restored)."""
    return 1000.0 * u * ub / total_time_ms(N, u, C, X)


def transfer_overhead(u, C, X, training=True):
    """Fraction of extra time caused by transfers relative to pure compute."""
    return (2 * X) / (4 * u * C) if training else X / (u * C)


# --------------------------------------------------------------------------- error measure used by parity tests
def rel_l2(a, b):
    """|| a - b ||_2 / || b ||_2 with b the oracle value."""
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def max_rel(a, b):
    """max | a - b | / max | b | with b the oracle value: the largest single error, in units of the tensor's
    largest entry.  Unlike rel_l2 it cannot be averaged away: a few wrong rows of a large tensor show up in full."""
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    if a.size == 0:
        return 0.0
    mb = float(np.abs(b).max())
    return float(np.abs(a - b).max() / mb) if mb > 0 else float(np.abs(a).max())

