"""Plain float64 definition of one pipeline stage of pre-LN GPT transformer layers.

Test infrastructure only (see package docstring).

The paper treats a stage ("nn_shard", Sec. 3.1, Alg. 1) as a contiguous subset of
transformer layers with Forward(msg) / Backward(msg) entry points (Alg. 2) and defers
the layer mathematics to the original transformer paper (Sec. 6.1).  The layer written
here is the standard pre-LayerNorm GPT block:

    u   = LN(x; g1, b1)
    qkv = u W_qkv + b_qkv          columns [0,h)=Q, [h,2h)=K, [2h,3h)=V, head j owns
                                    columns j*d..(j+1)*d-1 of each third
    o   = causal softmax(q k^T / sqrt(d)) v   per (batch, head)
    y   = x + o W_o + b_o
    w   = LN(y; g2, b2)
    pre = w W_1 + b_1 ;  g = GeLU(pre)  (exact erf form)
    z   = y + g W_2 + b_2

Weights are stored [in, out].  The backward pass is the exact reverse-mode derivative
(Sec. 2.1, "Forward and backward pass").  Gradients of a batch are the plain sum of
the per-microbatch gradients (Sec. 2.2 "Inter-layer parallelism"; Sec. 4.2: any 1/M
factor lives in the upstream gradients).

No blocking, fusion or reordering: attention materialises the full s x s matrices.
"""
import numpy as np
from scipy.special import erf as _erf

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")

_F = np.float64


# ----------------------------------------------------------------- LayerNorm
def layernorm_fwd(x, gamma, beta, eps):
    """Per-token LayerNorm over the last axis, biased variance, eps inside the root.

    Returns (out, xhat, rstd)."""
    x = np.asarray(x, _F)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def layernorm_bwd(dout, xhat, rstd, gamma):
    """Derivative of layernorm_fwd.  Returns (dx, dgamma, dbeta)."""
    dxhat = dout * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    red = tuple(range(dout.ndim - 1))
    return dx, (dout * xhat).sum(axis=red), dout.sum(axis=red)


# ---------------------------------------------------------------------- GeLU
def gelu(x):
    """GeLU(x) = x * Phi(x), Phi the standard normal CDF (exact erf form)."""
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    """d/dx GeLU(x) = Phi(x) + x * phi(x)."""
    return 0.5 * (1.0 + _erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)


# ----------------------------------------------------------------- attention
def _split_heads(t, n_heads):
    b, s, h = t.shape
    return t.reshape(b, s, n_heads, h // n_heads).transpose(0, 2, 1, 3)  # [b,a,s,d]


def _merge_heads(t):
    b, a, s, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, s, a * d)


def causal_attention_fwd(q, k, v, n_heads):
    """q,k,v: [b,s,h].  Returns (o [b,s,h], P [b,a,s,s]).

    Scores are scaled by 1/sqrt(d); positions j>i are excluded from the softmax
    (their probability is exactly 0)."""
    qh, kh, vh = (_split_heads(t, n_heads) for t in (q, k, v))
    d = qh.shape[-1]
    s = qh.shape[2]
    S = qh @ kh.transpose(0, 1, 3, 2) / np.sqrt(_F(d))
    allowed = np.tril(np.ones((s, s), dtype=bool))
    S = np.where(allowed, S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.where(allowed, np.exp(S), 0.0)
    P = E / E.sum(axis=-1, keepdims=True)
    return _merge_heads(P @ vh), P


def causal_attention_bwd(do, q, k, v, P, n_heads):
    """Returns (dq, dk, dv), each [b,s,h]."""
    qh, kh, vh, doh = (_split_heads(t, n_heads) for t in (q, k, v, do))
    d = qh.shape[-1]
    dV = P.transpose(0, 1, 3, 2) @ doh
    dP = doh @ vh.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dS = dS / np.sqrt(_F(d))
    dQ = dS @ kh
    dK = dS.transpose(0, 1, 3, 2) @ qh
    return _merge_heads(dQ), _merge_heads(dK), _merge_heads(dV)


# --------------------------------------------------------------------- layer
def layer_forward(x, p, n_heads, eps):
    """One pre-LN block.  x: [b,s,h]; p: dict over PARAM_NAMES.  Returns (z, cache)."""
    x = np.asarray(x, _F)
    h = x.shape[-1]
    u, xhat1, rstd1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = u @ p["w_qkv"] + p["b_qkv"]
    q, k, v = qkv[..., :h], qkv[..., h:2 * h], qkv[..., 2 * h:]
    o, P = causal_attention_fwd(q, k, v, n_heads)
    y = x + o @ p["w_o"] + p["b_o"]
    w, xhat2, rstd2 = layernorm_fwd(y, p["ln2_g"], p["ln2_b"], eps)
    pre = w @ p["w_fc1"] + p["b_fc1"]
    g = gelu(pre)
    z = y + g @ p["w_fc2"] + p["b_fc2"]
    cache = dict(xhat1=xhat1, rstd1=rstd1, u=u, q=q, k=k, v=v, P=P, o=o,
                 xhat2=xhat2, rstd2=rstd2, w=w, pre=pre, g=g)
    return z, cache


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_backward(dz, cache, p, n_heads):
    """Reverse-mode derivative of layer_forward.  Returns (dx, grads dict)."""
    c = cache
    dz = np.asarray(dz, _F)
    gr = {}
    # z = y + g W2 + b2
    gr["w_fc2"] = _flat(c["g"]).T @ _flat(dz)
    gr["b_fc2"] = _flat(dz).sum(axis=0)
    dg = dz @ p["w_fc2"].T
    dpre = dg * gelu_grad(c["pre"])
    gr["w_fc1"] = _flat(c["w"]).T @ _flat(dpre)
    gr["b_fc1"] = _flat(dpre).sum(axis=0)
    dw = dpre @ p["w_fc1"].T
    dy_ln, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dw, c["xhat2"], c["rstd2"], p["ln2_g"])
    dy = dz + dy_ln
    # y = x + o Wo + bo
    gr["w_o"] = _flat(c["o"]).T @ _flat(dy)
    gr["b_o"] = _flat(dy).sum(axis=0)
    do = dy @ p["w_o"].T
    dq, dk, dv = causal_attention_bwd(do, c["q"], c["k"], c["v"], c["P"], n_heads)
    dqkv = np.concatenate([dq, dk, dv], axis=-1)
    gr["w_qkv"] = _flat(c["u"]).T @ _flat(dqkv)
    gr["b_qkv"] = _flat(dqkv).sum(axis=0)
    du = dqkv @ p["w_qkv"].T
    dx_ln, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(du, c["xhat1"], c["rstd1"], p["ln1_g"])
    return dy + dx_ln, gr


# --------------------------------------------------------------------- stage
def stage_forward(x, layers, n_heads, eps):
    """Forward(msg) of a stage: layers applied in order.  Returns (output, caches).

    No final LayerNorm, LM head or loss: those belong to the last pipeline stage."""
    caches = []
    a = np.asarray(x, _F)
    for p in layers:
        a, c = layer_forward(a, p, n_heads, eps)
        caches.append(c)
    return a, caches


def stage_backward(dy, caches, layers, n_heads):
    """Backward(msg) of a stage.  Returns (dx, [per-layer grads dict])."""
    d = np.asarray(dy, _F)
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        d, grads[i] = layer_backward(d, caches[i], layers[i], n_heads)
    return d, grads


def stage_batch(xs, dys, layers, n_heads, eps):
    """All microbatches of a batch, sequentially.  Returns (outputs, dxs, summed grads)."""
    layers = [{k: np.asarray(v, _F) for k, v in p.items()} for p in layers]
    tot = [{k: np.zeros_like(v) for k, v in p.items()} for p in layers]
    outs, dxs = [], []
    for x, dy in zip(xs, dys):
        z, caches = stage_forward(x, layers, n_heads, eps)
        dx, grads = stage_backward(dy, caches, layers, n_heads)
        del caches
        outs.append(z)
        dxs.append(dx)
        for t, g in zip(tot, grads):
            for k in t:
                t[k] += g[k]
    return outs, dxs, tot


# ------------------------------------------------------- activation checkpointing
# Sec. 5.1: with stride ac (a factor of the layer count) only the outputs of layers
# ac, 2ac, ... are kept by the forward pass; a layer's other activations are regenerated
# from the nearest kept tensor when its backward pass runs.  For a stage, the output of
# the previous stage's last layer (the stage input) is the first kept tensor, and the
# stage's own last output is sent onwards rather than kept.
def stage_forward_checkpointed(x, layers, n_heads, eps, ac):
    """Forward(msg) keeping only the inputs of layers 0, ac, 2ac, ...

    Returns (output, kept) where kept[j] is the input of layer j*ac."""
    n = len(layers)
    if ac < 1 or n % ac != 0:
        raise ValueError("the checkpointing stride must be a factor of the layer count")
    kept = []
    a = np.asarray(x, _F)
    for i, p in enumerate(layers):
        if i % ac == 0:
            kept.append(a)
        a, _ = layer_forward(a, p, n_heads, eps)   # the cache is dropped at once
    return a, kept


def stage_backward_checkpointed(dy, kept, layers, n_heads, eps, ac, live_log=None):
    """Backward(msg) from the kept tensors: segment by segment from the last, the
    segment's ac layers are run forward again from its kept input, then differentiated.

    live_log, if a list, receives the number of layer caches alive after each
    regeneration (the "+ ac" term of Eq. 1).  Returns (dx, [per-layer grads dict])."""
    n = len(layers)
    d = np.asarray(dy, _F)
    grads = [None] * n
    for j in reversed(range(n // ac)):
        lo = j * ac
        _, caches = stage_forward(kept[j], layers[lo:lo + ac], n_heads, eps)
        if live_log is not None:
            live_log.append(len(caches))
        d, grads[lo:lo + ac] = stage_backward(d, caches, layers[lo:lo + ac], n_heads)
        del caches
    return d, grads


def activation_memory(n_layers, g_inter, ac):
    """Eq. 1 up to its constant of proportionality, in units of one layer's activations:
    g_inter microbatches in flight, each holding n_layers / (g_inter * ac) kept tensors,
    plus the layer being processed, plus the ac regenerated layers of one segment."""
    return g_inter * (n_layers / (g_inter * ac)) + 1 + ac


def checkpoint_stride(n_layers, g_inter):
    """Sec. 5.1: the factor of the per-GPU layer count n_layers / g_inter closest to
    sqrt(n_layers) (ties: the smaller factor)."""
    per_gpu = n_layers // g_inter
    factors = [a for a in range(1, per_gpu + 1) if per_gpu % a == 0]
    return min(factors, key=lambda a: (abs(a - np.sqrt(n_layers)), a))
