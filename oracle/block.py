"""fp64 CPU oracle: forward and reverse-mode gradient of one pipeline stage's layers.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this package; it exists
so that the HIP stage can be compared with a slow, plain statement of what it computes.
It shares no code with the HIP path.

The paper (Sections 3.1 and 5) treats a stage as a stack of transformer blocks with
Megatron-like dimensions and says nothing about the block's inside.  The block taken here
is the pre-LayerNorm one the workload descriptions name:

    a  = LN(x; g1, s1)                       LN(z) = g * (z - mean) / sqrt(var + eps) + s,
    [q|k|v] = a Wqkv + bqkv                   var biased, over the hidden dimension
    S  = q k^T / sqrt(dh) per head, masked keys excluded, P = softmax_rows(S), o = P v
    x1 = x + o Wo + bo
    c  = LN(x1; g2, s2)
    u  = c W1 + b1
    y  = x1 + GELU(u) W2 + b2                 GELU(u) = u/2 (1 + erf(u / sqrt 2))

Masks: none; causal (key j visible to query i iff j <= i); key padding (key j of sequence n
visible iff j < len_n, for every query row, padded query rows included).

The backward functions are the textbook reverse-mode derivative of exactly these equations.
Pins (tests/test_oracle_*.py): central finite differences, an autograd evaluation of the
same block with library routines, closed-form special cases, mask invariances.
No printed numeric example of a transformer stage exists in the paper.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import erf

MASK_NONE, MASK_CAUSAL, MASK_PADDING = 0, 1, 2

_LAYER_TENSORS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                  "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def layer_shapes(h: int, f: int) -> List[Tuple[str, Tuple[int, ...]]]:
    shapes = {"ln1_g": (h,), "ln1_b": (h,), "wqkv": (h, 3 * h), "bqkv": (3 * h,),
              "wo": (h, h), "bo": (h,), "ln2_g": (h,), "ln2_b": (h,),
              "w1": (h, f), "b1": (f,), "w2": (f, h), "b2": (h,)}
    return [(n, shapes[n]) for n in _LAYER_TENSORS]


def n_params(n_layers: int, h: int, f: int) -> int:
    return n_layers * sum(int(np.prod(s)) for _, s in layer_shapes(h, f))


def unflatten(flat: np.ndarray, n_layers: int, h: int, f: int) -> List[Dict[str, np.ndarray]]:
    """Views into a flat parameter (or gradient) vector: one dict per layer."""
    assert flat.ndim == 1 and flat.size == n_params(n_layers, h, f)
    layers, off = [], 0
    for _ in range(n_layers):
        d = {}
        for name, shape in layer_shapes(h, f):
            n = int(np.prod(shape))
            d[name] = flat[off:off + n].reshape(shape)
            off += n
        layers.append(d)
    return layers


# ----------------------------------------------------------------------------- sub-operations

def layernorm_fwd(x, gain, shift, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gain * xhat + shift, (xhat, rstd)


def layernorm_bwd(dy, saved, gain):
    xhat, rstd = saved
    dxhat = dy * gain
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / math.sqrt(2.0)))


def gelu_grad(u):
    cdf = 0.5 * (1.0 + erf(u / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return cdf + u * pdf


def visibility(mask_mode: int, s: int, length: Optional[int]) -> np.ndarray:
    """[s, s] boolean: entry (i, j) says whether query i may attend to key j."""
    if mask_mode == MASK_NONE:
        return np.ones((s, s), dtype=bool)
    if mask_mode == MASK_CAUSAL:
        return np.tril(np.ones((s, s), dtype=bool))
    if mask_mode == MASK_PADDING:
        assert length is not None and 1 <= length <= s
        return np.broadcast_to(np.arange(s)[None, :] < length, (s, s))
    raise ValueError(mask_mode)


def attention_fwd(q, k, v, vis):
    """q, k, v: [heads, s, dh] of one sequence; vis: [s, s].  Returns o and the probabilities."""
    dh = q.shape[-1]
    S = (q @ k.transpose(0, 2, 1)) / math.sqrt(dh)
    S = np.where(vis[None], S, -np.inf)           # exp(-inf) = 0: masked keys leave max and sum
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    P = E / E.sum(axis=-1, keepdims=True)
    return P @ v, P


def attention_bwd(do, q, k, v, P):
    dh = q.shape[-1]
    dv = P.transpose(0, 2, 1) @ do
    dP = do @ v.transpose(0, 2, 1)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dS = dS / math.sqrt(dh)
    return dS @ k, dS.transpose(0, 2, 1) @ q, dv


# ----------------------------------------------------------------------------- one block

def block_fwd(p: Dict[str, np.ndarray], x: np.ndarray, lens, mask_mode: int, n_heads: int,
              ln_eps: float):
    """x: [b, s, h] fp64.  Returns y and everything the backward needs."""
    b, s, h = x.shape
    dh = h // n_heads
    a, ln1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], ln_eps)
    qkv = a @ p["wqkv"] + p["bqkv"]
    # columns are Q|K|V, each head-major
    q, k, v = (qkv[..., i * h:(i + 1) * h].reshape(b, s, n_heads, dh).transpose(0, 2, 1, 3)
               for i in range(3))
    o = np.empty((b, n_heads, s, dh))
    probs = []
    for n in range(b):
        vis = visibility(mask_mode, s, None if lens is None else int(lens[n]))
        o[n], P = attention_fwd(q[n], k[n], v[n], vis)
        probs.append(P)
    o2 = o.transpose(0, 2, 1, 3).reshape(b, s, h)
    x1 = x + o2 @ p["wo"] + p["bo"]
    c, ln2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], ln_eps)
    u = c @ p["w1"] + p["b1"]
    g = gelu(u)
    y = x1 + g @ p["w2"] + p["b2"]
    cache = dict(ln1=ln1, a=a, q=q, k=k, v=v, probs=probs, o2=o2, ln2=ln2, c=c, u=u, g=g,
                 n_heads=n_heads)
    return y, cache


def block_bwd(p: Dict[str, np.ndarray], cache, dy: np.ndarray):
    """Returns dx and a dict of parameter gradients (summed over the microbatch's tokens)."""
    b, s, h = dy.shape
    n_heads = cache["n_heads"]
    dh = h // n_heads
    tok = lambda z: z.reshape(b * s, -1)
    gr = {}
    # y = x1 + g W2 + b2
    gr["w2"] = tok(cache["g"]).T @ tok(dy)
    gr["b2"] = tok(dy).sum(axis=0)
    dg = dy @ p["w2"].T
    du = dg * gelu_grad(cache["u"])
    gr["w1"] = tok(cache["c"]).T @ tok(du)
    gr["b1"] = tok(du).sum(axis=0)
    dc = du @ p["w1"].T
    dx1_ln, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dc, cache["ln2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    # x1 = x + o Wo + bo
    gr["wo"] = tok(cache["o2"]).T @ tok(dx1)
    gr["bo"] = tok(dx1).sum(axis=0)
    do2 = dx1 @ p["wo"].T
    do = do2.reshape(b, s, n_heads, dh).transpose(0, 2, 1, 3)
    dq = np.empty_like(do)
    dk = np.empty_like(do)
    dv = np.empty_like(do)
    for n in range(b):
        dq[n], dk[n], dv[n] = attention_bwd(do[n], cache["q"][n], cache["k"][n], cache["v"][n],
                                            cache["probs"][n])
    back = lambda z: z.transpose(0, 2, 1, 3).reshape(b, s, h)
    dqkv = np.concatenate([back(dq), back(dk), back(dv)], axis=-1)
    gr["wqkv"] = tok(cache["a"]).T @ tok(dqkv)
    gr["bqkv"] = tok(dqkv).sum(axis=0)
    da = dqkv @ p["wqkv"].T
    dx_ln, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(da, cache["ln1"], p["ln1_g"])
    return dx1 + dx_ln, gr


# ----------------------------------------------------------------------------- one stage

class Stage:
    """A stack of blocks: the function F(W; X) one pipeline stage evaluates, and its VJP."""

    def __init__(self, n_layers: int, hidden: int, n_heads: int, ffn: int, mask_mode: int,
                 ln_eps: float = 1e-5):
        assert hidden % n_heads == 0
        self.L, self.h, self.a, self.f = n_layers, hidden, n_heads, ffn
        self.mask_mode, self.ln_eps = mask_mode, ln_eps
        self.n_params = n_params(n_layers, hidden, ffn)

    def forward(self, w_flat: np.ndarray, x: np.ndarray, lens=None):
        w = np.asarray(w_flat, dtype=np.float64)
        layers = unflatten(w, self.L, self.h, self.f)
        z = np.asarray(x, dtype=np.float64)
        caches = []
        for p in layers:
            z, c = block_fwd(p, z, lens, self.mask_mode, self.a, self.ln_eps)
            caches.append(c)
        return z, caches

    def backward(self, w_flat: np.ndarray, caches, dy: np.ndarray):
        w = np.asarray(w_flat, dtype=np.float64)
        layers = unflatten(w, self.L, self.h, self.f)
        g_flat = np.zeros(self.n_params)
        g_layers = unflatten(g_flat, self.L, self.h, self.f)
        d = np.asarray(dy, dtype=np.float64)
        for p, c, g in zip(reversed(layers), reversed(caches), reversed(g_layers)):
            d, gr = block_bwd(p, c, d)
            for name, val in gr.items():
                g[name][...] = val
        return d, g_flat

    def vjp(self, w_flat, x, dy, lens=None):
        """(Y, dX, g): output, activation gradient and weight gradient for boundary gradient dY."""
        y, caches = self.forward(w_flat, x, lens)
        dx, g = self.backward(w_flat, caches, dy)
        return y, dx, g
