"""Pins for oracle/block.py (CPU only): each check is independent of the oracle's own formulas.

* central finite differences of every sub-operation, of a block and of a stage;
* the same block written with a library's routines (torch CPU, fp64) and differentiated by
  its autograd;
* special cases with closed forms (one key => attention is the identity on v; W1 = 0 => the
  MLP branch is a constant; GELU and LayerNorm values known from the normal distribution);
* mask properties: causal (no information flows backwards), key padding (valid positions see
  the truncated sequence's result).
"""
import math

import numpy as np
import pytest

from oracle import block as ob


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


def rand_params(rng, L, h, f, scale=0.3):
    flat = rng.standard_normal(ob.n_params(L, h, f)) * scale
    for p in ob.unflatten(flat, L, h, f):
        p["ln1_g"] += 1.0
        p["ln2_g"] += 1.0
    return flat


def fd_grad(fun, x, eps=1e-6):
    """Central differences of a scalar function of an array."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = fun()
        x[i] = old - eps
        fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


# ----------------------------------------------------------------------------- closed forms

def test_gelu_known_values():
    # Phi(1) from tables of the normal distribution
    assert ob.gelu(np.array(0.0)) == 0.0
    assert abs(ob.gelu(np.array(1.0)) - 0.8413447460685429) < 1e-15
    u = np.linspace(-4, 4, 33)
    assert np.allclose(ob.gelu(u) - ob.gelu(-u), u, atol=1e-15)          # u Phi(u) - (-u) Phi(-u) = u
    assert abs(ob.gelu_grad(np.array(0.0)) - 0.5) < 1e-16
    # derivative against central differences
    e = 1e-6
    assert np.allclose(ob.gelu_grad(u), (ob.gelu(u + e) - ob.gelu(u - e)) / (2 * e), atol=1e-9)


def test_layernorm_statistics():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 5, 16)) * 3 + 2
    y, _ = ob.layernorm_fwd(x, np.ones(16), np.zeros(16), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    assert np.allclose((y ** 2).mean(-1), 1, atol=1e-13)               # biased variance
    # eps enters under the root: a constant row has variance 0 and maps to the shift
    y, _ = ob.layernorm_fwd(np.full((1, 8), 7.0), np.full(8, 2.0), np.arange(8.0), 1e-5)
    assert np.allclose(y, np.arange(8.0))
    # two-element row (-1, 1): mean 0, var 1 -> values +-1/sqrt(1+eps)
    y, _ = ob.layernorm_fwd(np.array([[-1.0, 1.0]]), np.ones(2), np.zeros(2), 0.25)
    assert np.allclose(y, np.array([[-1, 1]]) / math.sqrt(1.25))


def test_attention_single_key_is_identity():
    rng = np.random.default_rng(2)
    q, k, v = (rng.standard_normal((3, 1, 4)) for _ in range(3))
    o, P = ob.attention_fwd(q, k, v, ob.visibility(ob.MASK_NONE, 1, None))
    assert np.array_equal(P, np.ones((3, 1, 1)))
    assert np.allclose(o, v)


def test_attention_uniform_scores_average_values():
    # q = 0 -> all visible keys get equal probability; causal row i averages v[0..i]
    rng = np.random.default_rng(3)
    s, dh = 6, 4
    k, v = rng.standard_normal((2, s, dh)), rng.standard_normal((2, s, dh))
    q = np.zeros((2, s, dh))
    o, _ = ob.attention_fwd(q, k, v, ob.visibility(ob.MASK_CAUSAL, s, None))
    want = np.cumsum(v, axis=1) / np.arange(1, s + 1)[None, :, None]
    assert np.allclose(o, want, atol=1e-14)
    o, P = ob.attention_fwd(q, k, v, ob.visibility(ob.MASK_PADDING, s, 4))
    assert np.allclose(o, np.broadcast_to(v[:, :4].mean(axis=1, keepdims=True), o.shape), atol=1e-14)
    assert np.all(P[:, :, 4:] == 0.0)                                   # masked keys: exactly zero


def test_attention_score_scale():
    # two keys, scores differ by d: p0/p1 = exp(d / sqrt(dh))
    dh = 16
    q = np.zeros((1, 1, dh)); q[0, 0, 0] = 2.0
    k = np.zeros((1, 2, dh)); k[0, 0, 0] = 3.0
    v = np.zeros((1, 2, dh))
    _, P = ob.attention_fwd(q, k, v, np.ones((1, 2), dtype=bool))
    assert abs(P[0, 0, 0] / P[0, 0, 1] - math.exp(6.0 / 4.0)) < 1e-12


def test_block_mlp_branch_constant_when_w1_zero():
    rng = np.random.default_rng(4)
    h, f, a = 8, 16, 2
    flat = rand_params(rng, 1, h, f)
    p = ob.unflatten(flat, 1, h, f)[0]
    p["w1"][...] = 0.0
    x = rng.standard_normal((2, 3, h))
    y, cache = ob.block_fwd(p, x, None, ob.MASK_NONE, a, 1e-5)
    # x1 recovered from the attention branch alone
    a_ln, _ = ob.layernorm_fwd(x, p["ln1_g"], p["ln1_b"], 1e-5)
    assert np.allclose(cache["a"], a_ln)
    const = ob.gelu(p["b1"]) @ p["w2"] + p["b2"]
    x1 = y - const
    # with s = 1 per sequence the attention output is v itself: check on a second input
    x_s1 = rng.standard_normal((3, 1, h))
    y1, _ = ob.block_fwd(p, x_s1, None, ob.MASK_NONE, a, 1e-5)
    a1, _ = ob.layernorm_fwd(x_s1, p["ln1_g"], p["ln1_b"], 1e-5)
    vproj = a1 @ p["wqkv"][:, 2 * h:] + p["bqkv"][2 * h:]
    assert np.allclose(y1, x_s1 + vproj @ p["wo"] + p["bo"] + const, atol=1e-13)
    assert x1.shape == x.shape


# ----------------------------------------------------------------------------- finite differences

def test_fd_layernorm():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 3, 6))
    g, s = rng.standard_normal(6) + 1, rng.standard_normal(6)
    w = rng.standard_normal((2, 3, 6))
    loss = lambda: float((ob.layernorm_fwd(x, g, s, 1e-5)[0] * w).sum())
    _, saved = ob.layernorm_fwd(x, g, s, 1e-5)
    dx, dg, ds = ob.layernorm_bwd(w, saved, g)
    assert rel(dx, fd_grad(loss, x)) < 1e-7
    assert rel(dg, fd_grad(loss, g)) < 1e-7
    assert rel(ds, fd_grad(loss, s)) < 1e-7


@pytest.mark.parametrize("mask,length", [(ob.MASK_NONE, None), (ob.MASK_CAUSAL, None), (ob.MASK_PADDING, 3)])
def test_fd_attention(mask, length):
    rng = np.random.default_rng(6)
    s, dh = 5, 4
    q, k, v = (rng.standard_normal((2, s, dh)) for _ in range(3))
    w = rng.standard_normal((2, s, dh))
    vis = ob.visibility(mask, s, length)
    loss = lambda: float((ob.attention_fwd(q, k, v, vis)[0] * w).sum())
    _, P = ob.attention_fwd(q, k, v, vis)
    dq, dk, dv = ob.attention_bwd(w, q, k, v, P)
    assert rel(dq, fd_grad(loss, q)) < 1e-7
    assert rel(dk, fd_grad(loss, k)) < 1e-7
    assert rel(dv, fd_grad(loss, v)) < 1e-7


@pytest.mark.parametrize("mask", [ob.MASK_NONE, ob.MASK_CAUSAL, ob.MASK_PADDING])
def test_fd_stage(mask):
    """Whole stage, two layers: every parameter tensor and dX against central differences."""
    rng = np.random.default_rng(7)
    L, h, a, f, s, b = 2, 8, 2, 16, 4, 2
    st = ob.Stage(L, h, a, f, mask)
    w = rand_params(rng, L, h, f)
    x = rng.standard_normal((b, s, h))
    dy = rng.standard_normal((b, s, h))
    lens = np.array([3, 4]) if mask == ob.MASK_PADDING else None
    _, dx, g = st.vjp(w, x, dy, lens)
    loss = lambda: float((st.forward(w, x, lens)[0] * dy).sum())
    assert rel(dx, fd_grad(loss, x)) < 1e-6
    gfd = fd_grad(loss, w)
    assert rel(g, gfd) < 1e-6
    # per tensor, so that a small tensor's error cannot hide behind a large one's norm
    for pl, pf in zip(ob.unflatten(g, L, h, f), ob.unflatten(gfd, L, h, f)):
        for name in pl:
            assert rel(pl[name], pf[name]) < 1e-5, name


# ----------------------------------------------------------------------------- library cross-check

def _torch_block(p, x, lens, mask, n_heads, eps):
    import torch
    import torch.nn.functional as F
    b, s, h = x.shape
    dh = h // n_heads
    a = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], eps)
    qkv = F.linear(a, p["wqkv"].t(), p["bqkv"])
    q, k, v = (z.reshape(b, s, n_heads, dh).permute(0, 2, 1, 3) for z in qkv.split(h, dim=-1))
    sc = q @ k.transpose(-1, -2) / math.sqrt(dh)
    if mask == ob.MASK_CAUSAL:
        sc = sc.masked_fill(torch.triu(torch.ones(s, s, dtype=torch.bool), 1), float("-inf"))
    elif mask == ob.MASK_PADDING:
        dead = torch.arange(s)[None, :] >= torch.as_tensor(lens)[:, None]       # [b, s]
        sc = sc.masked_fill(dead[:, None, None, :], float("-inf"))
    o = torch.softmax(sc, dim=-1) @ v
    o = o.permute(0, 2, 1, 3).reshape(b, s, h)
    x1 = x + F.linear(o, p["wo"].t(), p["bo"])
    c = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], eps)
    u = F.linear(c, p["w1"].t(), p["b1"])
    return x1 + F.linear(F.gelu(u), p["w2"].t(), p["b2"])          # default gelu = erf form


@pytest.mark.parametrize("mask", [ob.MASK_NONE, ob.MASK_CAUSAL, ob.MASK_PADDING])
def test_stage_against_autograd(mask):
    import torch
    rng = np.random.default_rng(8)
    L, h, a, f, s, b = 2, 32, 4, 64, 12, 3
    st = ob.Stage(L, h, a, f, mask)
    w = rand_params(rng, L, h, f, scale=0.2)
    x = rng.standard_normal((b, s, h))
    dy = rng.standard_normal((b, s, h))
    lens = np.array([12, 5, 9]) if mask == ob.MASK_PADDING else None
    y, dx, g = st.vjp(w, x, dy, lens)

    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    z, off = xt, 0
    for _ in range(L):
        p = {}
        for name, shape in ob.layer_shapes(h, f):
            n = int(np.prod(shape))
            p[name] = wt[off:off + n].reshape(shape)
            off += n
        z = _torch_block(p, z, lens, mask, a, 1e-5)
    (z * torch.tensor(dy)).sum().backward()
    assert rel(y, z.detach().numpy()) < 1e-13
    assert rel(dx, xt.grad.numpy()) < 1e-12
    assert rel(g, wt.grad.numpy()) < 1e-12
    for pl, pf in zip(ob.unflatten(g, L, h, f), ob.unflatten(wt.grad.numpy(), L, h, f)):
        for name in pl:
            assert rel(pl[name], pf[name]) < 1e-11, name


# ----------------------------------------------------------------------------- masks

def test_causal_no_flow_from_future():
    rng = np.random.default_rng(9)
    L, h, a, f, s, b = 2, 16, 2, 32, 8, 1
    st = ob.Stage(L, h, a, f, ob.MASK_CAUSAL)
    w = rand_params(rng, L, h, f)
    x = rng.standard_normal((b, s, h))
    y0, _ = st.forward(w, x)
    x2 = x.copy()
    x2[0, 5] += 1.0
    y1, _ = st.forward(w, x2)
    assert np.array_equal(y0[0, :5], y1[0, :5])
    assert not np.allclose(y0[0, 5:], y1[0, 5:])
    # and the gradient wrt x at position j only gathers from positions >= j
    dy = np.zeros((b, s, h)); dy[0, 3] = rng.standard_normal(h)
    _, dx, _ = st.vjp(w, x, dy)
    assert np.all(dx[0, 4:] == 0.0) and np.any(dx[0, :4] != 0.0)


def test_padding_equals_truncated_sequence():
    rng = np.random.default_rng(10)
    L, h, a, f, s = 2, 16, 2, 32, 8
    st = ob.Stage(L, h, a, f, ob.MASK_PADDING)
    w = rand_params(rng, L, h, f)
    x = rng.standard_normal((2, s, h))
    dy = rng.standard_normal((2, s, h))
    lens = np.array([5, 8])
    dy[0, 5:] = 0.0
    y, dx, g = st.vjp(w, x, dy, lens)
    # sequence 0 truncated to its 5 valid tokens, sequence 1 whole, no mask at all
    st0 = ob.Stage(L, h, a, f, ob.MASK_NONE)
    ya, dxa, ga = st0.vjp(w, x[:1, :5], dy[:1, :5])
    yb, dxb, gb = st0.vjp(w, x[1:], dy[1:])
    assert rel(y[0, :5], ya[0]) < 1e-13 and rel(y[1], yb[0]) < 1e-13
    assert rel(dx[0, :5], dxa[0]) < 1e-12 and rel(dx[1], dxb[0]) < 1e-12
    assert np.all(dx[0, 5:] == 0.0)
    assert rel(g, ga + gb) < 1e-12


def test_flat_layout_matches_generator():
    """The oracle's own description of the flat parameter format agrees with the generator's."""
    from paper_2006_09503_amd import synth
    assert [(n, tuple(s)) for n, s in ob.layer_shapes(24, 40)] == \
           [(n, tuple(s)) for n, s in synth.layer_layout(24, 40)]
    cfg = synth.PRESETS["C1"]
    assert ob.n_params(cfg.n_layers, cfg.hidden, cfg.ffn) == synth.param_count(cfg) == 396544
