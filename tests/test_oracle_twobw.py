"""Pins for oracle/twobw.py (CPU only).

* the version rule against the paper's worked example (tests/golden/version_rule_m4.txt);
* the delayed recurrence W(t+1) = W(t) - nu grad f(W(t-1)) in closed form on a scalar
  quadratic, and the vanilla recurrence of the flush variant beside it;
* a three-update trace of a tiny stage unrolled by hand (no replay loop, its own Adam);
* coalescing m microbatches of b samples equals one batch of m*b samples;
* Adam's closed forms; at most two live versions; independence of the in-flight depth;
* planted mistakes (wrong version, missing 1/m, update from the wrong buffer) move the
  result by far more than the parity tolerances, so the parity tests can see them.
"""
import os

import numpy as np
import pytest

from oracle import block as ob
from oracle import twobw as tb
from paper_2006_09503_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


# ----------------------------------------------------------------------------- version rule

def test_version_rule_paper_example():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "version_rule_m4.txt")) if l[0] != "#"]
    assert len(rows) == 9
    for k, v in rows:
        assert tb.weight_version(int(k), 4) == int(v)


def test_version_rule_properties():
    for m in (1, 2, 4, 7, 16):
        vs = [tb.weight_version(k, m) for k in range(1, 8 * m + 1)]
        assert vs[:2 * m] == [0] * (2 * m)                 # batches 0 and 1 run on the initial weights
        assert all(b - a in (0, 1) for a, b in zip(vs, vs[1:]))
        for t in range(2, 8):
            assert set(vs[t * m:(t + 1) * m]) == {t - 1}   # batch t reads the 1-stale version
        # any m consecutive ids (an in-flight window) span at most two versions
        assert all(len(set(vs[i:i + m])) <= 2 for i in range(len(vs) - m))
        assert [tb.weight_version_flush(k, m) for k in range(1, 3 * m + 1)] == \
               [0] * m + [1] * m + [2] * m


# ----------------------------------------------------------------------------- delayed recurrence

def _quadratic_vjp(c):
    # f(w) = c w^2 / 2 per microbatch; "Y" and "dX" are unused here
    return lambda w, *_: (None, None, c * w)


def test_delay1_recurrence_scalar_closed_form():
    """nu*c = 0.1, w0 = 1: delayed gives 0.9, 0.8, 0.71; vanilla gives 0.9, 0.81, 0.729."""
    c, nu, m = 2.0, 0.05, 3
    mbs = [()] * (3 * m)
    tr = tb.replay(_quadratic_vjp(c), np.array([1.0]), mbs, m, tb.Sgd(nu))
    assert np.allclose([w[0] for w in tr.W], [1.0, 0.9, 0.8, 0.71], atol=1e-15)
    tr = tb.replay(_quadratic_vjp(c), np.array([1.0]), mbs, m, tb.Sgd(nu),
                   version_rule=tb.weight_version_flush)
    assert np.allclose([w[0] for w in tr.W], [1.0, 0.9, 0.81, 0.729], atol=1e-15)


def test_delay1_recurrence_long_run_matches_linear_recursion():
    # w(t+1) = w(t) - a w(t-1), a = nu c: iterate the two-term recursion directly
    a, n, m = 0.07, 25, 2
    want = [1.0, 1.0 - a]
    for _ in range(n - 1):
        want.append(want[-1] - a * want[-2])
    tr = tb.replay(_quadratic_vjp(1.0), np.array([1.0]), [()] * (n * m), m, tb.Sgd(a))
    assert np.allclose([w[0] for w in tr.W], want, atol=1e-14)


def test_momentum_uses_stale_gradient_single_state():
    # beta = 0.5, nu = 0.2, c = 1, w0 = 1:
    # g0 = 1 (at W0): m1 = .5        W1 = 1 - .2*.5   = 0.9
    # g1 = 1 (at W0): m2 = .25+.5=.75 W2 = .9 - .15   = 0.75
    # g2 = .9 (at W1): m3 = .375+.45  W3 = .75 - .165 = 0.585
    tr = tb.replay(_quadratic_vjp(1.0), np.array([1.0]), [()] * 3, 1, tb.Momentum(0.2, 0.5))
    assert np.allclose([w[0] for w in tr.W], [1.0, 0.9, 0.75, 0.585], atol=1e-15)
    assert np.allclose([s["m"][0] for s in tr.opt_state], [0.5, 0.75, 0.825], atol=1e-15)


# ----------------------------------------------------------------------------- Adam closed forms

def test_adam_first_step_closed_form():
    rng = np.random.default_rng(0)
    w, g = rng.standard_normal(50), rng.standard_normal(50) * 1e-3
    opt = tb.Adam(1e-3, 0.9, 0.999, 1e-8)
    st = opt.init(w)
    w1 = opt.step(w, g, st, 0)
    assert np.allclose(w1 - w, -1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-12, atol=0)
    assert np.allclose(st["m"], 0.1 * g) and np.allclose(st["v"], 0.001 * g * g)


def test_adam_constant_gradient_and_sign_limit():
    g = np.array([0.3, -2.0, 1e-4])
    opt = tb.Adam(0.01, 0.9, 0.999, 0.0)
    st, w = opt.init(g), np.zeros(3)
    for t in range(6):
        w = opt.step(w, g, st, t)
        # bias-corrected moments equal g and g^2 at every step -> each step moves by lr*sign(g)
        assert np.allclose(w, -0.01 * (t + 1) * np.sign(g), rtol=1e-12)
    opt = tb.Adam(0.5, 0.0, 0.0, 0.0)                                   # beta = 0: sign descent
    st = opt.init(g)
    assert np.allclose(opt.step(np.zeros(3), g, st, 3), -0.5 * np.sign(g))


def test_adam_eps_outside_root():
    # g = 0 -> update exactly 0 (0/(0+eps)); tiny g: step = lr*g/(|g|+eps)
    opt = tb.Adam(1.0, 0.9, 0.999, 1e-8)
    g = np.array([0.0, 1e-8])
    w1 = opt.step(np.zeros(2), g, opt.init(g), 0)
    assert w1[0] == 0.0 and abs(w1[1] + 0.5) < 1e-12


# ----------------------------------------------------------------------------- tiny stage

def tiny():
    cfg = synth.StageConfig(n_layers=2, hidden=16, n_heads=2, ffn=32, seq=6, microbatch=2, m=3,
                            max_inflight=2, mask_mode=synth.MASK_CAUSAL, lr=1e-2)
    gen = synth.StageInputs(cfg, seed=3)
    w0 = gen.weights().astype(np.float64)
    st = ob.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.mask_mode, cfg.ln_eps)
    return cfg, gen, w0, st


def test_three_step_trace_unrolled_by_hand():
    cfg, gen, w0, st = tiny()
    m = cfg.m
    mbs = gen.microbatches(3 * m)
    vjp = lambda w, x, dy, lens: st.vjp(w, x, dy, lens)
    tr = tb.replay(vjp, w0, mbs, m, tb.Adam(cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps), inflight=2)

    def batch_grad(w, t):                       # mean over the m microbatches of batch t
        return sum(st.vjp(w, *mbs[t * m + j])[2] for j in range(m)) / m

    b1, b2, eps, lr = cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.lr
    g0 = batch_grad(w0, 0)                      # batch 0 on W(0)
    M1 = (1 - b1) * g0
    V1 = (1 - b2) * g0 ** 2
    W1 = w0 - lr * (M1 / (1 - b1)) / (np.sqrt(V1 / (1 - b2)) + eps)
    g1 = batch_grad(w0, 1)                      # batch 1 still on W(0): W(-1) := W(0)
    M2 = b1 * M1 + (1 - b1) * g1
    V2 = b2 * V1 + (1 - b2) * g1 ** 2
    W2 = W1 - lr * (M2 / (1 - b1 ** 2)) / (np.sqrt(V2 / (1 - b2 ** 2)) + eps)
    g2 = batch_grad(W1, 2)                      # batch 2 on W(1), applied to W(2)
    M3 = b1 * M2 + (1 - b1) * g2
    V3 = b2 * V2 + (1 - b2) * g2 ** 2
    W3 = W2 - lr * (M3 / (1 - b1 ** 3)) / (np.sqrt(V3 / (1 - b2 ** 3)) + eps)

    for got, want in zip(tr.W, [w0, W1, W2, W3]):
        assert rel(got, want) < 1e-14
    for got, want in zip(tr.G, [g0 * m, g1 * m, g2 * m]):
        assert rel(got, want) < 1e-13
    assert rel(tr.opt_state[2]["m"], M3) < 1e-13 and rel(tr.opt_state[2]["v"], V3) < 1e-13
    assert [tr.version_used[k] for k in range(1, 3 * m + 1)] == [0] * (2 * m) + [1] * m
    assert tr.max_live_versions <= 2


def test_coalesced_microbatches_equal_one_large_batch():
    cfg, gen, w0, st = tiny()
    m = 4
    mbs = gen.microbatches(m)
    G = sum(st.vjp(w0, *mb)[2] for mb in mbs)
    xs = np.concatenate([mb[0] for mb in mbs], axis=0).astype(np.float64)
    dys = np.concatenate([mb[1] for mb in mbs], axis=0).astype(np.float64)
    y_big, dx_big, g_big = st.vjp(w0, xs, dys / m)
    assert rel(G / m, g_big) < 1e-13
    b = cfg.microbatch
    for j, mb in enumerate(mbs):
        y, dx, _ = st.vjp(w0, *mb)
        assert rel(y, y_big[j * b:(j + 1) * b]) < 1e-14
        assert rel(dx / m, dx_big[j * b:(j + 1) * b]) < 1e-13


def test_batches_zero_and_one_share_initial_weights():
    cfg, gen, w0, st = tiny()
    m = cfg.m
    first = gen.microbatches(m)
    mbs = first + first + gen.microbatches(m)
    tr = tb.replay(lambda w, *mb: st.vjp(w, *mb), w0, mbs, m, tb.Adam(cfg.lr))
    assert np.array_equal(tr.G[0], tr.G[1])
    for j in range(1, m + 1):
        assert np.array_equal(tr.Y[j], tr.Y[m + j]) and np.array_equal(tr.dX[j], tr.dX[m + j])


def test_inflight_depth_does_not_change_results_and_two_versions_suffice():
    cfg, gen, w0, st = tiny()
    m = cfg.m
    mbs = gen.microbatches(4 * m)
    vjp = lambda w, *mb: st.vjp(w, *mb)
    ref = tb.replay(vjp, w0, mbs, m, tb.Adam(cfg.lr), inflight=1)
    for p in (2, m):
        tr = tb.replay(vjp, w0, mbs, m, tb.Adam(cfg.lr), inflight=p)
        assert tr.max_live_versions <= 2
        for a_, b_ in zip(tr.W, ref.W):
            assert np.array_equal(a_, b_)
        for k in ref.Y:
            assert np.array_equal(tr.Y[k], ref.Y[k]) and np.array_equal(tr.dX[k], ref.dX[k])


def test_padding_lengths_reach_the_stage():
    cfg = synth.StageConfig(1, 16, 2, 32, 8, 3, 2, 2, synth.MASK_PADDING, min_len=3)
    gen = synth.StageInputs(cfg, seed=1)
    w0 = gen.weights().astype(np.float64)
    x, dy, lens = gen.microbatch()
    assert lens.shape == (3,) and lens.min() >= 3 and lens.max() <= 8
    assert all(np.all(dy[n, lens[n]:] == 0) for n in range(3))
    st = ob.Stage(1, 16, 2, 32, cfg.mask_mode)
    _, dx, _ = st.vjp(w0, x, dy, lens)
    assert all(np.all(dx[n, lens[n]:] == 0) for n in range(3))


# ----------------------------------------------------------------------------- planted mistakes

def test_parity_metrics_see_planted_mistakes():
    """Each wrong variant must sit far outside the bar of the parity test that guards it.

    A wrong weight version changes the coalesced gradient by about |W(1) - W(0)| / |W|, i.e.
    roughly lr / 0.02 per step: at lr = 1e-3 that is ~1e-2, a hundred times the fp32 bar (1e-4)
    but inside the bf16 bar (2e-2); the bf16 version test therefore runs at lr = 2e-2.
    """
    cfg, gen, w0, st = tiny()
    m = cfg.m
    mbs = gen.microbatches(3 * m)
    vjp = lambda w, *mb: st.vjp(w, *mb)
    good = tb.replay(vjp, w0, mbs, m, tb.Adam(1e-3))
    # (1) newest version instead of the 1-stale one: shows in G of batches 1 and 2
    flush = tb.replay(vjp, w0, mbs, m, tb.Adam(1e-3), version_rule=tb.weight_version_flush)
    assert rel(flush.G[1], good.G[1]) > 50 * 1e-4 and rel(flush.G[2], good.G[2]) > 50 * 1e-4
    good_hi = tb.replay(vjp, w0, mbs, m, tb.Adam(2e-2))
    flush_hi = tb.replay(vjp, w0, mbs, m, tb.Adam(2e-2), version_rule=tb.weight_version_flush)
    assert rel(flush_hi.G[1], good_hi.G[1]) > 5 * 2e-2 and rel(flush_hi.G[2], good_hi.G[2]) > 5 * 2e-2
    # (2) forgetting the 1/m: Adam is scale-free at step 1 (only eps sees it), so look at m, v
    class NoMean(tb.Adam):
        def step(self, w, g, state, t):
            return super().step(w, g * m, state, t)
    nomean = tb.replay(vjp, w0, mbs, m, NoMean(1e-3))
    assert rel(nomean.opt_state[0]["v"], good.opt_state[0]["v"]) > 1.0
    assert rel(nomean.opt_state[0]["m"], good.opt_state[0]["m"]) > 1.0
    # (3) update applied to W(t-1) instead of W(t): shows in dW of the second update, while the
    # raw weights move by only ~lr/0.02 -- compare dW, not W
    dW_good = good.W[2] - good.W[1]
    assert rel(good.W[2] - good.W[0], dW_good) > 0.5
    assert rel(good.W[0] + dW_good, good.W[2]) < 2e-1


# ----------------------------------------------------------------------------- the composition, against library routines

@pytest.mark.parametrize("mask", [ob.MASK_CAUSAL, ob.MASK_PADDING])
def test_whole_stage_under_2bw_against_autograd_and_torch_adam(mask):
    """The composition itself -- a transformer stage trained under the version rule with coalescing and
    Adam -- against an implementation that shares nothing with the oracle: the block written with torch
    functions, gradients from autograd, the update from torch.optim.Adam, and the delay written out as in
    Section 3.1: the gradient of batch t is taken at W(t-1) (W(0) for the first two batches), averaged over
    the m microbatches, and applied to W(t)."""
    import torch
    from test_oracle_block import _torch_block, rand_params
    rng = np.random.default_rng(21)
    L, h, a, f, s, b, m, n_batches = 2, 32, 4, 64, 10, 2, 3, 5
    lr = 1e-2
    st = ob.Stage(L, h, a, f, mask)
    w0 = rand_params(rng, L, h, f, scale=0.2)
    mbs = []
    for _ in range(m * n_batches):
        x, dy = rng.standard_normal((b, s, h)), rng.standard_normal((b, s, h))
        lens = rng.integers(3, s + 1, size=b) if mask == ob.MASK_PADDING else None
        mbs.append((x, dy, lens))
    tr = tb.replay(lambda w, x, dy, lens: st.vjp(w, x, dy, lens), w0, mbs, m, tb.Adam(lr), inflight=2)

    def grad_at(w, x, dy, lens):
        wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
        z, off = torch.tensor(x, dtype=torch.float64), 0
        for _ in range(L):
            p = {}
            for name, shape in ob.layer_shapes(h, f):
                n = int(np.prod(shape))
                p[name] = wt[off:off + n].reshape(shape)
                off += n
            z = _torch_block(p, z, lens, mask, a, 1e-5)
        (z * torch.tensor(dy)).sum().backward()
        return wt.grad.numpy()

    W = [np.array(w0)]
    newest = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.Adam([newest], lr=lr, betas=(0.9, 0.999), eps=1e-8)
    for t in range(n_batches):
        stale = W[max(t - 1, 0)]
        g = sum(grad_at(stale, *mbs[t * m + j]) for j in range(m)) / m
        newest.grad = torch.tensor(g)
        opt.step()
        W.append(newest.detach().numpy().copy())
    # Adam's quotient mhat / (sqrt(vhat) + eps) is +-1 on the first step wherever |g| >> eps, and entries with
    # |g| near eps carry the gradients' rounding (1e-16 relative to the largest entry) at full size: 1e-8 is
    # far above that and far below what any mistake in the rule would give (compared below).
    for t in range(n_batches + 1):
        assert rel(tr.W[t], W[t]) < 1e-8, t
    # what the bar separates: one update more or less is five orders of magnitude away, and so is a replay
    # with a mistake planted in the rule (no delay; the delay one batch too long)
    assert rel(W[2], W[1]) > 1e-3
    for wrong in (lambda k, m_: (k - 1) // m_, lambda k, m_: max((k - 1) // m_ - 2, 0)):
        bad = tb.replay(lambda w, x, dy, lens: st.vjp(w, x, dy, lens), w0, mbs, m, tb.Adam(lr), inflight=1,
                        version_rule=wrong)
        assert max(rel(bad.W[t], W[t]) for t in range(n_batches + 1)) > 1e-4
