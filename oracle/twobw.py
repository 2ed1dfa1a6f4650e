"""fp64 CPU oracle: the 2BW schedule, its weight-version rule and its delayed update.

TEST INFRASTRUCTURE ONLY (see oracle/block.py).  Shares no code with the HIP path.

What the paper fixes (Section 3.1):
* microbatch k (1-indexed) runs its forward and its backward on weight version
  max(floor((k-1)/m) - 1, 0), m being the number of microbatches per batch;
* weight gradients of the m microbatches of a batch are accumulated into one coalesced
  gradient, averaged over m, and applied once per batch;
* the update reads the newest weights but a gradient taken one version earlier:
  W(t+1) = W(t) - nu * grad f(W(t-1)); with momentum m_t = beta m_(t-1) + (1-beta) grad f(W(t-1))
  and W(t+1) = W(t) - nu m_t; Adam is treated the same way, with one copy of optimizer state;
* at most two weight versions are alive at a worker at any time (for m >= in-flight depth);
* the flush variant (Section 3.2) keeps one version and has W(t+1) = W(t) - nu grad f(W(t)).

Readings where the paper is silent: the accumulator holds the sum and the update divides
by m; W(-1) := W(0) (forced by the max(., 0) of the version rule); Adam uses bias
correction with step index t+1 and adds eps outside the square root; no weight decay.

Pins (tests/test_oracle_twobw.py): the paper's worked example of the version rule; the
closed form of the delayed recurrence on a scalar quadratic; a hand-unrolled three-step trace;
Adam's closed forms; coalescing m microbatches equals one batch of m*b samples.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np


def weight_version(k: int, m: int) -> int:
    """Version used by microbatch k (1-indexed), forward and backward alike (Section 3.1)."""
    assert k >= 1 and m >= 1
    return max((k - 1) // m - 1, 0)


def weight_version_flush(k: int, m: int) -> int:
    """Flush variant (Section 3.2): every batch runs on the weights the previous update left."""
    assert k >= 1 and m >= 1
    return (k - 1) // m


# ----------------------------------------------------------------------------- optimizers

@dataclass
class Sgd:
    lr: float

    def init(self, w):
        return {}

    def step(self, w, g, state, t):
        """t: index of the batch being applied (0-based).  Returns the next weights."""
        return w - self.lr * g


@dataclass
class Momentum:
    """m_t = beta m_(t-1) + (1 - beta) g;  W <- W - lr m_t  (Section 3.1, no bias correction)."""
    lr: float
    beta: float = 0.9

    def init(self, w):
        return {"m": np.zeros_like(w)}

    def step(self, w, g, state, t):
        state["m"] = self.beta * state["m"] + (1.0 - self.beta) * g
        return w - self.lr * state["m"]


@dataclass
class Adam:
    lr: float
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8

    def init(self, w):
        return {"m": np.zeros_like(w), "v": np.zeros_like(w)}

    def step(self, w, g, state, t):
        state["m"] = self.beta1 * state["m"] + (1.0 - self.beta1) * g
        state["v"] = self.beta2 * state["v"] + (1.0 - self.beta2) * g * g
        mhat = state["m"] / (1.0 - self.beta1 ** (t + 1))
        vhat = state["v"] / (1.0 - self.beta2 ** (t + 1))
        return w - self.lr * mhat / (np.sqrt(vhat) + self.eps)


# ----------------------------------------------------------------------------- replay

@dataclass
class Trace:
    """Everything a replay produced, for element-wise comparison."""
    Y: Dict[int, np.ndarray] = field(default_factory=dict)        # per microbatch id k
    dX: Dict[int, np.ndarray] = field(default_factory=dict)
    version_used: Dict[int, int] = field(default_factory=dict)
    G: List[np.ndarray] = field(default_factory=list)             # coalesced sum, per batch
    W: List[np.ndarray] = field(default_factory=list)             # W[t], t = 0..n
    opt_state: List[Dict[str, np.ndarray]] = field(default_factory=list)   # after each update
    max_live_versions: int = 0


def replay(vjp: Callable, w0: np.ndarray, microbatches: Sequence, m: int, optimizer,
           inflight: int = 1, version_rule: Callable[[int, int], int] = weight_version) -> Trace:
    """Run a stage through len(microbatches)/m batches under the 1F1B order of one worker.

    vjp(W, *microbatches[k-1]) -> (Y_k, dX_k, g_k).
    inflight = p: the forward of microbatch k is issued p - 1 microbatches before its backward,
    as on a stage that has p inputs in flight; the backward then uses the weights tagged at
    the forward.  The numbers do not depend on p.
    Versions are kept in a dict and dropped as soon as no present or future microbatch can
    read them; the peak count is recorded so the two-version claim can be checked.
    """
    n_mb = len(microbatches)
    assert n_mb % m == 0 and 1 <= inflight <= m
    tr = Trace()
    w0 = np.asarray(w0, dtype=np.float64)
    live = {0: w0}                      # version id -> weights
    tr.W.append(w0)
    state = optimizer.init(w0)
    t = 0                               # updates applied so far; newest version id
    G = np.zeros_like(w0)
    n_acc = 0
    pending = {}                        # k -> (version tag, result of the vjp)

    def do_forward(k):
        ver = version_rule(k, m)
        assert ver in live, f"microbatch {k} needs version {ver}, live: {sorted(live)}"
        # The forward and the backward of k see the same weights, so evaluating both here,
        # at the forward's place in the order, gives what a split evaluation would.
        y, dx, g = vjp(live[ver], *microbatches[k - 1])
        tr.Y[k], tr.version_used[k] = y, ver
        pending[k] = (ver, dx, g)

    def do_backward(k):
        nonlocal G, n_acc, t, state
        ver, dx, g = pending.pop(k)
        tr.dX[k] = dx
        G = G + g
        n_acc += 1
        if n_acc == m:
            tr.G.append(G)
            w_next = optimizer.step(live[t], G / m, state, t)
            t += 1
            live[t] = w_next
            tr.W.append(w_next)
            tr.opt_state.append({k_: v.copy() for k_, v in state.items()})
            G = np.zeros_like(w0)
            n_acc = 0
            # drop versions no in-flight or future microbatch reads
            first_future = k + 1 + len(pending)
            needed = {tag for tag, _, _ in pending.values()}
            needed.add(version_rule(first_future, m))
            needed.add(t)               # the newest is read by the next update
            for vid in [vid for vid in live if vid < min(needed)]:
                del live[vid]
        tr.max_live_versions = max(tr.max_live_versions, len(live))

    for k in range(1, n_mb + 1):
        if k > inflight:
            do_backward(k - inflight)
        do_forward(k)
    for k in range(max(n_mb - inflight, 0) + 1, n_mb + 1):
        do_backward(k)
    return tr
