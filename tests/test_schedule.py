"""The library's 2BW bookkeeping (host only) against the paper's rule and the oracle's replay."""
import numpy as np
import pytest

from oracle import twobw as tb
from paper_2006_09503_amd import binding as B


def drive(m, p, n_batches):
    """1F1B order of one worker; returns the log of (event, k, version, buffer)."""
    s = B.Sched(m, p)
    log = []
    n = n_batches * m
    def back(k):
        rc, slot, ver, buf, first = s.backward(k)
        assert rc == 0, (k, rc)
        assert first == (1 if (k - 1) % m == 0 else 0)
        log.append(("B", k, ver, buf))
        if k % m == 0:
            t = s.query(B.Q_UPDATES)
            rc, rb, wb, step = s.coalesce_update()
            assert rc == 0 and step == t + 1
            assert rb == t % 2 and wb == (t + 1) % 2          # reads W(t), writes the other buffer
            log.append(("U", step, rb, wb))
    for k in range(1, n + 1):
        if k > p:
            back(k - p)
        if (k - 1) % m == 0 and (k - 1) // m >= 2:
            assert s.swap_versions() == 0
        rc, slot, ver, buf = s.forward(k)
        assert rc == 0, (k, rc)
        assert s.query(B.Q_INFLIGHT) <= p
        log.append(("F", k, ver, buf))
    for k in range(n - p + 1, n + 1):
        back(k)
    assert s.query(B.Q_INFLIGHT) == 0 and s.query(B.Q_UPDATES) == n_batches
    s.close()
    return log


@pytest.mark.parametrize("m,p", [(4, 4), (4, 1), (4, 2), (8, 4), (3, 3), (1, 1), (16, 4)])
def test_1f1b_order_follows_version_rule(m, p):
    log = drive(m, p, 6)
    fwd = {k: (v, b) for e, k, v, b in log if e == "F"}
    bwd = {k: (v, b) for e, k, v, b in log if e == "B"}
    for k in fwd:
        assert fwd[k][0] == tb.weight_version(k, m)           # Section 3.1 rule
        assert bwd[k] == fwd[k]                               # same version for both passes
        assert fwd[k][1] == fwd[k][0] % 2
    # no update overwrites a buffer that a microbatch in flight still reads
    inflight = {}
    for e, k, a, b in log:
        if e == "F":
            inflight[k] = b
        elif e == "B":
            del inflight[k]
        else:
            assert b not in inflight.values(), (k, inflight)


def test_paper_example_m4_d4():
    """m = d = 4: inputs 1..8 on version 0; the version made after input 4 is first used by input
    9; version 0's buffer is overwritten only after the backward of input 8 (Section 3.1)."""
    log = drive(4, 4, 4)
    assert [v for e, k, v, b in log if e == "F"][:9] == [0] * 8 + [1]
    idx_b8 = log.index(("B", 8, 0, 0))
    second_update = [i for i, ev in enumerate(log) if ev[0] == "U" and ev[1] == 2][0]
    assert second_update == idx_b8 + 1 and log[second_update] == ("U", 2, 1, 0)


def test_schedule_violations_are_refused():
    s = B.Sched(2, 2)
    assert s.coalesce_update()[0] == B.ERR_BAD_STATE          # nothing accumulated
    assert s.swap_versions() == B.ERR_BAD_STATE               # nothing newer
    assert s.backward(1)[0] == B.ERR_BAD_STATE                # not in flight
    assert s.forward(0)[0] == B.ERR_INVALID_ARG
    assert s.forward(1)[0] == 0
    assert s.forward(1)[0] == B.ERR_BAD_STATE                 # already in flight
    assert s.forward(2)[0] == 0
    assert s.forward(3)[0] == B.ERR_BAD_STATE                 # no free stash slot
    assert s.backward(1)[0] == 0
    assert s.coalesce_update()[0] == B.ERR_BAD_STATE          # 1 of 2 accumulated
    assert s.forward(3)[0] == 0                               # batch 1 still reads version 0
    assert s.backward(3)[0] == B.ERR_BAD_STATE                # batch 1 before batch 0 is complete
    assert s.backward(2)[0] == 0
    assert s.backward(3)[0] == B.ERR_BAD_STATE                # full batch waits for its update
    assert s.coalesce_update()[:3] == (0, 0, 1)
    assert s.forward(5)[0] == B.ERR_BAD_STATE                 # needs version 1: swap first
    assert s.forward(4)[0] == 0
    assert s.backward(3)[0] == 0 and s.backward(4)[0] == 0
    assert s.coalesce_update()[:3] == (0, 1, 0)               # W(2) overwrites buffer 0
    assert s.forward(5)[0] == B.ERR_BAD_STATE                 # version 0 is dead and 5 needs version 1
    assert s.swap_versions() == 0
    rc, slot, ver, buf = s.forward(5)
    assert (rc, ver, buf) == (0, 1, 1)
    assert s.forward(7)[0] == B.ERR_BAD_STATE                 # runs ahead: needs version 2
    assert s.swap_versions() == 0                             # r = 2 = t
    assert s.swap_versions() == B.ERR_BAD_STATE
    assert s.forward(6)[0] == B.ERR_BAD_STATE                 # 6 needs version 1, r moved on
    s.close()


def test_update_refused_while_shadow_version_in_flight():
    # contrived: in-flight depth equal to m, but the driver swaps late
    s = B.Sched(2, 2)
    for k in (1, 2):
        assert s.forward(k)[0] == 0
    for k in (1, 2):
        assert s.backward(k)[0] == 0
    assert s.coalesce_update()[0] == 0                        # t = 1
    for k in (3, 4):
        assert s.forward(k)[0] == 0                           # version 0, buffer 0
    assert s.backward(3)[0] == 0
    # 4 is still in flight on version 0; a second update would need n_acc == 2 -> refused anyway
    assert s.coalesce_update()[0] == B.ERR_BAD_STATE
    assert s.backward(4)[0] == 0
    assert s.coalesce_update()[:3] == (0, 1, 0)
    s.close()


def test_matches_oracle_replay_versions():
    m, p, nb = 3, 2, 5
    log = drive(m, p, nb)
    used = {k: v for e, k, v, b in log if e == "F"}
    tr = tb.replay(lambda w, *_: (None, None, w * 0), np.zeros(1), [()] * (m * nb), m, tb.Sgd(0.1), inflight=p)
    assert used == tr.version_used


@pytest.mark.parametrize("m,p", [(4, 4), (4, 2), (3, 1), (8, 4)])
def test_flush_variant_keeps_one_version_and_drains_every_batch(m, p):
    """Section 3.2: microbatch k runs on version floor((k-1)/m); the next batch cannot start before
    the update; one buffer; no swap."""
    s = B.Sched(m, p, flush=True)
    for b in range(4):
        first = b * m + 1
        # the whole batch in 1F1B order, drained at its end
        for k in range(first, first + m):
            if k - p >= first:
                rc, slot, ver, buf, is_first = s.backward(k - p)
                assert rc == 0 and ver == b and buf == 0 and is_first == (1 if k - p == first else 0)
            rc, slot, ver, buf = s.forward(k)
            assert rc == 0 and ver == tb.weight_version_flush(k, m) == b and buf == 0
        # a forward pass of the next batch is refused while this batch's update is outstanding
        assert s.forward(first + m)[0] == B.ERR_BAD_STATE
        assert s.coalesce_update()[0] == B.ERR_BAD_STATE          # backward passes still missing
        for k in range(max(first + m - p, first), first + m):
            rc, slot, ver, buf, _ = s.backward(k)
            assert rc == 0 and ver == b and buf == 0
        assert s.query(B.Q_INFLIGHT) == 0
        rc, rb, wb, step = s.coalesce_update()
        assert rc == 0 and rb == 0 and wb == 0 and step == b + 1   # in place
        assert s.query(B.Q_READ_VERSION) == b + 1                  # current at once
        assert s.swap_versions() == B.ERR_BAD_STATE
    s.close()
