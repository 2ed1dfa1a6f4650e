"""The planner (host only): the library's cost functions and sweep against the brute-force oracle,
and the oracle against hand-computed values of the appendix's closed forms."""
import numpy as np
import pytest

from oracle import planner as op
from paper_2006_09503_amd import binding as B


def profile(**kw):
    base = dict(n_blocks=24, n_gpus=8, gpus_per_server=8, microbatch_sizes=[1, 2, 4, 8],
                block_time_s=[1.0e-3, 1.8e-3, 3.4e-3, 6.6e-3], weight_bytes=600e6, state_bytes=0.0,
                act_bytes_per_sample=480e6, input_bytes_per_sample=1e6, boundary_bytes_per_sample=2e6,
                bw_high=100e9, bw_low=10e9, memory_capacity=16e9, global_batch=64, c_extra=4.0 / 3.0)
    base.update(kw)
    return op.Profile(**base)


def test_oracle_cost_functions_match_hand_computation():
    """Appendix closed forms with the numbers plugged in by hand."""
    p = profile()
    # d=4, w=2, b=4, pipelined: 6 blocks/stage * 3.4 ms = 20.4 ms compute; boundary 2*2e6*4/100e9 = 0.16 ms;
    # all-reduce 2*(1/2)*(600e6/4)/100e9 = 1.5 ms every m = 64/(2*4) = 8 microbatches -> 0.1875 ms.
    t = 20.4e-3 + 0.16e-3
    assert op.throughput(p, 2, 4, 4, op.PIPELINE) == pytest.approx(2 * 4 / t, rel=1e-12)
    # without pipelining the 4 stages run one after the other
    assert op.throughput(p, 2, 4, 4, op.NO_PIPELINE) == pytest.approx(2 * 4 / (4 * t), rel=1e-12)
    # recomputation: compute * 4/3, communication unchanged
    assert op.throughput(p, 2, 4, 4, op.PIPELINE_RECOMPUTE) == pytest.approx(8 / (20.4e-3 * 4 / 3 + 0.16e-3), rel=1e-12)
    # MEMORY: 2|W|/d + d|A_total|/d + d|A_input|  and  2|W|/d + |A_total|/d + d|A_input|
    assert op.memory(p, 2, 4, 4, op.PIPELINE) == pytest.approx(2 * 600e6 / 4 + 480e6 * 4 + 4 * 1e6 * 4)
    assert op.memory(p, 2, 4, 4, op.PIPELINE_RECOMPUTE) == pytest.approx(2 * 600e6 / 4 + 480e6 * 4 / 4 + 4 * 1e6 * 4)
    assert op.memory(p, 2, 4, 4, op.NO_PIPELINE) == pytest.approx(600e6 / 4 + 480e6 * 4 / 4)
    # one GPU: no communication at all, throughput = b / (blocks * block time)
    assert op.throughput(p, 1, 1, 8, op.PIPELINE) == pytest.approx(8 / (24 * 6.6e-3))


def test_oracle_all_reduce_bound_and_server_boundary():
    # communication-bound replica: tiny compute, big weights, one microbatch per update
    p = profile(block_time_s=[1e-6, 2e-6, 4e-6, 8e-6], global_batch=8, weight_bytes=8e9)
    t_ar = 2 * (7 / 8) * 8e9 / 100e9
    assert op.throughput(p, 8, 1, 1, op.PIPELINE) == pytest.approx(8 * 1 / t_ar)       # m(b) = 1
    # 16 GPUs in servers of 8: w=2, d=8 keeps each pipeline in a server (stage traffic fast, all-reduce slow) or
    # the stage replicas together (all-reduce fast, stage traffic slow); the better orientation counts
    q = profile(n_gpus=16, global_batch=64)
    t_depth_inside = max(3 * 3.4e-3 + 2 * 2e6 * 4 / 100e9, (2 * 0.5 * 600e6 / 8 / 10e9) / 8)
    t_width_inside = max(3 * 3.4e-3 + 2 * 2e6 * 4 / 10e9, (2 * 0.5 * 600e6 / 8 / 100e9) / 8)
    assert op.throughput(q, 2, 8, 4, op.PIPELINE) == pytest.approx(8 / min(t_depth_inside, t_width_inside))


def test_oracle_partition_prefers_what_fits():
    # memory so small that only recomputation (or a deep pipeline) fits the larger microbatches
    p = profile(memory_capacity=1.5e9)
    w, d, b, mode, g, thr, mem = op.partition(p)
    assert mem <= 1.5e9 and w * d <= 8 and 24 % d == 0 and g == 64 // (w * d * b)
    # nothing can beat the sum of all GPUs' compute
    assert thr <= 8 * max(bb / (24 * t) for bb, t in zip(p.microbatch_sizes, p.block_time_s)) * (1 + 1e-12)
    # more memory never lowers the optimum
    assert op.partition(profile(memory_capacity=64e9))[5] >= thr


def tiny(**kw):
    """Two GPUs in one server, two blocks, b in {1, 2}, B = 4; sizes in bytes, bandwidth in bytes/s."""
    base = dict(n_blocks=2, n_gpus=2, gpus_per_server=2, microbatch_sizes=[1, 2], block_time_s=[1.0, 1.6],
                weight_bytes=8.0, state_bytes=0.0, act_bytes_per_sample=6.0, input_bytes_per_sample=1.0,
                boundary_bytes_per_sample=1.0, bw_high=8.0, bw_low=8.0, memory_capacity=100.0, global_batch=4,
                c_extra=4.0 / 3.0)
    base.update(kw)
    return op.Profile(**base)


NO, PIPE, RECOMP = op.NO_PIPELINE, op.PIPELINE, op.PIPELINE_RECOMPUTE


def test_oracle_partition_hand_worked_sweep():
    """The whole sweep of the partitioning algorithm on a profile small enough to do on paper.

    (w, d) in {(1,1), (1,2), (2,1)}, b in {1, 2}; g = 4/(w d b) is whole for all six.
    THROUGHPUT (appendix), samples/s = w b / t:
      (1,1): no communication, t = 2 blocks * time(b) = 2 | 3.2          -> 0.5 | 0.625; recompute t*4/3 -> 0.375 | 0.46875
      (1,2): t = 1 block + 2*1*b/8 = 1.25 | 2.1                          -> 0.8 | 0.95238 pipelined,
             the two stages in turn without pipelining                   -> 0.4 | 0.47619,
             recompute 4/3 + 0.25 = 1.58333 | 2.13333 + 0.5 = 2.63333    -> 0.63158 | 0.75949
      (2,1): all-reduce 2*(1/2)*8/8 = 1 s every m = 4/(2b) = 2 | 1 microbatches = 0.5 | 1 s < compute 2 | 3.2
                                                                         -> 1.0 | 1.25; recompute -> 0.75 | 0.9375
    MEMORY (appendix; without pipelining one version and one activation set), order none / pipelined / recompute:
      d=1: 8+6b | 16+6b+b | 16+6b+b = 14, 23, 23 (b=1); 20, 30, 30 (b=2)
      d=2: 4+3b | 8+6b+2b | 8+3b+2b = 7, 16, 13 (b=1); 10, 24, 18 (b=2)
    """
    # the cost functions at the hand-computed points
    assert op.throughput(tiny(), 1, 2, 2, PIPE) == pytest.approx(2 / 2.1)
    assert op.throughput(tiny(), 1, 2, 1, RECOMP) == pytest.approx(1 / (4 / 3 + 0.25))
    assert op.throughput(tiny(), 2, 1, 2, NO) == pytest.approx(1.25)
    assert [op.memory(tiny(), 1, 2, b, mode) for b in (1, 2) for mode in (NO, PIPE, RECOMP)] == [7, 16, 13, 10, 24, 18]
    assert [op.memory(tiny(), 2, 1, b, mode) for b in (1, 2) for mode in (NO, PIPE, RECOMP)] == [14, 23, 23, 20, 30, 30]
    # everything fits: two replicas at the larger microbatch (the first of the two tied modes at d = 1)
    assert op.partition(tiny()) == pytest.approx((2, 1, 2, NO, 1, 1.25, 20.0))
    # M = 19 rules out b = 2 at d = 1 (20) and the pipelined (1,2,2) (24): replicas at b = 1
    assert op.partition(tiny(memory_capacity=19.0)) == pytest.approx((2, 1, 1, NO, 2, 1.0, 14.0))
    # M = 13.5 leaves only d = 2: none 7 | 10 (0.4 | 0.476) and recompute at b = 1 (13, 0.63158).  Dropping the
    # recompute mode would give (1,2,2,none); a sweep of d that stops below N/w would find nothing
    assert op.partition(tiny(memory_capacity=13.5)) == pytest.approx((1, 2, 1, RECOMP, 2, 1 / (4 / 3 + 0.25), 13.0))
    # nothing fits below the smallest footprint
    assert op.partition(tiny(memory_capacity=6.9)) is None


def test_oracle_partition_picks_each_mode_and_depth_when_forced():
    """Variants of the same profile whose optimum sits somewhere else; each fails if a mode is
    dropped or if w or d is swept over the wrong set."""
    # |W| = 80: the all-reduce takes 2*(1/2)*80/8 = 10 s per update, 5 | 10 s per microbatch: (2,1) falls to
    # 2/5 | 4/10 = 0.4.  Memory (M = 100): (1,2,2) pipelined 80+12+4 = 96 fits -> 2/2.1 wins over (1,1,2) 0.625
    # (80+12 = 92) and over recompute 0.75949 (80+6+4 = 90).  Without the pipelined mode the answer would be
    # the recompute one; without d = 2, (1,1,2).
    assert op.partition(tiny(weight_bytes=80.0)) == pytest.approx((1, 2, 2, PIPE, 1, 2 / 2.1, 96.0))
    # slow links everywhere (bandwidth 0.5): (1,2) pays 4b s of stage traffic -> 1/5 | 2/9.6; (2,1) pays
    # 16 s / m -> 2/8 | 4/16 = 0.25; one GPU alone at b = 2 is best, which a sweep forced to use all GPUs
    # (w d = N) would never see
    assert op.partition(tiny(bw_high=0.5, bw_low=0.5)) == pytest.approx((1, 1, 2, NO, 2, 0.625, 20.0))
    # B = 2: (1,2,2) would need g = 2/(1*2*2) = 1/2, i.e. m = 1 < d = 2 microbatches per update: not admissible
    # (Section 3.1 needs m >= d), and (2,1,2) likewise.  With the slow all-reduce of |W| = 80 (10 s per update,
    # m = 1 at (2,1,1): 2/10 = 0.2) the best is the pipelined (1,2,1): 0.8, memory 80+6+2 = 88, g = 1
    assert op.partition(tiny(weight_bytes=80.0, global_batch=2)) == pytest.approx((1, 2, 1, PIPE, 1, 0.8, 88.0))


def test_oracle_bandwidth_reading_at_the_server_boundary():
    """A group that fills a server exactly is charged the high bandwidth (the printed case expression
    is strict there; the departure is stated in the oracle's header)."""
    p = tiny(gpus_per_server=2, bw_high=8.0, bw_low=0.5, weight_bytes=80.0)
    # (2,1,1): all-reduce at the HIGH bandwidth: 10 s / m(=2) = 5 s -> 2/5; at the low one it would be 160/2 = 80 s
    assert op.throughput(p, 2, 1, 1, PIPE) == pytest.approx(2 / 5)
    q = tiny(gpus_per_server=1, bw_high=8.0, bw_low=0.5, weight_bytes=80.0)
    assert op.throughput(q, 2, 1, 1, PIPE) == pytest.approx(2 / 80)


def test_library_planner_on_the_hand_worked_sweep():
    for kw, want in ((dict(), (2, 1, 2, NO, 1, 1.25, 20.0)),
                     (dict(memory_capacity=19.0), (2, 1, 1, NO, 2, 1.0, 14.0)),
                     (dict(memory_capacity=13.5), (1, 2, 1, RECOMP, 2, 1 / (4 / 3 + 0.25), 13.0)),
                     (dict(weight_bytes=80.0), (1, 2, 2, PIPE, 1, 2 / 2.1, 96.0)),
                     (dict(bw_high=0.5, bw_low=0.5), (1, 1, 2, NO, 2, 0.625, 20.0)),
                     (dict(weight_bytes=80.0, global_batch=2), (1, 2, 1, PIPE, 1, 0.8, 88.0))):
        rc, got = B.Planner(tiny(**kw)).partition()
        assert rc == 0 and got == pytest.approx(want), kw
    assert B.Planner(tiny(memory_capacity=6.9)).partition()[0] == -2


def rand_profile(rng):
    sizes = sorted(rng.choice(np.arange(1, 33), size=int(rng.integers(1, 6)), replace=False).tolist())
    t1 = float(rng.uniform(0.2e-3, 3e-3))
    times = [t1 * s ** float(rng.uniform(0.7, 1.0)) for s in sizes]
    gps = int(rng.choice([1, 2, 4, 8]))
    n_gpus = gps * int(rng.choice([1, 2, 4]))
    return profile(n_blocks=int(rng.choice([12, 24, 30, 48])), n_gpus=n_gpus, gpus_per_server=gps,
                   microbatch_sizes=sizes, block_time_s=times, weight_bytes=float(rng.uniform(0.1e9, 20e9)),
                   state_bytes=float(rng.choice([0.0, 1.0])) * float(rng.uniform(0.1e9, 40e9)),
                   act_bytes_per_sample=float(rng.uniform(50e6, 2e9)), input_bytes_per_sample=float(rng.uniform(0.1e6, 20e6)),
                   boundary_bytes_per_sample=float(rng.uniform(0.1e6, 40e6)), bw_high=float(rng.uniform(20e9, 900e9)),
                   bw_low=float(rng.uniform(1e9, 20e9)), memory_capacity=float(rng.uniform(2e9, 288e9)),
                   global_batch=int(rng.choice([32, 64, 96, 512, 2048])), c_extra=float(rng.uniform(1.0, 1.6)))


@pytest.mark.parametrize("seed", range(40))
def test_library_planner_matches_the_brute_force_oracle(seed):
    rng = np.random.default_rng(seed)
    p = rand_profile(rng)
    pl = B.Planner(p)
    # cost functions on every admissible point
    for w in range(1, p.n_gpus + 1):
        for d in range(1, p.n_gpus // w + 1):
            if p.n_blocks % d:
                assert pl.throughput(w, d, p.microbatch_sizes[0], 1)[0] == B.ERR_INVALID_ARG
                continue
            for b in p.microbatch_sizes:
                if w * b > p.global_batch:
                    continue
                for mode in (0, 1, 2):
                    rc, thr = pl.throughput(w, d, b, mode)
                    assert rc == 0 and thr == pytest.approx(op.throughput(p, w, d, b, mode), rel=1e-12)
                    rc, mem = pl.memory(w, d, b, mode)
                    assert rc == 0 and mem == pytest.approx(op.memory(p, w, d, b, mode), rel=1e-12)
    rc, got = pl.partition()
    want = op.partition(p)
    if want is None:
        assert rc == -2
    else:
        assert rc == 0
        assert got[5] == pytest.approx(want[5], rel=1e-12)           # same optimum (ties may pick another point)
        assert got[6] <= p.memory_capacity and got[4] == p.global_batch // (got[0] * got[1] * got[2])


def test_library_planner_rejects_bad_input():
    p = profile()
    pl = B.Planner(p)
    assert pl.throughput(3, 3, 4, 1)[0] == B.ERR_INVALID_ARG        # 9 GPUs > 8
    assert pl.throughput(1, 5, 4, 1)[0] == B.ERR_INVALID_ARG        # 5 does not divide 24 blocks
    assert pl.throughput(1, 4, 3, 1)[0] == B.ERR_INVALID_ARG        # 3 is not a candidate size
    assert pl.memory(1, 4, 4, 7)[0] == B.ERR_INVALID_ARG
    assert B.Planner(profile(memory_capacity=1e6)).partition()[0] == -2


def test_plan_with_the_measured_mi355x_profile():
    """The example profile (this build's measured block times and stage sizes, 288 GB per GPU): a model that
    fits in one GPU is replicated, not pipelined; one that does not is split into the shallowest pipeline
    that fits, exactly what the brute-force oracle picks."""
    from paper_2006_09503_amd import plan_mi355x as pm
    rc, (w, d, b, mode, g, thr, mem) = pm.plan(8, 24, 512)
    assert rc == 0 and (w, d, mode) == (8, 1, B.PLANNER_NO_PIPELINE) and w * d * b * g == 512
    for n_gpus, n_blocks, batch in ((64, 768, 2048), (16, 1536, 512)):
        prof = pm.Mi355xProfile(n_blocks=n_blocks, n_gpus=n_gpus, global_batch=batch)
        rc, got = pm.plan(n_gpus, n_blocks, batch)
        want = op.partition(prof)
        assert rc == 0 and got[1] > 1 and got[3] != B.PLANNER_NO_PIPELINE
        assert got[5] == pytest.approx(want[5], rel=1e-12) and got[6] <= prof.memory_capacity
