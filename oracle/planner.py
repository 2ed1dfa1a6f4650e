"""Reference planner: the closed-form THROUGHPUT and MEMORY cost functions and the partitioning
algorithm of the paper's appendix "Planner, Additional Details", written out plainly and searched
by brute force.  Test infrastructure only: nothing in the product imports this.

Readings (the appendix leaves them open): equal stages, d divides the number of blocks; every
stage pays 2|A_inp+out(b)|/bandwidth when d > 1; the all-reduce moves 2(w-1)/w of a stage's weight
bytes (the closed form of the PipeDream paper the appendix cites); of the two ways to lay the
w x d grid over the servers the better one is taken; throughput is that of the whole job (w b / t).

Degree of gradient accumulation: the partitioning algorithm's last line gives g = B / (N b), and
Section 5.2 fixes its meaning through the batch size b w d g of a pipeline whose m = d g
microbatches are averaged per update.  So g = B / (w d b) for the (w, d) chosen (the printed N when
every GPU is used), a configuration is admissible iff that is a whole number >= 1, and then
m = d g >= d, the condition Section 3.1 needs for two weight versions to suffice.

One departure from a printed form, on purpose: the appendix's bandwidth case expression gives
the high bandwidth for w strictly below the number of GPUs in a server.  A group that fills a
server exactly still communicates inside it, so the test used here is group size <= server size;
at equality the printed form would charge the low bandwidth."""
from dataclasses import dataclass
from typing import Sequence

NO_PIPELINE, PIPELINE, PIPELINE_RECOMPUTE = 0, 1, 2


@dataclass
class Profile:
    n_blocks: int
    n_gpus: int
    gpus_per_server: int
    microbatch_sizes: Sequence[int]
    block_time_s: Sequence[float]
    weight_bytes: float
    state_bytes: float
    act_bytes_per_sample: float
    input_bytes_per_sample: float
    boundary_bytes_per_sample: float
    bw_high: float
    bw_low: float
    memory_capacity: float
    global_batch: int
    c_extra: float = 4.0 / 3.0


def _bw(p: Profile, group: int) -> float:
    return p.bw_high if group <= p.gpus_per_server else p.bw_low


def throughput(p: Profile, w: int, d: int, b: int, mode: int) -> float:
    t_block = p.block_time_s[list(p.microbatch_sizes).index(b)]
    blocks_per_stage = p.n_blocks // d
    best = 0.0
    # two orientations of the grid: stage replicas inside a server, or whole pipelines inside a server
    for bw_depth, bw_width in ((_bw(p, w * d), _bw(p, w)), (_bw(p, d), _bw(p, w * d))):
        per_stage = []
        for _stage in range(d):
            t_comp = blocks_per_stage * t_block
            if mode == PIPELINE_RECOMPUTE:
                t_comp *= p.c_extra
            t_act = 2.0 * p.boundary_bytes_per_sample * b / bw_depth if d > 1 else 0.0
            m_b = p.global_batch / (w * b)
            t_allreduce = 2.0 * (w - 1) / w * (p.weight_bytes / d) / bw_width if w > 1 else 0.0
            per_stage.append(max(t_comp + t_act, t_allreduce / m_b))
        t = sum(per_stage) if mode == NO_PIPELINE else max(per_stage)
        best = max(best, w * b / t)
    return best


def memory(p: Profile, w: int, d: int, b: int, mode: int) -> float:
    W, A, A_in = p.weight_bytes, p.act_bytes_per_sample * b, p.input_bytes_per_sample * b
    if mode == NO_PIPELINE:
        footprint = W / d + A / d
    elif mode == PIPELINE:
        footprint = 2.0 * W / d + d * A / d + d * A_in
    else:
        footprint = 2.0 * W / d + A / d + d * A_in
    return footprint + p.state_bytes / d


def partition(p: Profile):
    """Every (w, d, b, mode) that is admissible and fits, by brute force; returns the best as
    (w, d, b, mode, g, throughput, memory) or None."""
    best = None
    for w in range(1, p.n_gpus + 1):
        for d in range(1, p.n_gpus // w + 1):
            if p.n_blocks % d:
                continue
            for b in p.microbatch_sizes:
                if p.global_batch % (w * d * b):        # g = B / (w d b) must be a whole number >= 1
                    continue
                for mode in (NO_PIPELINE, PIPELINE, PIPELINE_RECOMPUTE):
                    mem = memory(p, w, d, b, mode)
                    if mem > p.memory_capacity:
                        continue
                    thr = throughput(p, w, d, b, mode)
                    if best is None or thr > best[5]:
                        best = (w, d, b, mode, p.global_batch // (w * d * b), thr, mem)
    return best
