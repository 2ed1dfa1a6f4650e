"""The planner (Section 3.4, appendix "Planner, Additional Details") fed with what this build measured
on one MI355X: forward + backward time of one BERT-Large-shaped block (h = 1024, 16 heads, f = 4096,
s = 512) at microbatch sizes 8, 16, 32 (`bench.py --microbatch b`, step time / (m * L)), and the sizes
the stage reports (`stage_query`).  Host only.

    python -m paper_2006_09503_amd.plan_mi355x [n_gpus] [n_blocks] [global_batch]
"""
from __future__ import annotations

import sys
from dataclasses import dataclass, field
from typing import List

from . import binding as B

H, F, S = 1024, 4096, 512
PARAMS_PER_BLOCK = 4 * H * H + 2 * H * F + 9 * H + F          # 12.6 M


@dataclass
class Mi355xProfile:
    """planner_input_t for a model of `n_blocks` such blocks on `n_gpus` MI355X (8 per server)."""
    n_blocks: int = 24
    n_gpus: int = 8
    gpus_per_server: int = 8
    microbatch_sizes: List[int] = field(default_factory=lambda: [8, 16, 32])
    # one block, forward + backward, two streams: 21.2 / 42.5 / 72.9 ms per step of m = 8 microbatches x 6 blocks
    block_time_s: List[float] = field(default_factory=lambda: [21.2e-3 / 48, 42.5e-3 / 48, 72.9e-3 / 48])
    weight_bytes: float = 0.0            # one bf16 version
    state_bytes: float = 0.0             # fp32 master, Adam m and v, gradient accumulator: 16 B / parameter
    act_bytes_per_sample: float = 0.0    # stash of the whole model per sample: 18.9 MB per block (0.9 GB per slot of 6 blocks x 8)
    input_bytes_per_sample: float = S * H * 2.0
    boundary_bytes_per_sample: float = 2 * S * H * 2.0
    bw_high: float = 300e9               # xGMI inside a server (a ring's share of 7 links x 153 GB/s, both directions)
    bw_low: float = 50e9                 # one 400 Gb/s NIC per GPU between servers
    memory_capacity: float = 288e9
    global_batch: int = 512
    c_extra: float = 4.0 / 3.0           # measured here: 1.28 .. 1.35

    def __post_init__(self):
        p = PARAMS_PER_BLOCK * self.n_blocks
        self.weight_bytes = 2.0 * p
        self.state_bytes = 16.0 * p
        self.act_bytes_per_sample = 18.9e6 * self.n_blocks


MODES = {B.PLANNER_NO_PIPELINE: "no pipelining", B.PLANNER_PIPELINE: "2BW pipeline",
         B.PLANNER_PIPELINE_RECOMPUTE: "2BW pipeline + recomputation"}


def plan(n_gpus: int = 8, n_blocks: int = 24, global_batch: int = 512):
    """(rc, (w, d, b, mode, g, samples_per_s, bytes_per_gpu)) of the partitioning algorithm."""
    return B.Planner(Mi355xProfile(n_blocks=n_blocks, n_gpus=n_gpus, global_batch=global_batch)).partition()


def main(argv):
    n_gpus = int(argv[1]) if len(argv) > 1 else 8
    n_blocks = int(argv[2]) if len(argv) > 2 else 24
    batch = int(argv[3]) if len(argv) > 3 else 512
    rc, c = plan(n_gpus, n_blocks, batch)
    if rc != 0:
        print(f"no configuration fits (code {rc})")
        return 1
    w, d, b, mode, g, thr, mem = c
    print(f"{n_blocks} blocks on {n_gpus} MI355X, global batch {batch}: w = {w} replicas of a d = {d} stage pipeline, "
          f"microbatch b = {b}, m = d g = {d * g} microbatches per update, {MODES[mode]}: {thr:.0f} samples/s predicted, "
          f"{mem / 2**30:.1f} GiB per GPU")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
