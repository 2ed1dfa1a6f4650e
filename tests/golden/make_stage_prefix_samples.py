#!/usr/bin/env python3
"""Writes tests/golden/stage_prefix_<workload>.txt: sampled values of what the fp64 oracle gives
for the FIRST microbatch through ONE layer of each workload shape (seed 0, the seeded generator's
own draws; in bf16 mode the inputs are the bf16-rounded ones): stage output Y, input gradient dX
and weight gradient G at 1024 evenly spaced flat positions each.

Calls only oracle/ and the input generator.  The GPU-side callers (bench.py's prefix check, a GPU
test) run the same one-layer stage and compare at the same positions, so that a throughput run on
the full configuration is tied to oracle-checked numbers at the real layer shape without paying
for the oracle (up to a minute of CPU per shape) in that run.

    python tests/golden/make_stage_prefix_samples.py [C1 C2 ...]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import block as ob                      # noqa: E402
from paper_2006_09503_amd import synth              # noqa: E402

N_SAMPLES = 1024


def positions(size: int) -> np.ndarray:
    return np.linspace(0, size - 1, N_SAMPLES).astype(np.int64)


def main(names):
    for name in names:
        cfg = synth.PRESETS[name].with_(n_layers=1, m=1, max_inflight=1, recompute=0)
        gen = synth.StageInputs(cfg, 0)
        w0 = gen.weights().astype(np.float64)
        x, dy, lens = gen.microbatch()
        st = ob.Stage(1, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.mask_mode, cfg.ln_eps)
        t0 = time.perf_counter()
        y, dx, g = st.vjp(w0, x, dy, lens)
        dt = time.perf_counter() - t0
        path = os.path.join(HERE, f"stage_prefix_{name}.txt")
        with open(path, "w") as f:
            f.write(f"# {name}: one layer h={cfg.hidden} a={cfg.n_heads} f={cfg.ffn} s={cfg.seq} b={cfg.microbatch} "
                    f"mask={cfg.mask_mode} precision={cfg.precision}, seed 0, microbatch 1, weights W(0)\n")
            f.write("# fp64 oracle (oracle/block.py Stage.vjp); written by tests/golden/make_stage_prefix_samples.py\n")
            f.write("# columns: tensor  flat_index  value\n")
            for tag, arr in (("Y", y), ("dX", dx), ("G", g)):
                flat = np.asarray(arr).reshape(-1)
                for i in positions(flat.size):
                    f.write(f"{tag} {i} {flat[i]:.10e}\n")
        print(f"{name}: oracle {dt:.1f} s -> {path}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or ["C1", "C2", "C3", "C4", "C5"])
