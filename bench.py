#!/usr/bin/env python3
"""Throughput of one 2BW pipeline stage on one MI355X.

A "step" is one batch of the stage's steady-state 1F1B stream (Section 3.1 of the paper): m
forward passes, m backward passes with in-place gradient coalescing, one Adam update into the
other weight buffer and the version swap, with `max_inflight` microbatches in flight.  The
default workload is the largest of the five configurations, C5: 2 layers, h=8192, 64 heads,
f=32768, s=2048, b=1, m=64, causal mask, bf16 compute with fp32 master weights (1.61 G
parameters); `--workload C2` is the BERT-Large-shaped stage, C3 / C4 the GPT-shaped ones.

Prints ONE JSON line: stage samples/s (value), model TFLOP/s, fraction of the bf16 MFMA peak,
a `roofline` object for the dominant kernel class (HIP-event timing of every launch of that
class inside a second timed region of the same length), a `cpu_baseline` object (the fp64
oracle timed on this host on a bounded sample of the same workload) and a `prefix_check` object:
before the timed run, the first microbatch goes through a one-layer stage of the workload's
shape and its output, input gradient and weight gradient are compared at 1024 positions each
with values the oracle computed for exactly that case (tests/golden/stage_prefix_*.txt).

All inputs are seeded, synthetic and resident in HBM before the clock starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch (read + write) of kernel instances, per workload at its default flags, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the same counters read
# for the library's plain copy kernel of known size; see profiles/ for the runs.  A workload, flag
# set or kernel that was not profiled reports null.
TRAFFIC_BYTES_PER_LAUNCH = {
    "C5": {
        # weight-gradient GEMM launches: the 8 products of the stage's 2 layers over 8 microbatches' tokens each
        # (reduction length 16384) go out in 6 launches of 16 rounds of tiles (FC2; FC1; out-projection + QKV, per
        # layer); average per launch: L2-miss read traffic 1.65e10 (the operand panels of products this size pass
        # through the 4 MB L2 of every XCD once per block of 32 tiles; the counter sees what misses L2, whether HBM or
        # the memory-side cache serves it) + 1.07e9 written.  Algorithmic minimum 3.58e9: operands once + fp32
        # accumulator read-modify-write.  (4 microbatches and all 8 products in one launch of 96 rounds: 8.75e10 ..
        # 9.93e10 per 4 microbatches instead of 5.3e10, see the stage's flush of pending products.)
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, true, false, 3>": 1.7651e+10,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 2>": 1.9206e+09,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 1>": 1.9351e+09,
        # forward projections and the data gradients (the latter on the transposed weight copy): averages
        # over the six shapes this instance serves
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 0>": 1.2583e+09,
    },
    "C4": {
        # (activation recomputation: the forward GEMMs run twice per microbatch; 4 layers x 4 products over 4 passes,
        # reduction length 16384, in 6 weight-gradient launches of 8 rounds)
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, true, false, 3>": 7.5253e+09,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 2>": 1.0826e+09,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 1>": 1.0772e+09,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 0>": 6.6144e+08,
    },
    "C2": {
        # grouped weight-gradient GEMM (the 24 products of the stage's 6 layers over 4 microbatches' tokens each,
        # reduction length 16384): FETCH_SIZE x 1.997 (copy-kernel factor) + WRITE_SIZE x 1.000; algorithmic minimum
        # 3.825e9 (operands once + fp32 accumulator read-modify-write)
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, true, false, 3>": 4.3746e+09,
        # the other GEMM instances (averages over the shapes each serves)
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 2>": 1.2830e+08,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 1>": 1.2617e+08,
        "gemm_bf16_ring_kernel<128, 128, 32, 64, 64, 4, false, false, 0>": 8.6542e+07,
        "gemm_bf16_ring_kernel<128, 128, 32, 64, 64, 4, false, true, 0>": 8.0722e+07,
        "gemm_bf16_ring_kernel<256, 256, 128, 64, 32, 4, false, false, 0>": 7.3567e+07,
    },
}


def measured_traffic(args, kernel):
    """Counter-measured HBM bytes per launch, or None unless this run is the profiled configuration."""
    if args.flush or args.recompute is not None or args.microbatch is not None or args.wgrad_group is not None:
        return None
    return TRAFFIC_BYTES_PER_LAUNCH.get(args.workload, {}).get(kernel)


def model_flops_per_microbatch(cfg) -> float:
    """3 x forward FLOPs; attention counted dense (4 b s^2 h per layer), no credit for recompute."""
    T, h, f, s, b = cfg.tokens, cfg.hidden, cfg.ffn, cfg.seq, cfg.microbatch
    fwd = cfg.n_layers * (2.0 * T * h * (3 * h) + 2.0 * T * h * h + 4.0 * T * h * f + 4.0 * b * s * s * h)
    return 3.0 * fwd


def cpu_baseline(cfg, seed):
    """The oracle as it stands on this host: one layer x one microbatch forward+backward plus one
    Adam step over the stage's parameters, extrapolated linearly in L and m."""
    import numpy as np
    from oracle import block as ob
    from oracle import twobw as tb
    from paper_2006_09503_amd import synth
    one = cfg.with_(n_layers=1)
    gen = synth.StageInputs(one, seed)
    w = gen.weights().astype(np.float64)
    x, dy, lens = gen.microbatch()
    st = ob.Stage(1, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.mask_mode, cfg.ln_eps)
    # one layer, microbatch after microbatch, until about 12 s of oracle time have been sampled
    n_mb, t_total = 0, 0.0
    while t_total < 12.0 and n_mb < 64:
        t0 = time.perf_counter()
        st.vjp(w, x, dy, lens)
        t_total += time.perf_counter() - t0
        n_mb += 1
        x, dy, lens = gen.microbatch()
    t_layer_mb = t_total / n_mb
    # the update is element-wise: a slice of at most 2^26 parameters is timed and scaled to all P
    P = synth.param_count(cfg)
    n_slice = min(P, 1 << 26)
    rng = np.random.default_rng(seed)
    wf, g = rng.standard_normal(n_slice), rng.standard_normal(n_slice)
    opt = tb.Adam(cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps)
    state = opt.init(wf)
    t0 = time.perf_counter()
    opt.step(wf, g, state, 0)
    t_adam = (time.perf_counter() - t0) * (P / n_slice)
    t_step = cfg.n_layers * cfg.m * t_layer_mb + t_adam
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": cfg.microbatch * cfg.m / t_step, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"fp64 numpy oracle: 1 layer x {n_mb} microbatches fwd+bwd ({t_layer_mb:.2f} s each) and one Adam step over "
                      f"{n_slice} of the {P} parameters (scaled to all: {t_adam:.2f} s), extrapolated linearly to "
                      f"L={cfg.n_layers}, m={cfg.m}"}


def prefix_check(workload, cfg, seed):
    """First microbatch through a one-layer stage of the workload's shape against the oracle's stored
    samples (tests/golden/stage_prefix_<workload>.txt; seed 0 only).  Returns relative L2 errors over
    the sampled positions, or None if no stored samples apply."""
    import numpy as np
    import torch
    from paper_2006_09503_amd import binding as B
    from paper_2006_09503_amd import synth
    path = os.path.join(ROOT, "tests", "golden", f"stage_prefix_{workload}.txt")
    if seed != 0 or not os.path.exists(path) or workload not in synth.PRESETS:
        return None
    base = synth.PRESETS[workload]
    if (cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.microbatch, cfg.mask_mode, cfg.precision) != \
            (base.hidden, base.n_heads, base.ffn, base.seq, base.microbatch, base.mask_mode, base.precision):
        return None
    want = {"Y": ([], []), "dX": ([], []), "G": ([], [])}
    for line in open(path):
        if line.startswith("#"):
            continue
        tag, idx, val = line.split()
        want[tag][0].append(int(idx))
        want[tag][1].append(float(val))
    one = base.with_(n_layers=1, m=1, max_inflight=1, recompute=0)
    gen = synth.StageInputs(one, 0)
    w0 = gen.weights()
    x, dy, lens = gen.microbatch()
    dt = torch.bfloat16 if one.precision == synth.PREC_BF16 else torch.float32
    st = B.Stage(one, w0)
    del w0
    X, DY = (torch.from_numpy(a).cuda().to(dt) for a in (x, dy))
    LEN = None if lens is None else torch.from_numpy(lens).cuda()
    Y, DX = torch.empty_like(X), torch.empty_like(X)
    st.forward(1, X, LEN, Y)
    st.backward(1, DY, DX)
    torch.cuda.synchronize()
    got = {"Y": Y.float().cpu().numpy().reshape(-1), "dX": DX.float().cpu().numpy().reshape(-1),
           "G": st.read_grad_accum()}
    st.close()
    out = {}
    for tag, (idx, val) in want.items():
        g, w = got[tag][np.asarray(idx)].astype(np.float64), np.asarray(val)
        out["rel_l2_" + tag] = float(np.linalg.norm(g - w) / np.linalg.norm(w))
    bar = 2e-2 if one.precision == synth.PREC_BF16 else 1e-4
    out["bar"] = bar
    out["ok"] = bool(max(out["rel_l2_Y"], out["rel_l2_dX"], out["rel_l2_G"]) <= bar)
    out["what"] = "one layer of the workload's shape, microbatch 1 of seed 0, 1024 sampled positions per tensor vs the fp64 oracle"
    return out


def pipeline_bench(args, cfg, w0):
    """d stages of the workload's shape chained in one process (the whole model has d * L layers)."""
    import torch
    from paper_2006_09503_amd import synth
    from paper_2006_09503_amd.pipeline import Pipeline
    d, m, K, W = args.stages, cfg.m, args.steps, args.warmup
    assert not cfg.flush and m >= d
    pipe = Pipeline(cfg, [w0] * d)
    dt = torch.bfloat16 if cfg.precision == synth.PREC_BF16 else torch.float32
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    shape = (cfg.microbatch, cfg.seq, cfg.hidden)
    X = [torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(dt) for _ in range(m)]
    TG = [torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(dt) for _ in range(m)]
    LEN = [None] * m
    if cfg.mask_mode == synth.MASK_PADDING:
        LEN = [torch.randint(cfg.min_len, cfg.seq + 1, (cfg.microbatch,), generator=g, device="cuda", dtype=torch.int32)
               for _ in range(m)]
    scale = 1.0 / (cfg.microbatch * cfg.seq * cfg.hidden)
    torch.cuda.synchronize()

    def run(first_batch, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipe.run(first_batch * m + 1, n * m, lambda k: (X[(k - 1) % m], LEN[(k - 1) % m]), lambda k: TG[(k - 1) % m], scale)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run(0, W)
    elapsed = run(W, K)
    flops_step = model_flops_per_microbatch(cfg) * m * d
    alloc = sum(st.query(4) for st in pipe.stages)
    pipe.close()
    print(json.dumps({
        "metric": "pipeline samples/sec (d stages of the workload's shape on 1 MI355X, one stream per stage, 2BW)",
        "value": cfg.microbatch * m * K / elapsed, "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.precision == synth.PREC_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} x {d} stages: {d * cfg.n_layers} layers h={cfg.hidden} a={cfg.n_heads} "
                               f"f={cfg.ffn} s={cfg.seq} b={cfg.microbatch} m={m}, in-process pipeline, squared-error loss",
                   "samples_per_step": cfg.microbatch * m, "model_flops_per_step": flops_step, "bytes_allocated": alloc},
        "model_tflops": flops_step * K / elapsed / 1e12,
        "frac_of_bf16_mfma_peak": flops_step * K / elapsed / 1e12 / PEAK_BF16_TFLOPS}))


def probe_gemm(spec):
    """`--probe-gemm f32,4096,4096,4096` (or bf16,...): one GEMM kernel alone, the three forms the stage issues,
    warm operands, HIP-event average over 20 launches; prints one JSON line."""
    import torch
    from paper_2006_09503_amd import binding as B
    name, M, N, K = spec.split(",")
    M, N, K = int(M), int(N), int(K)
    dt, code, peak = (torch.float32, 0, 157.3) if name == "f32" else (torch.bfloat16, 1, PEAK_BF16_TFLOPS)
    L = B.lib()
    g = torch.Generator(device="cuda").manual_seed(0)
    rnd = lambda *shape: torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(dt)
    out = {}
    forms = {"forward (A[M,K] B[K,N])": (0, 0, 0, rnd(M, K), K, rnd(K, N), N, torch.empty(M, N, device="cuda", dtype=dt)),
             "data gradient (A[M,K] B[N,K]^T)": (0, 1, 0, rnd(M, K), K, rnd(N, K), K, torch.empty(M, N, device="cuda", dtype=dt)),
             "weight gradient (A[K,M]^T B[K,N], fp32 +=)": (1, 0, 3, rnd(K, M), M, rnd(K, N), N,
                                                           torch.zeros(M, N, device="cuda", dtype=torch.float32))}
    for form, (ta, tb, epi, A, lda, Bm, ldb, Cm) in forms.items():
        def launch():
            rc = L.k2bw_gemm(code, ta, tb, epi, M, N, K, A.data_ptr(), lda, Bm.data_ptr(), ldb, Cm.data_ptr(), N, None, None,
                             None, 1 if epi == 3 else 0, None)
            assert rc == 0, rc
        for _ in range(3):
            launch()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(20):
            launch()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) / 20 * 1e3
        tf = 2.0 * M * N * K / (us * 1e-6) / 1e12
        out[form] = {"us": us, "tflops": tf, "frac_of_peak": tf / peak}
    print(json.dumps({"probe": f"k2bw_gemm {name} M={M} N={N} K={K}", "peak_tflops": peak, "forms": out}))


def event_pair_gap_us(stream, n=200):
    """Median time between two HIP events recorded back to back on `stream` with nothing in between."""
    import torch
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    with torch.cuda.stream(stream):
        for a, b in pairs:
            a.record()
            b.record()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in pairs)[n // 2] * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5", help="C1..C5 (see paper_2006_09503_amd/synth.py)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--flush", action="store_true", help="PipeDream-Flush (Section 3.2) instead of 2BW: one version, drain per batch")
    ap.add_argument("--recompute", type=int, default=None, help="override the workload's activation recomputation (0/1)")
    ap.add_argument("--microbatch", type=int, default=None, help="override the workload's microbatch size b (an extra "
                    "measurement: recomputation frees the memory for a larger b, Section 4.1 and the appendix)")
    ap.add_argument("--stages", type=int, default=1, help="d > 1: a d-stage 2BW pipeline of such stages in this process, one "
                    "HIP stream per stage, squared-error loss behind the last (an extra measurement, not the headline)")
    ap.add_argument("--streams", type=int, default=0, choices=(0, 1, 2),
                    help="2: backward passes and updates on a stream of their own, so that the forward and backward "
                         "passes of different microbatches overlap (the per-kernel timing region always runs on one "
                         "stream: each kernel then has the GPU to itself); 0 (default): what the workload's shape "
                         "recommends (two streams unless every projection gives each CU a 256x256 tile)")
    ap.add_argument("--wgrad-group", type=int, default=None, help="override how many microbatches' weight-gradient "
                    "products one launch covers (reduction length j*T; default: the library's choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefix-check", action="store_true")
    ap.add_argument("--probe-gemm", default=None, help="dtype,M,N,K: time one GEMM kernel alone (e.g. f32,4096,4096,4096) "
                    "instead of the stage; an extra measurement, not the headline")
    ap.add_argument("--no-kernel-timing", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(no collectives or multi-GPU sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2006_09503_amd import binding as B
    from paper_2006_09503_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.probe_gemm:
        probe_gemm(args.probe_gemm)
        return
    cfg = synth.PRESETS[args.workload]
    if args.flush:
        cfg = cfg.with_(flush=1)
    if args.recompute is not None:
        cfg = cfg.with_(recompute=args.recompute)
    if args.microbatch is not None:
        cfg = cfg.with_(microbatch=args.microbatch)
    if args.wgrad_group is not None:
        cfg = cfg.with_(wgrad_group=args.wgrad_group)
    if args.streams == 0:
        args.streams = cfg.recommended_streams
    p, m = cfg.max_inflight, cfg.m
    K, W = args.steps, args.warmup
    assert K >= 1 and W >= 2, "two warm-up batches are needed before the version rule leaves version 0"

    check = None if args.no_prefix_check else prefix_check(args.workload, cfg, args.seed)
    gen = synth.StageInputs(cfg, args.seed)
    w0 = gen.weights()
    if args.stages > 1:
        pipeline_bench(args, cfg, w0)
        return
    fwd_stream = torch.cuda.Stream()
    st = B.Stage(cfg, w0, fwd_stream)
    if args.streams == 2:
        bwd_stream = torch.cuda.Stream()
        st.set_backward_stream(bwd_stream)
    del w0
    # a pool of m distinct microbatches, resident in HBM, reused batch after batch
    dt = torch.bfloat16 if cfg.precision == synth.PREC_BF16 else torch.float32
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    shape = (cfg.microbatch, cfg.seq, cfg.hidden)
    X = [torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(dt) for _ in range(m)]
    DY = [(torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * 1e-2).to(dt) for _ in range(m)]
    LEN = [None] * m
    if cfg.mask_mode == synth.MASK_PADDING:
        LEN = [torch.randint(cfg.min_len, cfg.seq + 1, (cfg.microbatch,), generator=g, device="cuda",
                             dtype=torch.int32) for _ in range(m)]
        for j in range(m):
            keep = torch.arange(cfg.seq, device="cuda")[None, :] < LEN[j][:, None]
            DY[j] = (DY[j] * keep[:, :, None]).contiguous()
    Y = [torch.empty(shape, device="cuda", dtype=dt) for _ in range(p + 1)]
    DX = torch.empty(shape, device="cuda", dtype=dt)

    drained = [0]   # microbatches up to this one have had their backward pass (see drain())

    def iteration(k):
        """One slot of the worker's 1F1B stream: backward of k-p, maybe update, maybe swap, forward of k."""
        kb = k - p
        if kb > drained[0]:
            st.backward(kb, DY[(kb - 1) % m], DX)
            if kb % m == 0:
                st.coalesce_update()
        if (k - 1) % m == 0 and (k - 1) // m >= 2:
            st.swap_versions()
        st.forward(k, X[(k - 1) % m], LEN[(k - 1) % m], Y[k % (p + 1)])

    def flush_batch(b):
        """One batch under the flush schedule: 1F1B inside the batch, drained before the update."""
        first = b * m + 1
        for k in range(first, first + m):
            if k - p >= first:
                st.backward(k - p, DY[(k - p - 1) % m], DX)
            st.forward(k, X[(k - 1) % m], LEN[(k - 1) % m], Y[k % (p + 1)])
        for k in range(first + m - p, first + m):
            st.backward(k, DY[(k - 1) % m], DX)
        st.coalesce_update()

    def drain(last):
        """Backward passes of the microbatches still in flight after forward pass `last` (a batch end)."""
        if not cfg.flush:
            for kb in range(max(last - p, drained[0]) + 1, last + 1):
                st.backward(kb, DY[(kb - 1) % m], DX)
                if kb % m == 0:
                    st.coalesce_update()
        drained[0] = last
        torch.cuda.synchronize()

    def run_steps(first_step, n_steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if cfg.flush:
            for b in range(first_step, first_step + n_steps):
                flush_batch(b)
        else:
            for k in range(first_step * m + 1, (first_step + n_steps) * m + 1):
                iteration(k)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run_steps(0, W)
    elapsed = run_steps(W, K)
    ms_per_step = elapsed / K * 1e3
    samples_per_s = cfg.microbatch * m * K / elapsed
    flops_step = model_flops_per_microbatch(cfg) * m
    tflops = flops_step * K / elapsed / 1e12

    roofline, kernels = None, None
    steps_done = W + K
    if not args.no_kernel_timing:
        # Per-kernel durations (HIP events around every launch, on the stream it is launched on) come
        # from a second region of K steps on ONE stream, where each kernel has the GPU to itself;
        # one untimed batch refills the pipeline after the switch.
        if args.streams == 2:
            drain(steps_done * m)
            st.set_backward_stream(fwd_stream)
        run_steps(steps_done, 1)
        launches_per_step = m * cfg.n_layers * 64 + 16
        st.timing_enable(True, launches_per_step * K + 64)
        run_steps(steps_done + 1, K)
        steps_done += 1 + K
        per_kernel = st.timing_collect_kernels()
        tm = st.timing_collect()
        st.timing_enable(False)
        kernels = {}
        for name, r in tm.items():
            if r["launches"] == 0:
                continue
            e = {"launches_per_step": r["launches"] / K, "ms_per_step": r["ms"] / K,
                 "avg_us": r["ms"] / r["launches"] * 1e3}
            if r["flops"] > 0:
                e["tflops"] = r["flops"] / (r["ms"] * 1e-3) / 1e12
                e["frac_of_bf16_peak"] = e["tflops"] / PEAK_BF16_TFLOPS
            if r["bytes"] > 0:
                e["gbs"] = r["bytes"] / (r["ms"] * 1e-3) / 1e9
                e["frac_of_hbm_peak"] = e["gbs"] / PEAK_HBM_GBS
            kernels[name] = e
        # dominant kernel = the single kernel instance (name as rocprofv3 prints it) with the most
        # time in the timed region; its algorithmic FLOPs per launch = 2*M*N*K summed over the
        # problems of the launch, averaged over its launches
        # (an event pair costs a few microseconds per launch, which would tip the choice towards the
        # kernel with the most launches: the time of an empty pair is taken off for the choice only)
        gap_ms = event_pair_gap_us(fwd_stream) * 1e-3
        gemm_inst = {n: r for n, r in per_kernel.items() if n.startswith("gemm_") and r["flops"] > 0}
        dom = max(gemm_inst, key=lambda n: gemm_inst[n]["ms"] - gemm_inst[n]["launches"] * gap_ms)
        r = gemm_inst[dom]
        achieved = r["flops"] / (r["ms"] * 1e-3) / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(args, dom),
                    "avg_launch_us": r["ms"] / r["launches"] * 1e3, "launches_per_step": r["launches"] / K,
                    "flops_per_launch": r["flops"] / r["launches"], "empty_event_pair_us": gap_ms * 1e3,
                    "share_of_step": r["ms"] / K / ms_per_step}
        kernels["_by_instance"] = {n: {"launches_per_step": v["launches"] / K, "avg_us": v["ms"] / v["launches"] * 1e3,
                                       **({"tflops": v["flops"] / (v["ms"] * 1e-3) / 1e12} if v["flops"] > 0 else {}),
                                       **({"gbs": v["bytes"] / (v["ms"] * 1e-3) / 1e9} if v["bytes"] > 0 else {})}
                                   for n, v in per_kernel.items()}

    # drain the microbatches still in flight so the stage ends at a batch boundary
    drain(steps_done * m)
    finite = bool(torch.isfinite(DX.float()).all().item())
    alloc = st.query(B.Q_BYTES_ALLOCATED)
    st.close()

    out = {
        "metric": "stage samples/sec + % bf16 MFMA peak (1 MI355X), 2BW fwd/bwd/update step",
        "value": samples_per_s, "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.precision == synth.PREC_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: one pipeline stage, L={cfg.n_layers} h={cfg.hidden} a={cfg.n_heads} "
                               f"f={cfg.ffn} s={cfg.seq} b={cfg.microbatch} m={cfg.m} inflight={p} "
                               f"mask={('none', 'causal', 'padding')[cfg.mask_mode]} recompute={cfg.recompute} "
                               f"schedule={'flush' if cfg.flush else '2bw'} streams={args.streams}",
                   "samples_per_step": cfg.microbatch * m, "model_flops_per_step": flops_step,
                   "stage_bytes_allocated": alloc},
        "model_tflops": tflops, "frac_of_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS, "outputs_finite": finite,
        "prefix_check": check, "roofline": roofline, "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
