"""A d-stage 2BW pipeline inside one process on one GPU: one library stage per pipeline stage, each
on its own HIP stream, driven in the 1F1B order of Section 3.1 (stage i has d - i microbatches in
flight), with a squared-error loss behind the last stage.  Orchestration only: every tensor
operation is a library kernel; torch supplies buffers, streams and events."""
from __future__ import annotations

from typing import Callable, List, Optional

import numpy as np
import torch

from . import binding as B
from . import synth


class Pipeline:
    def __init__(self, cfg: synth.StageConfig, stage_weights: List[np.ndarray]):
        """cfg: the shape of every stage (n_layers = layers per stage); max_inflight is set per
        stage to d - i.  stage_weights: one flat fp32 vector per stage."""
        d = len(stage_weights)
        assert d >= 1 and cfg.m >= d, "2BW generates a version every m >= d microbatches (Section 3.1)"
        assert not cfg.flush, "this driver streams batches back to back; the flush schedule drains per batch"
        self.d, self.cfg = d, cfg
        self.dtype = torch.bfloat16 if cfg.precision == synth.PREC_BF16 else torch.float32
        self.streams = [torch.cuda.Stream() for _ in range(d)]
        self.stages = [B.Stage(cfg.with_(max_inflight=d - i), stage_weights[i], stream=self.streams[i]) for i in range(d)]
        shape = (cfg.microbatch, cfg.seq, cfg.hidden)
        self.ring = d + 1
        # act[i][r]: output of stage i = input of stage i + 1; grad[i][r]: gradient w.r.t. that tensor
        self.act = [[torch.empty(shape, device="cuda", dtype=self.dtype) for _ in range(self.ring)] for _ in range(d)]
        self.grad = [[torch.empty(shape, device="cuda", dtype=self.dtype) for _ in range(self.ring)] for _ in range(d)]
        self.dx0 = [torch.empty(shape, device="cuda", dtype=self.dtype) for _ in range(self.ring)]
        torch.cuda.synchronize()

    def close(self):
        torch.cuda.synchronize()
        for st in self.stages:
            st.close()

    def stage_order(self, i: int, first: int, last: int):
        """1F1B at stage i: d - 1 - i warm-up forward passes, then forward/backward in turn."""
        ops, fw, bw = [], first, first
        for _ in range(min(self.d - 1 - i, last - first + 1)):
            ops.append(("F", fw)); fw += 1
        while bw <= last:
            if fw <= last:
                ops.append(("F", fw)); fw += 1
            ops.append(("B", bw)); bw += 1
        return ops

    def run(self, first_mb: int, count: int, get_input: Callable, get_target: Callable, loss_scale: float,
            on_output: Optional[Callable] = None, on_input_grad: Optional[Callable] = None,
            on_update: Optional[Callable] = None):
        """Microbatches first_mb .. first_mb + count - 1 (first_mb - 1 a multiple of m; nothing in flight).
        get_input(k) -> (x, seqlens) device tensors; get_target(k) -> device tensor like the output.
        on_output(k, y, stream) / on_input_grad(k, dx, stream) get tensors that are written on `stream` and
        stay valid until d more microbatches have passed; on_update(stage, t) is called right after an
        update has been enqueued."""
        d, m, R = self.d, self.cfg.m, self.ring
        assert (first_mb - 1) % m == 0 and count % m == 0
        last = first_mb + count - 1
        order = [self.stage_order(i, first_mb, last) for i in range(d)]
        pos = [0] * d
        issued = set()
        ev = {}

        def event(key, stream):
            e = torch.cuda.Event()
            e.record(stream)
            ev[key] = e

        def ready(i, op, k):
            if op == "F":
                return i == 0 or ("F", i - 1, k) in issued
            return ("F", i, k) in issued and (i == d - 1 or ("B", i + 1, k) in issued)

        n_elem = self.cfg.microbatch * self.cfg.seq * self.cfg.hidden
        dt = B.DT_BF16 if self.cfg.precision == synth.PREC_BF16 else B.DT_F32
        remaining = sum(len(o) for o in order)
        while remaining:
            progressed = False
            for i in range(d):
                if pos[i] == len(order[i]):
                    continue
                op, k = order[i][pos[i]]
                if not ready(i, op, k):
                    continue
                st, s = self.stages[i], self.streams[i]
                if op == "F":
                    x, lens = get_input(k)
                    if i > 0:
                        x = self.act[i - 1][k % R]
                        s.wait_event(ev[("F", i - 1, k)])
                    if i + 1 < d and ("F", i + 1, k - R) in ev:
                        s.wait_event(ev[("F", i + 1, k - R)])       # the reader of the slot being overwritten
                    if (k - 1) % m == 0 and (k - 1) // m >= 2:
                        st.swap_versions()
                    y = self.act[i][k % R]
                    st.forward(k, x, lens, y)
                    if i == d - 1:
                        B.check(B.lib().k2bw_squared_error_grad(dt, n_elem, y.data_ptr(), get_target(k).data_ptr(),
                                                                loss_scale, self.grad[i][k % R].data_ptr(), s.cuda_stream),
                                "k2bw_squared_error_grad")
                        if on_output is not None:
                            on_output(k, y, s)
                    event(("F", i, k), s)
                else:
                    if i + 1 < d:
                        s.wait_event(ev[("B", i + 1, k)])
                    dx = self.dx0[k % R] if i == 0 else self.grad[i - 1][k % R]
                    if i > 0 and ("B", i - 1, k - R) in ev:
                        s.wait_event(ev[("B", i - 1, k - R)])
                    st.backward(k, self.grad[i][k % R], dx)
                    event(("B", i, k), s)
                    if i == 0 and on_input_grad is not None:
                        on_input_grad(k, dx, s)
                    if k % m == 0:
                        st.coalesce_update()
                        if on_update is not None:
                            on_update(i, k // m)
                issued.add((op, i, k))
                pos[i] += 1
                remaining -= 1
                progressed = True
            assert progressed, "dependency cycle in the issue order"
            # drop events nobody can wait for any more
            for key in [key for key in ev if key[2] < k - 2 * R]:
                del ev[key]
        for s in self.streams:
            torch.cuda.current_stream().wait_stream(s)
