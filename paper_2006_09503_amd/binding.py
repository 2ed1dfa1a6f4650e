"""ctypes binding over lib2bw.so: the same entry points as include/stage2bw.h and
include/stage2bw_kernels.h, argument marshalling only.  Every step of the stage runs in the
library's HIP kernels; PyTorch supplies device buffers and the stream.

There is no fallback: if the library has not been built (python -m paper_2006_09503_amd.build)
loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib2bw.so")

STAGE_OK, ERR_INVALID_ARG, ERR_BAD_STATE, ERR_OOM, ERR_HIP = 0, -1, -2, -3, -4
WEIGHTS_BUF0, WEIGHTS_BUF1, WEIGHTS_MASTER = 0, 1, 2
(Q_UPDATES, Q_READ_VERSION, Q_INFLIGHT, Q_ACCUMULATED, Q_BYTES_ALLOCATED, Q_BYTES_WEIGHTS,
 Q_BYTES_STASH, Q_BUFFER_OF_NEWEST, Q_BUFFER_OF_READ) = range(9)
KERNEL_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd",
                  "bias_grad", "adam", "other")


class StageConfigC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_heads", "ffn", "seq", "microbatch", "m",
                                         "max_inflight", "mask_mode", "precision", "recompute")] + \
               [(n, C.c_float) for n in ("lr", "beta1", "beta2", "adam_eps", "ln_eps")] + \
               [("flush", C.c_int32), ("optimizer", C.c_int32), ("wgrad_group", C.c_int32)]


class PlannerInputC(C.Structure):
    _fields_ = [("n_blocks", C.c_int32), ("n_gpus", C.c_int32), ("gpus_per_server", C.c_int32), ("n_sizes", C.c_int32),
                ("microbatch_sizes", C.POINTER(C.c_int32)), ("block_time_s", C.POINTER(C.c_double)),
                ("weight_bytes", C.c_double), ("state_bytes", C.c_double), ("act_bytes_per_sample", C.c_double),
                ("input_bytes_per_sample", C.c_double), ("boundary_bytes_per_sample", C.c_double),
                ("bw_high", C.c_double), ("bw_low", C.c_double), ("memory_capacity", C.c_double),
                ("global_batch", C.c_int64), ("c_extra", C.c_double)]


class PlannerChoiceC(C.Structure):
    _fields_ = [("w", C.c_int32), ("d", C.c_int32), ("b", C.c_int32), ("mode", C.c_int32), ("g", C.c_int64),
                ("throughput", C.c_double), ("memory", C.c_double)]


class StageError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib_handle = None


def lib() -> C.CDLL:
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2006_09503_amd.build`; "
                               "there is no non-HIP path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        sig = {
            "stage_param_count": (i64, [C.POINTER(StageConfigC)]),
            "stage_create": (C.c_int, [C.POINTER(StageConfigC), vp, vp, C.POINTER(vp)]),
            "stage_forward": (C.c_int, [vp, i64, vp, vp, vp]),
            "stage_backward": (C.c_int, [vp, i64, vp, vp]),
            "stage_coalesce_update": (C.c_int, [vp]),
            "stage_swap_versions": (C.c_int, [vp]),
            "stage_set_backward_stream": (C.c_int, [vp, vp]),
            "stage_destroy": (C.c_int, [vp]),
            "stage_read_weights": (C.c_int, [vp, C.c_int, vp]),
            "stage_read_grad_accum": (C.c_int, [vp, vp]),
            "stage_read_adam": (C.c_int, [vp, vp, vp]),
            "stage_query": (C.c_int, [vp, C.c_int, C.POINTER(i64)]),
            "stage_strerror": (C.c_char_p, [C.c_int]),
            "stage_timing_enable": (C.c_int, [vp, C.c_int, i32]),
            "stage_timing_collect": (C.c_int, [vp, vp, vp, vp, vp]),
            "stage_timing_collect_kernels": (C.c_int, [vp, i32, vp, vp, vp, vp, vp, C.POINTER(i32)]),
            "stage_sched_create": (C.c_int, [i32, i32, i32, C.POINTER(vp)]),
            "stage_sched_forward": (C.c_int, [vp, i64, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]),
            "stage_sched_backward": (C.c_int, [vp, i64, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32),
                                               C.POINTER(i32)]),
            "stage_sched_coalesce_update": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]),
            "stage_sched_swap_versions": (C.c_int, [vp]),
            "stage_sched_query": (C.c_int, [vp, C.c_int, C.POINTER(i64)]),
            "stage_sched_destroy": (C.c_int, [vp]),
            "k2bw_gemm": (C.c_int, [C.c_int] * 7 + [vp, C.c_int, vp, C.c_int, vp, C.c_int, vp, vp, vp, C.c_int, vp]),
            "k2bw_gemm_wgrad_segmented": (C.c_int, [C.c_int] * 4 + [vp, C.c_int, i64, vp, vp, C.c_int, i64, vp, vp, C.c_int,
                                                      C.c_int, vp]),
            "k2bw_layernorm_fwd": (C.c_int, [C.c_int, C.c_int, C.c_int, f32, vp, vp, vp, vp, vp, vp, vp]),
            "k2bw_gemm_dgrad_gelu_bias_workspace": (i64, [C.c_int, C.c_int]),
            "k2bw_gemm_dgrad_gelu_bias": (C.c_int, [C.c_int, C.c_int, C.c_int, vp, C.c_int, vp, C.c_int, vp, C.c_int, vp, vp, C.c_int, vp, vp]),
            "k2bw_layernorm_bwd_workspace": (i64, [C.c_int]),
            "k2bw_layernorm_bwd": (C.c_int, [C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, vp]),
            "k2bw_bias_grad_workspace": (i64, [C.c_int]),
            "k2bw_bias_grad": (C.c_int, [C.c_int, C.c_int, C.c_int, vp, vp, C.c_int, vp, vp]),
            "k2bw_bias_grad_static_max_cols": (C.c_int, []),
            "k2bw_bias_grad_static": (C.c_int, [C.c_int, C.c_int, C.c_int, vp, vp, C.c_int, vp]),
            "k2bw_attention_fwd": (C.c_int, [C.c_int] * 6 + [vp, vp, vp, vp, vp]),
            "k2bw_attention_bwd_workspace": (i64, [C.c_int] * 4),
            "k2bw_attention_bwd": (C.c_int, [C.c_int] * 6 + [vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, vp]),
            "k2bw_adam": (C.c_int, [i64, vp, vp, vp, vp, vp, vp, f32, f32, f32, f32, C.c_int, i64, vp]),
            "k2bw_momentum": (C.c_int, [i64, vp, vp, vp, vp, vp, f32, f32, C.c_int, vp]),
            "k2bw_squared_error_grad": (C.c_int, [C.c_int, i64, vp, vp, f32, vp, vp]),
            "k2bw_copy": (C.c_int, [vp, vp, i64, vp]),
            "k2bw_tune_gemm_tile": (C.c_int, [C.c_int]),
            "planner_throughput": (C.c_int, [C.POINTER(PlannerInputC), i32, i32, i32, i32, C.POINTER(C.c_double)]),
            "planner_memory": (C.c_int, [C.POINTER(PlannerInputC), i32, i32, i32, i32, C.POINTER(C.c_double)]),
            "planner_search": (C.c_int, [C.POINTER(PlannerInputC), i32, i32, C.POINTER(PlannerChoiceC)]),
            "planner_partition": (C.c_int, [C.POINTER(PlannerInputC), C.POINTER(PlannerChoiceC)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib_handle = L
    return _lib_handle


def strerror(code: int) -> str:
    return lib().stage_strerror(code).decode()


DT_F32, DT_BF16 = 0, 1      # dtype codes of the k2bw_* kernel calls


def _check(code: int, where: str):
    if code != STAGE_OK:
        raise StageError(code, where)


def _ptr(t) -> Optional[int]:
    """Device (torch tensor) or host (numpy array) address; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    assert t.is_contiguous()
    return t.data_ptr()


check = _check


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def config_struct(cfg) -> StageConfigC:
    """cfg: any object with the stage_config_t field names (e.g. synth.StageConfig)."""
    c = StageConfigC()
    for name, _ in StageConfigC._fields_:
        setattr(c, name, getattr(cfg, name))
    return c


# ----------------------------------------------------------------------------- stage calls

def stage_param_count(cfg) -> int:
    n = lib().stage_param_count(C.byref(config_struct(cfg)))
    if n < 0:
        raise StageError(int(n), "stage_param_count")
    return int(n)


def stage_create(cfg, init_weights_host: np.ndarray, stream=None) -> int:
    w = np.ascontiguousarray(init_weights_host, dtype=np.float32)
    assert w.size == stage_param_count(cfg)
    h = C.c_void_p()
    _check(lib().stage_create(C.byref(config_struct(cfg)), w.ctypes.data, _stream_ptr(stream), C.byref(h)),
           "stage_create")
    return h.value


def stage_forward(st: int, mb: int, x, seqlens, y):
    _check(lib().stage_forward(st, mb, _ptr(x), _ptr(seqlens), _ptr(y)), f"stage_forward({mb})")


def stage_backward(st: int, mb: int, dy, dx):
    _check(lib().stage_backward(st, mb, _ptr(dy), _ptr(dx)), f"stage_backward({mb})")


def stage_coalesce_update(st: int):
    _check(lib().stage_coalesce_update(st), "stage_coalesce_update")


def stage_swap_versions(st: int):
    _check(lib().stage_swap_versions(st), "stage_swap_versions")


def stage_set_backward_stream(st: int, stream):
    _check(lib().stage_set_backward_stream(st, _stream_ptr(stream)), "stage_set_backward_stream")


def stage_destroy(st: int):
    _check(lib().stage_destroy(st), "stage_destroy")


def stage_query(st: int, what: int) -> int:
    out = C.c_int64()
    _check(lib().stage_query(st, what, C.byref(out)), "stage_query")
    return out.value


def stage_read_weights(st: int, which: int, n_params: int) -> np.ndarray:
    out = np.empty(n_params, dtype=np.float32)
    _check(lib().stage_read_weights(st, which, out.ctypes.data), "stage_read_weights")
    return out


def stage_read_grad_accum(st: int, n_params: int) -> np.ndarray:
    out = np.empty(n_params, dtype=np.float32)
    _check(lib().stage_read_grad_accum(st, out.ctypes.data), "stage_read_grad_accum")
    return out


def stage_read_adam(st: int, n_params: int, second_moment: bool = True):
    m = np.empty(n_params, dtype=np.float32)
    v = np.empty(n_params, dtype=np.float32) if second_moment else None
    _check(lib().stage_read_adam(st, m.ctypes.data, v.ctypes.data if second_moment else None), "stage_read_adam")
    return m, v


def stage_timing_enable(st: int, enable: bool, capacity: int = 0):
    _check(lib().stage_timing_enable(st, int(enable), capacity), "stage_timing_enable")


def stage_timing_collect(st: int):
    """{class: dict(ms, launches, flops, bytes)} since the last collect."""
    n = len(KERNEL_CLASSES)
    ms, fl, by = (np.zeros(n, dtype=np.float64) for _ in range(3))
    cnt = np.zeros(n, dtype=np.int64)
    _check(lib().stage_timing_collect(st, ms.ctypes.data, cnt.ctypes.data, fl.ctypes.data, by.ctypes.data),
           "stage_timing_collect")
    return {k: dict(ms=float(ms[i]), launches=int(cnt[i]), flops=float(fl[i]), bytes=float(by[i]))
            for i, k in enumerate(KERNEL_CLASSES)}


def stage_timing_collect_kernels(st: int, capacity: int = 64):
    """{kernel instance name: dict(ms, launches, flops, bytes)}; call before stage_timing_collect."""
    names = C.create_string_buffer(capacity * 96)
    ms, fl, by = (np.zeros(capacity, dtype=np.float64) for _ in range(3))
    cnt = np.zeros(capacity, dtype=np.int64)
    n = C.c_int32()
    _check(lib().stage_timing_collect_kernels(st, capacity, C.addressof(names), ms.ctypes.data, cnt.ctypes.data,
                                              fl.ctypes.data, by.ctypes.data, C.byref(n)), "stage_timing_collect_kernels")
    out = {}
    for i in range(n.value):
        name = names.raw[i * 96:(i + 1) * 96].split(b"\0")[0].decode()
        out[name] = dict(ms=float(ms[i]), launches=int(cnt[i]), flops=float(fl[i]), bytes=float(by[i]))
    return out


# ----------------------------------------------------------------------------- schedule alone (host)

class Sched:
    """The library's 2BW bookkeeping without any device: each method returns (code, outputs...)."""

    def __init__(self, m: int, max_inflight: int, flush: bool = False):
        h = C.c_void_p()
        _check(lib().stage_sched_create(m, max_inflight, int(flush), C.byref(h)), "stage_sched_create")
        self.h = h.value

    def forward(self, mb):
        slot, ver, buf = C.c_int32(), C.c_int64(), C.c_int32()
        rc = lib().stage_sched_forward(self.h, mb, C.byref(slot), C.byref(ver), C.byref(buf))
        return rc, slot.value, ver.value, buf.value

    def backward(self, mb):
        slot, ver, buf, first = C.c_int32(), C.c_int64(), C.c_int32(), C.c_int32()
        rc = lib().stage_sched_backward(self.h, mb, C.byref(slot), C.byref(ver), C.byref(buf), C.byref(first))
        return rc, slot.value, ver.value, buf.value, first.value

    def coalesce_update(self):
        rb, wb, step = C.c_int32(), C.c_int32(), C.c_int64()
        rc = lib().stage_sched_coalesce_update(self.h, C.byref(rb), C.byref(wb), C.byref(step))
        return rc, rb.value, wb.value, step.value

    def swap_versions(self):
        return lib().stage_sched_swap_versions(self.h)

    def query(self, what):
        out = C.c_int64()
        _check(lib().stage_sched_query(self.h, what, C.byref(out)), "stage_sched_query")
        return out.value

    def close(self):
        if self.h:
            lib().stage_sched_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ----------------------------------------------------------------------------- convenience wrapper

class Stage:
    """Owns a stage handle; methods are the C calls.  `run_1f1b` issues them in the order one
    worker of a 1F1B pipeline would (Section 3.1), with `inflight` microbatches in flight."""

    def __init__(self, cfg, init_weights_host: np.ndarray, stream=None):
        self.cfg = cfg
        self.n_params = stage_param_count(cfg)
        self.h = stage_create(cfg, init_weights_host, stream)

    def forward(self, mb, x, seqlens, y): stage_forward(self.h, mb, x, seqlens, y)
    def backward(self, mb, dy, dx): stage_backward(self.h, mb, dy, dx)
    def coalesce_update(self): stage_coalesce_update(self.h)
    def swap_versions(self): stage_swap_versions(self.h)
    def set_backward_stream(self, stream): stage_set_backward_stream(self.h, stream)
    def query(self, what): return stage_query(self.h, what)
    def read_weights(self, which): return stage_read_weights(self.h, which, self.n_params)
    def read_grad_accum(self): return stage_read_grad_accum(self.h, self.n_params)
    def read_adam(self): return stage_read_adam(self.h, self.n_params, getattr(self.cfg, "optimizer", 0) == 0)
    def timing_enable(self, enable, capacity=0): stage_timing_enable(self.h, enable, capacity)
    def timing_collect(self): return stage_timing_collect(self.h)
    def timing_collect_kernels(self, capacity=64): return stage_timing_collect_kernels(self.h, capacity)

    def close(self):
        if self.h:
            stage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def run_1f1b(self, first_mb: int, count: int, get_inputs, get_outputs, inflight: int, on_update=None):
        """Microbatches first_mb .. first_mb+count-1 (first_mb - 1 a multiple of m, nothing in flight).

        get_inputs(k) -> (x, seqlens, dy) device tensors; get_outputs(k) -> (y, dx) device tensors.
        on_update(t) is called right after update number t has been enqueued.  In flush mode the
        in-flight microbatches are drained at every batch end before the update (Section 3.2).
        """
        m = self.cfg.m
        assert (first_mb - 1) % m == 0 and 1 <= inflight <= m
        last = first_mb + count - 1

        def back(k):
            _, _, dy = get_inputs(k)
            _, dx = get_outputs(k)
            self.backward(k, dy, dx)
            if k % m == 0:
                self.coalesce_update()
                if on_update is not None:
                    on_update(k // m)

        if getattr(self.cfg, "flush", 0):
            for b0 in range(first_mb, last + 1, m):
                b1 = min(b0 + m - 1, last)
                for k in range(b0, b1 + 1):
                    if k - inflight >= b0:
                        back(k - inflight)
                    x, lens, _ = get_inputs(k)
                    y, _ = get_outputs(k)
                    self.forward(k, x, lens, y)
                for k in range(max(b1 - inflight + 1, b0), b1 + 1):
                    back(k)
            return

        for k in range(first_mb, last + 1):
            if k - inflight >= first_mb:
                back(k - inflight)
            if (k - 1) % m == 0 and (k - 1) // m >= 2:
                self.swap_versions()
            x, lens, _ = get_inputs(k)
            y, _ = get_outputs(k)
            self.forward(k, x, lens, y)
        for k in range(max(last - inflight + 1, first_mb), last + 1):
            back(k)


# ----------------------------------------------------------------------------- planner (host)

PLANNER_NO_PIPELINE, PLANNER_PIPELINE, PLANNER_PIPELINE_RECOMPUTE = 0, 1, 2


class Planner:
    """The library's planner (Section 3.4 / appendix); `profile` is any object with the fields of
    planner_input_t (microbatch_sizes and block_time_s as sequences)."""

    def __init__(self, profile):
        n = len(profile.microbatch_sizes)
        self._sizes = (C.c_int32 * n)(*profile.microbatch_sizes)
        self._times = (C.c_double * n)(*profile.block_time_s)
        c = PlannerInputC()
        for name, _ in PlannerInputC._fields_:
            if name == "n_sizes":
                c.n_sizes = n
            elif name == "microbatch_sizes":
                c.microbatch_sizes = self._sizes
            elif name == "block_time_s":
                c.block_time_s = self._times
            else:
                setattr(c, name, getattr(profile, name))
        self._c = c

    def throughput(self, w, d, b, mode):
        out = C.c_double()
        rc = lib().planner_throughput(C.byref(self._c), w, d, b, mode, C.byref(out))
        return rc, out.value

    def memory(self, w, d, b, mode):
        out = C.c_double()
        rc = lib().planner_memory(C.byref(self._c), w, d, b, mode, C.byref(out))
        return rc, out.value

    @staticmethod
    def _choice(rc, c):
        return rc, (None if rc else (c.w, c.d, c.b, c.mode, c.g, c.throughput, c.memory))

    def search(self, w, d):
        c = PlannerChoiceC()
        return self._choice(lib().planner_search(C.byref(self._c), w, d, C.byref(c)), c)

    def partition(self):
        c = PlannerChoiceC()
        return self._choice(lib().planner_partition(C.byref(self._c), C.byref(c)), c)
