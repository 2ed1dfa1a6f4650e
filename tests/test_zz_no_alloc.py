"""The allocation-free bias-gradient entry point (partial rows in a device array inside the library
image) against the workspace-taking entry point it mirrors and against the fp64 column sums:
two calls in a row, the second on a smaller input, so that what the first left in the shared
array must not leak into the second.  Collected last: it runs both alone and after everything else."""
import numpy as np
import pytest
import torch

from paper_2006_09503_amd import binding as B
from paper_2006_09503_amd.synth import round_to_bf16

from gpu_util import rel, to_dev, to_host

pytestmark = pytest.mark.gpu

F32, BF16 = 0, 1


def _case(L, dtype, rows, n, seed, accumulate_on):
    rng = np.random.default_rng(seed)
    y = rng.standard_normal((rows, n)).astype(np.float32)
    if dtype == BF16:
        y = round_to_bf16(y)
    Yd = to_dev(y, dtype)
    ws = torch.empty(L.k2bw_bias_grad_workspace(n), device="cuda")
    start = None if accumulate_on is None else torch.from_numpy(accumulate_on[:n].copy()).cuda()
    want_dev = torch.full((n,), float("nan"), device="cuda") if start is None else start.clone()
    got_dev = torch.full((n,), float("nan"), device="cuda") if start is None else start.clone()
    acc = 0 if start is None else 1
    print(f"no-alloc case dtype={dtype} rows={rows} n={n} accumulate={acc}", flush=True)
    assert L.k2bw_bias_grad(dtype, rows, n, Yd.data_ptr(), want_dev.data_ptr(), acc, ws.data_ptr(), None) == 0
    assert L.k2bw_bias_grad_static(dtype, rows, n, Yd.data_ptr(), got_dev.data_ptr(), acc, None) == 0
    torch.cuda.synchronize()
    got, want = to_host(got_dev), to_host(want_dev)
    exact = y.astype(np.float64).sum(0) + (0.0 if accumulate_on is None else accumulate_on[:n].astype(np.float64))
    assert np.array_equal(got, want)                 # same kernels, same order of additions
    assert rel(got, exact) < 1e-5                    # fp32 sums of <= 4096 terms; the fp32 bar is 1e-4
    return got


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_static_scratch_bias_gradient_two_calls_second_smaller(dtype):
    L = B.lib()
    assert L.k2bw_bias_grad_static_max_cols() == 32768
    first = _case(L, dtype, 4096, 3080, 1, None)
    _case(L, dtype, 150, 72, 2, None)                # smaller in both extents: fewer partial rows, narrower rows
    _case(L, dtype, 1000, 1024, 3, first)            # accumulate form on top of earlier sums


def test_static_scratch_rejects_sizes_beyond_the_array():
    L = B.lib()
    y = torch.zeros(8, 8, device="cuda")
    out = torch.zeros(40000, device="cuda")
    assert L.k2bw_bias_grad_static(F32, 8, 32768 + 8, y.data_ptr(), out.data_ptr(), 0, None) == B.ERR_INVALID_ARG
    assert L.k2bw_bias_grad_static(F32, 8, 0, y.data_ptr(), out.data_ptr(), 0, None) == B.ERR_INVALID_ARG
    assert L.k2bw_bias_grad_static(F32, 8, 8, y.data_ptr(), None, 0, None) == B.ERR_INVALID_ARG
    torch.cuda.synchronize()


def test_static_scratch_at_the_maximum_width():
    L = B.lib()
    _case(L, BF16, 70, 32768, 4, None)
    _case(L, BF16, 64, 256, 5, None)
