"""Each HIP kernel, called through the C ABI, against the oracle's statement of the same step
(oracle/block.py, oracle/twobw.py) on seeded inputs: several tiles plus ragged tails.
fp32 kernels must meet 1e-4, bf16 kernels 2e-2 (relative L2); in practice they sit far below."""
import math

import numpy as np
import pytest
import torch

from oracle import block as ob
from oracle import twobw as tb
from paper_2006_09503_amd import binding as B
from paper_2006_09503_amd.synth import round_to_bf16

from gpu_util import rel, to_dev, to_host

pytestmark = pytest.mark.gpu

F32, BF16 = 0, 1
TOL = {F32: 1e-4, BF16: 2e-2}
TIGHT = {F32: 2e-6, BF16: 6e-3}     # what the arithmetic should actually achieve on one kernel


def rnd(rng, shape, dtype, scale=1.0):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return round_to_bf16(a) if dtype == BF16 else a


def dev(a, dtype):
    return to_dev(a, dtype)


def empty(shape, dtype):
    return torch.full(shape, float("nan"), device="cuda", dtype=torch.bfloat16 if dtype == BF16 else torch.float32)


def sync():
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- GEMM

GEMM_SHAPES = [
    # (M, N, K)   small ragged; several 128-tiles; 256x256-tile path (>= 144 big tiles), ragged; more than two
    # rounds of 256 tiles (the tile -> XCD mapping in whole blocks, then in runs, then the halved tail)
    (70, 40, 24), (300, 264, 200), (512, 384, 256), (4000, 3080, 136), (4100, 8200, 64),
]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("epi", [0, 1])
def test_gemm_forward_form(dtype, M, N, K, epi):
    """X[M,K] W[K,N] + b (+ residual) and the FC1 form with GELU."""
    rng = np.random.default_rng(M + N + K + epi)
    x, w, b = rnd(rng, (M, K), dtype), rnd(rng, (K, N), dtype, 0.1), rnd(rng, (N,), dtype)
    res = rnd(rng, (M, N), dtype)
    want_u = x.astype(np.float64) @ w.astype(np.float64) + b
    X, W, Bv, R = dev(x, dtype), dev(w, dtype), dev(b, dtype), dev(res, dtype)
    Cc, G = empty((M, N), dtype), empty((M, N), dtype)
    L = B.lib()
    if epi == 0:
        rc = L.k2bw_gemm(dtype, 0, 0, 0, M, N, K, X.data_ptr(), K, W.data_ptr(), N, Cc.data_ptr(), N,
                         Bv.data_ptr(), R.data_ptr(), None, 0, None)
        assert rc == 0
        sync()
        assert rel(to_host(Cc), want_u + res) < TIGHT[dtype]
    else:
        rc = L.k2bw_gemm(dtype, 0, 0, 1, M, N, K, X.data_ptr(), K, W.data_ptr(), N, Cc.data_ptr(), N,
                         Bv.data_ptr(), None, G.data_ptr(), 0, None)
        assert rc == 0
        sync()
        assert rel(to_host(Cc), want_u) < TIGHT[dtype]
        assert rel(to_host(G), ob.gelu(want_u)) < TIGHT[dtype]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("epi", [0, 2])
def test_gemm_data_gradient_form(dtype, M, N, K, epi):
    """dY[M,K'] W[N,K']^T, optionally times GELU'(u): here the ABI's N is the weight's row count."""
    rng = np.random.default_rng(7 * M + N + K + epi)
    dy, w = rnd(rng, (M, K), dtype), rnd(rng, (N, K), dtype, 0.1)
    u = rnd(rng, (M, N), dtype)
    want = dy.astype(np.float64) @ w.astype(np.float64).T
    if epi == 2:
        want = want * ob.gelu_grad(u.astype(np.float64))
    DY, W, U = dev(dy, dtype), dev(w, dtype), dev(u, dtype)
    Cc = empty((M, N), dtype)
    rc = B.lib().k2bw_gemm(dtype, 0, 1, epi, M, N, K, DY.data_ptr(), K, W.data_ptr(), K, Cc.data_ptr(), N, None,
                           U.data_ptr() if epi == 2 else None, None, 0, None)
    assert rc == 0
    sync()
    assert rel(to_host(Cc), want) < TIGHT[dtype]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_data_gradient_through_gelu_on_a_transposed_weight_copy(dtype, M, N, K):
    """(dY[M,K'] Wt[K',N]) * GELU'(u): the form the bf16 stage issues, reading its transposed copy of the weights
    (the forward's operand form with the data-gradient epilogue)."""
    rng = np.random.default_rng(11 * M + N + K)
    dy, wt = rnd(rng, (M, K), dtype), rnd(rng, (K, N), dtype, 0.1)
    u = rnd(rng, (M, N), dtype)
    want = (dy.astype(np.float64) @ wt.astype(np.float64)) * ob.gelu_grad(u.astype(np.float64))
    DY, WT, U = dev(dy, dtype), dev(wt, dtype), dev(u, dtype)
    Cc = empty((M, N), dtype)
    assert B.lib().k2bw_gemm(dtype, 0, 0, 2, M, N, K, DY.data_ptr(), K, WT.data_ptr(), N, Cc.data_ptr(), N, None,
                             U.data_ptr(), None, 0, None) == 0
    sync()
    assert rel(to_host(Cc), want) < TIGHT[dtype]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("M,N,K", [(72, 40, 150), (264, 136, 150), (512, 384, 1000), (4096, 3080, 130)])
def test_gemm_weight_gradient_form_coalesces_in_place(dtype, M, N, K):
    """G[M,N] (fp32) = X[K,M]^T dY[K,N], then += a second product (Section 3.1 coalescing)."""
    rng = np.random.default_rng(M + 3 * N + K)
    x1, d1 = rnd(rng, (K, M), dtype), rnd(rng, (K, N), dtype)
    x2, d2 = rnd(rng, (K, M), dtype), rnd(rng, (K, N), dtype)
    G = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
    L = B.lib()
    X1, D1, X2, D2 = dev(x1, dtype), dev(d1, dtype), dev(x2, dtype), dev(d2, dtype)
    assert L.k2bw_gemm(dtype, 1, 0, 3, M, N, K, X1.data_ptr(), M, D1.data_ptr(), N, G.data_ptr(), N, None, None,
                       None, 0, None) == 0
    sync()
    g1 = x1.astype(np.float64).T @ d1.astype(np.float64)
    assert rel(to_host(G), g1) < 2e-6           # fp32 accumulation of exact bf16 products either way
    assert L.k2bw_gemm(dtype, 1, 0, 3, M, N, K, X2.data_ptr(), M, D2.data_ptr(), N, G.data_ptr(), N, None, None,
                       None, 1, None) == 0
    sync()
    assert rel(to_host(G), g1 + x2.astype(np.float64).T @ d2.astype(np.float64)) < 2e-6


@pytest.mark.parametrize("tile", [2, 3, 6, 22, 23])
@pytest.mark.parametrize("M,N,K", [(296, 264, 200), (328, 272, 192), (136, 520, 64), (264, 136, 96), (136, 264, 32)])
def test_gemm_every_tile_variant(tile, M, N, K):
    """Each tile shape / staging variant of the bf16 kernel, forced, on ragged shapes in all three forms:
    K = 200 is not a multiple of the K step (the direct-to-LDS variants fall back), K = 192 is three K
    steps (uneven halves for the variant with two K groups), K = 64 leaves its second group empty;
    K = 96 and 32 are three tiles and one tile of the four-stage ring (fewer than it prefetches)."""
    rng = np.random.default_rng(tile * 1000 + M + N + K)
    L = B.lib()
    assert L.k2bw_tune_gemm_tile(tile) == 0
    try:
        x, w, b = rnd(rng, (M, K), BF16), rnd(rng, (K, N), BF16, 0.1), rnd(rng, (N,), BF16)
        X, W, Bv = dev(x, BF16), dev(w, BF16), dev(b, BF16)
        U, Gl = empty((M, N), BF16), empty((M, N), BF16)
        assert L.k2bw_gemm(BF16, 0, 0, 1, M, N, K, X.data_ptr(), K, W.data_ptr(), N, U.data_ptr(), N, Bv.data_ptr(),
                           None, Gl.data_ptr(), 0, None) == 0
        sync()
        want_u = x.astype(np.float64) @ w.astype(np.float64) + b
        assert rel(to_host(U), want_u) < TIGHT[BF16]
        assert rel(to_host(Gl), ob.gelu(want_u)) < TIGHT[BF16]

        wt = rnd(rng, (N, K), BF16, 0.1)
        Wt, Cc = dev(wt, BF16), empty((M, N), BF16)
        u_host = to_host(U)
        assert L.k2bw_gemm(BF16, 0, 1, 2, M, N, K, X.data_ptr(), K, Wt.data_ptr(), K, Cc.data_ptr(), N, None,
                           U.data_ptr(), None, 0, None) == 0
        sync()
        want = (x.astype(np.float64) @ wt.astype(np.float64).T) * ob.gelu_grad(u_host.astype(np.float64))
        assert rel(to_host(Cc), want) < TIGHT[BF16]

        xt, dy = rnd(rng, (K, M), BF16), rnd(rng, (K, N), BF16)
        G = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
        Xt, DY = dev(xt, BF16), dev(dy, BF16)
        for acc in (0, 1):
            assert L.k2bw_gemm(BF16, 1, 0, 3, M, N, K, Xt.data_ptr(), M, DY.data_ptr(), N, G.data_ptr(), N, None,
                               None, None, acc, None) == 0
        sync()
        assert rel(to_host(G), 2.0 * (xt.astype(np.float64).T @ dy.astype(np.float64))) < 2e-6
    finally:
        assert L.k2bw_tune_gemm_tile(0) == 0


@pytest.mark.parametrize("M,N,K", [(4360, 4096, 64), (4096, 4360, 96)])
def test_gemm_balanced_tail_of_a_256_tile_launch(M, N, K):
    """A launch whose last round of 256x256 tiles would leave most CUs idle gives the rows of those tiles to
    half-height tiles: 4360 x 4096 is 18 x 16 = 288 tiles (the last two tile rows, 264 rows, are split off and
    halved: 128 + 128 + 8 rows); 4096 x 4360 is 16 x 18 (the last tile row halved).  All three forms, the
    two-output epilogue and in-place accumulation."""
    test_gemm_every_tile_variant(23, M, N, K)


def _random_gemm_shapes():
    """Seeded shapes (multiples of 8) across the regimes of the tile choice: a few 128-tiles, about one 128-tile
    per CU, and 256-tile launches of one to two rounds, where the last round is or is not given to half-height
    tiles; K from one K tile of the ring to a few, with and without a remainder for either K tile."""
    rng = np.random.default_rng(2006)
    shapes = []
    for lo, hi in [(8, 400), (400, 1500), (1500, 2600), (3300, 4700), (3300, 4700), (3300, 4700)]:
        for _ in range(3):
            M, N = (int(rng.integers(lo, hi)) // 8 * 8 + 8 for _ in range(2))
            K = int(rng.choice([32, 64, 96, 128, 136, 192, 256, 320]))
            shapes.append((M, N, K))
    return shapes


@pytest.mark.parametrize("M,N,K", _random_gemm_shapes())
def test_gemm_random_shapes_with_the_built_in_tile_choice(M, N, K):
    """The bf16 GEMM as the stage calls it (tile chosen by the library), all three forms, against fp64."""
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    L = B.lib()
    x, w, b = rnd(rng, (M, K), BF16), rnd(rng, (K, N), BF16, 0.1), rnd(rng, (N,), BF16)
    r = rnd(rng, (M, N), BF16)
    X, W, Bv, R = dev(x, BF16), dev(w, BF16), dev(b, BF16), dev(r, BF16)
    Y = empty((M, N), BF16)
    assert L.k2bw_gemm(BF16, 0, 0, 0, M, N, K, X.data_ptr(), K, W.data_ptr(), N, Y.data_ptr(), N, Bv.data_ptr(),
                       R.data_ptr(), None, 0, None) == 0
    sync()
    assert rel(to_host(Y), x.astype(np.float64) @ w.astype(np.float64) + b + r) < TIGHT[BF16]

    wt = rnd(rng, (N, K), BF16, 0.1)
    Wt, D = dev(wt, BF16), empty((M, N), BF16)
    assert L.k2bw_gemm(BF16, 0, 1, 0, M, N, K, X.data_ptr(), K, Wt.data_ptr(), K, D.data_ptr(), N, None, None, None,
                       0, None) == 0
    sync()
    assert rel(to_host(D), x.astype(np.float64) @ wt.astype(np.float64).T) < TIGHT[BF16]

    xt, dy = rnd(rng, (K, M), BF16), rnd(rng, (K, N), BF16)
    G = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
    Xt, DY = dev(xt, BF16), dev(dy, BF16)
    for acc in (0, 1):
        assert L.k2bw_gemm(BF16, 1, 0, 3, M, N, K, Xt.data_ptr(), M, DY.data_ptr(), N, G.data_ptr(), N, None, None,
                           None, acc, None) == 0
    sync()
    assert rel(to_host(G), 2.0 * (xt.astype(np.float64).T @ dy.astype(np.float64))) < 2e-6


@pytest.mark.parametrize("M,N,K", [(296, 264, 200), (4096, 1032, 136), (520, 4096, 64), (4360, 4096, 64)])
def test_gemm_gelu_gradient_with_fused_bias_gradient(M, N, K):
    """du = (dy W^T) * GELU'(u) and db = colsum(du) from the same pass (bf16), overwrite then accumulate.
    The last shape is 288 tiles of 256x256: its last two tile rows (264 rows) run as five rows of
    half-height tiles, split off as a problem of their own with its own partial-sum rows."""
    rng = np.random.default_rng(M + N + K)
    dy, w, u = rnd(rng, (M, K), BF16), rnd(rng, (N, K), BF16, 0.1), rnd(rng, (M, N), BF16)
    want = (dy.astype(np.float64) @ w.astype(np.float64).T) * ob.gelu_grad(u.astype(np.float64))
    L = B.lib()
    DY, W, U = dev(dy, BF16), dev(w, BF16), dev(u, BF16)
    DU = empty((M, N), BF16)
    db = torch.full((N,), float("nan"), device="cuda")
    ws = torch.empty(L.k2bw_gemm_dgrad_gelu_bias_workspace(M, N), device="cuda")
    for acc in (0, 1):
        assert L.k2bw_gemm_dgrad_gelu_bias(M, N, K, DY.data_ptr(), K, W.data_ptr(), K, DU.data_ptr(), N, U.data_ptr(),
                                           db.data_ptr(), acc, ws.data_ptr(), None) == 0
    sync()
    assert rel(to_host(DU), want) < TIGHT[BF16]
    scale = np.sqrt((want ** 2).sum(0)).max()
    assert np.abs(to_host(db) - 2.0 * want.sum(0)).max() < 1e-5 * scale * np.sqrt(M)


def test_gemm_rejects_shapes_it_cannot_take():
    L = B.lib()
    a = torch.zeros(64 * 64, device="cuda", dtype=torch.bfloat16)
    p = a.data_ptr()
    assert L.k2bw_gemm(BF16, 0, 0, 0, 8, 8, 12, p, 12, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG  # K % 8
    assert L.k2bw_gemm(BF16, 0, 0, 0, 8, 8, 8, p + 2, 8, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG  # alignment
    assert L.k2bw_gemm(BF16, 1, 1, 0, 8, 8, 8, p, 8, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG    # form never issued
    assert L.k2bw_gemm(F32, 0, 0, 0, 0, 8, 8, p, 8, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG     # empty
    assert L.k2bw_gemm(F32, 0, 0, 1, 8, 8, 8, p, 8, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG     # GELU without bias
    assert L.k2bw_gemm(3, 0, 0, 0, 8, 8, 8, p, 8, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG
    big = 1 << 27   # 8 rows of 2^27 bf16 = 2 GiB: past the kernels' 32-bit byte offsets
    assert L.k2bw_gemm(BF16, 0, 0, 0, 8, 8, 8, p, big, p, 8, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG
    assert L.k2bw_gemm(BF16, 0, 0, 0, 8, 8, 8, p, 8, p, big, p, 8, None, None, None, 0, None) == B.ERR_INVALID_ARG


# ----------------------------------------------------------------------------- LayerNorm

@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("rows,h", [(150, 72), (130, 128), (1030, 1024), (300, 2560), (260, 4096), (70, 8192),
                                    (33, 12288), (1030, 2048), (777, 8192), (2100, 4096), (4100, 2048)])
# (from (1030, 2048) on: several trips per workgroup; the last two: three trips with two and four rows per workgroup and
# trip, so that rows requested a trip ahead are used, and the last trip is ragged)
def test_layernorm_forward_backward(dtype, rows, h):
    rng = np.random.default_rng(rows + h)
    x = rnd(rng, (rows, h), dtype, 2.0)
    g, s = rnd(rng, (h,), dtype, 0.2) + np.float32(1), rnd(rng, (h,), dtype, 0.2)
    if dtype == BF16:
        g = round_to_bf16(g)
    else:
        x = (x + np.float32(0.5)).astype(np.float32)
    dy, dres = rnd(rng, (rows, h), dtype), rnd(rng, (rows, h), dtype)
    eps = 1e-5
    y_want, saved = ob.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), s.astype(np.float64), eps)
    dx_want, dg_want, ds_want = ob.layernorm_bwd(dy.astype(np.float64), saved, g.astype(np.float64))

    L = B.lib()
    X, Gn, Sh, DY, DR = (dev(a, dtype) for a in (x, g, s, dy, dres))
    Y, DX = empty((rows, h), dtype), empty((rows, h), dtype)
    mean = torch.empty(rows, device="cuda"); rstd = torch.empty(rows, device="cuda")
    assert L.k2bw_layernorm_fwd(dtype, rows, h, eps, X.data_ptr(), Gn.data_ptr(), Sh.data_ptr(), Y.data_ptr(),
                                mean.data_ptr(), rstd.data_ptr(), None) == 0
    sync()
    assert rel(to_host(Y), y_want) < TIGHT[dtype]
    assert np.abs(to_host(mean) - x.astype(np.float64).mean(-1)).max() < 1e-5
    assert rel(to_host(rstd), saved[1][:, 0]) < 1e-5

    ws = torch.empty(L.k2bw_layernorm_bwd_workspace(h), device="cuda")
    dgs = torch.full((2 * h,), float("nan"), device="cuda")
    dxs = torch.full((h,), float("nan"), device="cuda")
    assert L.k2bw_layernorm_bwd(dtype, rows, h, DY.data_ptr(), X.data_ptr(), mean.data_ptr(), rstd.data_ptr(),
                                Gn.data_ptr(), DR.data_ptr(), DX.data_ptr(), dgs.data_ptr(), dxs.data_ptr(), 0,
                                ws.data_ptr(), None) == 0
    sync()
    assert rel(to_host(DX), dx_want + dres) < TIGHT[dtype]
    assert rel(to_host(dgs)[:h], dg_want) < 1e-5 and rel(to_host(dgs)[h:], ds_want) < 1e-5
    # column sums of the result (a bias gradient in the stage), taken before dx is rounded
    cs_want = (dx_want + dres).sum(0)
    assert np.abs(to_host(dxs) - cs_want).max() < 1e-5 * np.abs(dx_want + dres).sum(0).max() + 1e-4 * np.sqrt(rows)
    # accumulate on top, no residual, no column sums
    assert L.k2bw_layernorm_bwd(dtype, rows, h, DY.data_ptr(), X.data_ptr(), mean.data_ptr(), rstd.data_ptr(),
                                Gn.data_ptr(), None, DX.data_ptr(), dgs.data_ptr(), None, 1, ws.data_ptr(),
                                None) == 0
    sync()
    assert rel(to_host(DX), dx_want) < TIGHT[dtype]
    assert rel(to_host(dgs)[:h], 2 * dg_want) < 1e-5 and rel(to_host(dgs)[h:], 2 * ds_want) < 1e-5


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("rows,n", [(150, 72), (4096, 1024), (1000, 3080), (70, 32768)])
def test_bias_gradient_column_sums(dtype, rows, n):
    rng = np.random.default_rng(rows + n)
    y = rnd(rng, (rows, n), dtype)
    Yd = dev(y, dtype)
    L = B.lib()
    ws = torch.empty(L.k2bw_bias_grad_workspace(n), device="cuda")
    out = torch.full((n,), float("nan"), device="cuda")
    assert L.k2bw_bias_grad(dtype, rows, n, Yd.data_ptr(), out.data_ptr(), 0, ws.data_ptr(), None) == 0
    assert L.k2bw_bias_grad(dtype, rows, n, Yd.data_ptr(), out.data_ptr(), 1, ws.data_ptr(), None) == 0
    sync()
    assert rel(to_host(out), 2 * y.astype(np.float64).sum(0)) < 1e-5


@pytest.mark.parametrize("M,N,T,idx_a,idx_b", [
    (520, 264, 128, [3, 0, 2], [0, 1, 2]),                 # 128x128 ring tiles, K tiles of 64
    (264, 520, 64, [1], [2]),                              # one piece: the plain product
    (3080, 3072, 96, [5, 1, 4, 0], [3, 2, 1, 0]),          # 256x256 ring tiles (K tiles of 32), ragged M
    (2048, 2304, 64, [0, 1, 2, 3, 4, 5, 6, 7], [7, 6, 5, 4, 3, 2, 1, 0]),   # the maximum number of pieces
])
def test_gemm_weight_gradient_over_several_microbatches(M, N, T, idx_a, idx_b):
    """sum_s X_s^T dY_s with the pieces in separate buffers at a constant stride, in one product."""
    n_seg, n_buf = len(idx_a), 8
    rng = np.random.default_rng(M + N + T + n_seg)
    xs = rnd(rng, (n_buf, T, M), BF16)
    dys = rnd(rng, (n_buf, T, N), BF16, 0.1)
    g0 = rng.standard_normal((M, N)).astype(np.float32)
    want = sum(xs[a].astype(np.float64).T @ dys[b].astype(np.float64) for a, b in zip(idx_a, idx_b))
    X, DY = dev(xs, BF16), dev(dys, BF16)
    assert (T * M * 2) % 256 == 0 and (T * N * 2) % 256 == 0
    ia, ib = np.array(idx_a, dtype=np.uint8), np.array(idx_b, dtype=np.uint8)
    L = B.lib()
    for acc in (0, 1):
        G = torch.from_numpy(g0.copy()).cuda()
        assert L.k2bw_gemm_wgrad_segmented(M, N, T, n_seg, X.data_ptr(), M, T * M * 2, ia.ctypes.data, DY.data_ptr(), N,
                                           T * N * 2, ib.ctypes.data, G.data_ptr(), N, acc, None) == 0
        sync()
        assert rel(to_host(G), want + (g0 if acc else 0)) < 2e-6
    # refused: pieces that are not whole K tiles, an index beyond 15, a stride off the 256-byte grid
    G = torch.zeros((M, N), device="cuda")
    bad = np.array([16] * n_seg, dtype=np.uint8)
    if n_seg > 1:
        assert L.k2bw_gemm_wgrad_segmented(M, N, T, n_seg, X.data_ptr(), M, T * M * 2, bad.ctypes.data, DY.data_ptr(), N,
                                           T * N * 2, ib.ctypes.data, G.data_ptr(), N, 0, None) == B.ERR_INVALID_ARG
        assert L.k2bw_gemm_wgrad_segmented(M, N, T, n_seg, X.data_ptr(), M, T * M * 2 + 16, ia.ctypes.data, DY.data_ptr(), N,
                                           T * N * 2, ib.ctypes.data, G.data_ptr(), N, 0, None) == B.ERR_INVALID_ARG
        assert L.k2bw_gemm_wgrad_segmented(M, N, 40, n_seg, X.data_ptr(), M, T * M * 2, ia.ctypes.data, DY.data_ptr(), N,
                                           T * N * 2, ib.ctypes.data, G.data_ptr(), N, 0, None) == B.ERR_INVALID_ARG
    sync()


@pytest.mark.parametrize("dtype,dh", [(F32, 16), (BF16, 64)])
def test_attention_key_lengths_outside_the_sequence_are_clamped(dtype, dh):
    """A length of 0 or below acts as 1, a length above s as s: same bits as the clamped lengths."""
    b, s, a = 4, 96, 2
    h = a * dh
    rng = np.random.default_rng(5)
    QKV, DO = dev(rnd(rng, (b, s, 3 * h), dtype), dtype), dev(rnd(rng, (b, s, h), dtype), dtype)
    L = B.lib()
    outs = []
    for lens in ([0, s + 7, -3, 50], [1, s, 1, 50]):
        LEN = torch.tensor(lens, dtype=torch.int32, device="cuda")
        O, DQKV = empty((b, s, h), dtype), empty((b, s, 3 * h), dtype)
        lse = torch.empty((b, a, s), device="cuda"); delta = torch.empty((b, a, s), device="cuda")
        assert L.k2bw_attention_fwd(dtype, b, s, a, dh, 2, LEN.data_ptr(), QKV.data_ptr(), O.data_ptr(),
                                    lse.data_ptr(), None) == 0
        assert L.k2bw_attention_bwd(dtype, b, s, a, dh, 2, LEN.data_ptr(), QKV.data_ptr(), O.data_ptr(),
                                    lse.data_ptr(), DO.data_ptr(), DQKV.data_ptr(), delta.data_ptr(), None, 0, None,
                                    None) == 0
        sync()
        outs.append((to_host(O), to_host(lse), to_host(DQKV)))
    for got, want in zip(*outs):
        assert np.isfinite(got).all() and np.array_equal(got, want)


def test_momentum_sgd_kernel():
    rng = np.random.default_rng(11)
    n, m_micro, lr, beta = 4096 * 5 + 8, 4, 0.05, 0.9
    w = rng.standard_normal(n).astype(np.float32); mom = rng.standard_normal(n).astype(np.float32) * 0.1
    G = rng.standard_normal(n).astype(np.float32)
    W, M, Gd = (torch.from_numpy(a).cuda() for a in (w, mom, G))
    Wn = torch.empty_like(W); Wlp = torch.empty(n, device="cuda", dtype=torch.bfloat16)
    assert B.lib().k2bw_momentum(n, W.data_ptr(), Wn.data_ptr(), Wlp.data_ptr(), M.data_ptr(), Gd.data_ptr(), lr, beta,
                                 m_micro, None) == 0
    sync()
    b = float(np.float32(beta)); l = float(np.float32(lr))
    m_want = b * mom.astype(np.float64) + (1.0 - b) * G.astype(np.float64) / m_micro
    w_want = w.astype(np.float64) - l * m_want
    assert rel(to_host(M), m_want) < 1e-6 and rel(to_host(Wn), w_want) < 1e-6
    assert np.array_equal(to_host(Wlp), round_to_bf16(to_host(Wn)))


# ----------------------------------------------------------------------------- attention

ATTN_SHAPES = [  # b, s, a, dh   (the last: three 256-row blocks per head, several heads and sequences)
    (2, 50, 3, 24), (1, 200, 2, 64), (2, 130, 2, 80), (1, 257, 2, 128), (3, 64, 4, 32), (2, 700, 3, 64),
]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("b,s,a,dh", ATTN_SHAPES)
@pytest.mark.parametrize("mask", [0, 1, 2])
def test_attention_forward_backward(dtype, b, s, a, dh, mask):
    rng = np.random.default_rng(b * 1000 + s + a + dh + mask)
    h = a * dh
    qkv = rnd(rng, (b, s, 3 * h), dtype)
    d_o = rnd(rng, (b, s, h), dtype)
    lens = rng.integers(max(1, s // 3), s + 1, size=b).astype(np.int32) if mask == 2 else None
    split = lambda z, i: z[..., i * h:(i + 1) * h].reshape(b, s, a, dh).transpose(0, 2, 1, 3).astype(np.float64)
    q, k, v = (split(qkv, i) for i in range(3))
    do = d_o.reshape(b, s, a, dh).transpose(0, 2, 1, 3).astype(np.float64)
    o_want = np.empty((b, a, s, dh)); lse_want = np.empty((b, a, s))
    dq, dk, dv = np.empty_like(o_want), np.empty_like(o_want), np.empty_like(o_want)
    for n in range(b):
        vis = ob.visibility(mask, s, None if lens is None else int(lens[n]))
        o_want[n], P = ob.attention_fwd(q[n], k[n], v[n], vis)
        dq[n], dk[n], dv[n] = ob.attention_bwd(do[n], q[n], k[n], v[n], P)
        S = np.where(vis[None], q[n] @ k[n].transpose(0, 2, 1) / math.sqrt(dh), -np.inf)
        lse_want[n] = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    back = lambda z: z.transpose(0, 2, 1, 3).reshape(b, s, h)

    L = B.lib()
    QKV, DO = dev(qkv, dtype), dev(d_o, dtype)
    LEN = None if lens is None else torch.from_numpy(lens).cuda()
    O, DQKV = empty((b, s, h), dtype), empty((b, s, 3 * h), dtype)
    lse = torch.empty((b, a, s), device="cuda"); delta = torch.empty((b, a, s), device="cuda")
    lp = None if LEN is None else LEN.data_ptr()
    assert L.k2bw_attention_fwd(dtype, b, s, a, dh, mask, lp, QKV.data_ptr(), O.data_ptr(), lse.data_ptr(), None) == 0
    sync()
    assert rel(to_host(O), back(o_want)) < TIGHT[dtype]
    assert rel(to_host(lse), lse_want) < 1e-5 if dtype == F32 else rel(to_host(lse), lse_want) < 1e-3
    # the backward consumes the forward's own O (as the stage does), compared with the exact one
    fused = dtype == BF16 and dh in (32, 64, 80, 128)       # the MFMA kernels also emit the QKV bias gradient
    db = torch.full((3 * h,), float("nan"), device="cuda") if fused else None
    ws = torch.empty(L.k2bw_attention_bwd_workspace(b, s, a, dh), device="cuda") if fused else None
    for acc in ((0, 1) if fused else (0,)):
        assert L.k2bw_attention_bwd(dtype, b, s, a, dh, mask, lp, QKV.data_ptr(), O.data_ptr(), lse.data_ptr(),
                                    DO.data_ptr(), DQKV.data_ptr(), delta.data_ptr(),
                                    None if db is None else db.data_ptr(), acc,
                                    None if ws is None else ws.data_ptr(), None) == 0
    sync()
    got = to_host(DQKV)
    if fused:
        want_db = 2.0 * np.concatenate([back(dq), back(dk), back(dv)], axis=-1).reshape(-1, 3 * h).sum(0)
        assert rel(to_host(db), want_db) < 1.2e-2
    tol = 5e-6 if dtype == F32 else 1.2e-2
    assert rel(got[..., :h], back(dq)) < tol
    assert rel(got[..., h:2 * h], back(dk)) < tol
    assert rel(got[..., 2 * h:], back(dv)) < tol
    if mask == 2:       # masked keys receive exactly zero gradient
        for n in range(b):
            assert np.all(got[n, lens[n]:, h:] == 0.0)


# ----------------------------------------------------------------------------- Adam

@pytest.mark.parametrize("lp", [False, True])
def test_adam_kernel_three_steps(lp):
    rng = np.random.default_rng(5)
    n, m_micro = 4 * 100_003, 4
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    f32 = lambda z: float(np.float32(z))        # the ABI carries the hyper-parameters as floats
    opt = tb.Adam(f32(1e-3), f32(0.9), f32(0.999), f32(1e-8))
    state = opt.init(w0.astype(np.float64))
    w_or = w0.astype(np.float64)
    Wc, Wn = torch.from_numpy(w0).cuda(), torch.empty(n, device="cuda")
    Wlp = torch.empty(n, device="cuda", dtype=torch.bfloat16) if lp else None
    M, V = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    L = B.lib()
    for t in range(3):
        G = (rng.standard_normal(n) * 1e-3 * m_micro).astype(np.float32)
        G[::7] = 0.0
        w_prev = w_or
        w_or = opt.step(w_or, G.astype(np.float64) / m_micro, state, t)
        Gd = torch.from_numpy(G).cuda()
        src, dst = (Wc, Wc) if lp else ((Wc, Wn) if t % 2 == 0 else (Wn, Wc))
        assert L.k2bw_adam(n, src.data_ptr(), dst.data_ptr(), None if Wlp is None else Wlp.data_ptr(), M.data_ptr(),
                           V.data_ptr(), Gd.data_ptr(), 1e-3, 0.9, 0.999, 1e-8, m_micro, t + 1, None) == 0
        sync()
        assert rel(to_host(M), state["m"]) < 1e-6 and rel(to_host(V), state["v"]) < 1e-6
        assert rel(to_host(dst).astype(np.float64) - w_prev, w_or - w_prev) < 1e-4
        if lp:
            assert np.array_equal(to_host(Wlp), round_to_bf16(to_host(dst)))
        else:
            assert rel(to_host(src), w_prev) < 1e-7          # W(t) is left intact: the other buffer was written
