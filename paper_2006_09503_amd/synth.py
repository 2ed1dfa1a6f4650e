"""Seeded synthetic inputs for one 2BW pipeline stage.

This module holds no arithmetic of the method: it only describes stage shapes,
the flat parameter layout (a storage format) and draws random tensors.  Both the
CPU oracle's tests and the HIP path's tests/bench feed on the arrays it returns;
neither side's code is imported here.

Input recipe (the paper trains transformer language models on OpenWebText with
sequence length 512, Section 5; throughput of a stage depends on shapes only, so
Gaussian tensors of the same shapes stand in):

* weights and biases ~ N(0, 0.02^2); LayerNorm gain = 1 + N(0, 0.02^2),
  LayerNorm shift ~ N(0, 0.02^2) (no parameter sits at a degenerate value);
* boundary activation X_k ~ N(0, 1), shape [microbatch, seq, hidden];
* boundary gradient dY_k ~ N(0, (1e-2)^2), rows of padded positions zeroed;
* key-padding lengths uniform in [min_len, seq] per sequence.

Draw order from one PCG64 stream: weights in flat-layout order, then for
k = 1, 2, ...: X_k, dY_k, len_k.
"""
from __future__ import annotations

from dataclasses import dataclass, replace, asdict
from typing import Dict, List, Optional, Tuple

import numpy as np

MASK_NONE = 0
MASK_CAUSAL = 1
MASK_PADDING = 2

PREC_FP32 = 0
PREC_BF16 = 1

OPT_ADAM = 0
OPT_MOMENTUM = 1


@dataclass(frozen=True)
class StageConfig:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    seq: int
    microbatch: int
    m: int                      # microbatches per coalesced update (Section 3.1)
    max_inflight: int           # activation stash slots (in-flight microbatches, Section 3.1)
    mask_mode: int = MASK_NONE
    precision: int = PREC_FP32
    recompute: int = 0          # Section 4.1: stash only the stage input
    flush: int = 0              # Section 3.2: one weight version, pipeline flush per batch
    optimizer: int = 0          # 0 Adam, 1 SGD with momentum (Section 3.1's printed form, beta = beta1)
    wgrad_group: int = 0        # backward passes per grouped weight-gradient launch (0: the library's choice)
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    ln_eps: float = 1e-5
    min_len: int = 0            # only used to draw padding lengths

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    @property
    def tokens(self) -> int:
        return self.microbatch * self.seq

    def with_(self, **kw) -> "StageConfig":
        return replace(self, **kw)

    @property
    def recommended_streams(self) -> int:
        """1 or 2 HIP streams for a lone stage.  A backward stream of its own lets the forward pass of one
        microbatch fill what the backward kernels of another leave idle: ramps and drains, and the CUs that a
        launch of fewer than one 256x256 tile per CU does not use (measured +7 % at h = 1024 and 2560 with 4096
        tokens).  Once the smallest projection gives every CU a tile, two GEMM launches that run side by side
        only take CUs from each other, and the 32 tiles an XCD runs at a time no longer form one block that
        shares operand panels in its L2: measured, one stream is then 3 % (h = 8192, 2048 tokens) and 1.4 %
        (h = 4096, 4096 tokens) faster than two."""
        tiles = -(-self.tokens // 256) * -(-self.hidden // 256)
        return 1 if tiles >= 256 else 2

    def as_dict(self) -> Dict:
        return asdict(self)


# The five workload shapes (tiny parity case; BERT-Large quarter; GPT h=2560; GPT h=4096 with
# activation recomputation; memory stress).
PRESETS: Dict[str, StageConfig] = {
    "C1": StageConfig(2, 128, 4, 512, 64, 2, 4, 2, MASK_NONE, PREC_FP32),
    "C2": StageConfig(6, 1024, 16, 4096, 512, 8, 8, 4, MASK_PADDING, PREC_BF16, min_len=384),
    "C3": StageConfig(8, 2560, 32, 10240, 1024, 4, 16, 4, MASK_CAUSAL, PREC_BF16),
    "C4": StageConfig(4, 4096, 32, 16384, 2048, 2, 32, 4, MASK_CAUSAL, PREC_BF16, recompute=1),
    "C5": StageConfig(2, 8192, 64, 32768, 2048, 1, 64, 4, MASK_CAUSAL, PREC_BF16),
}


def layer_layout(hidden: int, ffn: int) -> List[Tuple[str, Tuple[int, ...]]]:
    """Per-layer tensors of the flat fp32 parameter vector, in storage order.

    Matrices are row-major [in, out] (y = x W + b); Wqkv's columns are Q|K|V, each
    head-major.
    """
    h, f = hidden, ffn
    return [
        ("ln1_g", (h,)), ("ln1_b", (h,)),
        ("wqkv", (h, 3 * h)), ("bqkv", (3 * h,)),
        ("wo", (h, h)), ("bo", (h,)),
        ("ln2_g", (h,)), ("ln2_b", (h,)),
        ("w1", (h, f)), ("b1", (f,)),
        ("w2", (f, h)), ("b2", (h,)),
    ]


def layer_param_count(hidden: int, ffn: int) -> int:
    return sum(int(np.prod(s)) for _, s in layer_layout(hidden, ffn))


def param_count(cfg: StageConfig) -> int:
    return cfg.n_layers * layer_param_count(cfg.hidden, cfg.ffn)


def param_slices(cfg: StageConfig) -> List[Dict[str, Tuple[int, Tuple[int, ...]]]]:
    """[{name: (offset, shape)}] per layer, offsets into the flat vector."""
    out, off = [], 0
    for _ in range(cfg.n_layers):
        d = {}
        for name, shape in layer_layout(cfg.hidden, cfg.ffn):
            d[name] = (off, shape)
            off += int(np.prod(shape))
        out.append(d)
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bfloat16 (round to nearest even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(a.shape)


class StageInputs:
    """Stream of seeded inputs for one stage; see the module docstring for the recipe."""

    def __init__(self, cfg: StageConfig, seed: int = 0):
        self.cfg = cfg
        self.rng = np.random.Generator(np.random.PCG64(seed))
        self._weights_drawn = False
        self._quantise = cfg.precision == PREC_BF16

    def _q(self, a: np.ndarray) -> np.ndarray:
        return round_to_bf16(a) if self._quantise else a

    def weights(self) -> np.ndarray:
        assert not self._weights_drawn, "weights are the first draw of the stream"
        self._weights_drawn = True
        cfg = self.cfg
        w = np.empty(param_count(cfg), dtype=np.float32)
        for layer in param_slices(cfg):
            for name, (off, shape) in layer.items():
                n = int(np.prod(shape))
                v = self.rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
                if name in ("ln1_g", "ln2_g"):
                    v += np.float32(1.0)
                w[off:off + n] = v
        return self._q(w)

    def microbatch(self) -> Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]:
        """Next (X_k, dY_k, len_k); len_k is None unless the mask is key-padding."""
        assert self._weights_drawn, "draw weights() first to keep the stream order fixed"
        cfg = self.cfg
        shape = (cfg.microbatch, cfg.seq, cfg.hidden)
        x = self.rng.standard_normal(shape, dtype=np.float32)
        dy = self.rng.standard_normal(shape, dtype=np.float32) * np.float32(1e-2)
        lens = None
        if cfg.mask_mode == MASK_PADDING:
            lo = cfg.min_len if cfg.min_len > 0 else 1
            lens = self.rng.integers(lo, cfg.seq + 1, size=cfg.microbatch).astype(np.int32)
            for n in range(cfg.microbatch):
                dy[n, lens[n]:, :] = 0.0
        return self._q(x), self._q(dy), lens

    def microbatches(self, count: int):
        return [self.microbatch() for _ in range(count)]
