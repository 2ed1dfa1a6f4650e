"""The C-ABI library loads and exports every symbol the headers declare (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2006_09503_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b((?:stage|k2bw)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    L = binding.lib()
    names = declared_functions()
    assert len(names) >= 30
    for n in names:
        assert hasattr(L, n), n


def test_binding_covers_every_declared_symbol():
    L = binding.lib()
    for n in declared_functions():
        assert getattr(L, n).argtypes is not None, f"binding has no signature for {n}"


def test_strerror_and_codes():
    assert binding.strerror(0) == "ok"
    assert "schedule" in binding.strerror(binding.ERR_BAD_STATE)
    assert "invalid" in binding.strerror(binding.ERR_INVALID_ARG)


def test_param_counts_of_the_workload_shapes():
    want = {"C1": 396_544, "C2": 75_577_344, "C3": 629_411_840, "C4": 805_519_360, "C5": 1_610_825_728}
    for name, n in want.items():
        cfg = synth.PRESETS[name]
        assert binding.stage_param_count(cfg) == n == synth.param_count(cfg)


def test_stream_recommendation_follows_the_smallest_projection():
    """Two streams while the smallest projection (T x h outputs) leaves CUs without a 256x256 tile, one from 256
    tiles on: 16 x 4, 16 x 10, 16 x 16 and 8 x 32 tiles at the four large workload shapes."""
    want = {"C2": 2, "C3": 2, "C4": 1, "C5": 1}
    for name, n in want.items():
        assert synth.PRESETS[name].recommended_streams == n
    assert synth.PRESETS["C2"].with_(microbatch=32).recommended_streams == 1   # 64 x 4 tiles


@pytest.mark.parametrize("bad", [dict(hidden=100), dict(n_heads=3), dict(m=1, max_inflight=2), dict(mask_mode=5),
                                 dict(precision=7), dict(n_layers=0), dict(ffn=12), dict(hidden=16, n_heads=4),
                                 dict(beta1=1.0), dict(recompute=2),
                                 dict(hidden=16384, n_heads=128, ffn=65536),          # h*f = 2^30 elements
                                 dict(seq=4096, microbatch=1024, ffn=256)])           # T*f = 2^30 elements
def test_invalid_configs_are_rejected(bad):
    cfg = synth.PRESETS["C1"].with_(**bad)
    with pytest.raises(binding.StageError) as e:
        binding.stage_param_count(cfg)
    assert e.value.code == binding.ERR_INVALID_ARG


def test_config_struct_layout_matches_header():
    # 14 int32 + 5 float, no padding
    assert ctypes.sizeof(binding.StageConfigC) == 19 * 4
    text = open(os.path.join(ROOT, "include", "stage2bw.h")).read()
    body = text[text.index("typedef struct {"):text.index("} stage_config_t;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.replace("typedef struct {", "").strip()
        if not decl:
            continue
        parts = decl.replace(",", " ").split()
        fields += parts[1:]
    assert fields == [n for n, _ in binding.StageConfigC._fields_]


def test_null_arguments_return_invalid_arg():
    L = binding.lib()
    assert L.stage_forward(None, 1, None, None, None) == binding.ERR_INVALID_ARG
    assert L.stage_backward(None, 1, None, None) == binding.ERR_INVALID_ARG
    assert L.stage_coalesce_update(None) == binding.ERR_INVALID_ARG
    assert L.stage_swap_versions(None) == binding.ERR_INVALID_ARG
    assert L.stage_set_backward_stream(None, None) == binding.ERR_INVALID_ARG
    assert L.stage_destroy(None) == binding.ERR_INVALID_ARG
    assert L.stage_sched_swap_versions(None) == binding.ERR_INVALID_ARG
    h = ctypes.c_void_p()
    assert L.stage_sched_create(2, 3, 0, ctypes.byref(h)) == binding.ERR_INVALID_ARG   # m < in-flight depth
