"""CPU-side checks of the boundary: the library loads and exports exactly what
include/qzo.h declares; host-only entry points behave; argument errors are
reported before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2505_13430_amd import binding as qb
from paper_2505_13430_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "qzo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qzo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = qb.lib()
    names = _declared()
    assert "qzo_step" in names and "qzo_dequant_gemm" in names and "qzo_forward_loss" in names
    assert "qzo_model_create" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(qb.EXPORTS) == names


def test_scale_count_is_table2(oracle):
    assert qb.qzo_model_scale_count(synth.SHAPES["llama-2-7b"]) == 50593792
    opt67 = dict(arch="opt", n_layers=32, d_model=4096, n_heads=32, d_ffn=16384, vocab=50272, max_seq=64)
    assert qb.qzo_model_scale_count(opt67) == 50331648
    for name in ("tiny", "tiny_opt", "opt-1.3b", "llama-2-13b"):
        assert qb.qzo_model_scale_count(synth.SHAPES[name]) == synth.n_scales(synth.SHAPES[name])


def test_config_errors_are_reported():
    bad = dict(synth.SHAPES["tiny"], d_model=200)
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_model_scale_count(bad)
    assert e.value.status == qb.QZO_ERR_SHAPE and "128" in str(e.value)
    bad = dict(synth.SHAPES["tiny"], n_heads=16)      # head size 16
    with pytest.raises(qb.QzoError):
        qb.qzo_model_scale_count(bad)
    cfg = qb.make_config(synth.SHAPES["tiny"])
    cfg.struct_size = 4
    out = C.c_uint64(0)
    assert qb.lib().qzo_model_scale_count(C.byref(cfg), C.byref(out)) == qb.QZO_ERR_ARG
    # null pointers never reach a kernel
    assert qb.lib().qzo_dequant_gemm(None, None, None, 0, 1, 8, 128, 128, C.c_uint64(0),
                                     C.c_float(0), 1, None, None, None) == qb.QZO_ERR_ARG
    assert qb.lib().qzo_step(None, None, 1, 2, C.c_uint64(0), C.c_float(0), C.c_float(0),
                             C.c_float(1), None, C.c_uint64(0), None, None) == qb.QZO_ERR_ARG
