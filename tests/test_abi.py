"""The C-ABI library loads, exports every symbol the header declares, and validates its arguments
on the host before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import partime_streams as ps
from paper_2210_09147_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "partime.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(partime_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = header_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_binding_constants_match_header():
    src = open(os.path.join(ROOT, "include", "partime.h")).read()
    for name in ("PT_DENSE", "PT_CONV3X3", "PT_GAP_DENSE", "PT_ID", "PT_RELU", "PT_GELU", "PT_LOSS_NONE",
                 "PT_LOSS_MSE", "PT_LOSS_CE", "PT_F32", "PT_BF16", "PT_EXEC_AUTO", "PT_EXEC_LAUNCH_PER_TICK",
                 "PT_EXEC_PERSISTENT", "PT_OK", "PT_EINVAL", "PT_ESHAPE", "PT_ENOMEM", "PT_EHIP", "PT_EUNSUPPORTED"):
        m = re.search(r"\b%s\s*=\s*(-?\d+)" % name, src)
        assert m and int(m.group(1)) == getattr(B, name), name


def _init(layers, **kw):
    Ws, bs = ps.init_weights(layers, 0)
    return B.partime_init(layers, Ws, bs, **kw)


def test_init_rejects_bad_arguments_on_the_host():
    good = ps.mlp([8, 8, 4], ps.ACT_RELU)
    cases = [
        (dict(n_streams=0), B.PT_EINVAL),
        (dict(w_dtype=7), B.PT_EINVAL),
        (dict(loss=9), B.PT_EINVAL),
        (dict(target_delay=-1), B.PT_EINVAL),
        (dict(exec_mode=5), B.PT_EINVAL),
        (dict(balance=[1, 2]), B.PT_ESHAPE),
        (dict(balance=[0, 2]), B.PT_EINVAL),
    ]
    for kw, code in cases:
        with pytest.raises(B.PartimeError) as e:
            _init(good, **kw)
        assert e.value.code == code, (kw, str(e.value))
        assert B.partime_last_error()
    bad_chain = [ps.LayerSpec(ps.DENSE, ps.ACT_RELU, 8, 8), ps.LayerSpec(ps.DENSE, ps.ACT_ID, 7, 4)]
    with pytest.raises(B.PartimeError) as e:
        _init(bad_chain)
    assert e.value.code == B.PT_ESHAPE
    bad_act = [ps.LayerSpec(ps.DENSE, 5, 8, 8)]
    with pytest.raises(B.PartimeError) as e:
        _init(bad_act)
    assert e.value.code == B.PT_EINVAL
    wide = [ps.LayerSpec(ps.DENSE, ps.ACT_ID, 5000, 8)]
    with pytest.raises(B.PartimeError) as e:
        _init(wide)
    assert e.value.code == B.PT_EUNSUPPORTED


def test_init_rejects_unsupported_combinations_on_the_host():
    """Stream counts, Adam and skip connections are checked before anything touches the GPU."""
    good = ps.mlp([8, 8, 8, 4], ps.ACT_RELU)
    adam = (0.9, 0.999, 1e-8)

    def skip(dst, src, layers=None):
        ls = ps.mlp([8, 8, 8, 4], ps.ACT_RELU) if layers is None else layers
        ls[dst].skip_from = src
        return ls

    cases = [
        (good, dict(n_streams=48, w_dtype=B.PT_BF16), B.PT_EUNSUPPORTED),     # neither 32 nor a multiple of 64
        (good, dict(n_streams=2048, w_dtype=B.PT_BF16), B.PT_EUNSUPPORTED),   # beyond the largest batch
        (good, dict(n_streams=64), B.PT_EUNSUPPORTED),                         # several streams take bf16 weights
        (good, dict(adam=(1.0, 0.999, 1e-8)), B.PT_EINVAL),
        (good, dict(adam=(0.9, 0.999, 0.0)), B.PT_EINVAL),
        (good, dict(adam=adam, exec_mode=B.PT_EXEC_PERSISTENT), B.PT_EUNSUPPORTED),
        (skip(1, 1), {}, B.PT_EINVAL),                                         # not an earlier layer
        (skip(2, 0), {}, B.PT_EUNSUPPORTED),                                   # into the last layer
        (skip(1, 0, ps.mlp([8, 6, 8, 4], ps.ACT_RELU)), {}, B.PT_ESHAPE),      # sizes differ
    ]
    for layers, kw, code in cases:
        with pytest.raises(B.PartimeError) as e:
            _init(layers, **kw)
        assert e.value.code == code, (kw, str(e.value))


def test_null_context_calls_return_errors():
    lib = B.load()
    assert lib.partime_step(None, None, None, 1, None, None) == B.PT_EINVAL
    assert lib.partime_infer(None, None, 1, None) == B.PT_EINVAL
    assert lib.partime_get_state(None, 0, None, None) == B.PT_EINVAL
    assert lib.partime_reset(None) == B.PT_EINVAL
    assert lib.partime_set_lr(None, 0.1) == B.PT_EINVAL
    lib.partime_destroy(None)
    assert b"null" in lib.partime_last_error()


def test_no_gpu_means_a_loud_failure_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.PartimeError) as e:
        _init(ps.mlp([8, 8, 4], ps.ACT_RELU))
    assert e.value.code in (B.PT_EHIP, B.PT_ENOMEM)
    from paper_2210_09147_amd import Pipeline
    layers = ps.mlp([8, 8, 4], ps.ACT_RELU)
    Ws, bs = ps.init_weights(layers, 0)
    with pytest.raises(RuntimeError):
        Pipeline(layers, Ws, bs)


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2210_09147_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in txt and "partime_oracle" not in txt, f
