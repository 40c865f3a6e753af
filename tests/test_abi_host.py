"""Host-only checks of the C ABI: the built library exports every function the header declares,
and argument validation answers before any device call (so it works without a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2111_00705_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            text = open(os.path.join(inc, header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(comp_ams_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 18
    L = P.lib()
    for name in names:
        assert hasattr(L, name), name
    assert sorted(P.EXPORTS) == names        # the Python binding covers the same set


@pytest.mark.parametrize("args", [
    dict(d=0), dict(d=2 ** 31), dict(n=0), dict(n=70000), dict(compressor=7),
    dict(compressor=P.TOPK, k_or_block=0), dict(compressor=P.TOPK, k_or_block=101),
    dict(compressor=P.BLOCKSIGN, k_or_block=0),
    dict(beta1=1.0), dict(beta1=-0.1), dict(beta2=1.5), dict(beta2=float("nan")),
    dict(eps=0.0), dict(eps=-1e-8), dict(eps=float("inf")), dict(lr=0.0), dict(lr=float("nan")),
])
def test_create_rejects_invalid_arguments_on_the_host(args):
    kw = dict(d=100, n=2, compressor=P.TOPK, k_or_block=10, beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3)
    kw.update(args)
    with pytest.raises(P.CompAmsError) as ei:
        P.CompAms(**kw)
    assert ei.value.code == P.EINVAL
    assert str(ei.value)


def test_create_with_null_out_pointer_and_null_handles():
    L = P.lib()
    assert L.comp_ams_create(None, 10, 1, 0, 1, 0.9, 0.999, 1e-8, 1e-3) == P.EINVAL
    assert L.comp_ams_last_error(None)
    buf = np.zeros(4, np.float32)
    assert L.comp_ams_step(None, buf.ctypes.data, None) == P.EINVAL
    assert L.comp_ams_get_theta(None, buf.ctypes.data, 0) == P.EINVAL
    assert L.comp_ams_set_lr(None, 0.1) == P.EINVAL
    assert L.comp_ams_n_blocks(None) == P.EINVAL
    assert L.comp_ams_step_bf16(None, buf.ctypes.data, None) == P.EINVAL
    assert L.comp_ams_step_f16(None, buf.ctypes.data, None) == P.EINVAL
    assert L.comp_ams_set_method(None, P.METHOD_CD) == P.EINVAL
    assert L.comp_ams_set_rand(None, 1, 0) == P.EINVAL
    assert L.comp_ams_set_streaming(None, -1, -1) == P.EINVAL
    assert L.comp_ams_set_tile_order(None, -1) == P.EINVAL
    assert L.comp_ams_set_pass_lds(None, -1) == P.EINVAL
    assert L.comp_ams_set_eps_mode(None, 1) == P.EINVAL
    L.comp_ams_destroy(None)                       # no-op


def test_valid_create_without_gpu_reports_a_device_error_not_a_crash():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(P.CompAmsError) as ei:
        P.CompAms(100, 2, P.TOPK, 10)
    assert ei.value.code == P.EDEVICE
