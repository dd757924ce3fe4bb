"""The C-ABI library loads, exports every symbol include/hfta.h declares, and
rejects bad arguments before any launch (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2102_02344_amd import binding
    return binding


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "hfta.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(hfta_[a-z0-9_]+)\s*\(", src)))


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 25
    raw = lib.raw()
    for n in names:
        assert hasattr(raw, n), n
    assert set(names) == set(lib.EXPORTS)
    assert lib.version() >= 100
    assert lib.status_string(0) == "ok" and "workspace" in lib.status_string(-3)


def test_validation_precedes_launch(lib):
    raw = lib.raw()
    s4 = (C.c_int64 * 4)(12, 24, 4, 1)
    bad_l = (C.c_int64 * 4)(12, 24, 4, 2)
    one = C.c_void_p(16)      # never dereferenced: validation fails first
    # B <= 0, null pointers, bad dtype
    assert raw.hfta_linear_fwd(0, 4, 4, 4, 0, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 0, None, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 7, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 4, 4, 4, 0, one, one, None, one, 99, 0.0, None) == lib.EINVAL
    assert raw.hfta_linear_fwd(1, 1 << 20, 1 << 12, 4, 0, one, one, None, one, 0, 0.0, None) == lib.EINVAL
    # stride_l != 1 is not implemented for the conv family
    assert raw.hfta_conv1x1_fwd(1, 2, 3, 4, 4, 0, one, bad_l, one, None, one, s4, 0, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_conv1x1_fwd(1, 2, 3, 4, 4, 0, one, None, one, None, one, s4, 0, 0.0, None) == lib.EINVAL
    # workspace too small / missing
    need = raw.hfta_conv1x1_bwd_workspace_bytes(8, 32, 128, 1024, 2500, 1)
    assert need > 0
    assert raw.hfta_conv1x1_bwd(8, 32, 128, 1024, 2500, 1, one, s4, one, one, s4, None, None, one, None,
                                None, 0, None) == lib.EWORKSPACE
    assert raw.hfta_conv1x1_bwd(8, 32, 128, 1024, 2500, 1, one, s4, one, one, s4, None, None, one, None,
                                one, need - 1, None) == lib.EWORKSPACE
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, bad_l, one, one, 1e-5, 0.1, None, None, one, one, one, bad_l,
                           0, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, s4, one, one, 1e-5, 0.1, one, None, one, one, one, s4,
                           0, 0.0, None) == lib.EINVAL
    assert raw.hfta_bn_fwd(1, 2, 3, 4, 0, one, s4, one, one, 1e-5, 0.1, None, None, one, one, one, s4,
                           lib.ACT_TANH, 0.0, None) == lib.EUNSUPPORTED
    assert raw.hfta_adam_step(2, 8, 0, one, one, one, one, None, one, one, one, one, one, 0, 0, None) == lib.EINVAL
    assert raw.hfta_adam_step(2, 0, 0, one, one, one, one, None, one, one, one, one, one, 1, 0, None) == lib.EINVAL
    assert raw.hfta_maxpool_points(1, 1, 1, 0, 0, one, s4, one, one, (C.c_int64 * 3)(1, 1, 1), None) == lib.EINVAL
    assert raw.hfta_dropout(8, 0, one, one, 1.0, one, None) == lib.EINVAL
    assert raw.hfta_act_bwd(8, 0, one, one, one, lib.ACT_GELU, 0.0, 1, None) == lib.EUNSUPPORTED
    assert raw.hfta_layernorm_bwd(1, 4, 8, 0, one, one, one, one, one, one, one, one, None, 0, None) == lib.EWORKSPACE
