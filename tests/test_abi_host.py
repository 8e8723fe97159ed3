"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_1608_00895_amd import binding as rl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "rlstm.h")).read()
    return re.findall(r"RLSTM_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 12
    L = ctypes.CDLL(rl.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(names) == sorted(rl.EXPORTS)


def test_version_and_error_strings():
    assert rl.version() == "0.3"
    for code in range(0, -7, -1):
        assert "unknown" not in rl.strerror(code)
    assert "unknown" in rl.strerror(-99)


def test_sizes_and_descriptor_validation():
    d = rl.rlstm_desc(T=20, B=2, D=8, H=16, direction=1)
    assert rl.rlstm_reserve_bytes(d) >= 20 * 2 * 64 * 4
    assert rl.rlstm_workspace_bytes(d) > 0
    for bad in (dict(T=0), dict(B=-1), dict(H=0), dict(direction=0), dict(direction=2), dict(operand_dtype=7),
                dict(engine=9), dict(ldx=4), dict(ldy=3)):
        kw = dict(T=20, B=2, D=8, H=16, direction=1)
        kw.update(bad)
        assert rl.rlstm_reserve_bytes(rl.rlstm_desc(**kw)) == 0, bad
        assert rl.rlstm_workspace_bytes(rl.rlstm_desc(**kw)) == 0, bad
    s = rl.rblstm_desc(L=4, T=1000, B=32, D=40, H=500)
    per_layer = 1000 * 32 * (2 * 2000 + 2 * 500 + 1000) * 4     # gates and cells of both directions, the layer's output
    top_y = 1000 * 32 * 1000 * 4                                 # the top layer's output is the caller's y_top
    assert 4 * per_layer - top_y <= rl.rblstm_reserve_bytes(s) < 4 * per_layer
    assert rl.rblstm_workspace_bytes(s) >= 2 * 1000 * 32 * 1000 * 4
    assert rl.rblstm_reserve_bytes(rl.rblstm_desc(L=0, T=1, B=1, D=1, H=1)) == 0


def test_argument_errors_are_returned_before_any_device_work():
    L = rl.lib()
    d = rl.rlstm_desc(T=4, B=2, D=3, H=4, direction=1)
    nulls = [None] * 14
    assert L.lstm_fwd(None, *nulls) == -1
    assert L.lstm_fwd(ctypes.byref(d), *nulls) == -1
    assert L.lstm_fwd(ctypes.byref(rl.rlstm_desc(T=0, B=2, D=3, H=4, direction=1)), *nulls) == -2
    assert L.lstm_fwd(ctypes.byref(rl.rlstm_desc(T=4, B=2, D=3, H=4, direction=3)), *nulls) == -3
    assert L.lstm_bwd(ctypes.byref(d), *([None] * 20)) == -1
    s = rl.rblstm_desc(L=1, T=4, B=2, D=3, H=4)
    assert L.blstm_stack_fwd_bwd(ctypes.byref(s), None, None, None, None, None, None, None, None, None, None, None) == -1
    assert L.blstm_stack_fwd_bwd(ctypes.byref(rl.rblstm_desc(L=1, T=4, B=0, D=3, H=4)),
                                 None, None, None, None, None, None, None, None, None, None, None) == -2
    assert L.rlstm_gemm_f32(0, 0, 4, 4, 4, None, 4, None, 4, None, 4, None, 0, None, 0, None) == -1
    assert L.rlstm_last_timeout(None) == -1


def test_binding_refuses_host_tensors():
    import torch
    d = rl.rlstm_desc(T=4, B=2, D=3, H=4, direction=1)
    t = torch.zeros(8)
    with pytest.raises(ValueError):
        rl.lstm_fwd(d, t, t, t, t, None, None, t, t, t, None, None, t, t, stream=object())
