"""lstm_fwd_noalloc (the entry point for callers that cannot allocate: its scratch is a device array inside the
library) against lstm_fwd, through the C ABI, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_1608_00895_amd import binding as rl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(T, B, D, H, direction, seed, engine):
    rng = np.random.Generator(np.random.Philox(seed))
    host = dict(x=rng.standard_normal((T, B, D)), W=rng.uniform(-0.3, 0.3, (D, 4 * H)), R=rng.uniform(-0.3, 0.3, (H, 4 * H)),
                b=rng.uniform(-0.3, 0.3, (4 * H,)), h0=rng.uniform(-0.5, 0.5, (B, H)), c0=rng.uniform(-0.5, 0.5, (B, H)))
    t = {k: torch.from_numpy(v.astype(np.float32)).to(DEV) for k, v in host.items()}
    lens = rng.integers(0, T + 1, B).astype(np.int32)
    lens[0] = T
    t["lens"] = torch.from_numpy(lens).to(DEV)
    desc = rl.rlstm_desc(T=T, B=B, D=D, H=H, direction=direction, operand_dtype=0, ldx=0, ldy=0, engine=engine)
    return desc, t


def _outputs(T, B, H, desc):
    nan = float("nan")
    return dict(y=torch.full((T, B, H), nan, device=DEV), c=torch.full((T, B, H), nan, device=DEV),
                hT=torch.full((B, H), nan, device=DEV), cT=torch.full((B, H), nan, device=DEV),
                reserve=torch.full((rl.rlstm_reserve_bytes(desc) // 4,), nan, device=DEV))


@pytest.mark.parametrize("engine", [rl.RLSTM_ENGINE_PERSISTENT, rl.RLSTM_ENGINE_STEPWISE])
def test_noalloc_forward_equals_lstm_fwd_on_two_calls_in_a_row(engine):
    # the second call is smaller in every dimension and finds the first call's contents in the scratch
    for k, (T, B, D, H, direction) in enumerate([(37, 21, 12, 72, 1), (19, 5, 7, 36, -1)]):
        desc, t = _case(T, B, D, H, direction, 900 + k, engine)
        need = rl.rlstm_noalloc_scratch_bytes(desc)
        assert 0 < need <= rl.RLSTM_NOALLOC_SCRATCH_LIMIT
        ref = _outputs(T, B, H, desc)
        ws = torch.empty(rl.rlstm_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
        rl.lstm_fwd(desc, t["x"], t["W"], t["R"], t["b"], t["h0"], t["c0"], t["lens"], ref["y"], ref["c"], ref["hT"],
                    ref["cT"], ref["reserve"], ws)
        assert rl.rlstm_last_timeout(ws) == 0
        got = _outputs(T, B, H, desc)
        before = torch.cuda.memory_allocated()
        rl.lstm_fwd_noalloc(desc, t["x"], t["W"], t["R"], t["b"], t["h0"], t["c0"], t["lens"], got["y"], got["c"],
                            got["hT"], got["cT"], got["reserve"])
        assert torch.cuda.memory_allocated() == before
        assert rl.rlstm_last_timeout_on(None) == 0
        for name in ("y", "c", "hT", "cT", "reserve"):
            a, b = got[name].cpu().numpy(), ref[name].cpu().numpy()
            if name == "reserve":                    # the activated gates [T,B,4H]; the rest of the buffer is alignment
                a, b = a[:T * B * 4 * H], b[:T * B * 4 * H]
            assert not np.isnan(a).any(), name
            # the same kernels with the same launch shapes ran on the same inputs: the same bits, which is within any bar
            assert np.array_equal(a, b), (name, float(np.abs(a - b).max()))


def test_noalloc_rejects_shapes_beyond_its_scratch_and_bad_arguments():
    big = rl.rlstm_desc(T=8, B=64, D=8, H=4096, direction=1, operand_dtype=0, ldx=0, ldy=0, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.rlstm_noalloc_scratch_bytes(big) > rl.RLSTM_NOALLOC_SCRATCH_LIMIT
    t = torch.zeros(16, device=DEV)
    assert rl.lstm_fwd_noalloc(big, t, t, t, t, None, None, t, t, t, None, None, t, check=False) == -4
    ok = rl.rlstm_desc(T=4, B=2, D=3, H=4, direction=1, operand_dtype=0, ldx=0, ldy=0, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.lstm_fwd_noalloc(ok, None, t, t, t, None, None, t, t, t, None, None, t, check=False) == -1
    bad = rl.rlstm_desc(T=0, B=2, D=3, H=4, direction=1, operand_dtype=0, ldx=0, ldy=0, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.lstm_fwd_noalloc(bad, t, t, t, t, None, None, t, t, t, None, None, t, check=False) == -2
    assert rl.rlstm_noalloc_scratch_bytes(bad) == 0
