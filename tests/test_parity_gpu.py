"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Tolerances (max abs difference over max abs oracle
value, per tensor): 1e-5 forward, 1e-4 gradients for fp32."""
import numpy as np
import pytest
import torch

from oracle import lstm_backward, lstm_forward
from paper_1608_00895_amd import binding as rl
from paper_1608_00895_amd import synth

import gpu_harness as gh

pytestmark = pytest.mark.gpu

TOL_FWD = 1e-5
TOL_GRAD = 1e-4
ENGINES = [rl.RLSTM_ENGINE_PERSISTENT, rl.RLSTM_ENGINE_STEPWISE]


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _check_layer(got, fwd, grad, lens, tag):
    print(tag, flush=True)
    for k in ("y", "c", "hT", "cT"):
        assert gh.rel_err(got[k], fwd[k]) < TOL_FWD, (tag, k, gh.rel_err(got[k], fwd[k]))
    T = got["y"].shape[0]
    for n, ln in enumerate(lens):
        assert np.all(got["y"][ln:, n] == 0.0), (tag, "y not zero at padded frames")
    if grad is None:
        return
    for k in ("dx", "dW", "dR", "db", "dh0", "dc0"):
        if k in got:
            assert gh.rel_err(got[k], grad[k]) < TOL_GRAD, (tag, k, gh.rel_err(got[k], grad[k]))
    if "dx" in got:
        for n, ln in enumerate(lens):
            assert np.all(got["dx"][ln:, n] == 0.0), (tag, "dx not zero at padded frames")


@pytest.mark.parametrize("engine", ENGINES)
def test_config1_single_layer(engine):
    """Config 1: T=20, B=2, D=8, H=16, all lengths 20, loss = sum(y), seed 0."""
    wl = synth.config1()
    (W, R, b), = wl.params[0]
    fwd = lstm_forward(wl.x, W, R, b, wl.seq_lens, 1)
    grad = lstm_backward(fwd, np.ones((wl.T, wl.B, wl.H)))
    got = gh.run_lstm_layer(wl.x, W, R, b, wl.seq_lens, 1, dy=np.ones((wl.T, wl.B, wl.H), np.float32), engine=engine)
    _check_layer(got, fwd, grad, wl.seq_lens, f"config1 engine={engine}")


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("shape", [
    # T, B, D, H, lens, ldx, ldy
    (13, 5, 12, 20, (13, 7, 1, 0, 9), 0, 0),        # ragged, a zero-length sequence
    (9, 3, 7, 17, (4, 6, 2), 0, 0),                 # odd H and D (scalar loads), T beyond the longest sequence
    (11, 18, 16, 36, None, 24, 80),                 # B spans two 16-row tiles, padded row strides
    (1, 2, 4, 8, (1, 1), 0, 0),                     # single frame
    (6, 1, 5, 130, (6,), 0, 0),                     # one sequence, several workgroups
    (40, 33, 8, 64, None, 0, 0),                    # B spans three tiles
])
def test_single_layer_shapes(engine, direction, shape):
    T, B, D, H, lens, ldx, ldy = shape
    rng = _rng(1000 + T * 7 + B * 3 + H + (direction > 0))
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    W = rng.uniform(-0.3, 0.3, (D, 4 * H)).astype(np.float32)
    R = rng.uniform(-0.3, 0.3, (H, 4 * H)).astype(np.float32)
    b = rng.uniform(-0.3, 0.3, (4 * H,)).astype(np.float32)
    h0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    lens = np.array(lens if lens is not None else rng.integers(0, T + 1, B), dtype=np.int32)
    dy = rng.standard_normal((T, B, H)).astype(np.float32)
    dhT = rng.standard_normal((B, H)).astype(np.float32)
    dcT = rng.standard_normal((B, H)).astype(np.float32)
    fwd = lstm_forward(x, W, R, b, lens, direction, h0, c0)
    grad = lstm_backward(fwd, dy, dhT, dcT)
    got = gh.run_lstm_layer(x, W, R, b, lens, direction, h0, c0, dy, dhT, dcT, engine=engine, ldx=ldx, ldy=ldy)
    _check_layer(got, fwd, grad, lens, f"shape={shape} dir={direction} engine={engine}")
    if ldy:
        assert np.all(np.isnan(got["y_pad"])), "padding columns of y were written"


def test_null_optional_arguments():
    """h0/c0/dhT/dcT null means zeros; hT/cT/dx/dh0/dc0 null means not wanted."""
    rng = _rng(7)
    T, B, D, H = 8, 4, 6, 12
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    W = rng.uniform(-0.3, 0.3, (D, 4 * H)).astype(np.float32)
    R = rng.uniform(-0.3, 0.3, (H, 4 * H)).astype(np.float32)
    b = rng.uniform(-0.3, 0.3, (4 * H,)).astype(np.float32)
    lens = np.array([8, 3, 5, 8], np.int32)
    dy = rng.standard_normal((T, B, H)).astype(np.float32)
    fwd = lstm_forward(x, W, R, b, lens, -1)
    grad = lstm_backward(fwd, dy)
    got = gh.run_lstm_layer(x, W, R, b, lens, -1, dy=dy, want_dx=False)
    _check_layer(got, fwd, grad, lens, "null optionals")
    assert "dx" not in got


@pytest.mark.parametrize("engine", ENGINES)
def test_small_stack(engine):
    wl = synth.small_blstm(seed=11, L=3, B=5, D=12, H=20, len_lo=0, len_hi=37, T=40)
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=engine)
    run.step()
    got = run.results()
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD
    assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD
    for i, (g, r) in enumerate(zip(got["grads"], ref["grads"])):
        assert gh.rel_err(g, r) < TOL_GRAD, (i, gh.rel_err(g, r))


def test_stack_one_stream_and_no_dx_match_two_streams():
    """The schedule changes no result beyond rounding: with two streams the products run beside the recurrent
    kernels with one slab in flight, with one stream with two (the same sums in the same order), and the two-stream
    pass adds the bias gradient piece by piece."""
    wl = synth.small_blstm(seed=12, L=2, B=7, D=9, H=24, len_lo=2, len_hi=30)
    a = gh.StackRun(wl, two_streams=True)
    a.step()
    ra = a.results()
    b = gh.StackRun(wl, two_streams=False, want_dx=False)
    b.step()
    rb = b.results()
    assert gh.rel_err(ra["y"], rb["y"]) < 2e-6
    for g1, g2 in zip(ra["grads"], rb["grads"]):
        assert gh.rel_err(g1, g2) < 2e-6
    # the forward-only entry point writes the same outputs as the one-stream pass, bit for bit
    c = gh.StackRun(wl)
    c.forward_only()
    assert np.array_equal(c.results()["y"], rb["y"])


@pytest.mark.parametrize("mode", [1, 2])
def test_overlap_modes_against_oracle(mode):
    """Products one after the other on one stream (overlap_mode 1) or beside the recurrent kernels with the passes cut
    into pieces (2): the same results, up to the order of sums."""
    wl = synth.make_workload("overlap", L=3, B=20, D=16, H=72, len_lo=10, len_hi=300, wscale=0.1, seed=41)
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, two_streams=True, overlap_mode=mode, first_piece=64)
    run.step()
    got = run.results()
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD
    assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD
    for g1, g2 in zip(got["grads"], ref["grads"]):
        assert gh.rel_err(g1, g2) < TOL_GRAD
    # tuning values outside their ranges are refused before anything is enqueued
    for bad in (dict(overlap_mode=3), dict(overlap_mode=-1), dict(first_piece=-2), dict(batch_groups=9), dict(bwd_exchange=3),
                dict(gemm_variant=-1), dict(gemm_variant=4)):
        d = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0, engine=0, **bad)
        assert rl.rblstm_workspace_bytes(d) == 0, bad
        assert rl.blstm_stack_fwd(d, run.x, run.params, run.seq_lens, run.y_top, run.reserve, run.ws, None, check=False) == -3, bad


def test_shared_call_where_only_the_fp32_instruction_products_fit_beside_the_recurrent_kernels():
    """640 units per direction: the recurrent workgroups hold 100 KB of LDS, so the default product kernel for fp32
    operands (three bf16 parts, 72 KB) does not fit on a CU beside them; a two-stream call then shares the CUs with the
    kernels on the fp32 matrix instructions (33 KB) instead of falling back to the serial schedule.  Against the
    oracle, and bit-equal to the same call with those kernels asked for by gemm_variant 3."""
    wl = synth.make_workload("wide_shared", L=2, B=16, D=24, H=640, len_lo=40, len_hi=200, wscale=0.05, seed=43)
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, two_streams=True, overlap_mode=2, first_piece=64)
    run.step()
    got = run.results()
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD
    assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD
    for g1, g2 in zip(got["grads"], ref["grads"]):
        assert gh.rel_err(g1, g2) < TOL_GRAD
    same = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, two_streams=True, overlap_mode=2, first_piece=64, gemm_variant=3)
    same.step()
    again = same.results()
    assert np.array_equal(again["y"], got["y"]) and np.array_equal(again["dx"], got["dx"])
    for g1, g2 in zip(again["grads"], got["grads"]):
        assert np.array_equal(g1, g2)


def test_groups_of_more_than_16_sequences_as_three_parts_and_on_the_fp32_instructions():
    """fp32 operands, 40 sequences = 2 groups of 20 per direction, i.e. two 16-row tiles per workgroup: by default the
    recurrent kernels exchange h_t / d a_t and keep R as three bf16 parts each (rblstm_plan reports form 2, and the
    products use the three-part kernel as well); gemm_variant 3 keeps both on the fp32 matrix instructions (form 0).
    Both against the oracle at the unchanged bars; the default twice, bit for bit; and the two agree with each other
    more closely than either has to agree with the oracle."""
    wl = synth.make_workload("two_tiles", L=2, B=40, D=24, H=200, len_lo=30, len_hi=150, wscale=0.08, seed=47)
    ref = gh.oracle_stack(wl)
    res = {}
    for variant in (0, 3):
        run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, gemm_variant=variant)
        assert rl.rblstm_plan(run.desc)["recurrent_operand_form"] == (2 if variant == 0 else 0)
        assert rl.rblstm_plan(run.desc)["rows"] == 32
        run.step()
        got = run.results()
        assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD, variant
        assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD, variant
        for g1, g2 in zip(got["grads"], ref["grads"]):
            assert gh.rel_err(g1, g2) < TOL_GRAD, variant
        res[variant] = got
        if variant == 0:
            run.step()
            again = run.results()
            assert np.array_equal(again["y"], got["y"]) and np.array_equal(again["dx"], got["dx"])
            for g1, g2 in zip(again["grads"], got["grads"]):
                assert np.array_equal(g1, g2)
    print("three parts vs fp32 instructions: y", gh.rel_err(res[0]["y"], res[3]["y"]), flush=True)
    assert gh.rel_err(res[0]["y"], res[3]["y"]) < 2e-6


def test_plan_reports_the_form_of_the_recurrent_product():
    """rblstm_plan's last field: groups of 16 sequences (the benchmark stack) keep fp32 values on the fp32 matrix
    instructions (0), groups of 41 (the paper's batch of 81 segments) exchange three bf16 parts (2) unless a gemm_variant
    asks for the fp32 instructions, bf16 operands are 1; more than 512 units keep the fp32 instructions."""
    def form(**kw):
        return rl.rblstm_plan(rl.rblstm_desc(**kw))["recurrent_operand_form"]
    assert form(L=4, T=1000, B=32, D=40, H=500, operand_dtype=0, engine=0) == 0
    assert form(L=3, T=250, B=81, D=45, H=512, operand_dtype=0, engine=0) == 2
    for v in (1, 2, 3):
        assert form(L=3, T=250, B=81, D=45, H=512, operand_dtype=0, engine=0, gemm_variant=v) == 0
    assert form(L=3, T=250, B=81, D=45, H=512, operand_dtype=1, engine=0) == 1
    assert form(L=2, T=100, B=40, D=40, H=640, operand_dtype=0, engine=0) == 0


def test_config2_blstm():
    """Config 2: 1-layer BLSTM, D=40, H=256 per direction, B=16, lengths uniform in [100, 500]."""
    wl = synth.config2()
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl)
    run.step()
    got = run.results()
    errs = dict(y=gh.rel_err(got["y"], ref["y"]), dx=gh.rel_err(got["dx"], ref["dx"]))
    for i, (g, r) in enumerate(zip(got["grads"], ref["grads"])):
        errs[f"g{i}"] = gh.rel_err(g, r)
    print("config2 errors", errs, flush=True)
    assert errs["y"] < TOL_FWD
    assert all(v < TOL_GRAD for k, v in errs.items() if k != "y"), errs
    # run-to-run reproducibility: no atomics on floating-point data anywhere
    run.step()
    again = run.results()
    assert np.array_equal(again["y"], got["y"])
    for g1, g2 in zip(again["grads"], got["grads"]):
        assert np.array_equal(g1, g2)


def test_engines_agree_on_medium_stack():
    wl = synth.make_workload("medium", L=2, B=24, D=40, H=100, len_lo=20, len_hi=120, wscale=0.1, seed=5)
    a = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT)
    a.step()
    ra = a.results()
    b = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_STEPWISE)
    b.step()
    rb = b.results()
    assert gh.rel_err(ra["y"], rb["y"]) < 2 * TOL_FWD
    for g1, g2 in zip(ra["grads"], rb["grads"]):
        assert gh.rel_err(g1, g2) < 2 * TOL_GRAD


@pytest.mark.parametrize("case", [
    # trans_a, trans_b, M, N, K
    (0, 0, 300, 200, 40), (0, 0, 257, 129, 1000), (0, 1, 260, 40, 512), (1, 0, 100, 260, 5000),
    (1, 1, 64, 64, 64), (0, 0, 33, 17, 19), (1, 0, 37, 50, 4100), (0, 1, 128, 128, 16),
    # the pipelined kernel (whole float4s along the contiguous dimension): K tails that are no multiple of the slab,
    # one slab, fewer K than a slab, M and N tails, split-K with a K that is no multiple of 4
    (0, 0, 260, 132, 1004), (0, 1, 200, 260, 36), (1, 0, 132, 260, 4098), (1, 1, 260, 136, 520), (0, 0, 128, 128, 4),
    (1, 0, 516, 1028, 20250), (0, 1, 1000, 36, 2000), (1, 1, 4, 4, 8),
    # few columns on both sides and a long sum (one tile for the whole result): full and ragged tiles, a K that is
    # no multiple of the 32-row chunk
    (1, 0, 68, 160, 40000), (1, 0, 80, 160, 16500), (1, 0, 36, 84, 20001), (1, 0, 4, 4, 16384),
])
@pytest.mark.parametrize("variant", [0, 2, 3])
def test_gemm_against_numpy(case, variant):
    """variant 0: the product from three bf16 parts per operand (its pipelined form where the operands allow); 2: the
    plain kernel on the fp32 matrix instructions; 3: those instructions, the pipelined kernel where the operands allow."""
    ta, tb, M, N, K = case
    rng = _rng(sum(case))
    A = rng.standard_normal((K, M) if ta else (M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K) if tb else (K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    ref = (A.T if ta else A).astype(np.float64) @ (Bm.T if tb else Bm).astype(np.float64) + bias
    Ad, Bd, biasd = gh.dev(A), gh.dev(Bm), gh.dev(bias)
    C = torch.full((M, N), float("nan"), device=gh.DEV)
    ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
    rl.rlstm_gemm_f32(ta, tb, M, N, K, Ad, A.shape[1], Bd, Bm.shape[1], C, N, biasd, ws, variant=variant)
    torch.cuda.synchronize()
    assert gh.rel_err(C.cpu().numpy(), ref) < 1e-5, (case, variant)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("side", ["a", "b"])
def test_gemm_three_part_product_keeps_all_24_bits(ta, tb, side):
    """The default fp32 product cuts every operand value into three bf16 parts.  One operand holds numbers that use all
    24 significant bits over a range of exponents, the other picks and scales them (one entry +-2^e per column or row):
    every output is then a single product that fp32 holds exactly, so the result must equal it bit for bit - a lost or
    misplaced part would show.  Both operand sides, all four storage orders, shapes with tile tails (the kernel with
    range-checked loads) and without whole float4s (the plain-load kernel)."""
    for (M, N, K) in [(260, 132, 72), (131, 67, 45)]:
        rng = _rng(1000 * ta + 100 * tb + M)
        full_shape = (M, K) if side == "a" else (K, N)
        mant = rng.integers(2 ** 23, 2 ** 24, size=full_shape).astype(np.float64)          # 24 significant bits
        full = (mant * np.exp2(rng.integers(-40, 17, size=full_shape)) * rng.choice([-1.0, 1.0], size=full_shape))
        if side == "a":
            pick = np.zeros((K, N))
            rows = rng.integers(0, K, size=N)
            pick[rows, np.arange(N)] = np.exp2(rng.integers(-6, 7, size=N)) * rng.choice([-1.0, 1.0], size=N)
            A, Bm = full, pick
        else:
            pick = np.zeros((M, K))
            cols = rng.integers(0, K, size=M)
            pick[np.arange(M), cols] = np.exp2(rng.integers(-6, 7, size=M)) * rng.choice([-1.0, 1.0], size=M)
            A, Bm = pick, full
        ref = (A @ Bm).astype(np.float32)
        assert np.array_equal(ref.astype(np.float64), A @ Bm)                                # exact in fp32
        As = np.ascontiguousarray(A.T if ta else A).astype(np.float32)
        Bs = np.ascontiguousarray(Bm.T if tb else Bm).astype(np.float32)
        C = torch.full((M, N), float("nan"), device=gh.DEV)
        rl.rlstm_gemm_f32(ta, tb, M, N, K, gh.dev(As), As.shape[1], gh.dev(Bs), Bs.shape[1], C, N, None, None, variant=0)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), ref), (ta, tb, side, M, N, K)


@pytest.mark.parametrize("case", [(0, 0, 1024, 768, 1000), (0, 1, 1000, 500, 2000), (1, 0, 500, 1000, 32000), (1, 1, 260, 132, 516)])
def test_gemm_three_part_product_is_as_close_to_fp64_as_the_fp32_instructions(case):
    """Against the fp64 product, entry by entry in units of sum_k |a||b| (the scale rounding errors of a sum of products
    are measured in), the default fp32 product (three bf16 parts per operand, six of the nine part products) must be as
    close as the kernels on the fp32 matrix instructions (largest error at most 1.5 times, root mean square at most 1.25
    times theirs),
    on normal operands and on operands whose rows carry scales from 2^-30 to 2^30."""
    ta, tb, M, N, K = case
    for spread in (0, 30):
        rng = _rng(sum(case) + spread)
        A = rng.standard_normal((M, K)) * np.exp2(rng.integers(-spread, spread + 1, size=(M, 1)))
        Bm = rng.standard_normal((K, N)) * np.exp2(rng.integers(-spread, spread + 1, size=(1, N)))
        A, Bm = A.astype(np.float32), Bm.astype(np.float32)
        ref = A.astype(np.float64) @ Bm.astype(np.float64)
        scale = np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64)
        As = np.ascontiguousarray(A.T) if ta else A
        Bs = np.ascontiguousarray(Bm.T) if tb else Bm
        Ad, Bd = gh.dev(As), gh.dev(Bs)
        ws = torch.empty(64 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
        err = {}
        for variant in (0, 3):
            C = torch.full((M, N), float("nan"), device=gh.DEV)
            rl.rlstm_gemm_f32(ta, tb, M, N, K, Ad, As.shape[1], Bd, Bs.shape[1], C, N, None, ws, variant=variant)
            torch.cuda.synchronize()
            e = np.abs(C.cpu().numpy().astype(np.float64) - ref) / scale
            err[variant] = (e.max(), np.sqrt(np.mean(e * e)))
        print("three-part vs fp32 instructions", case, "spread", spread, err, flush=True)
        assert err[0][0] <= 1.5 * err[3][0] and err[0][1] <= 1.25 * err[3][1], (case, spread, err)
        assert err[0][0] < 5e-6


def test_gemm_tall_skinny_many_slices():
    """The one-tile kernel with 512 K slices and the 16-group sum of the slices, as the two-dimensional layer's
    weight gradients use it; twice, for bit reproducibility."""
    M, N, K = 68, 160, 300000
    rng = _rng(5)
    A = rng.standard_normal((K, M)).astype(np.float32)
    Bm = rng.standard_normal((K, N)).astype(np.float32)
    ref = A.T.astype(np.float64) @ Bm.astype(np.float64)
    Ad, Bd = gh.dev(A), gh.dev(Bm)
    ws = torch.empty(512 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
    outs = []
    for _ in range(2):
        C = torch.full((M, N), float("nan"), device=gh.DEV)
        rl.rlstm_gemm_f32(1, 0, M, N, K, Ad, M, Bd, N, C, N, None, ws)
        torch.cuda.synchronize()
        outs.append(C.cpu().numpy())
    assert gh.rel_err(outs[0], ref) < 1e-5
    assert np.array_equal(outs[0], outs[1])


def test_engine_resolution_and_unsupported_shape():
    d = rl.rlstm_desc(T=4, B=2, D=3, H=16, direction=1, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.rlstm_resolve_engine(d) == rl.RLSTM_ENGINE_PERSISTENT
    # 100 sequences: dealt out to two groups of workgroups
    mid = rl.rlstm_desc(T=4, B=100, D=3, H=16, direction=1, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.rlstm_resolve_engine(mid) == rl.RLSTM_ENGINE_PERSISTENT
    # more sequences than 8 groups of 64 can hold
    big = rl.rlstm_desc(T=4, B=600, D=3, H=16, direction=1, engine=rl.RLSTM_ENGINE_AUTO)
    assert rl.rlstm_resolve_engine(big) == rl.RLSTM_ENGINE_STEPWISE
    big.engine = rl.RLSTM_ENGINE_PERSISTENT
    assert rl.rlstm_resolve_engine(big) == -5


def test_config3_full_size_against_oracle_samples():
    """The benchmark workload at full size, in the launch configuration bench.py times (persistent
    engine, two streams): sampled entries of every output against values the oracle wrote
    (tests/golden/make_config3_golden.py), plus properties that hold at any size."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config3_oracle_samples.npz")
    g = np.load(path)
    wl = synth.config3()
    assert np.array_equal(g["seq_lens"], wl.seq_lens)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, want_dx=True, two_streams=True)
    run.step()
    got = run.results()

    def check(name, arr, tol):
        err = np.abs(arr.reshape(-1)[g[name + "_idx"]].astype(np.float64) - g[name + "_val"]).max() / float(g[name + "_max"])
        print(f"config3 {name}: sampled rel err {err:.2e}", flush=True)
        assert err < tol, (name, err)

    check("y", got["y"], TOL_FWD)
    check("dx", got["dx"], TOL_GRAD)
    k = 0
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR", "db"):
                check(f"{nm}_{l}_{d}", got["grads"][k], TOL_GRAD)
                k += 1
    # whole frames on either side of the places the passes are cut, both ends of the time axis, every sequence's last
    # valid and first padded frame, units 496..499 next to the padding of H, every bias gradient whole
    gh.check_structured_samples(g, "", run.y_top, run.dx, run.grads, wl.seq_lens, wl.L, TOL_FWD, TOL_GRAD, "config3")
    for n, ln in enumerate(wl.seq_lens):
        assert np.all(got["y"][ln:, n] == 0.0) and np.all(got["dx"][ln:, n] == 0.0)
    assert all(np.isfinite(a).all() for a in got["grads"])
    # second call on the same buffers gives bit-identical results
    run.step()
    again = run.results()
    assert np.array_equal(again["y"], got["y"])
    assert all(np.array_equal(a, b) for a, b in zip(again["grads"], got["grads"]))


def _round_bf16(a):
    """fp32 -> bf16 (round to nearest even) -> fp32, in numpy (the definition of the format)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


@pytest.mark.parametrize("case", [
    (0, 0, 300, 200, 40), (0, 0, 257, 129, 1000), (0, 1, 260, 40, 512), (1, 0, 100, 260, 5000),
    (1, 1, 64, 64, 64), (0, 0, 33, 17, 19), (1, 0, 37, 50, 4100), (0, 1, 128, 128, 32),
    # enough tiles for the 256 x 256 kernel: ragged edges in m, n and k, every operand layout, split-K
    (0, 0, 3000, 2900, 100), (0, 1, 2830, 3100, 77), (1, 0, 2900, 2950, 4100), (1, 1, 2820, 2900, 40),
])
def test_gemm_bf16_against_numpy(case):
    """bf16-operand product: equal to the fp64 product of the bf16-rounded operands up to fp32
    accumulation, and within 2e-2 of the unrounded product."""
    ta, tb, M, N, K = case
    rng = _rng(sum(case) + 1)
    A = rng.standard_normal((K, M) if ta else (M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K) if tb else (K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    Ar, Br = _round_bf16(A).astype(np.float64), _round_bf16(Bm).astype(np.float64)
    ref_rounded = (Ar.T if ta else Ar) @ (Br.T if tb else Br) + bias
    ref = (A.T if ta else A).astype(np.float64) @ (Bm.T if tb else Bm).astype(np.float64) + bias
    C = torch.full((M, N), float("nan"), device=gh.DEV)
    ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
    rl.rlstm_gemm_bf16(ta, tb, M, N, K, gh.dev(A), A.shape[1], gh.dev(Bm), Bm.shape[1], C, N, gh.dev(bias), ws)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert gh.rel_err(got, ref_rounded) < 1e-5, case
    assert gh.rel_err(got, ref) < 2e-2, case


@pytest.mark.parametrize("case", [
    # every operand layout; ragged tiles in m and n; K tails inside a slab of 32; split-K
    (0, 0, 3000, 2904, 104), (0, 1, 2832, 3104, 72), (1, 0, 2904, 2952, 4104), (1, 1, 2824, 2904, 40), (1, 0, 1000, 4000, 16384),
])
def test_gemm_bf16_operands_read_as_bf16_from_memory(case):
    """The product kernel that takes bf16 copies of its operands from memory: the bits of the kernel that reads fp32 and
    rounds on the way into LDS (the same rounding, the same order of sums), and the fp64 product of the rounded operands
    up to fp32 accumulation.  The copy itself against the definition of the format."""
    ta, tb, M, N, K = case
    rng = _rng(sum(case) + 7)
    A = rng.standard_normal((K, M) if ta else (M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K) if tb else (K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    Ad, Bd, biasd = gh.dev(A), gh.dev(Bm), gh.dev(bias)
    A16 = torch.zeros(A.shape, dtype=torch.int16, device=gh.DEV)
    B16 = torch.zeros(Bm.shape, dtype=torch.int16, device=gh.DEV)
    A16t = torch.zeros(A.shape[::-1], dtype=torch.int16, device=gh.DEV)
    B16t = torch.zeros(Bm.shape[::-1], dtype=torch.int16, device=gh.DEV)
    rl.rlstm_to_bf16(A16, Ad)
    rl.rlstm_to_bf16_2d(B16, B16t, Bd, Bm.shape[0], Bm.shape[1], Bm.shape[1])
    rl.rlstm_to_bf16_2d(None, A16t, Ad, A.shape[0], A.shape[1], A.shape[1])
    torch.cuda.synchronize()
    bits = lambda a: (_round_bf16(a).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(A16.cpu().numpy().view(np.uint16), bits(A))
    assert np.array_equal(B16.cpu().numpy().view(np.uint16), bits(Bm))
    assert np.array_equal(A16t.cpu().numpy().view(np.uint16), bits(A).T)
    assert np.array_equal(B16t.cpu().numpy().view(np.uint16), bits(Bm).T)
    ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
    Cref = torch.full((M, N), float("nan"), device=gh.DEV)
    rl.rlstm_gemm_bf16(ta, tb, M, N, K, Ad, A.shape[1], Bd, Bm.shape[1], Cref, N, biasd, ws)
    torch.cuda.synchronize()
    ref = Cref.cpu().numpy()
    Ar, Br = _round_bf16(A).astype(np.float64), _round_bf16(Bm).astype(np.float64)
    assert gh.rel_err(ref, (Ar.T if ta else Ar) @ (Br.T if tb else Br) + bias) < 1e-5, case
    # the same product from the copies as stored, and from the transposed copies with the transposition flags flipped
    # (every combination of layouts goes through a different pair of loaders)
    for fa in (0, 1):
        for fb in (0, 1):
            a16, b16 = (A16t if fa else A16), (B16t if fb else B16)
            C = torch.full((M, N), float("nan"), device=gh.DEV)
            rl.rlstm_gemm_bf16_mem(ta ^ fa, tb ^ fb, M, N, K, a16, a16.shape[1], b16, b16.shape[1], C, N, biasd, ws)
            torch.cuda.synchronize()
            assert np.array_equal(C.cpu().numpy(), ref), (case, fa, fb)
    # the other forms of the kernel give the same bits: one workgroup per tile instead of one per CU walking through
    # its tiles (3), slabs staged through registers instead of the ring of LDS slabs filled by direct loads (4)
    for variant in (3, 4):
        C = torch.full((M, N), float("nan"), device=gh.DEV)
        rl.rlstm_gemm_bf16_mem(ta ^ 1, tb ^ 1, M, N, K, A16t, A16t.shape[1], B16t, B16t.shape[1], C, N, biasd, ws, variant=variant)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), ref), (case, variant)
    assert rl.rlstm_gemm_bf16_mem(0, 0, M, N, K, A16, A.shape[1], B16, Bm.shape[1], C, N, None, None, check=False, variant=1) == -3
    # a shape without the tiles for that kernel, or a K that is no multiple of 8, is refused, not silently rerouted
    assert rl.rlstm_gemm_bf16_mem(0, 0, 64, 64, 64, A16, 64, B16, 64, C, N, None, None, check=False) == -3
    if not ta and not tb:
        assert rl.rlstm_gemm_bf16_mem(0, 0, M, N, K - 4, A16, A.shape[1], B16, Bm.shape[1], C, N, None, None, check=False) == -3
    # the converter refuses what it cannot write in whole aligned groups
    assert rl.rlstm_to_bf16_2d(B16, B16t, Bd, Bm.shape[0] - 4, Bm.shape[1], Bm.shape[1], check=False) == -2


def test_gemm_bf16_copies_with_row_strides_and_offsets():
    """The bf16-copy product on operands that are windows of larger arrays, as the stack's weight gradients use them
    (rows of T*B values of which a product takes (T-1)*B, starting B values in): row strides beyond K, starts that are
    16-byte but not row aligned, K with a tail inside a slab, split K.  Against the fp64 product of the same bf16 values."""
    rng = _rng(77)
    bits = lambda a: torch.from_numpy((a.view(np.uint32) >> 16).astype(np.uint16).view(np.int16)).to(gh.DEV)
    for M, N, K, ld in ((2904, 3000, 8 * 130, 8 * 140), (1000, 4000, 16384 + 24, 16384 + 96)):
        A = _round_bf16(rng.standard_normal((M, ld)).astype(np.float32))
        Bm = _round_bf16(rng.standard_normal((N, ld)).astype(np.float32))
        A16, B16 = bits(A), bits(Bm)
        ws = torch.empty(16 * M * N * 4, dtype=torch.uint8, device=gh.DEV)
        for oa, ob in ((64, 0), (0, 64), (8, 24)):
            C = torch.full((M, N), float("nan"), device=gh.DEV)
            rl.rlstm_gemm_bf16_mem(0, 1, M, N, K, A16.reshape(-1)[oa:], ld, B16.reshape(-1)[ob:], ld, C, N, None, ws)
            torch.cuda.synchronize()
            ref = A[:, oa:oa + K].astype(np.float64) @ Bm[:, ob:ob + K].astype(np.float64).T
            assert gh.rel_err(C.cpu().numpy(), ref) < 1e-5, (M, N, K, oa, ob)


TOL_BF16 = 2e-2


@pytest.mark.parametrize("engine", ENGINES)
@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("shape", [
    (13, 5, 12, 20, (13, 7, 1, 0, 9)),
    (11, 18, 16, 36, None),
    (25, 40, 24, 136, None),
])
def test_single_layer_bf16_operands(engine, direction, shape):
    """operand_dtype = 1: matrix-product operands rounded to bf16, fp32 accumulation and cell state;
    checked against the unrounded fp64 oracle within 2e-2."""
    T, B, D, H, lens = shape
    rng = _rng(2000 + T + B + H + (direction > 0))
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    W = rng.uniform(-0.3, 0.3, (D, 4 * H)).astype(np.float32)
    R = rng.uniform(-0.3, 0.3, (H, 4 * H)).astype(np.float32)
    b = rng.uniform(-0.3, 0.3, (4 * H,)).astype(np.float32)
    h0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    lens = np.array(lens if lens is not None else rng.integers(0, T + 1, B), dtype=np.int32)
    dy = rng.standard_normal((T, B, H)).astype(np.float32)
    dhT = rng.standard_normal((B, H)).astype(np.float32)
    dcT = rng.standard_normal((B, H)).astype(np.float32)
    fwd = lstm_forward(x, W, R, b, lens, direction, h0, c0)
    grad = lstm_backward(fwd, dy, dhT, dcT)
    got = gh.run_lstm_layer(x, W, R, b, lens, direction, h0, c0, dy, dhT, dcT, engine=engine, operand_dtype=1)
    errs = {k: gh.rel_err(got[k], (fwd if k in fwd else grad)[k])
            for k in ("y", "c", "hT", "cT", "dx", "dW", "dR", "db", "dh0", "dc0")}
    print(f"bf16 shape={shape} dir={direction} engine={engine}", {k: f"{v:.1e}" for k, v in errs.items()}, flush=True)
    assert all(v < TOL_BF16 for v in errs.values()), errs
    # rounding must actually happen: the result differs from the fp32 path
    assert errs["y"] > 1e-5
    for n, ln in enumerate(lens):
        assert np.all(got["y"][ln:, n] == 0.0) and np.all(got["dx"][ln:, n] == 0.0)


@pytest.mark.parametrize("engine", ENGINES)
def test_small_stack_bf16_operands(engine):
    wl = synth.small_blstm(seed=13, L=3, B=20, D=12, H=40, len_lo=0, len_hi=37, T=40, wscale=0.2)
    wl.operand_dtype = 1
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=engine)
    run.step()
    got = run.results()
    errs = [gh.rel_err(got["y"], ref["y"]), gh.rel_err(got["dx"], ref["dx"])] + \
           [gh.rel_err(g, r) for g, r in zip(got["grads"], ref["grads"])]
    print("bf16 stack", engine, [f"{e:.1e}" for e in errs], flush=True)
    assert max(errs) < TOL_BF16


def test_stack_bf16_operands_with_bf16_copies():
    """A bf16-operand stack large enough that the library keeps bf16 copies of the products' operands (T*B >= 16384,
    H >= 256): a conversion pass writes them, as stored and transposed, and the projections and input gradients
    read them (the weight gradients of this shape have too few tiles for that kernel and read fp32).  Every output against the oracle, the padding zero, and
    the same call twice bit for bit."""
    wl = synth.make_workload("bf16_copies", L=2, B=64, D=40, H=256, len_lo=40, len_hi=264, wscale=0.06, seed=17,
                             operand_dtype=1, bias_scale=0.1)
    assert wl.T * wl.B >= 16384
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT)
    run.step()
    got = run.results()
    errs = [gh.rel_err(got["y"], ref["y"]), gh.rel_err(got["dx"], ref["dx"])] + \
           [gh.rel_err(g, r) for g, r in zip(got["grads"], ref["grads"])]
    print("bf16 stack with copies", [f"{e:.1e}" for e in errs], flush=True)
    assert max(errs) < TOL_BF16
    for n, ln in enumerate(wl.seq_lens):
        assert np.all(got["y"][ln:, n] == 0.0) and np.all(got["dx"][ln:, n] == 0.0)
    run.step()
    again = run.results()
    assert np.array_equal(again["y"], got["y"]) and np.array_equal(again["dx"], got["dx"])
    for a, b in zip(again["grads"], got["grads"]):
        assert np.array_equal(a, b)


def _golden(name):
    import os
    return np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name))


def test_config4_network_on_short_sequences_against_oracle_samples():
    """Config 4's network (6 layers, H=1000, B=64, bf16 operands) on short sequences: every output,
    sampled, against values the oracle wrote (tests/golden/make_config4_golden.py)."""
    g = _golden("config4_oracle_samples.npz")
    wl = synth.config4_short()
    assert np.array_equal(g["short_seq_lens"], wl.seq_lens)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, want_dx=True, two_streams=True)
    run.step()
    got = run.results()
    errs = {}

    def check(name, arr):
        key = "short_" + name
        errs[name] = np.abs(arr.reshape(-1)[g[key + "_idx"]].astype(np.float64) - g[key + "_val"]).max() / float(g[key + "_max"])

    check("y", got["y"])
    check("dx", got["dx"])
    k = 0
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR", "db"):
                check(f"{nm}_{l}_{d}", got["grads"][k])
                k += 1
    print("config4 short: worst sampled rel err", max(errs.values()), "y", errs["y"], flush=True)
    assert max(errs.values()) < TOL_BF16, errs


def test_config4_full_size_against_oracle_samples():
    """Config 4 at full size (T=1500, B=64, bf16 operands), in the two-stream persistent launch configuration, against
    values the oracle wrote (tests/golden/make_config4_golden.py ran the minibatch in groups of 8 sequences and added
    the groups' weight gradients): random samples of y_top and dx from every sequence, of dW and dR of every layer and
    direction, every db whole, whole first / last frames, every sequence's last valid and first padded frame, and the
    rows / columns of the last units; all at the 2e-2 of the bf16-operand variant."""
    g = _golden("config4_oracle_samples.npz")
    wl = synth.config4()
    assert np.array_equal(g["full_seq_lens"], wl.seq_lens)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, want_dx=True, two_streams=True)
    run.step()
    torch.cuda.synchronize()
    assert rl.rlstm_last_timeout(run.ws) == 0
    errs = {}

    def check(name, t):
        key = "full_" + name
        idx = torch.from_numpy(g[key + "_idx"]).to(gh.DEV)
        got = t.reshape(-1)[idx].cpu().numpy().astype(np.float64)
        errs[name] = float(np.abs(got - g[key + "_val"]).max() / float(g[key + "_max"]))

    check("y", run.y_top)
    check("dx", run.dx)
    k = 0
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR"):
                check(f"{nm}_{l}_{d}", run.grads[k])
                k += 1
            k += 1
    worst = max(errs, key=lambda n: errs[n])
    print(f"config4 full size: y {errs['y']:.2e}, dx {errs['dx']:.2e}, worst weight gradient {worst} {errs[worst]:.2e}", flush=True)
    assert max(errs.values()) < TOL_BF16, errs
    gh.check_structured_samples(g, "full_", run.y_top, run.dx, run.grads, wl.seq_lens, wl.L, TOL_BF16, TOL_BF16, "config4")
    lens = torch.from_numpy(wl.seq_lens.astype(np.int64)).to(gh.DEV)
    pad = torch.arange(wl.T, device=gh.DEV)[:, None] >= lens[None, :]
    assert bool((run.y_top[pad] == 0).all()) and bool((run.dx[pad] == 0).all())
    assert all(bool(torch.isfinite(gr).all()) for gr in run.grads)


def test_bounded_waits_turn_a_silent_workgroup_into_an_error_flag():
    """Failure path, forced from the host: one workgroup of the persistent kernels withholds its step
    flags and the wait bound is 2 ms.  Every kernel must still end normally, rlstm_last_timeout()
    must report it, and the next ordinary call must work again."""
    import time
    wl = synth.small_blstm(seed=14, L=1, B=6, D=8, H=40, len_lo=5, len_hi=30)
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT)
    try:
        rl.rlstm_test_hook(3, 200_000)
        t0 = time.time()
        run.step()
        torch.cuda.synchronize()
        assert time.time() - t0 < 5.0
        assert rl.rlstm_last_timeout(run.ws) == 1
    finally:
        rl.rlstm_test_hook(-1, 0)
    run.step()
    got = run.results()          # asserts that no wait expired
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD


@pytest.mark.parametrize("bwd_exchange", [1, 2])
@pytest.mark.parametrize("operand_dtype", [0, 1])
def test_a_late_workgroup_changes_no_bit(operand_dtype, bwd_exchange):
    """Race check of the exchange between the workgroups of the persistent kernels, forced from the host: one
    workgroup publishes every step 3 us late (several times the step itself).  A consumer that read its producers'
    data without having waited for them would take the values of two steps ago; with correct waits every output has
    the bits of the undisturbed call.  Every kernel still ends normally and no wait expires."""
    if operand_dtype == 1 and bwd_exchange == 2:
        pytest.skip("one exchange per step exists for fp32 operands only")
    import dataclasses
    wl = dataclasses.replace(synth.small_blstm(seed=33, L=2, B=11, D=8, H=44, len_lo=3, len_hi=40), operand_dtype=operand_dtype)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, bwd_exchange=bwd_exchange)
    run.step()
    base = run.results()
    plan = rl.rblstm_plan(run.desc)
    members = plan["members_fwd"]            # workgroups 0 .. members-1 exist in every launch (index = member * groups + group)
    assert members >= 4
    assert rl.rlstm_test_delay(0, 100001) == -2
    for slow in (0, 3, members - 1):
        try:
            rl.rlstm_test_delay(slow, 300)
            run.step()
            got = run.results()          # asserts that no wait expired
        finally:
            rl.rlstm_test_delay(-1, 0)
        assert np.array_equal(got["y"], base["y"]), slow
        assert np.array_equal(got["dx"], base["dx"]), slow
        for a, b in zip(got["grads"], base["grads"]):
            assert np.array_equal(a, b), slow


@pytest.mark.parametrize("bwd_exchange", [1, 2])
@pytest.mark.parametrize("first", [-1, 3, 7, 64])
def test_stack_results_do_not_depend_on_how_the_passes_are_cut(first, bwd_exchange):
    """Two streams + persistent engine: the recurrent passes are cut into pieces (first, first, 2*first, ...; -1: not
    cut) that the feeding matrix products run ahead of.  Every cut must give the oracle's results, and the
    same bits as the uncut passes except for the order of the bias gradient's sums.  (The bits are compared with
    one product kernel for every piece: by default the first piece's product, which runs while the chain waits
    for it, uses the pipelined kernel and the others the plain one, and the two add in different orders.)  With
    one and with two exchanges per step in the backward kernel."""
    wl = synth.small_blstm(seed=21, L=3, B=9, D=11, H=36, len_lo=0, len_hi=61, T=61)
    ref = gh.oracle_stack(wl)
    dflt = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, first_piece=first, overlap_mode=2, bwd_exchange=bwd_exchange)
    dflt.step()
    rd = dflt.results()
    assert gh.rel_err(rd["y"], ref["y"]) < TOL_FWD and gh.rel_err(rd["dx"], ref["dx"]) < TOL_GRAD
    for i, (g, r) in enumerate(zip(rd["grads"], ref["grads"])):
        assert gh.rel_err(g, r) < TOL_GRAD, (i, gh.rel_err(g, r))
    base = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, first_piece=-1, overlap_mode=2, gemm_variant=2, bwd_exchange=bwd_exchange)
    base.step()
    rb = base.results()
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, first_piece=first, overlap_mode=2, gemm_variant=2, bwd_exchange=bwd_exchange)
    run.step()
    got = run.results()
    run.step()                      # a second step reuses the scratch the first one left behind
    again = run.results()
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD
    assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD
    for i, (g, r) in enumerate(zip(got["grads"], ref["grads"])):
        assert gh.rel_err(g, r) < TOL_GRAD, (i, gh.rel_err(g, r))
    assert np.array_equal(got["y"], rb["y"]) and np.array_equal(got["dx"], rb["dx"])
    for i, (g1, g2) in enumerate(zip(got["grads"], rb["grads"])):
        if i % 3 == 2:
            assert gh.rel_err(g1, g2) < 1e-6
        else:
            assert np.array_equal(g1, g2), i
    assert np.array_equal(again["y"], got["y"]) and np.array_equal(again["dx"], got["dx"])
    for g1, g2 in zip(again["grads"], got["grads"]):
        assert np.array_equal(g1, g2)


@pytest.mark.parametrize("groups", [1, 2, 4])
@pytest.mark.parametrize("shape", [
    dict(B=24, D=10, H=72, len_lo=0, len_hi=45, T=45),      # groups of 24 / 12 / 6 sequences
    dict(B=9, D=7, H=130, len_lo=3, len_hi=33),             # 4 groups: 3, 3, 3, 0 sequences
])
@pytest.mark.parametrize("bwd_exchange", [1, 2])
def test_stack_results_do_not_depend_on_the_groups_of_sequences(groups, shape, bwd_exchange):
    """The persistent engine deals the sequences out to groups of workgroups that run independently; the backward
    kernel with two exchanges per step and (where the groups hold at most 16 sequences) with one."""
    wl = synth.small_blstm(seed=23, L=2, **shape)
    ref = gh.oracle_stack(wl)
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, batch_groups=groups, bwd_exchange=bwd_exchange)
    run.step()
    got = run.results()
    plan = rl.rblstm_plan(run.desc)
    assert plan["bwd_exchanges_per_step"] == (1 if bwd_exchange == 2 and plan["sequences_per_group"] <= 16 else 2)
    assert gh.rel_err(got["y"], ref["y"]) < TOL_FWD
    assert gh.rel_err(got["dx"], ref["dx"]) < TOL_GRAD
    for i, (g, r) in enumerate(zip(got["grads"], ref["grads"])):
        assert gh.rel_err(g, r) < TOL_GRAD, (i, gh.rel_err(g, r))


@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("shape", [
    # T, B, D, H: unit counts that take every slice width (4, 8, 16 units per workgroup) and padded product width
    (13, 5, 12, 20), (9, 16, 7, 130), (11, 7, 16, 256), (7, 12, 5, 300), (6, 3, 5, 500), (5, 10, 8, 600), (4, 2, 3, 1024),
])
def test_single_layer_backward_with_one_exchange_per_step(direction, shape):
    """bwd_exchange = 2 (applies up to H = 512): every workgroup multiplies its own columns of d a_t with its rows of R^T and hands pieces of
    the result to the owners of the units, one exchange between workgroups per step instead of two; ragged lengths with
    an empty sequence, initial and final states and their gradients."""
    T, B, D, H = shape
    rng = _rng(2500 + T + B + H + (direction > 0))
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    s = 0.3 if H < 200 else 0.08
    W = rng.uniform(-s, s, (D, 4 * H)).astype(np.float32)
    R = rng.uniform(-s, s, (H, 4 * H)).astype(np.float32)
    b = rng.uniform(-0.3, 0.3, (4 * H,)).astype(np.float32)
    h0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    lens = rng.integers(0, T + 1, B).astype(np.int32)
    lens[0], lens[-1] = T, 0
    dy = rng.standard_normal((T, B, H)).astype(np.float32)
    dhT = rng.standard_normal((B, H)).astype(np.float32)
    dcT = rng.standard_normal((B, H)).astype(np.float32)
    fwd = lstm_forward(x, W, R, b, lens, direction, h0, c0)
    grad = lstm_backward(fwd, dy, dhT, dcT)
    got = gh.run_lstm_layer(x, W, R, b, lens, direction, h0, c0, dy, dhT, dcT, engine=rl.RLSTM_ENGINE_PERSISTENT, bwd_exchange=2)
    _check_layer(got, fwd, grad, lens, f"one exchange per step, shape={shape} dir={direction}")
    two = gh.run_lstm_layer(x, W, R, b, lens, direction, h0, c0, dy, dhT, dcT, engine=rl.RLSTM_ENGINE_PERSISTENT, bwd_exchange=1)
    assert np.array_equal(got["y"], two["y"])                       # the same forward kernel
    # H <= 512 runs the other kernel (another order of sums); above that the request falls back to two exchanges
    assert gh.rel_err(got["dW"], two["dW"]) < 1e-5 and np.array_equal(got["dR"], two["dR"]) == (H > 512)


@pytest.mark.parametrize("groups", [2, 8])
@pytest.mark.parametrize("direction", [1, -1])
@pytest.mark.parametrize("bwd_exchange", [1, 2])
def test_single_layer_initial_and_final_state_with_groups_of_sequences(groups, direction, bwd_exchange):
    T, B, D, H = 28, 19, 6, 44
    rng = _rng(2400 + groups + (direction > 0))
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    W = rng.uniform(-0.3, 0.3, (D, 4 * H)).astype(np.float32)
    R = rng.uniform(-0.3, 0.3, (H, 4 * H)).astype(np.float32)
    b = rng.uniform(-0.3, 0.3, (4 * H,)).astype(np.float32)
    h0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, (B, H)).astype(np.float32)
    lens = rng.integers(0, T + 1, B).astype(np.int32)
    dy = rng.standard_normal((T, B, H)).astype(np.float32)
    dhT = rng.standard_normal((B, H)).astype(np.float32)
    dcT = rng.standard_normal((B, H)).astype(np.float32)
    fwd = lstm_forward(x, W, R, b, lens, direction, h0, c0)
    grad = lstm_backward(fwd, dy, dhT, dcT)
    got = gh.run_lstm_layer(x, W, R, b, lens, direction, h0, c0, dy, dhT, dcT, engine=rl.RLSTM_ENGINE_PERSISTENT,
                            batch_groups=groups, bwd_exchange=bwd_exchange)
    _check_layer(got, fwd, grad, lens, f"groups={groups} dir={direction} bwd_exchange={bwd_exchange}")


def test_plan_query_and_exchange_floor_probe():
    """Measurement aids: the plan the persistent engine uses for config 3, and the bare-exchange probe
    (argument checks; a run ends normally and reports a plausible time per step)."""
    wl = synth.config3()
    desc = rl.rblstm_desc(L=wl.L, T=wl.T, B=wl.B, D=wl.D, H=wl.H, operand_dtype=0, engine=rl.RLSTM_ENGINE_AUTO)
    plan = rl.rblstm_plan(desc)
    assert plan["groups"] * plan["members_fwd"] <= 256 and plan["groups"] * plan["members_bwd"] <= 256
    assert plan["members_fwd"] * plan["units_per_workgroup"] >= wl.H
    assert plan["groups"] // 2 * plan["sequences_per_group"] >= wl.B
    assert rl.rlstm_exchange_floor_bytes(9, 4, 64) == 0 and rl.rlstm_exchange_floor_bytes(2, 4, 24) == 0
    ws = torch.empty(rl.rlstm_exchange_floor_bytes(2, 16, 256), dtype=torch.uint8, device=gh.DEV)
    assert rl.rlstm_exchange_floor(2, 16, 256, 16 * 256 + 16, 100, ws, check=False) == -2      # reads past the tiles
    assert rl.rlstm_exchange_floor(2, 16, 256, 16 * 256, 100, ws[:1024], check=False) == -4    # workspace too small
    assert rl.rlstm_exchange_floor(2, 200, 256, 256, 100, ws, check=False) in (-4, -5)
    us = rl.rlstm_exchange_floor(2, 16, 256, 16 * 256, 200, ws)
    assert 0.2 < us < 100.0, us
