"""Chunking: pins of the oracle (CPU), the library's host-side segment table against the oracle (CPU, integer
work only), and the device gather against the oracle (GPU, bit-exact)."""
import math

import numpy as np
import pytest

from oracle import chunk_batch, chunk_table
from paper_1608_00895_amd import binding as rl
from paper_1608_00895_amd import synth


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def test_oracle_segments_cover_every_frame_and_nothing_else():
    rng = _rng(1)
    lens = np.array([0, 1, 7, 250, 251, 499, 500, 738, 1203])
    T, D = int(lens.max()), 3
    x = rng.standard_normal((T, len(lens), D))
    for size, step in ((250, 250), (250, 125), (100, 30), (7, 7), (5, 9)):
        xc, (seq, start, length) = chunk_batch(x, lens, size, step)
        for b, n in enumerate(lens):
            mine = np.nonzero(seq == b)[0]
            assert len(mine) == math.ceil(n / step)                      # one segment per step, none for an empty sequence
            assert list(start[mine]) == [k * step for k in range(len(mine))]
            covered = np.zeros(n, int)
            for k in mine:
                assert 1 <= length[k] <= size and start[k] + length[k] <= n
                assert length[k] == size or start[k] + length[k] == n      # only the tail of a sequence is short
                covered[start[k]:start[k] + length[k]] += 1
                assert np.array_equal(xc[:length[k], k], x[start[k]:start[k] + length[k], b])
                assert not xc[length[k]:, k].any()                          # zero frames where the sequence has ended
            if step <= size:
                assert covered.min(initial=1) >= 1                          # every frame is in some segment
            if step == size:
                assert covered.max(initial=1) == 1                          # exactly once without overlap


def test_oracle_without_overlap_is_a_reshape():
    rng = _rng(2)
    x = rng.standard_normal((1000, 2, 4))
    xc, (seq, start, length) = chunk_batch(x, [1000, 750], 250, 250)
    assert xc.shape == (250, 7, 4) and list(length) == [250] * 7
    assert np.array_equal(xc[:, :4], x[:, 0].reshape(4, 250, 4).transpose(1, 0, 2))
    assert np.array_equal(xc[:, 4:], x[:750, 1].reshape(3, 250, 4).transpose(1, 0, 2))


@pytest.mark.parametrize("size,step", [(250, 250), (250, 100), (64, 200), (1, 1)])
def test_library_segment_table_equals_the_oracle(size, step):
    lens = _rng(3).integers(0, 1500, 50)
    lens[:3] = (0, 1, size)
    got = rl.rlstm_chunk_plan(lens, size, step)
    ref = chunk_table(lens, size, step)
    for g, r in zip(got, ref):
        assert g.dtype == np.int32 and np.array_equal(g, r)


def test_paper_shaped_workload_is_a_batch_of_81_segments():
    """The oracle cuts the corpus; the shared generator only draws the network for the batch it is handed."""
    corpus_x, corpus_lens = synth.paper_corpus()
    xc, (seq, start, length) = chunk_batch(corpus_x, corpus_lens, synth.PAPER_SEGMENT_FRAMES, synth.PAPER_SEGMENT_FRAMES)
    assert len(seq) >= synth.PAPER_BATCH_SEGMENTS
    wl = synth.paper_workload(xc[:, :81], length[:81])
    assert (wl.T, wl.B, wl.D, wl.L, wl.H) == (250, 81, 45, 3, 512)
    assert wl.seq_lens.max() == 250 and wl.seq_lens.min() >= 1
    assert np.array_equal(wl.x, xc[:, :81]) and not wl.G[wl.seq_lens[5]:, 5].any()


@pytest.mark.gpu
@pytest.mark.parametrize("size,step,ldx", [(250, 250, 0), (100, 30, 0), (16, 40, 12)])
def test_device_gather_is_bit_exact(size, step, ldx):
    import torch
    rng = _rng(4)
    lens = np.array([0, 33, 250, 612, 17, 251])
    T, B, D = 612, len(lens), 9
    x = rng.standard_normal((T, B, D)).astype(np.float32)
    ref, _ = chunk_batch(x, lens, size, step)
    seq, start, length = rl.rlstm_chunk_plan(lens, size, step)
    lx = ldx or D
    xd = torch.full((T, B, lx), float("nan"), device="cuda:0")
    xd[:, :, :D] = torch.from_numpy(x)
    xc = torch.full((size, len(seq), D), float("nan"), device="cuda:0")
    dev = lambda a: torch.from_numpy(a).to("cuda:0")
    rl.rlstm_chunk_gather(xd, dev(seq), dev(start), dev(length), size, xc, ldx=ldx)
    torch.cuda.synchronize()
    assert np.array_equal(xc.cpu().numpy(), ref)
    # a table entry that points outside x is padding, not a fault
    bad_start = start.copy()
    bad_start[-1] = T + 5
    rl.rlstm_chunk_gather(xd, dev(seq), dev(bad_start), dev(length), size, xc, ldx=ldx)
    torch.cuda.synchronize()
    got = xc.cpu().numpy()
    assert np.array_equal(got[:, :-1], ref[:, :-1]) and not got[:, -1].any()


@pytest.mark.gpu
def test_paper_shaped_batch_against_oracle_samples():
    """The batch shape the paper's experiments time (81 segments of 250 frames, 3 x 512 BLSTM): the corpus is
    cut on the device (segment table + gather), the stack runs on the gathered batch, and sampled entries of
    every output are compared with values the oracle wrote (tests/golden/make_paper_chunks_golden.py)."""
    import os
    import sys
    import torch
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import gpu_harness as gh
    g = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_chunks_oracle_samples.npz"))
    # the batch is built by the library from the corpus (segment table + device gather)
    wl = gh.paper_batch_from_corpus()
    assert np.array_equal(g["seq_lens"], wl.seq_lens)
    ref_x, (_, _, ref_len) = chunk_batch(*synth.paper_corpus(), synth.PAPER_SEGMENT_FRAMES, synth.PAPER_SEGMENT_FRAMES)
    assert np.array_equal(wl.x, ref_x[:, :wl.B]) and np.array_equal(wl.seq_lens, ref_len[:wl.B])   # the oracle's cut, bit for bit
    run = gh.StackRun(wl, engine=rl.RLSTM_ENGINE_PERSISTENT, want_dx=True, two_streams=True)
    run.step()
    got = run.results()

    def check(name, arr, tol):
        err = np.abs(arr.reshape(-1)[g[name + "_idx"]].astype(np.float64) - g[name + "_val"]).max() / float(g[name + "_max"])
        assert err < tol, (name, err)

    check("y", got["y"], 1e-5)
    check("dx", got["dx"], 1e-4)
    k = 0
    for l in range(wl.L):
        for d in range(2):
            for nm in ("dW", "dR", "db"):
                check(f"{nm}_{l}_{d}", got["grads"][k], 1e-4)
                k += 1
    gh.check_structured_samples(g, "", run.y_top, run.dx, run.grads, wl.seq_lens, wl.L, 1e-5, 1e-4, "paper batch")
