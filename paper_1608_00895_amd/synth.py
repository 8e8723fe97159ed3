"""Seeded synthetic inputs for the LSTM / BLSTM hot path.

This module only draws random numbers and shapes them; it contains none of
the LSTM arithmetic.  It is the one module that both the CPU oracle's tests
and the HIP path's tests / benchmark may share, so that both sides see the
same arrays.

The workloads stand in for the speech features the paper trains on
(Sec. 6: ~40-dimensional acoustic frames, utterances of several hundred
frames, zero-padded into time-major batches): x ~ N(0,1) per feature,
uniform weights, sequence lengths uniform in a range, frames past a
sequence's length set to zero.

Draw order (one numpy Philox stream per workload, seeded by ``seed``):
seq_lens, x, then for every layer and direction (forward first) W, R, b,
then the loss weights G of the top layer.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass
class Workload:
    name: str
    L: int                 # stacked layers
    T: int                 # padded length (= max seq_lens)
    B: int                 # sequences per minibatch
    D: int                 # input feature width of layer 0
    H: int                 # units per direction
    bidirectional: bool
    operand_dtype: int     # 0: fp32 operands, 1: bf16 GEMM operands (fp32 accumulate / cell)
    seq_lens: np.ndarray   # int32 [B]
    x: np.ndarray          # float32 [T, B, D], zero past each sequence's length
    # params[l][d] = (W [D_l, 4H], R [H, 4H], b [4H]) float32; d = 0 forward, 1 backward
    params: List[List[Tuple[np.ndarray, np.ndarray, np.ndarray]]] = field(default_factory=list)
    G: Optional[np.ndarray] = None  # float32 [T, B, ndir*H]: loss = sum(y_top * G)

    @property
    def ndir(self) -> int:
        return 2 if self.bidirectional else 1

    @property
    def frames(self) -> int:
        return int(self.seq_lens.sum())


def make_workload(name: str, *, L: int, B: int, D: int, H: int, len_lo: int, len_hi: int,
                  wscale: float, seed: int, bidirectional: bool = True,
                  operand_dtype: int = 0, loss: str = "random", T: Optional[int] = None,
                  bias_scale: float = 0.0) -> Workload:
    """Draw one workload.  Lengths are uniform integers in [len_lo, len_hi]
    (both ends included); sequence 0 is forced to len_hi so that the padded
    length T = len_hi is the same for every seed.  ``loss`` = "ones" gives
    G = 1 (loss = sum of outputs), "random" gives G ~ N(0,1)."""
    rng = np.random.Generator(np.random.Philox(seed))
    seq_lens = rng.integers(len_lo, len_hi + 1, size=B).astype(np.int32)
    if B > 0:
        seq_lens[0] = len_hi
    Tp = int(len_hi if T is None else T)
    assert Tp >= len_hi
    x = rng.standard_normal((Tp, B, D)).astype(np.float32)
    tt = np.arange(Tp, dtype=np.int32)[:, None]
    x *= (tt < seq_lens[None, :])[:, :, None]
    ndir = 2 if bidirectional else 1
    params = []
    for l in range(L):
        Dl = D if l == 0 else ndir * H
        layer = []
        for _d in range(ndir):
            W = rng.uniform(-wscale, wscale, size=(Dl, 4 * H)).astype(np.float32)
            R = rng.uniform(-wscale, wscale, size=(H, 4 * H)).astype(np.float32)
            if bias_scale > 0.0:
                b = rng.uniform(-bias_scale, bias_scale, size=(4 * H,)).astype(np.float32)
            else:
                b = np.zeros((4 * H,), dtype=np.float32)
            layer.append((W, R, b))
        params.append(layer)
    if loss == "ones":
        G = np.ones((Tp, B, ndir * H), dtype=np.float32)
    else:
        G = rng.standard_normal((Tp, B, ndir * H)).astype(np.float32)
    return Workload(name=name, L=L, T=Tp, B=B, D=D, H=H, bidirectional=bidirectional,
                    operand_dtype=operand_dtype, seq_lens=seq_lens, x=x, params=params, G=G)


def config1() -> Workload:
    """1-layer unidirectional LSTM, T=20, B=2, D=8, H=16, all lengths 20, loss = sum(y), seed 0."""
    return make_workload("config1_lstm_T20_B2_D8_H16", L=1, B=2, D=8, H=16, len_lo=20, len_hi=20,
                         wscale=0.1, seed=0, bidirectional=False, loss="ones")


def config2() -> Workload:
    """1-layer BLSTM, D=40, H=256 per direction, B=16, lengths uniform in [100, 500]."""
    return make_workload("config2_blstm1x256_B16", L=1, B=16, D=40, H=256, len_lo=100, len_hi=500,
                         wscale=0.08, seed=2)


def config3() -> Workload:
    """4-layer BLSTM, D=40, H=500 per direction, B=32, lengths uniform in [300, 1000] (headline)."""
    return make_workload("config3_blstm4x500_B32", L=4, B=32, D=40, H=500, len_lo=300, len_hi=1000,
                         wscale=0.05, seed=3)


def config4() -> Workload:
    """6-layer BLSTM, D=40, H=1000 per direction, B=64, lengths in [500, 1500], bf16 GEMM operands."""
    return make_workload("config4_blstm6x1000_B64_bf16", L=6, B=64, D=40, H=1000, len_lo=500,
                         len_hi=1500, wscale=0.03, seed=4, operand_dtype=1)


def config4_short() -> Workload:
    """Config 4's network (6 layers, H=1000, B=64, bf16 operands) on short sequences (lengths uniform in
    [16, 48]) so that the CPU oracle can run the whole minibatch."""
    return make_workload("config4_short_blstm6x1000_B64_bf16", L=6, B=64, D=40, H=1000, len_lo=16, len_hi=48,
                         wscale=0.03, seed=44, operand_dtype=1)


def small_blstm(seed: int = 11, *, L: int = 2, B: int = 5, D: int = 12, H: int = 20,
                len_lo: int = 3, len_hi: int = 37, wscale: float = 0.3,
                bias_scale: float = 0.2, T: Optional[int] = None) -> Workload:
    """A ragged multi-layer BLSTM small enough for the oracle to finish in well under a second."""
    return make_workload(f"small_blstm_s{seed}", L=L, B=B, D=D, H=H, len_lo=len_lo, len_hi=len_hi,
                         wscale=wscale, seed=seed, bias_scale=bias_scale, T=T)


@dataclass
class ImageWorkload:
    """Batch of grayscale-like images for the two-dimensional LSTM layer (four scan directions)."""
    name: str
    Hh: int                # rows of every image
    Ww: int                # padded width (= max widths)
    B: int                 # images per minibatch
    D: int                 # values per pixel
    H: int                 # units per direction
    widths: np.ndarray     # int32 [B]
    x: np.ndarray          # float32 [Hh, Ww, B, D], zero beyond each image's width
    # params[d] = (W [D, 5H], Ru [H, 5H], Rv [H, 5H], b [5H]) float32, d over the four scan directions
    params: List[Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]] = field(default_factory=list)
    G: Optional[np.ndarray] = None  # float32 [Hh, Ww, B, 4H]: loss = sum(y * G)

    @property
    def pixels(self) -> int:
        return int(self.widths.sum()) * self.Hh


def make_image_workload(name: str, *, Hh: int, B: int, D: int, H: int, w_lo: int, w_hi: int, wscale: float,
                        seed: int, bias_scale: float = 0.0, forget_bias: float = 0.0) -> ImageWorkload:
    """Widths are uniform integers in [w_lo, w_hi]; image 0 is forced to w_hi so that the padded width is
    the same for every seed.  Pixel values are uniform in [0, 1).  Draw order: widths, x, then per scan
    direction W, Ru, Rv, b, then G.  ``forget_bias`` is added to the bias of both forget-gate blocks."""
    rng = np.random.Generator(np.random.Philox(seed))
    widths = rng.integers(w_lo, w_hi + 1, size=B).astype(np.int32)
    widths[0] = w_hi
    Ww = int(w_hi)
    x = rng.random((Hh, Ww, B, D), dtype=np.float32)
    for n in range(B):
        x[:, widths[n]:, n, :] = 0.0
    params = []
    for _ in range(4):
        W = rng.uniform(-wscale, wscale, (D, 5 * H)).astype(np.float32)
        Ru = rng.uniform(-wscale, wscale, (H, 5 * H)).astype(np.float32)
        Rv = rng.uniform(-wscale, wscale, (H, 5 * H)).astype(np.float32)
        b = (rng.uniform(-bias_scale, bias_scale, (5 * H,)) if bias_scale else np.zeros(5 * H)).astype(np.float32)
        b[H:3 * H] += np.float32(forget_bias)
        params.append((W, Ru, Rv, b))
    G = rng.standard_normal((Hh, Ww, B, 4 * H)).astype(np.float32)
    return ImageWorkload(name, Hh, Ww, B, D, H, widths, x, params, G)


def config5() -> ImageWorkload:
    """Config 5: two-dimensional LSTM, 4 scan directions, images of height 64 and width uniform in
    [200, 800], pixel values U(0,1), B = 8, H = 32 per direction, fp32.  Weights U(-0.1, 0.1); the two
    forget gates start at bias -1 (f_u + f_v < 1): with zero forget biases the cell state of a 64 x 800
    image is not contractive and float32 arithmetic itself is 1e-3 .. 1e-2 away from float64."""
    return make_image_workload("config5_mdlstm_h64_B8_H32", Hh=64, B=8, D=1, H=32, w_lo=200, w_hi=800,
                               wscale=0.1, seed=5, forget_bias=-1.0)


def config5_plain() -> ImageWorkload:
    """The shape of config 5 with the plain recipe: every bias zero, the forget gates' too (same draws as config 5).  Its results
    depend on their inputs much more strongly than config 5's (the cell state is not contractive), so it is a parity
    case with a tolerance of its own, not a benchmark workload."""
    return make_image_workload("config5_plain_mdlstm_h64_B8_H32", Hh=64, B=8, D=1, H=32, w_lo=200, w_hi=800,
                               wscale=0.1, seed=5, forget_bias=0.0)


def paper_corpus(n_seq: int = 40, seed: int = 6) -> Tuple[np.ndarray, np.ndarray]:
    """A corpus shaped like the one the paper's experiments use (Sec. 6): 45 values per frame, segment
    lengths around 738 frames with a spread of 291 (drawn normal, clipped to [100, 1600]).  Returns
    (x [T, n_seq, 45] float32 ~ N(0,1), zero past each length; lengths int32)."""
    rng = np.random.Generator(np.random.Philox(seed))
    lens = np.clip(np.rint(rng.normal(738.0, 291.0, n_seq)), 100, 1600).astype(np.int32)
    T = int(lens.max())
    x = rng.standard_normal((T, n_seq, 45), dtype=np.float32)
    for b in range(n_seq):
        x[lens[b]:, b, :] = 0.0
    return x, lens


PAPER_SEGMENT_FRAMES = 250     # Sec. 6: segments of 250 frames ...
PAPER_BATCH_SEGMENTS = 81      # ... 81 of them per batch


def paper_workload(x: np.ndarray, seq_lens: np.ndarray) -> Workload:
    """The network the paper times (Sec. 6: three bidirectional layers of 512 units, fp32) on a minibatch of
    segments that the caller has cut from paper_corpus(): x [250, 81, 45] with zeros past each segment's length,
    seq_lens [81].  Cutting the corpus is part of the method and is not done here: the oracle side calls
    oracle.chunk_batch, the HIP side rlstm_chunk_plan / rlstm_chunk_gather.  Draws the weights U(-0.05, 0.05) and the
    loss weights G ~ N(0,1) (zero past each segment's length)."""
    size, nb = x.shape[0], x.shape[1]
    seq_lens = np.asarray(seq_lens, np.int32)
    assert x.shape[2] == 45 and seq_lens.shape == (nb,)
    rng = np.random.Generator(np.random.Philox(66))
    L, D, H = 3, 45, 512
    params = []
    for l in range(L):
        din = D if l == 0 else 2 * H
        layer = []
        for _ in range(2):
            W = rng.uniform(-0.05, 0.05, (din, 4 * H)).astype(np.float32)
            R = rng.uniform(-0.05, 0.05, (H, 4 * H)).astype(np.float32)
            layer.append((W, R, np.zeros(4 * H, np.float32)))
        params.append(layer)
    G = rng.standard_normal((size, nb, 2 * H)).astype(np.float32)
    for b in range(nb):
        G[seq_lens[b]:, b, :] = 0.0
    return Workload("paper_3x512_81_segments_of_250", L, size, nb, D, H, True, 0, seq_lens,
                    np.ascontiguousarray(x, dtype=np.float32), params, G)


def output_layer(T: int, B: int, F: int, C: int, seed: int, wscale: float = 0.1):
    """Random output-layer weights Wo [F,C], bo [C] and frame labels [T,B] (uniform over the classes).  No arithmetic
    of the method: the caller decides which frames are valid."""
    rng = np.random.Generator(np.random.Philox(seed))
    Wo = rng.uniform(-wscale, wscale, (F, C)).astype(np.float32)
    bo = rng.uniform(-wscale, wscale, (C,)).astype(np.float32)
    labels = rng.integers(0, C, (T, B)).astype(np.int32)
    return Wo, bo, labels


@dataclass
class StreamWorkload:
    name: str
    L: int                 # stacked unidirectional layers
    S: int                 # segments
    Tc: int                # frames per segment
    B: int
    D: int
    H: int
    seq_lens: np.ndarray   # int32 [B], lengths of the whole sequences (<= S * Tc)
    x: np.ndarray          # float32 [S*Tc, B, D], zero past each sequence's length
    params: List[Tuple[np.ndarray, np.ndarray, np.ndarray]] = field(default_factory=list)   # per layer (W, R, b)
    G: Optional[np.ndarray] = None   # float32 [S*Tc, B, H]

    @property
    def frames(self) -> int:
        return int(self.seq_lens.sum())


def paper_stream() -> StreamWorkload:
    """Whole sequences of the corpus statistics of Sec. 6 (64 of them, lengths around 738 +- 291 frames, 45 values per
    frame) read in segments of 250 frames by three unidirectional layers of 512 units, fp32: the streaming mode's
    workload.  No arithmetic of the method here."""
    cx, lens = paper_corpus(n_seq=64, seed=8)
    Tc = 250
    S = (int(lens.max()) + Tc - 1) // Tc
    x = np.zeros((S * Tc, cx.shape[1], cx.shape[2]), np.float32)
    x[:cx.shape[0]] = cx
    rng = np.random.Generator(np.random.Philox(88))
    L, D, H = 3, 45, 512
    params = []
    for l in range(L):
        din = D if l == 0 else H
        params.append((rng.uniform(-0.05, 0.05, (din, 4 * H)).astype(np.float32),
                       rng.uniform(-0.05, 0.05, (H, 4 * H)).astype(np.float32), np.zeros(4 * H, np.float32)))
    G = rng.standard_normal((S * Tc, x.shape[1], H)).astype(np.float32)
    for b in range(x.shape[1]):
        G[lens[b]:, b, :] = 0.0
    return StreamWorkload(f"paper_stream_3x512_64_sequences_{S}_segments_of_250", L, S, Tc, x.shape[1], D, H, lens, x, params, G)
