"""Seeded synthetic inputs: network shapes, degrees, weights and noise.

This module only *draws data*.  It holds none of the sampler's arithmetic (no masks,
no forward pass, no decision rule) and imports neither the HIP binding nor the CPU
oracle, so both sides of a parity test can be handed the very same arrays.

Workload shapes follow the paper's autoregressive-sampling experiment (Section 5.3.1
and Appendix C.3: MADE over T = 784 raster-ordered pixels, about 100 images sampled
in parallel); the trained weights and the image data sets are replaced by seeded
random networks of the same shape.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import os

import numpy as np

SEED_BASE = 2002036290


@dataclass
class Workload:
    """One named synthetic workload (shape of the network plus batch and seeds)."""
    name: str
    D: int                      # number of positions (T in the paper)
    C: int                      # 1 = Bernoulli positions, >1 = C-way categorical positions
    hidden: List[int]           # widths of the hidden masked layers
    dtype: str                  # "f32" or "bf16" (weights and hidden activations)
    N: int                      # batch (independent samples drawn in parallel)
    degree_rule: str            # "cyclic" or "random"
    weight_rule: str            # "std0.1" or "fan_in"
    seed: int = SEED_BASE
    gain: float = 1.0           # extra factor on every weight (coupling strength sweeps)
    block_sizes: List[int] = field(default_factory=list)
    real: bool = False          # continuous states with logistic conditionals (C = 2 outputs per position)
    onehot: bool = False        # categorical symbols enter the network as one-hot vectors (D * C inputs)


def workload(name: str) -> Workload:
    """The benchmark configurations plus reduced versions used by the tests."""
    table = {
        # tiny fp32 MADE, natural ordering
        "cfg1": Workload("cfg1", 64, 1, [256], "f32", 16, "cyclic", "std0.1", SEED_BASE + 1),
        # MNIST-shaped binary MADE
        "cfg2": Workload("cfg2", 784, 1, [2000, 2000], "bf16", 128, "random", "fan_in", SEED_BASE + 2,
                         block_sizes=[16, 64, 196]),
        # 256-way categorical MADE
        "cfg4": Workload("cfg4", 1024, 256, [4096, 4096], "bf16", 64, "random", "fan_in", SEED_BASE + 4),
        # reduced shapes with ragged tiles (nothing is a multiple of 32)
        "small_f32": Workload("small_f32", 50, 1, [77, 45], "f32", 9, "random", "fan_in", SEED_BASE + 11, gain=3.0),
        "small_bf16": Workload("small_bf16", 100, 1, [203, 150], "bf16", 37, "random", "fan_in", SEED_BASE + 12,
                               gain=2.0),
        "mid_bf16": Workload("mid_bf16", 196, 1, [500, 500], "bf16", 70, "random", "fan_in", SEED_BASE + 13,
                             gain=2.0),
        "small_cat": Workload("small_cat", 24, 256, [96, 80], "bf16", 10, "random", "fan_in", SEED_BASE + 14,
                              gain=1.5),
        "small_cat_f32": Workload("small_cat_f32", 12, 5, [40], "f32", 7, "random", "fan_in", SEED_BASE + 15,
                                  gain=3.0),
        # the same categorical models with one-hot input (the alternative reading of the input encoding)
        "cfg4_onehot": Workload("cfg4_onehot", 1024, 256, [4096, 4096], "bf16", 64, "random", "fan_in", SEED_BASE + 7,
                                onehot=True),
        "small_cat_onehot": Workload("small_cat_onehot", 24, 256, [96, 80], "bf16", 10, "random", "fan_in",
                                     SEED_BASE + 18, gain=1.5, onehot=True),
        "small_cat_onehot_f32": Workload("small_cat_onehot_f32", 12, 5, [40], "f32", 7, "random", "fan_in",
                                         SEED_BASE + 19, gain=3.0, onehot=True),
        "mid_cat_onehot": Workload("mid_cat_onehot", 70, 7, [300, 130], "bf16", 45, "random", "fan_in",
                                   SEED_BASE + 21, gain=2.5, onehot=True),
        # first layers of several 512-unit chunks (three: an odd count, and two), which the one-hot kernel pairs up
        "wide_cat_onehot": Workload("wide_cat_onehot", 40, 7, [1400, 96], "bf16", 37, "random", "fan_in",
                                    SEED_BASE + 23, gain=2.0, onehot=True),
        "wide_cat_onehot_f32": Workload("wide_cat_onehot_f32", 30, 5, [700], "f32", 9, "random", "fan_in",
                                        SEED_BASE + 24, gain=2.5, onehot=True),
        # continuous states, logistic conditionals: the paper's own MADE (2 x 512 hidden, 100 images, T = 784)
        "made_logistic": Workload("made_logistic", 784, 2, [512, 512], "bf16", 100, "random", "fan_in", SEED_BASE + 6,
                                  real=True),
        "small_real_f32": Workload("small_real_f32", 50, 2, [77, 45], "f32", 9, "random", "fan_in", SEED_BASE + 16,
                                   gain=1.5, real=True),
        "small_real_bf16": Workload("small_real_bf16", 100, 2, [203, 150], "bf16", 37, "random", "fan_in",
                                    SEED_BASE + 17, gain=1.5, real=True),
    }
    return table[name]


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


def bf16_representable(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are the inputs rounded to the nearest bfloat16 (ties to even).

    Pure data preparation: the library and the oracle both receive these already
    representable numbers, so neither has to agree with the other on how to round weights.
    """
    out = np.array(a, dtype=np.float32, copy=True, order="C")
    _round_bf16_inplace(out)
    return out


def _round_bf16_inplace(out: np.ndarray) -> None:
    flat = out.reshape(-1).view(np.uint32)
    step = 1 << 24                                   # bounded temporaries for multi-GiB matrices
    for i in range(0, flat.size, step):
        bits = flat[i:i + step]
        lsb = (bits >> np.uint32(16)) & np.uint32(1)
        # no finite normal weight is within 0x8000 of the uint32 range's end, so this cannot wrap
        bits += np.uint32(0x7FFF) + lsb
        bits &= np.uint32(0xFFFF0000)


def hidden_degrees(rule: str, D: int, widths: List[int], seed: int) -> List[np.ndarray]:
    """Degree (1..D-1) of every hidden unit, one int32 array per hidden layer."""
    g = _rng(seed)
    out = []
    for H in widths:
        if D < 2:
            raise ValueError("need D >= 2 for hidden degrees")
        if rule == "cyclic":
            m = 1 + (np.arange(H) % (D - 1))
        elif rule == "random":
            m = g.integers(1, D, size=H)
        else:
            raise ValueError(rule)
        out.append(m.astype(np.int32))
    return out


def dense_weights(D: int, C: int, widths: List[int], rule: str, seed: int, gain: float = 1.0,
                  bf16: bool = False, onehot: bool = False) -> List[np.ndarray]:
    """Unmasked fp32 weight matrices, row-major [out, in], one per layer (L hidden + output).

    "std0.1": every entry N(0, 0.1^2).  "fan_in": N(0, 1/fan_in) with fan_in the dense
    input width of the layer.  The output layer has D*C rows, row index t*C + c.  With one-hot input
    the first layer has D*C columns (column t*C + c) of which D are active at a time: its fan_in is D.
    """
    g = _rng(seed)
    dims = [D * C if onehot else D] + list(widths) + [D * C]
    Ws = []
    for l in range(len(dims) - 1):
        fan_in, fan_out = dims[l], dims[l + 1]
        std = 0.1 if rule == "std0.1" else (1.0 / np.sqrt(D if (onehot and l == 0) else fan_in))
        scale = np.float32(std * gain)
        if fan_out * fan_in <= (1 << 26):
            w = g.standard_normal(size=(fan_out, fan_in), dtype=np.float32)
            w *= scale
            if bf16:
                _round_bf16_inplace(w)
        else:
            # multi-GiB layer: row blocks are drawn from jumped copies of the layer's own stream, in parallel
            w = np.empty((fan_out, fan_in), dtype=np.float32)
            rows = max(1, (1 << 24) // fan_in)

            def draw(i, w=w, rows=rows, l=l, scale=scale):
                blk = w[i * rows:(i + 1) * rows]
                gb = np.random.Generator(np.random.Philox(int(seed)).jumped(1 + 65536 * (l + 1) + i))
                gb.standard_normal(size=blk.shape, dtype=np.float32, out=blk)
                blk *= scale
                if bf16:
                    _round_bf16_inplace(blk)

            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
                list(pool.map(draw, range((fan_out + rows - 1) // rows)))
        Ws.append(w)
    return Ws


def uniform_noise(N: int, D: int, seed: int) -> np.ndarray:
    """u[N, D] fp32 in [0, 1): the fixed per-position noise of a Bernoulli sampler."""
    u = _rng(seed).random(size=(N, D), dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def gumbel_noise(N: int, D: int, C: int, seed: int) -> np.ndarray:
    """g[N, D, C] fp32 standard Gumbel values, computed once in fp64 from clamped uniforms."""
    u = _rng(seed).random(size=(N, D, C))
    u = np.clip(u, 2.0 ** -24, 1.0 - 2.0 ** -24)
    return (-np.log(-np.log(u))).astype(np.float32)


@dataclass
class Network:
    """Raw description handed to both `made_init` and the oracle."""
    D: int
    C: int
    hidden: List[int]
    dtype: str
    degrees: List[np.ndarray]
    W: List[np.ndarray]
    b: List[Optional[np.ndarray]]
    real: bool = False          # continuous states with logistic conditionals (then C = 2: mean and log-scale rows)
    onehot: bool = False        # W[0] is [hidden[0], D * C]: symbols enter as one-hot vectors


def make_network(w: Workload, with_bias: bool = False) -> Network:
    degs = hidden_degrees(w.degree_rule, w.D, w.hidden, w.seed + 1)
    Ws = dense_weights(w.D, w.C, w.hidden, w.weight_rule, w.seed, w.gain, bf16=(w.dtype == "bf16"), onehot=w.onehot)
    bs: List[Optional[np.ndarray]] = [None] * len(Ws)
    if with_bias:
        g = _rng(w.seed + 3)
        bs = []
        for W in Ws:
            b = (0.3 * g.standard_normal(size=W.shape[0])).astype(np.float32)
            bs.append(bf16_representable(b) if w.dtype == "bf16" else b)
    return Network(w.D, w.C, list(w.hidden), w.dtype, degs, Ws, bs, w.real, w.onehot)


def logistic_noise(N: int, D: int, seed: int) -> np.ndarray:
    """l[N, D] fp32 standard logistic variates log(u / (1 - u)), computed once in fp64 from clamped uniforms."""
    u = np.clip(_rng(seed).random(size=(N, D)), 2.0 ** -24, 1.0 - 2.0 ** -24)
    return np.log(u / (1.0 - u)).astype(np.float32)


def make_noise(w: Workload, rep: int = 0, N: Optional[int] = None) -> np.ndarray:
    n = w.N if N is None else N
    seed = w.seed + 2 + 10 * rep
    if w.real:
        return logistic_noise(n, w.D, seed)
    return uniform_noise(n, w.D, seed) if w.C == 1 else gumbel_noise(n, w.D, w.C, seed)


# ---------------------------------------------------------------------------------------------
# Hand-built networks whose dependency structure is one of the paper's worked examples
# (Section 4.1).  Only weights/biases are chosen here; what they imply is asserted in the tests.
# ---------------------------------------------------------------------------------------------

def independent_network(D: int, H: int, seed: int, dtype: str = "f32") -> Network:
    """Example 1: every weight zero, arbitrary output biases -> positions are independent."""
    degs = hidden_degrees("cyclic", D, [H], 0)
    W = [np.zeros((H, D), np.float32), np.zeros((D, H), np.float32)]
    bV = (2.0 * _rng(seed).standard_normal(size=D)).astype(np.float32)
    if dtype == "bf16":
        bV = bf16_representable(bV)
    return Network(D, 1, [H], dtype, degs, W, [np.zeros(H, np.float32), bV])


def first_only_network(D: int, H: int, seed: int, dtype: str = "f32") -> Network:
    """Example 2: only position 1 feeds the network; its own bias forces x_1 = 1."""
    g = _rng(seed)
    degs = hidden_degrees("cyclic", D, [H], 0)
    W1 = np.zeros((H, D), np.float32)
    W1[:, 0] = (1.0 + g.random(size=H)).astype(np.float32)
    WV = (4.0 * g.standard_normal(size=(D, H)) / np.sqrt(H)).astype(np.float32)
    bV = np.zeros(D, np.float32)
    bV[0] = 30.0
    if dtype == "bf16":
        W1, WV = bf16_representable(W1), bf16_representable(WV)
    return Network(D, 1, [H], dtype, degs, [W1, WV], [np.zeros(H, np.float32), bV])


def copy_chain_network(D: int, dtype: str = "f32") -> Network:
    """Example 3: a strict Markov chain.  Hidden unit k (degree k) copies x_k, output t+1 reads
    only that unit; biases make x_1 = 1 and x_t = x_{t-1}, so a 1 walks one position per pass."""
    H = D - 1
    degs = [np.arange(1, D, dtype=np.int32)]
    W1 = np.zeros((H, D), np.float32)
    WV = np.zeros((D, H), np.float32)
    for k in range(H):
        W1[k, k] = 1.0          # unit of degree k+1 reads position k+1 (0-based column k)
        WV[k + 1, k] = 64.0     # position k+2 (0-based row k+1) reads that unit
    bV = np.full(D, -32.0, np.float32)
    bV[0] = 32.0
    return Network(D, 1, [H], dtype, degs, [W1, WV], [np.zeros(H, np.float32), bV])


def skip_network(D: int, H: int, skip: int, seed: int, dtype: str = "f32") -> Network:
    """Position t reads only positions <= t - skip, so the dependency DAG's longest path has
    ceil(D / skip) state nodes (the critical-path remark of Section 4.1)."""
    g = _rng(seed)
    degs = hidden_degrees("cyclic", D, [H], 0)
    W1 = (3.0 * g.standard_normal(size=(H, D)) / np.sqrt(D)).astype(np.float32)
    WV = (6.0 * g.standard_normal(size=(D, H)) / np.sqrt(H)).astype(np.float32)
    m = degs[0]
    for t in range(1, D + 1):
        WV[t - 1, m > t - skip] = 0.0
    if dtype == "bf16":
        W1, WV = bf16_representable(W1), bf16_representable(WV)
    return Network(D, 1, [H], dtype, degs, [W1, WV], [np.zeros(H, np.float32), np.zeros(D, np.float32)])


# ---------------------------------------------------------------------------------------------
# Masked convolutional (PixelCNN-style) workloads: H x W images, 3 colours, one C-way state per sub-pixel
# ---------------------------------------------------------------------------------------------

@dataclass
class ConvWorkload:
    name: str
    H: int
    W: int
    C: int                      # classes per sub-pixel
    F: int                      # feature channels
    k: int                      # kernel size
    n_conv: int                 # masked k x k layers (first of type A, rest of type B); a 1 x 1 head follows
    dtype: str
    N: int
    seed: int
    gain: float = 1.0


def conv_workload(name: str) -> ConvWorkload:
    table = {
        # 32 x 32 x 3 image, 256-way sub-pixels, 8 masked 5 x 5 layers of 128 channels, batch 32
        # (about half of a layer's taps are visible and ReLU halves the variance again: gain 2 keeps the scale from
        # layer to layer; 2.3 gives logits of rms ~2, i.e. conditionals that are neither flat nor one-hot)
        "cfg5": ConvWorkload("cfg5", 32, 32, 256, 128, 5, 8, "bf16", 32, SEED_BASE + 5, gain=2.3),
        # reduced shapes for the parity tests (the width stays 32: one row of pixels per 32-row operand group)
        "small_conv": ConvWorkload("small_conv", 3, 32, 256, 64, 5, 3, "bf16", 3, SEED_BASE + 21, gain=1.5),
        "small_conv_f32": ConvWorkload("small_conv_f32", 2, 32, 256, 64, 3, 2, "f32", 2, SEED_BASE + 22, gain=2.0),
    }
    return table[name]


@dataclass
class ConvNetwork:
    H: int
    W: int
    C: int
    F: int
    k: int
    dtype: str
    W_: List[np.ndarray]        # [F, k, k, 3], (n_conv - 1) x [F, k, k, F], [3*C, 1, 1, F]; unmasked fp32
    b: List[Optional[np.ndarray]]

    @property
    def D(self) -> int:
        return self.H * self.W * 3


def make_conv_network(w: ConvWorkload, with_bias: bool = False) -> ConvNetwork:
    g = _rng(w.seed)
    shapes = [(w.F, w.k, w.k, 3)] + [(w.F, w.k, w.k, w.F)] * (w.n_conv - 1) + [(3 * w.C, 1, 1, w.F)]
    Ws, bs = [], []
    for shp in shapes:
        fan_in = shp[1] * shp[2] * shp[3]
        wt = g.standard_normal(size=shp, dtype=np.float32) * np.float32(w.gain / np.sqrt(fan_in))
        if w.dtype == "bf16":
            _round_bf16_inplace(wt)
        Ws.append(wt)
        if with_bias:
            bb = (0.2 * g.standard_normal(size=shp[0])).astype(np.float32)
            bs.append(bf16_representable(bb) if w.dtype == "bf16" else bb)
        else:
            bs.append(None)
    return ConvNetwork(w.H, w.W, w.C, w.F, w.k, w.dtype, Ws, bs)


def make_conv_noise(w: ConvWorkload, rep: int = 0, N: Optional[int] = None) -> np.ndarray:
    n = w.N if N is None else N
    return gumbel_noise(n, w.H * w.W * 3, w.C, w.seed + 2 + 10 * rep)


# ------------------------------------------------------------------------------------------------
# recurrent network of Section 5.1 (backward pass by Jacobi iteration)
# ------------------------------------------------------------------------------------------------
@dataclass
class RnnWorkload:
    """One-layer RNN fitted to pixel sequences (Section 5.1, Appendix C.1)."""
    name: str
    B: int                      # sequences handled in parallel (the paper trains with batch size 1)
    T: int                      # time steps = pixels of one flattened image
    H: int                      # hidden units
    I: int                      # inputs per step
    seed: int = SEED_BASE + 40
    w_std: float = 0.1          # all weights N(0, w_std^2), biases zero (Appendix C.1)


def rnn_workload(name: str) -> RnnWorkload:
    table = {
        # the paper's shape: 10 x 10 images read pixel by pixel, 128 hidden units, batch 1
        "rnn_paper": RnnWorkload("rnn_paper", 1, 100, 128, 1, SEED_BASE + 41),
        # the same network on a batch that fills the GPU (one sequence per workgroup)
        "rnn_batch": RnnWorkload("rnn_batch", 256, 100, 128, 1, SEED_BASE + 42),
        # reduced, ragged shapes for the tests (nothing a multiple of 32)
        "rnn_small": RnnWorkload("rnn_small", 5, 37, 40, 3, SEED_BASE + 43, w_std=0.2),
        "rnn_wide": RnnWorkload("rnn_wide", 3, 70, 100, 2, SEED_BASE + 44, w_std=0.12),
    }
    return table[name]


def make_rnn_params(w: RnnWorkload):
    """(W [H, H], U [H, I], b [H]) as float32."""
    r = _rng(w.seed)
    W = (r.standard_normal((w.H, w.H)) * w.w_std).astype(np.float32)
    U = (r.standard_normal((w.H, w.I)) * w.w_std).astype(np.float32)
    b = np.zeros((w.H,), dtype=np.float32)
    return W, U, b


def make_rnn_inputs(w: RnnWorkload, rep: int = 0):
    """(x [B, T, I], y [B, T, H]) as float32: x are flattened blob images with values in [0, 1] (stand-ins for the
    resized digits; for I > 1 the channels are shifted copies), y are the per-step targets of the squared loss the
    benchmark and the tests put on the hidden state."""
    r = _rng(w.seed + 1000 * (rep + 1))
    side = int(np.ceil(np.sqrt(w.T)))
    yy, xx = np.mgrid[0:side, 0:side].astype(np.float64)
    x = np.zeros((w.B, w.T, w.I), dtype=np.float64)
    for bi in range(w.B):
        img = np.zeros((side, side))
        for _ in range(2):
            cy, cx = r.uniform(0.2, 0.8, size=2) * (side - 1)
            s = r.uniform(0.8, 2.0)
            img += np.exp(-((yy - cy) ** 2 + (xx - cx) ** 2) / (2 * s * s))
        flat = np.clip(img, 0.0, 1.0).reshape(-1)[:w.T]
        for c in range(w.I):
            x[bi, :, c] = np.roll(flat, c)
    y = r.uniform(0.3, 1.2, size=(w.B, w.T, w.H))
    return x.astype(np.float32), y.astype(np.float32)
