"""Plain CPU oracle for autoregressive sampling from a PixelCNN-style masked convolutional network.

TEST INFRASTRUCTURE ONLY (see made_oracle.py for the rules; nothing in the product path imports this).

The paper's second sampling experiment (Section 5.3.2) uses a masked convolutional network whose states
are visited one pixel after the other in raster-scan order (Section 5.3).  That architecture
and its checkpoint are not available; this is a plain masked-convolution stand-in with the same kind of
state space: an H x W image with 3 channels, one state per sub-pixel in (row, column, channel) order,
C-way categorical states drawn by Gumbel-max from fixed noise (Appendix A.3).  The feedforward recurrence
(Eq. 1), Algorithm 1 and the fixed-point certificate are the same as for the MLP oracle; only the network
that yields the logits differs, so this module supplies the network and re-uses nothing else.

Network (all choices are this build's reading, the paper fixes none of them):
  * input: symbol v of every sub-pixel enters as (v - 128) / 128, 3 input channels;
  * F feature channels in three groups of sizes ceil(F/3), ceil((F - s0)/2), rest (group j serves colour j);
  * layer 1: k x k convolution 3 -> F of type A, layers 2..n_conv: k x k convolutions F -> F of type B, each
    followed by bias + ReLU; zero padding (k-1)/2;
  * head: 1 x 1 convolution F -> 3*C of type B; output block c (C logits) belongs to colour c;
  * masks: a tap strictly above, or in the same row strictly to the left, is fully visible; taps below or
    to the right are invisible; at the centre tap an output of group j sees inputs of group < j (type A;
    input colour c counts as group c) or <= j (type B).
The logits of state (y, x, c) therefore depend on earlier pixels and on colours < c of the same pixel only:
the triangular structure of Eq. 5.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .made_oracle import decide, round_to_bf16


def group_sizes(F: int) -> Tuple[int, int, int]:
    s0 = -(-F // 3)
    s1 = -(-(F - s0) // 2)
    return s0, s1, F - s0 - s1


def group_of_feature(F: int) -> np.ndarray:
    s0, s1, s2 = group_sizes(F)
    return np.concatenate([np.zeros(s0, int), np.ones(s1, int), np.full(s2, 2, int)])


def conv_mask(c_out_groups: np.ndarray, c_in_groups: np.ndarray, k: int, kind: str) -> np.ndarray:
    """Boolean [C_out, k, k, C_in]; tap (ky, kx) reads the input at offset (ky - k//2, kx - k//2)."""
    m = np.zeros((len(c_out_groups), k, k, len(c_in_groups)), dtype=bool)
    mid = k // 2
    for ky in range(k):
        for kx in range(k):
            if ky < mid or (ky == mid and kx < mid):
                m[:, ky, kx, :] = True
            elif ky == mid and kx == mid:
                if kind == "A":
                    m[:, ky, kx, :] = c_in_groups[None, :] < c_out_groups[:, None]
                else:
                    m[:, ky, kx, :] = c_in_groups[None, :] <= c_out_groups[:, None]
    return m


@dataclass
class ConvModel:
    H: int
    W: int
    C: int                      # classes per sub-pixel
    F: int                      # feature channels
    k: int                      # kernel size of the conv layers
    WM: List[np.ndarray]        # masked weights: n_conv arrays [F, k, k, C_in] + head [3*C, 1, 1, F], float64
    b: List[np.ndarray]
    act_round: Optional[str]

    @property
    def D(self) -> int:
        return self.H * self.W * 3


def build_conv_model(H: int, W: int, C: int, F: int, k: int, Wts: Sequence[np.ndarray],
                     b: Sequence[Optional[np.ndarray]], act_round: Optional[str] = None) -> ConvModel:
    """Wts[l] unmasked: [F, k, k, 3] for l = 0, [F, k, k, F] for the other conv layers, [3*C, 1, 1, F] last."""
    gf = group_of_feature(F)
    WM, bb = [], []
    n = len(Wts)
    for l, (Wl, bl) in enumerate(zip(Wts, b)):
        Wl = np.asarray(Wl, dtype=np.float64)
        if l == 0:
            mask = conv_mask(gf, np.arange(3), k, "A")
        elif l < n - 1:
            mask = conv_mask(gf, gf, k, "B")
        else:
            mask = conv_mask(np.repeat(np.arange(3), C), gf, 1, "B")
        assert Wl.shape == mask.shape, (l, Wl.shape, mask.shape)
        WM.append(np.where(mask, Wl, 0.0))
        bb.append(np.zeros(Wl.shape[0]) if bl is None else np.asarray(bl, dtype=np.float64))
    assert act_round in (None, "bf16")
    return ConvModel(H, W, C, F, k, WM, bb, act_round)


def conv_layer(a: np.ndarray, WM: np.ndarray, b: np.ndarray) -> np.ndarray:
    """a [N, H, W, C_in] -> [N, H, W, C_out]: out(y, x) = b + sum_taps WM[:, ky, kx, :] a(y + ky - mid, x + kx - mid),
    zero outside the image."""
    N, H, W, _ = a.shape
    k = WM.shape[1]
    mid = k // 2
    pad = np.zeros((N, H + 2 * mid, W + 2 * mid, a.shape[3]))
    pad[:, mid:mid + H, mid:mid + W, :] = a
    out = np.zeros((N, H, W, WM.shape[0])) + b
    for ky in range(k):
        for kx in range(k):
            w = WM[:, ky, kx, :]
            if not w.any():
                continue
            out += pad[:, ky:ky + H, kx:kx + W, :] @ w.T
    return out


def conv_logits_all(model: ConvModel, x: np.ndarray) -> np.ndarray:
    """x [N, D] symbols (D = H*W*3 in (y, x, colour) order) -> logits [N, D, C] from one pass."""
    N = x.shape[0]
    a = (np.asarray(x, dtype=np.float64).reshape(N, model.H, model.W, 3) - 128.0) / 128.0
    for WM, b in zip(model.WM[:-1], model.b[:-1]):
        a = np.maximum(conv_layer(a, WM, b), 0.0)
        if model.act_round == "bf16":
            a = round_to_bf16(a)
    z = conv_layer(a, model.WM[-1], model.b[-1])             # [N, H, W, 3*C]
    return z.reshape(N, model.D, model.C)


def conv_jacobi_pass(model: ConvModel, x: np.ndarray, noise: np.ndarray):
    return decide(conv_logits_all(model, x), noise, model.C)


def conv_fixed_point_check(model: ConvModel, x: np.ndarray, noise: np.ndarray):
    fx, margin = conv_jacobi_pass(model, x, noise)
    return fx == x, margin


def conv_sequential_sample(model: ConvModel, noise: np.ndarray):
    """Eq. 1: one state after the other (every step evaluates the network; only state t's logits are used)."""
    N, D = noise.shape[0], model.D
    x = np.zeros((N, D), dtype=np.uint8)
    margin = np.zeros((N, D))
    for t in range(D):
        z_t = conv_logits_all(model, x)[:, t]
        x[:, t], margin[:, t] = decide(z_t, noise[:, t], model.C)
    return x, margin


def conv_jacobi_reference(model: ConvModel, noise: np.ndarray, x_init: Optional[np.ndarray] = None,
                          max_iters: Optional[int] = None):
    """Algorithm 1, tolerance 0, per-sample stopping.  Returns (x, iters, converged, min_margin)."""
    N, D = noise.shape[0], model.D
    cap = D if (max_iters is None or max_iters <= 0) else min(max_iters, D)
    x = np.zeros((N, D), dtype=np.uint8) if x_init is None else np.array(x_init, dtype=np.uint8)
    iters = np.zeros(N, dtype=np.int32)
    done = np.zeros(N, dtype=bool)
    min_margin = np.full(N, np.inf)
    k = 0
    while not done.all() and k < cap:
        k += 1
        act = np.flatnonzero(~done)
        new, margin = conv_jacobi_pass(model, x[act], noise[act])
        min_margin[act] = np.minimum(min_margin[act], margin.min(axis=1))
        same = (new == x[act]).all(axis=1)
        x[act] = new
        iters[act] = k
        done[act[same]] = True
        if k == D:
            done[act] = True
    return x, iters, done, min_margin


def conv_jacobi_gs_reference(model: ConvModel, noise: np.ndarray, block: int, x_init: Optional[np.ndarray] = None,
                             max_iters: Optional[int] = None):
    """Algorithm 2 (Jacobi-GS) on the convolutional model, tolerance 0, per-image stopping.
    Returns (x, iters[N], done[N], min_margin[N]).

    The states are cut into consecutive blocks of `block` states (the last may be short).  Iteration k: every block
    [a, b) starts from the previous iterate s^{k-1} and is walked through state by state,
    s_j^k = h_j(u, s^{k-1}_{1:a-1}, s^k_{a:j-1}) -- the blocks independently of each other ("in parallel") -- and the
    blocks' new states together form s^k.  An image stops at the first k with s^k == s^{k-1} or at k = M (number of
    blocks), where the result is exact (Proposition 2).  The count includes the confirming iteration."""
    N, D = noise.shape[0], model.D
    parts = [(a, min(a + block, D)) for a in range(0, D, block)]
    M = len(parts)
    cap = M if (max_iters is None or max_iters <= 0) else min(max_iters, M)
    x = np.zeros((N, D), dtype=np.uint8) if x_init is None else np.array(x_init, dtype=np.uint8)
    iters = np.zeros(N, dtype=np.int32)
    done = np.zeros(N, dtype=bool)
    min_margin = np.full(N, np.inf)
    k = 0
    while not done.all() and k < cap:
        k += 1
        act = np.flatnonzero(~done)
        prev = x[act]
        new = prev.copy()
        for (a, b) in parts:
            mixed = prev.copy()                         # s^{k-1} everywhere, then the block's own new states
            for j in range(a, b):
                z_j = conv_logits_all(model, mixed)[:, j]
                mixed[:, j], margin = decide(z_j, noise[act][:, j], model.C)
                min_margin[act] = np.minimum(min_margin[act], margin)
            new[:, a:b] = mixed[:, a:b]
        same = (new == prev).all(axis=1)
        x[act] = new
        iters[act] = k
        done[act[same]] = True
        if k == M:
            done[act] = True
    return x, iters, done, min_margin
