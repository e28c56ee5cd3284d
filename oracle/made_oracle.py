"""Plain CPU oracle for autoregressive sampling from a MADE-style masked MLP.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it
exists so that tests, the smoke check and the benchmark's CPU-baseline leg have an
independent, slow, obviously-correct statement of what the HIP library must compute.
It shares no code with the HIP path.  Everything is float64 numpy.

What it states, and where the paper fixes it:

* The feedforward recurrence s_t = h_t(u, s_{1:t-1}) (Section 2.1, Eq. 1), evaluated one
  position at a time: `sequential_sample`.  This is the definition of the result; the
  Jacobi and GS-Jacobi methods reach exactly the same values (Propositions 1 and 2).
* h_t for ancestral sampling (Appendix A.3): position t is drawn from p(x_t | x_{<t})
  using the t-th entry of a fixed noise vector u.  Here p comes from a masked MLP
  (the MADE construction the paper cites in Section 5.3): `logits_at`, `decide`.
* Algorithm 1 (nonlinear Jacobi) and Algorithm 3 (GS-Jacobi) written out step by step
  with tolerance 0, so that iteration counts can be compared: `jacobi_reference`,
  `gs_jacobi_reference`.
* The chain rule p(x) = prod_t p(x_t | x_{<t}) (Appendix A.3) by enumeration:
  `joint_bruteforce`.

Readings the paper leaves open (mask rule, encodings, tie-breaks, per-sample stopping)
are documented next to the code that takes them.

Every function here is pinned by tests/test_oracle_*.py against hand-computed masks,
closed forms, a scalar by-definition evaluator, the paper's three worked examples
(Section 4.1) and brute-force enumeration; no function is left unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------------------
# bfloat16 rounding (used only to model the hidden activations of the bf16 network)
# --------------------------------------------------------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float64.

    bfloat16 keeps the top 16 bits of an IEEE float32.  The value is first rounded to
    float32, then to 16 bits.  (For the activations this oracle rounds, the double
    rounding differs from a direct rounding only on a measure-zero set of fp64 inputs.)
    """
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    keep = bits >> np.uint64(16)
    rem = bits & np.uint64(0xFFFF)
    up = (rem > 0x8000) | ((rem == 0x8000) & ((keep & np.uint64(1)) == 1))
    keep = keep + up.astype(np.uint64)
    out = (keep << np.uint64(16)).astype(np.uint32).view(np.float32)
    return out.astype(np.float64).reshape(np.shape(a))


# --------------------------------------------------------------------------------------
# The model
# --------------------------------------------------------------------------------------

@dataclass
class MadeModel:
    D: int                      # positions (T in the paper)
    C: int                      # 1: Bernoulli position, >1: C-way categorical position
    masks: List[np.ndarray]     # L+1 boolean masks, [out, in]
    WM: List[np.ndarray]        # L+1 masked weights (W * mask), [out, in], float64; a multi-GiB layer given as
                                # float32 is kept as float32 (an exact copy; all arithmetic on it is float64)
    b: List[np.ndarray]         # L+1 biases, float64
    act_round: Optional[str]    # None, or "bf16": round every hidden activation to bfloat16
    onehot: bool = False        # categorical symbols enter as one-hot vectors (D * C inputs) instead of one scalar each


def masks_from_degrees(D: int, C: int, degrees: Sequence[np.ndarray], onehot: bool = False) -> List[np.ndarray]:
    """Autoregressive masks of the masked MLP (the MADE construction cited in Section 5.3).

    Input position d (1-based) carries degree d.  A hidden unit of degree m may read a
    unit (or input) of degree <= m.  Output row (t, c) may read last-layer units of
    degree < t, strictly, so that the logits of position t are a function of x_{1:t-1}
    only -- the triangular structure of Eq. 5.  There are no direct input->output links.
    With one-hot input, position d owns the C inputs d*C .. d*C + C - 1, all of degree d.
    """
    prev = np.repeat(np.arange(1, D + 1), C) if onehot else np.arange(1, D + 1)
    masks = []
    for m in degrees:
        m = np.asarray(m, dtype=np.int64)
        masks.append(m[:, None] >= prev[None, :])
        prev = m
    t_of_row = np.repeat(np.arange(1, D + 1), C)       # row t*C + c belongs to position t
    masks.append(t_of_row[:, None] > prev[None, :])
    return masks


def build_model(D: int, C: int, degrees: Sequence[np.ndarray], W: Sequence[np.ndarray],
                b: Sequence[Optional[np.ndarray]], act_round: Optional[str] = None, onehot: bool = False) -> MadeModel:
    assert not onehot or C > 1
    masks = masks_from_degrees(D, C, degrees, onehot)
    assert len(W) == len(masks) == len(b)
    WM, bb = [], []
    for Wl, Ml, bl in zip(W, masks, b):
        assert Wl.shape == Ml.shape, (Wl.shape, Ml.shape)
        Wl = np.asarray(Wl)
        keep32 = Wl.dtype == np.float32 and Wl.size > (1 << 27)      # only multi-GiB layers stay float32
        masked = np.array(Wl, dtype=np.float32 if keep32 else np.float64, copy=True)
        rows = max(1, (1 << 26) // Wl.shape[1])         # row blocks only bound the temporaries
        for r0 in range(0, Wl.shape[0], rows):
            blk = masked[r0:r0 + rows]
            blk[~Ml[r0:r0 + rows]] = 0.0
        WM.append(masked)
        bb.append(np.zeros(Wl.shape[0]) if bl is None else np.asarray(bl, dtype=np.float64))
    assert act_round in (None, "bf16")
    return MadeModel(D, C, masks, WM, bb, act_round, onehot)


def encode(x: np.ndarray, C: int, onehot: bool = False) -> np.ndarray:
    """Network input for symbol values x: Bernoulli positions enter as 0/1, categorical
    positions as the scalar (x - 128) / 128 (one input per position, as in the paper's MADE
    whose states are scalar pixel intensities, Appendix C.3) -- or, in the one-hot reading, as the
    indicator vector of the symbol: input t*C + c is 1 iff x_t = c."""
    if onehot:
        x = np.asarray(x, dtype=np.int64)
        N, D = x.shape
        e = np.zeros((N, D * C))
        e[np.arange(N)[:, None], np.arange(D)[None, :] * C + x] = 1.0
        return e
    x = np.asarray(x, dtype=np.float64)
    return x if C == 1 else (x - 128.0) / 128.0


def affine(h: np.ndarray, WM: np.ndarray, b: np.ndarray) -> np.ndarray:
    """h (W * M)^T + b in float64.  Weights stored as float32 are widened (exactly) block of rows by block
    of rows, which only limits memory: every product and sum is float64."""
    if WM.dtype == np.float64:
        return h @ WM.T + b
    out = np.empty((h.shape[0], WM.shape[0]))
    rows = max(1, (1 << 25) // WM.shape[1])
    for r0 in range(0, WM.shape[0], rows):
        out[:, r0:r0 + rows] = h @ WM[r0:r0 + rows].astype(np.float64).T
    return out + b


def last_hidden(model: MadeModel, x: np.ndarray) -> np.ndarray:
    """h_L for a batch of symbol vectors x[N, D]: h_l = ReLU((W_l * M_l) h_{l-1} + b_l)."""
    h = encode(x, model.C, model.onehot)
    for WM, b in zip(model.WM[:-1], model.b[:-1]):
        h = np.maximum(affine(h, WM, b), 0.0)
        if model.act_round == "bf16":
            h = round_to_bf16(h)
    return h


def logits_all(model: MadeModel, x: np.ndarray) -> np.ndarray:
    """Logits of every position, z[N, D, C], from one pass over the whole network."""
    h = last_hidden(model, x)
    z = affine(h, model.WM[-1], model.b[-1])
    return z.reshape(x.shape[0], model.D, model.C)


def logits_at(model: MadeModel, x: np.ndarray, t: int) -> np.ndarray:
    """Logits of position t (0-based) only, z[N, C]: the quantity h_t needs."""
    h = last_hidden(model, x)
    rows = slice(t * model.C, (t + 1) * model.C)
    return affine(h, model.WM[-1][rows], model.b[-1][rows])


def decide(z: np.ndarray, noise: np.ndarray, C: int) -> Tuple[np.ndarray, np.ndarray]:
    """Turn logits and the fixed noise of the same positions into symbols.

    Bernoulli (C == 1; z[..., 1], noise u[...]): inverse-CDF draw, x = 1 iff u < sigmoid(z).
    Categorical (z[..., C], noise g[..., C] standard Gumbel): x = argmax_c (z_c + g_c), the
    lowest index winning ties (Gumbel-max draws from softmax(z)).
    Also returns the decision margin: |sigmoid(z) - u|, resp. best minus runner-up of z + g.
    """
    if C == 1:
        p = 1.0 / (1.0 + np.exp(-z[..., 0]))
        u = np.asarray(noise, dtype=np.float64)
        return (u < p).astype(np.uint8), np.abs(p - u)
    s = z + np.asarray(noise, dtype=np.float64)
    x = np.argmax(s, axis=-1)                          # first maximal index
    srt = np.sort(s, axis=-1)
    return x.astype(np.uint8), srt[..., -1] - srt[..., -2]


def _noise_at(noise: np.ndarray, t) -> np.ndarray:
    return noise[:, t]


# --------------------------------------------------------------------------------------
# The definition: sequential (feedforward) sampling, Eq. 1
# --------------------------------------------------------------------------------------

def sequential_sample(model: MadeModel, noise: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x[N, D] (uint8) and the decision margins [N, D], one position after the other."""
    N = noise.shape[0]
    x = np.zeros((N, model.D), dtype=np.uint8)
    margin = np.zeros((N, model.D))
    for t in range(model.D):
        z_t = logits_at(model, x, t)                    # depends on x[:, :t] only
        x[:, t], margin[:, t] = decide(z_t, _noise_at(noise, t), model.C)
    return x, margin


def jacobi_pass(model: MadeModel, x: np.ndarray, noise: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """F(x): every position re-drawn in parallel from the previous iterate (the body of
    Algorithm 1).  Returns the new symbols and the decision margins."""
    return decide(logits_all(model, x), noise, model.C)


def fixed_point_check(model: MadeModel, x: np.ndarray, noise: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """x solves the triangular system (Eq. 5) iff F(x) == x; the solution is unique, so this
    one pass certifies a sample of any size.  Returns (F(x) == x per position, margins at x)."""
    fx, margin = jacobi_pass(model, x, noise)
    return fx == x, margin


# --------------------------------------------------------------------------------------
# Algorithm 1: nonlinear Jacobi iteration, tolerance 0, each sample an independent system
# --------------------------------------------------------------------------------------

def jacobi_reference(model: MadeModel, noise: np.ndarray, x_init: Optional[np.ndarray] = None,
                     max_iters: Optional[int] = None, record: bool = False):
    """Returns (x, iters[N], converged[N], trajectory or None, min_margin[N]).

    Each sample stops at the first k with s^k == s^{k-1}, or at k = T (= D); `iters` is that
    stopping k, so it includes the pass that merely confirms the fixed point.  A sample
    that stopped is left untouched afterwards (it is a fixed point, so further passes would
    not change it).  With max_iters < D a sample may end unconverged (converged[n] False).
    trajectory[k] is s^k for the whole batch (stopped samples keep their value).
    min_margin[n] is the smallest decision margin sample n met in any of its passes.
    """
    N, D = noise.shape[0], model.D
    cap = D if (max_iters is None or max_iters <= 0) else min(max_iters, D)
    x = np.zeros((N, D), dtype=np.uint8) if x_init is None else np.array(x_init, dtype=np.uint8)
    iters = np.zeros(N, dtype=np.int32)
    done = np.zeros(N, dtype=bool)
    traj = [x.copy()] if record else None
    min_margin = np.full(N, np.inf)
    k = 0
    while not done.all() and k < cap:
        k += 1
        act = np.flatnonzero(~done)
        new, margin = jacobi_pass(model, x[act], noise[act])
        min_margin[act] = np.minimum(min_margin[act], margin.min(axis=1))
        same = (new == x[act]).all(axis=1)
        x[act] = new
        iters[act] = k
        done[act[same]] = True
        if k == D:
            done[act] = True                            # the "k = T" clause: exact by Prop. 1
        if record:
            traj.append(x.copy())
    return x, iters, done, traj, min_margin


# --------------------------------------------------------------------------------------
# Algorithm 3: GS-Jacobi (blocks swept in order, Jacobi inside a block)
# --------------------------------------------------------------------------------------

def block_partition(D: int, block: int) -> List[Tuple[int, int]]:
    """Consecutive intervals [a, b) of `block` positions covering 0..D-1; the last may be short."""
    return [(a, min(a + block, D)) for a in range(0, D, block)]


def gs_jacobi_reference(model: MadeModel, noise: np.ndarray, block: int,
                        x_init: Optional[np.ndarray] = None):
    """Returns (x, iters[N], per_block_iters[N, M], min_margin[N]).

    For block [a, b): the block's positions start from x_init (zeros by default), then
    s_j^k = h_j(u, s_{1:a-1} final, s^{k-1}_{a:j-1}) for all j in the block at once, until the
    block did not change or k = |block|.  Samples are independent systems; iters[n] is the
    sum over blocks of sample n's inner iteration counts.
    """
    N, D = noise.shape[0], model.D
    x = np.zeros((N, D), dtype=np.uint8) if x_init is None else np.array(x_init, dtype=np.uint8)
    parts = block_partition(D, block)
    per_block = np.zeros((N, len(parts)), dtype=np.int32)
    min_margin = np.full(N, np.inf)
    for i, (a, b) in enumerate(parts):
        done = np.zeros(N, dtype=bool)
        k = 0
        while not done.all():
            k += 1
            act = np.flatnonzero(~done)
            z = logits_all(model, x[act])[:, a:b]        # positions of this block only
            new, margin = decide(z, noise[act, a:b], model.C)
            min_margin[act] = np.minimum(min_margin[act], margin.min(axis=1))
            same = (new == x[act, a:b]).all(axis=1)
            xa = x[act]
            xa[:, a:b] = new
            x[act] = xa
            per_block[act, i] = k
            done[act[same]] = True
            if k == b - a:
                done[act] = True
    return x, per_block.sum(axis=1).astype(np.int32), per_block, min_margin


def jacobi_gs_reference(model: MadeModel, noise: np.ndarray, block: int,
                        x_init: Optional[np.ndarray] = None, max_iters: Optional[int] = None):
    """Algorithm 2 (Jacobi-GS), tolerance 0, per-sample stopping.  Returns (x, iters[N], done[N], min_margin[N]).

    Iteration k: every block [a, b) -- all blocks "in parallel", i.e. all from the same s^{k-1} -- is walked
    through position by position: s_j^k = h_j(u, s^{k-1}_{1:a-1}, s^k_{a:j-1}).  So position j of block i is
    evaluated on the mixed vector (previous iterate before the block, current iterate inside it).  Stop at the
    first k with s^k == s^{k-1} or at k = M (number of blocks), where the result is exact (Proposition 2).
    """
    N, D = noise.shape[0], model.D
    parts = block_partition(D, block)
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
            mixed = prev.copy()                         # s^{k-1} everywhere ...
            for j in range(a, b):                       # ... except the block's earlier positions
                z_j = logits_at(model, mixed, j)
                mixed[:, j], margin = decide(z_j, _noise_at(noise[act], j), model.C)
                min_margin[act] = np.minimum(min_margin[act], margin)
            new[:, a:b] = mixed[:, a:b]
        same = (new == prev).all(axis=1)
        x[act] = new
        iters[act] = k
        done[act[same]] = True
        if k == M:
            done[act] = True
    return x, iters, done, min_margin


# --------------------------------------------------------------------------------------
# The joint distribution by enumeration (chain rule, Appendix A.3)
# --------------------------------------------------------------------------------------

def conditional_probs(z: np.ndarray, C: int) -> np.ndarray:
    """p(x_t = v | x_{<t}) for v = 0..max(C,2)-1 from logits z[..., C]."""
    if C == 1:
        p1 = 1.0 / (1.0 + np.exp(-z[..., 0]))
        return np.stack([1.0 - p1, p1], axis=-1)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def joint_bruteforce(model: MadeModel) -> Tuple[np.ndarray, np.ndarray]:
    """All V^D states (V = 2 or C) as rows of `states`, and p(state) = prod_t p(x_t | x_{<t})."""
    V = 2 if model.C == 1 else model.C
    D = model.D
    assert V ** D <= 1 << 22, "enumeration is for tiny models"
    idx = np.arange(V ** D)
    states = np.stack([(idx // V ** (D - 1 - t)) % V for t in range(D)], axis=1).astype(np.uint8)
    z = logits_all(model, states)
    p = conditional_probs(z, model.C)                   # [S, D, V]
    chosen = np.take_along_axis(p, states[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    return states, chosen.prod(axis=1)
