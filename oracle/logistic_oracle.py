"""Plain CPU oracle for a MADE with continuous states and logistic conditionals, and Jacobi iteration with a
forward-difference tolerance.

TEST INFRASTRUCTURE ONLY (see made_oracle.py for the rules; nothing in the product path imports this).

The paper's own MADE experiment models every conditional with a logistic distribution (Appendix C.3) and stops
the iteration when the forward difference is below a tolerance eps (Algorithm 1; Sections 2.2 and 4.2).
States are reals: s_t = h_t(u, s_{1:t-1}) = mu_t + scale_t * l_t, the inverse-CDF draw of Appendix A.3, where
l_t = log(u_t / (1 - u_t)) is a standard logistic variate (passed in as the fixed noise) and (mu_t, a_t) are the
two outputs the masked network produces for position t from s_{1:t-1}.

Readings (the paper fixes none of them):
  * the network is the masked MLP of made_oracle with C = 2 output rows per position (row 2t = mu_t, row 2t+1 =
    a_t), same masks; a real state enters the network as itself (rounded to bf16 in bf16 mode, like every other
    activation the GPU stores in bf16);
  * scale_t = exp(clip(a_t, A_LO, A_HI));
  * forward difference = max-norm over the positions of one sample; a sample stops at the first k with
    |s^k - s^{k-1}|_inf <= eps, or at k = T.  With eps = 0 the result is the feedforward result (Proposition 1;
    in floating point: up to the rounding differences between two evaluation orders of the same sums).
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from .made_oracle import MadeModel, affine, round_to_bf16

A_LO, A_HI = -6.0, 3.0


def hidden_real(model: MadeModel, x: np.ndarray) -> np.ndarray:
    h = np.asarray(x, dtype=np.float64)
    if model.act_round == "bf16":
        h = round_to_bf16(h)
    for WM, b in zip(model.WM[:-1], model.b[:-1]):
        h = np.maximum(affine(h, WM, b), 0.0)
        if model.act_round == "bf16":
            h = round_to_bf16(h)
    return h


def params_all(model: MadeModel, x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(mu, a), each [N, D], of every position from one pass over the network."""
    assert model.C == 2
    z = affine(hidden_real(model, x), model.WM[-1], model.b[-1]).reshape(x.shape[0], model.D, 2)
    return z[:, :, 0], z[:, :, 1]


def params_at(model: MadeModel, x: np.ndarray, t: int) -> Tuple[np.ndarray, np.ndarray]:
    h = hidden_real(model, x)
    z = affine(h, model.WM[-1][2 * t:2 * t + 2], model.b[-1][2 * t:2 * t + 2])
    return z[:, 0], z[:, 1]


def draw(mu: np.ndarray, a: np.ndarray, l: np.ndarray) -> np.ndarray:
    """Inverse-CDF draw of Logistic(mu, scale) from the standard logistic variate l."""
    return mu + np.exp(np.clip(a, A_LO, A_HI)) * np.asarray(l, dtype=np.float64)


def sequential_sample_real(model: MadeModel, l: np.ndarray) -> np.ndarray:
    """Eq. 1: one position after the other."""
    N, D = l.shape
    x = np.zeros((N, D))
    for t in range(D):
        mu, a = params_at(model, x, t)
        x[:, t] = draw(mu, a, l[:, t])
    return x


def jacobi_pass_real(model: MadeModel, x: np.ndarray, l: np.ndarray) -> np.ndarray:
    mu, a = params_all(model, x)
    return draw(mu, a, l)


def jacobi_reference_real(model: MadeModel, l: np.ndarray, eps: float, x_init: Optional[np.ndarray] = None,
                          max_iters: Optional[int] = None, record: bool = False):
    """Algorithm 1 with tolerance eps, per-sample stopping.  Returns (x, iters[N], done[N], trajectory or None)."""
    N, D = l.shape
    cap = D if (max_iters is None or max_iters <= 0) else min(max_iters, D)
    x = np.zeros((N, D)) if x_init is None else np.array(x_init, dtype=np.float64)
    iters = np.zeros(N, dtype=np.int32)
    done = np.zeros(N, dtype=bool)
    traj = [x.copy()] if record else None
    k = 0
    while not done.all() and k < cap:
        k += 1
        act = np.flatnonzero(~done)
        new = jacobi_pass_real(model, x[act], l[act])
        small = np.abs(new - x[act]).max(axis=1) <= eps
        x[act] = new
        iters[act] = k
        done[act[small]] = True
        if k == D:
            done[act] = True
        if record:
            traj.append(x.copy())
    return x, iters, done, traj
