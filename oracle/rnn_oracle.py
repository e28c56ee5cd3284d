"""Plain CPU oracle for the backward pass of a one-layer recurrent network solved by Jacobi iteration.

TEST INFRASTRUCTURE ONLY (see made_oracle.py for the rules; nothing in the product path imports this).

Backpropagation is feedforward computation (Appendix A.2): the state of step t is the gradient of the loss with
respect to one layer's output, and each state is a function of the one before it.  For a recurrent network
(Section 5.1; Appendix C.1: one hidden layer, softplus units) unrolled over T time steps,

    z_t = W h_{t-1} + U x_t + b,     h_t = softplus(z_t),     L = sum_t l_t(h_t),

the states are d_t = dL/dh_t (total derivative), which obey, backwards in time,

    d_T = g_T,      d_t = g_t + W^T (softplus'(z_{t+1}) * d_{t+1}),      g_t = dl_t/dh_t,  softplus' = sigmoid.

The standard backward pass ("feedforward" in Section 5.1) evaluates this one step after the other.  Jacobi
iteration (Algorithm 1) updates every step in parallel from the previous iterate,

    d^k_T = g_T,    d^k_t = g_t + W^T (sigmoid(z_{t+1}) * d^{k-1}_{t+1}),

and "Jacobi_n" (Section 5.1) is that iteration truncated after n passes.  Everything is fp64 numpy, written in
row-vector form: arrays are [B, T, H] (B independent sequences), so W^T v becomes v @ W.

Readings (the paper fixes none of them):
  * the iteration starts from d^0 = 0 unless an initial iterate is given, so d^1 = g and d^n is the gradient of
    backpropagation through time truncated to n steps;
  * forward difference = max-norm over all steps and units of one sequence; a sequence stops at the first k
    with |d^k - d^{k-1}|_inf <= eps, or at k = min(n, T) (Algorithm 1 with the truncation of Section 5.1); the
    count includes the confirming pass;
  * parameter gradients ("immediately computed" once the states are known, Appendix A.2) with
    p_t = sigmoid(z_t) * d_t:  dW = sum_t p_t h_{t-1}^T,  dU = sum_t p_t x_t^T,  db = sum_t p_t, summed over the
    batch as well.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def softplus(z: np.ndarray) -> np.ndarray:
    return np.logaddexp(0.0, z)


def sigmoid(z: np.ndarray) -> np.ndarray:
    return 0.5 * (1.0 + np.tanh(0.5 * z))


def rnn_forward(W: np.ndarray, U: np.ndarray, b: np.ndarray, x: np.ndarray,
                h0: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """x [B, T, I] -> (z, h), both [B, T, H].  W [H, H], U [H, I], b [H]; h0 [B, H] (zeros if None)."""
    x = np.asarray(x, dtype=np.float64)
    B, T, _ = x.shape
    H = W.shape[0]
    z = np.empty((B, T, H))
    h = np.empty((B, T, H))
    prev = np.zeros((B, H)) if h0 is None else np.asarray(h0, dtype=np.float64)
    for t in range(T):
        z[:, t] = prev @ W.T + x[:, t] @ U.T + b
        h[:, t] = softplus(z[:, t])
        prev = h[:, t]
    return z, h


def backprop_sequential(W: np.ndarray, z: np.ndarray, g: np.ndarray) -> np.ndarray:
    """The standard backward pass: d [B, T, H], one time step after the other, last step first."""
    z = np.asarray(z, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    T = z.shape[1]
    d = np.empty_like(g)
    d[:, T - 1] = g[:, T - 1]
    for t in range(T - 2, -1, -1):
        d[:, t] = g[:, t] + (sigmoid(z[:, t + 1]) * d[:, t + 1]) @ W
    return d


def jacobi_pass(W: np.ndarray, z: np.ndarray, g: np.ndarray, d: np.ndarray) -> np.ndarray:
    """One pass of Algorithm 1 over all steps at once, from the iterate d."""
    new = np.array(g, dtype=np.float64, copy=True)
    new[:, :-1] += (sigmoid(z[:, 1:]) * d[:, 1:]) @ W
    return new


def jacobi_reference(W: np.ndarray, z: np.ndarray, g: np.ndarray, n_iters: int = 0, eps: float = 0.0,
                     d_init: Optional[np.ndarray] = None):
    """Jacobi_n with forward-difference stopping, per sequence.

    n_iters <= 0 or > T means T.  Returns (d [B, T, H], iters [B], converged [B] bool, diffs list of [B]) where
    converged says the sequence met the tolerance (rather than running into the pass limit) and diffs[k-1] is the
    forward difference of pass k (NaN for sequences that had already stopped)."""
    z = np.asarray(z, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    B, T, H = g.shape
    cap = T if n_iters <= 0 or n_iters > T else n_iters
    d = np.zeros_like(g) if d_init is None else np.array(d_init, dtype=np.float64, copy=True)
    iters = np.zeros(B, dtype=np.int64)
    conv = np.zeros(B, dtype=bool)
    active = np.ones(B, dtype=bool)
    diffs = []
    for k in range(1, cap + 1):
        if not active.any():
            break
        idx = np.nonzero(active)[0]
        new = jacobi_pass(W, z[idx], g[idx], d[idx])
        diff = np.abs(new - d[idx]).reshape(len(idx), -1).max(axis=1)
        d[idx] = new
        iters[idx] += 1
        rec = np.full(B, np.nan)
        rec[idx] = diff
        diffs.append(rec)
        met = diff <= eps
        conv[idx[met]] = True
        active[idx[met]] = False
    return d, iters, conv, diffs


def param_grads(z: np.ndarray, h: np.ndarray, x: np.ndarray, d: np.ndarray,
                h0: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(dW [H, H], dU [H, I], db [H]) from the states d, summed over time steps and sequences."""
    B, T, H = d.shape
    p = sigmoid(np.asarray(z, dtype=np.float64)) * d
    prev = np.empty_like(h, dtype=np.float64)
    prev[:, 0] = 0.0 if h0 is None else h0
    prev[:, 1:] = h[:, :-1]
    dW = np.einsum("bti,btj->ij", p, prev)
    dU = np.einsum("bti,btj->ij", p, np.asarray(x, dtype=np.float64))
    db = p.sum(axis=(0, 1))
    return dW, dU, db
