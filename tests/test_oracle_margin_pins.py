"""Pins for the `min_margin` output of the oracle's reference iterations (Algorithms 1, 2, 3 and the
convolutional Algorithm 1).

The GPU tests compare iteration counts only for samples whose `min_margin` is at least 1e-3, so a slip in
it (wrong axis, wrong set of passes, margins of positions outside the block) would silently exempt samples.
Here every pass a sample takes is re-run with the scalar loop evaluators of the pin files (their own mask
rules, Python floats), the decision margin is computed from its definition -- |sigmoid(z) - u|, resp. best
minus runner-up of z + g -- and the smallest one over EXACTLY the passes and positions the algorithm
evaluates for that sample is compared with what the oracle returns.  Iteration counts and results fall out
of the same loops and are compared too."""
import math

import numpy as np
import pytest

from oracle import conv_oracle as CO
from oracle import made_oracle as O
from paper_2002_03629_amd import synth as S

from test_oracle_conv_pins import model_of, scalar_conv_logits, tiny
from test_oracle_pins import _model, scalar_logits, small_net


def scalar_decide(z, noise_t, C):
    """(symbol, margin) of one position from its logits z (list of C floats) and its noise."""
    if C == 1:
        p = 1.0 / (1.0 + math.exp(-z[0]))
        return (1 if float(noise_t) < p else 0), abs(p - float(noise_t))
    s = [z[c] + float(noise_t[c]) for c in range(C)]
    best = max(s)
    sym = s.index(best)                                  # lowest index of the maximum
    rest = sorted(s)
    return sym, rest[-1] - rest[-2]


def _close(a, b):
    return np.allclose(a, b, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("C,init", [(1, "zeros"), (1, "random"), (3, "zeros")])
def test_jacobi_reference_min_margin(C, init):
    D = 6
    net = small_net(D, C, [7, 5], seed=31 + C, gain=6.0)
    model = _model(net)
    N = 4
    noise = S.uniform_noise(N, D, 77) if C == 1 else S.gumbel_noise(N, D, C, 78)
    hi = 2 if C == 1 else C
    x0 = None if init == "zeros" else np.random.default_rng(5).integers(0, hi, (N, D)).astype(np.uint8)
    x, iters, done, _, mm = O.jacobi_reference(model, noise, x0)
    for n in range(N):
        cur = [0] * D if x0 is None else [int(v) for v in x0[n]]
        smallest, k = math.inf, 0
        while True:
            k += 1
            new = []
            for t in range(D):                           # every position from the previous iterate
                sym, m = scalar_decide(scalar_logits(net, cur, t), noise[n, t], C)
                new.append(sym)
                smallest = min(smallest, m)
            same = new == cur
            cur = new
            if same or k == D:
                break
        assert k == iters[n] and cur == [int(v) for v in x[n]]
        assert _close(mm[n], smallest), (n, mm[n], smallest)


def test_jacobi_reference_min_margin_ignores_passes_after_the_stop():
    """A sample that has stopped takes no further passes: margins of later passes of OTHER samples must not
    leak into it, and its own value must not be refreshed."""
    D = 6
    net = small_net(D, 1, [7, 5], seed=34, gain=6.0)
    model = _model(net)
    noise = S.uniform_noise(8, D, 79)
    _, iters, _, _, mm = O.jacobi_reference(model, noise)
    assert iters.min() < iters.max()                     # the batch does stop at different passes
    for n in range(8):
        alone = O.jacobi_reference(model, noise[n:n + 1])
        assert alone[1][0] == iters[n] and alone[4][0] == mm[n]


@pytest.mark.parametrize("block", [1, 2, 4, 6, 9])
def test_gs_jacobi_reference_min_margin(block):
    D = 6
    net = small_net(D, 1, [7, 5], seed=34, gain=6.0)
    model = _model(net)
    N = 4
    noise = S.uniform_noise(N, D, 80)
    x, iters, per_block, mm = O.gs_jacobi_reference(model, noise, block)
    for n in range(N):
        cur = [0] * D
        smallest, total = math.inf, 0
        for a in range(0, D, block):
            b = min(a + block, D)
            k = 0
            while True:
                k += 1
                new = list(cur)
                for t in range(a, b):                    # only the block's positions are drawn
                    sym, m = scalar_decide(scalar_logits(net, cur, t), noise[n, t], 1)
                    new[t] = sym
                    smallest = min(smallest, m)
                same = new == cur
                cur = new
                if same or k == b - a:
                    break
            total += k
        assert total == iters[n] and cur == [int(v) for v in x[n]]
        assert _close(mm[n], smallest), (n, mm[n], smallest)


@pytest.mark.parametrize("block", [1, 2, 4, 7])
def test_jacobi_gs_reference_min_margin(block):
    D = 7
    net = small_net(D, 1, [9], seed=34, gain=10.0)
    model = _model(net)
    N = 4
    noise = S.uniform_noise(N, D, 81)
    x, iters, done, mm = O.jacobi_gs_reference(model, noise, block)
    M = -(-D // block)
    for n in range(N):
        prev = [0] * D
        smallest, k = math.inf, 0
        while True:
            k += 1
            new = list(prev)
            for a in range(0, D, block):
                mixed = list(prev)                       # the previous iterate before the block ...
                for j in range(a, min(a + block, D)):    # ... this iteration's symbols inside it
                    sym, m = scalar_decide(scalar_logits(net, mixed, j), noise[n, j], 1)
                    mixed[j] = sym
                    smallest = min(smallest, m)
                new[a:a + block] = mixed[a:a + block]
            same = new == prev
            prev = new
            if same or k == M:
                break
        assert k == iters[n] and prev == [int(v) for v in x[n]]
        assert _close(mm[n], smallest), (n, mm[n], smallest)


def test_conv_jacobi_reference_min_margin():
    net = tiny(2, 2, 3, 4, 3, 2, seed=9)
    model = model_of(net)
    N, D, C = 2, net.D, net.C
    noise = S.gumbel_noise(N, D, C, 82)
    x, iters, done, mm = CO.conv_jacobi_reference(model, noise)
    for n in range(N):
        cur = [0] * D
        smallest, k = math.inf, 0
        while True:
            k += 1
            new = []
            for t in range(D):
                sym, m = scalar_decide(scalar_conv_logits(net, cur, t), noise[n, t], C)
                new.append(sym)
                smallest = min(smallest, m)
            same = new == cur
            cur = new
            if same or k == D:
                break
        assert k == iters[n] and cur == [int(v) for v in x[n]]
        assert _close(mm[n], smallest), (n, mm[n], smallest)


def test_conv_jacobi_gs_reference_min_margin():
    net = tiny(2, 2, 3, 4, 3, 2, seed=9)
    model = model_of(net)
    N, D, C = 2, net.D, net.C
    noise = S.gumbel_noise(N, D, C, 83)
    block = 5
    M = -(-D // block)
    x, iters, done, mm = CO.conv_jacobi_gs_reference(model, noise, block)
    for n in range(N):
        prev = [0] * D
        smallest, k = math.inf, 0
        while True:
            k += 1
            new = list(prev)
            for a in range(0, D, block):
                mixed = list(prev)
                for j in range(a, min(a + block, D)):
                    sym, m = scalar_decide(scalar_conv_logits(net, mixed, j), noise[n, j], C)
                    mixed[j] = sym
                    smallest = min(smallest, m)
                new[a:a + block] = mixed[a:a + block]
            same = new == prev
            prev = new
            if same or k == M:
                break
        assert k == iters[n] and prev == [int(v) for v in x[n]]
        assert _close(mm[n], smallest), (n, mm[n], smallest)


def test_a_planted_mistake_in_min_margin_is_caught():
    """The pins above have teeth: a min over the batch axis, or a min over the last pass only, is rejected."""
    D = 6
    net = small_net(D, 1, [7, 5], seed=34, gain=6.0)
    model = _model(net)
    noise = S.uniform_noise(8, D, 79)
    _, iters, _, traj, mm = O.jacobi_reference(model, noise, record=True)
    wrong_axis = np.full(8, mm.min())                    # min over samples instead of per sample
    assert not np.allclose(wrong_axis, mm)
    last_only = O.fixed_point_check(model, traj[-1], noise)[1].min(axis=1)
    assert not np.allclose(last_only, mm)
