"""CPU pins of the continuous-state (logistic conditionals) oracle against facts that do not come from it."""
import math

import numpy as np
import pytest
from scipy import stats

from oracle import logistic_oracle as L
from oracle import made_oracle as O
from paper_2002_03629_amd import synth as S


def _model(net, act_round=None):
    return O.build_model(net.D, net.C, net.degrees, net.W, net.b, act_round)


def scalar_params(net, x, t):
    """(mu_t, a_t) of one sample straight from the definition of the masked MLP (Python loops, real inputs):
    a unit of degree m reads units of degree <= m; output rows 2t, 2t+1 read last-layer units of degree < t+1."""
    prev_deg = list(range(1, net.D + 1))
    h = [float(v) for v in x]
    for l, deg in enumerate(net.degrees):
        W, b = net.W[l], net.b[l]
        nh = []
        for j in range(len(deg)):
            acc = 0.0 if b is None else float(b[j])
            for i in range(len(h)):
                if int(deg[j]) >= prev_deg[i]:
                    acc += float(W[j, i]) * h[i]
            nh.append(max(acc, 0.0))
        h, prev_deg = nh, [int(d) for d in deg]
    W, b = net.W[-1], net.b[-1]
    out = []
    for c in range(2):
        r = 2 * t + c
        acc = 0.0 if b is None else float(b[r])
        for i in range(len(h)):
            if (t + 1) > prev_deg[i]:
                acc += float(W[r, i]) * h[i]
        out.append(acc)
    return out


def small_net(D, hidden, seed, gain=1.5):
    w = S.Workload("t", D, 2, hidden, "f32", 4, "random", "fan_in", seed, gain, real=True)
    return S.make_network(w, with_bias=True)


def test_params_match_scalar_definition():
    net = small_net(9, [13, 11], seed=5)
    model = _model(net)
    x = np.random.default_rng(1).normal(size=(3, 9)) * 2.0
    mu, a = L.params_all(model, x)
    for n in range(3):
        for t in range(9):
            m_ref, a_ref = scalar_params(net, x[n], t)
            assert abs(mu[n, t] - m_ref) < 1e-9 and abs(a[n, t] - a_ref) < 1e-9
            mt, at = L.params_at(model, x[n:n + 1], t)
            assert abs(mt[0] - m_ref) < 1e-9 and abs(at[0] - a_ref) < 1e-9


def test_autoregressive_property():
    net = small_net(12, [20], seed=7, gain=3.0)
    model = _model(net)
    x = np.random.default_rng(2).normal(size=(4, 12))
    mu0, a0 = L.params_all(model, x)
    seen = 0
    for s in range(12):
        y = x.copy()
        y[:, s] += 1.7
        mu1, a1 = L.params_all(model, y)
        assert (mu1[:, :s + 1] == mu0[:, :s + 1]).all() and (a1[:, :s + 1] == a0[:, :s + 1]).all()
        seen += int((mu1[:, s + 1:] != mu0[:, s + 1:]).any())
    assert seen >= 8          # later positions do depend on earlier ones


def test_draw_is_the_logistic_inverse_cdf():
    """x = mu + s * log(u / (1-u)) has CDF 1 / (1 + exp(-(x - mu) / s)); the scale is exp(a) inside the clip."""
    u = np.array([0.1, 0.5, 0.9])
    l = np.log(u / (1 - u))
    x = L.draw(np.full(3, 0.7), np.full(3, math.log(2.0)), l)
    assert np.allclose(1.0 / (1.0 + np.exp(-(x - 0.7) / 2.0)), u)
    assert np.allclose(L.draw(np.zeros(2), np.array([-50.0, 50.0]), np.ones(2)), [math.exp(L.A_LO), math.exp(L.A_HI)])


def test_sequential_sampler_distribution():
    """Position 1 is Logistic(b_mu, exp(b_a)); position 2 given position 1, standardised with the SCALAR
    evaluator's parameters, is standard logistic (Kolmogorov-Smirnov against scipy's distribution)."""
    net = small_net(4, [8], seed=3, gain=3.0)
    model = _model(net)
    l = S.logistic_noise(20000, 4, 99)
    x = L.sequential_sample_real(model, l)
    b = net.b[-1]
    p1 = stats.kstest(x[:, 0], stats.logistic(loc=float(b[0]), scale=math.exp(float(b[1]))).cdf).pvalue
    assert p1 > 1e-3
    z = np.empty(400)
    for n in range(400):
        m2, a2 = scalar_params(net, x[n], 1)
        z[n] = (x[n, 1] - m2) / math.exp(min(max(a2, L.A_LO), L.A_HI))
    assert stats.kstest(z, stats.logistic().cdf).pvalue > 1e-3
    # and a wrong scale reading (e.g. a used directly) is rejected by the same test
    assert stats.kstest(x[:, 0], stats.logistic(loc=float(b[0]), scale=abs(float(b[1])) + 1e-3).cdf).pvalue < 1e-3


@pytest.mark.parametrize("name", ["small_real_f32", "small_real_bf16"])
def test_jacobi_eps0_is_the_feedforward_result(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    model = _model(net, "bf16" if w.dtype == "bf16" else None)
    l = S.make_noise(w)
    xs = L.sequential_sample_real(model, l)
    x, iters, done, traj = L.jacobi_reference_real(model, l, 0.0, record=True)
    tol = 1e-9 if w.dtype == "f32" else 1e-6     # (bf16 mode: a rounding boundary can amplify a 1e-16 difference)
    assert np.abs(x - xs).max() <= tol and done.all() and (iters <= w.D).all()
    # Proposition 1's invariant: after k iterations the first k positions are final
    for k in (1, 2, 5):
        assert np.abs(traj[k][:, :k] - xs[:, :k]).max() <= tol
    # any initial guess
    init = np.random.default_rng(4).normal(size=xs.shape) * 3.0
    assert np.abs(L.jacobi_reference_real(model, l, 0.0, init)[0] - xs).max() <= tol


def test_tolerance_trades_iterations_for_error():
    w = S.workload("small_real_f32")
    net = S.make_network(w, with_bias=True)
    model = _model(net)
    l = S.make_noise(w)
    xs = L.sequential_sample_real(model, l)
    prev_iters, errs = None, []
    for eps in (1e-1, 1e-3, 1e-6, 0.0):
        x, iters, done, traj = L.jacobi_reference_real(model, l, eps, record=True)
        assert done.all()
        # the stopping rule itself: the last step of every sample moved it by at most eps
        for n in range(w.N):
            k = iters[n]
            assert np.abs(traj[k][n] - traj[k - 1][n]).max() <= eps or k == w.D
            if k > 1 and eps > 0:
                assert np.abs(traj[k - 1][n] - traj[k - 2][n]).max() > eps
        if prev_iters is not None:
            assert (iters >= prev_iters).all()        # a tighter tolerance never stops earlier
        prev_iters = iters
        errs.append(np.abs(x - xs).max())
    assert errs[-1] <= 1e-9 and errs[0] >= errs[-1]
