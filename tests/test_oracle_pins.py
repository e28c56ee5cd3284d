"""Pins for the CPU oracle: everything here runs without a GPU and compares the oracle with
things that are *not* the oracle: hand-written masks, closed forms, a scalar by-definition
evaluator written with Python loops, the iteration counts the paper prints for its worked
examples (Section 4.1), the propositions' guarantees, and brute-force enumeration."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
from scipy import stats

from oracle import made_oracle as O
from paper_2002_03629_amd import synth as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _model(net, act_round=None):
    return O.build_model(net.D, net.C, net.degrees, net.W, net.b, act_round, net.onehot)


# ------------------------------------------------------------------ a scalar evaluator
def scalar_logits(net, x, t):
    """Logits of position t (0-based) of one sample, straight from the definition of a masked
    MLP, with Python loops and no shared code with the oracle.  Connections are allowed when
    degree(out) >= degree(in) between hidden layers / from the inputs, and when
    t+1 > degree(in) for the output layer."""
    C = net.C
    prev_deg = list(range(1, net.D + 1))
    h = [float(v) if C == 1 else (float(v) - 128.0) / 128.0 for v in x]
    if net.onehot:      # input t*C + c is the indicator of x_t = c and carries the degree of position t
        prev_deg = [d for d in range(1, net.D + 1) for _ in range(C)]
        h = [1.0 if int(x[i // C]) == i % C else 0.0 for i in range(net.D * C)]
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
    for c in range(C):
        r = t * C + c
        acc = 0.0 if b is None else float(b[r])
        for i in range(len(h)):
            if (t + 1) > prev_deg[i]:
                acc += float(W[r, i]) * h[i]
        out.append(acc)
    return out


def small_net(D, C, hidden, seed, gain=3.0, bias=True, rule="random", onehot=False):
    w = S.Workload("t", D, C, hidden, "f32", 4, rule, "fan_in", seed, gain, onehot=onehot)
    return S.make_network(w, with_bias=bias)


# ------------------------------------------------------------------ masks
def test_masks_hand_example():
    # D = 3, hidden degrees [1, 2, 2], second hidden layer degrees [2, 1]; written out by hand.
    masks = O.masks_from_degrees(3, 1, [np.array([1, 2, 2]), np.array([2, 1])])
    m1 = np.array([[1, 0, 0], [1, 1, 0], [1, 1, 0]], bool)          # unit degree >= input position
    m2 = np.array([[1, 1, 1], [1, 0, 0]], bool)                     # degree >= previous degree
    mv = np.array([[0, 0], [0, 1], [1, 1]], bool)                   # position t > degree (strict)
    assert (masks[0] == m1).all() and (masks[1] == m2).all() and (masks[2] == mv).all()


def test_masks_categorical_rows_grouped_by_position():
    masks = O.masks_from_degrees(3, 2, [np.array([1, 2])])
    mv = np.array([[0, 0], [0, 0], [1, 0], [1, 0], [1, 1], [1, 1]], bool)
    assert (masks[1] == mv).all()


@pytest.mark.parametrize("C", [1, 4])
def test_logits_match_scalar_definition(C):
    net = small_net(6, C, [7, 5], seed=5 + C)
    model = _model(net)
    rng = np.random.default_rng(0)
    x = rng.integers(0, 2 if C == 1 else 256, size=(3, 6)).astype(np.uint8)
    z = O.logits_all(model, x)
    for n in range(3):
        for t in range(6):
            ref = scalar_logits(net, x[n], t)
            assert np.allclose(z[n, t], ref, rtol=1e-12, atol=1e-12)
            assert np.allclose(O.logits_at(model, x[n:n + 1], t)[0], ref, rtol=1e-12, atol=1e-12)


def test_logits_closed_form_all_ones():
    # One hidden layer, all weights 1, hidden bias 0.5, output bias -2, input all ones:
    # h_k = m(k) + 0.5 (it sees inputs 1..m(k)); z_t = sum_{k: m(k) < t} (m(k) + 0.5) - 2.
    D, H = 9, 14
    deg = S.hidden_degrees("random", D, [H], 3)
    W = [np.ones((H, D), np.float32), np.ones((D, H), np.float32)]
    b = [np.full(H, 0.5, np.float32), np.full(D, -2.0, np.float32)]
    model = O.build_model(D, 1, deg, W, b)
    z = O.logits_all(model, np.ones((1, D), np.uint8))[0, :, 0]
    m = deg[0]
    for t in range(1, D + 1):
        assert z[t - 1] == pytest.approx(sum(mk + 0.5 for mk in m if mk < t) - 2.0, abs=1e-12)


@pytest.mark.parametrize("C", [1, 3])
def test_autoregressive_property(C):
    net = small_net(8, C, [20, 16], seed=21 + C, rule="cyclic")   # every degree occurs in every layer
    model = _model(net)
    rng = np.random.default_rng(1)
    hi = 2 if C == 1 else 256
    x = rng.integers(0, hi, size=(5, 8)).astype(np.uint8)
    z = O.logits_all(model, x)
    seen = 0
    for t in range(8):
        y = x.copy()
        y[:, t:] = rng.integers(0, hi, size=(5, 8 - t))
        assert (O.logits_all(model, y)[:, t] == z[:, t]).all()       # exactly unchanged
        if t > 0:                                                    # and it does see x_{t-1}
            y = x.copy()
            y[:, t - 1] = ((y[:, t - 1].astype(np.int64) + 1) % hi).astype(np.uint8)
            seen += bool((O.logits_all(model, y)[:, t] != z[:, t]).any())
    assert seen >= 4                   # (a dead ReLU path may hide the link for a few t)


def test_first_position_is_bias_only():
    net = small_net(5, 1, [9], seed=2)
    z = O.logits_all(_model(net), np.ones((1, 5), np.uint8))
    assert z[0, 0, 0] == pytest.approx(float(net.b[-1][0]))


# ------------------------------------------------------------------ decisions
def test_decide_bernoulli_rule_and_margin():
    z = np.array([[0.0], [2.0], [-2.0]])
    u = np.array([0.5, 0.88, 0.1])
    x, margin = O.decide(z, u, 1)
    # sigmoid(0) = .5 -> u < p fails (strict); sigmoid(2) = .8808 -> .88 < p; sigmoid(-2) = .1192 -> .1 < p
    assert x.tolist() == [0, 1, 1]
    assert margin == pytest.approx([0.0, 1 / (1 + math.exp(-2)) - 0.88, 1 / (1 + math.exp(2)) - 0.1])


def test_decide_categorical_tie_and_margin():
    z = np.array([[1.0, 3.0, 3.0, 0.0]])
    g = np.array([[0.0, 0.0, 0.0, 0.5]])
    x, margin = O.decide(z, g, 4)
    assert x.tolist() == [1] and margin[0] == 0.0                    # lowest index wins a tie
    x, margin = O.decide(z, np.array([[0.0, 0.0, 0.25, 0.0]]), 4)
    assert x.tolist() == [2] and margin[0] == pytest.approx(0.25)


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_exhaustive_roundtrip_and_ties():
    pats = np.arange(1 << 16, dtype=np.uint32) << 16
    vals = pats.view(np.float32)
    finite = np.isfinite(vals)
    assert (O.round_to_bf16(vals[finite]) == vals[finite].astype(np.float64)).all()
    # 1 + 2^-8 is exactly between 1 and 1 + 2^-7: ties go to the even significand (1.0)
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert O.round_to_bf16(np.array([-(1.0 + 2.0 ** -8 + 2.0 ** -20)]))[0] == -(1.0 + 2.0 ** -7)


def test_bf16_against_torch_conversion():
    a = np.random.default_rng(3).standard_normal(200000).astype(np.float32) * 37.0
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert (O.round_to_bf16(a) == ref.astype(np.float64)).all()
    assert (S.bf16_representable(a) == ref).all()


# ------------------------------------------------------------------ distribution (chain rule)
def brute_joint(net):
    """p(x) = prod_t p(x_t | x_{<t}) with the scalar evaluator; tiny models only."""
    V = 2 if net.C == 1 else net.C
    out = {}
    for state in itertools.product(range(V), repeat=net.D):
        p = 1.0
        for t in range(net.D):
            z = scalar_logits(net, state, t)
            if net.C == 1:
                p1 = 1.0 / (1.0 + math.exp(-z[0]))
                p *= p1 if state[t] == 1 else 1.0 - p1
            else:
                mx = max(z)
                e = [math.exp(v - mx) for v in z]
                p *= e[state[t]] / sum(e)
        out[state] = p
    return out


def test_joint_sums_to_one_and_matches_scalar_enumeration():
    net = small_net(5, 1, [8, 6], seed=31)
    states, p = O.joint_bruteforce(_model(net))
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    ref = brute_joint(net)
    for s, ps in zip(states, p):
        assert ps == pytest.approx(ref[tuple(int(v) for v in s)], rel=1e-10)


def test_leaky_mask_breaks_normalisation():
    # The normalisation pin has teeth: let position t read itself and the "joint" no longer sums to 1.
    net = small_net(5, 1, [8], seed=32)
    model = _model(net)
    leaky = O.build_model(net.D, 1, net.degrees, net.W, net.b)
    leaky.WM[-1] = np.where(O.masks_from_degrees(net.D, 1, net.degrees)[-1] | (
        np.arange(1, 6)[:, None] >= net.degrees[0][None, :]), net.W[-1].astype(np.float64), 0.0)
    assert abs(O.joint_bruteforce(leaky)[1].sum() - 1.0) > 1e-4
    assert O.joint_bruteforce(model)[1].sum() == pytest.approx(1.0, abs=1e-12)


def _chi2(counts, probs):
    exp = probs * counts.sum()
    keep = exp > 5
    chi = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum() + \
        (counts[~keep].sum() - exp[~keep].sum()) ** 2 / max(exp[~keep].sum(), 1e-9) * (exp[~keep].sum() > 5)
    dof = int(keep.sum()) - (0 if (~keep).any() and exp[~keep].sum() > 5 else 1)
    return stats.chi2.sf(chi, max(dof, 1))


def test_sequential_sampler_distribution_bernoulli():
    D = 10
    net = small_net(D, 1, [24, 24], seed=41, gain=4.0)
    model = _model(net)
    states, p = O.joint_bruteforce(model)
    n = 200000
    x, _ = O.sequential_sample(model, S.uniform_noise(n, D, 777))
    code = (x.astype(np.int64) * (2 ** np.arange(D - 1, -1, -1))).sum(axis=1)
    counts = np.bincount(code, minlength=2 ** D).astype(np.float64)
    assert _chi2(counts, p) > 1e-3
    tv = 0.5 * np.abs(counts / n - p).sum()
    assert tv < 0.5 * np.sqrt(p * (1 - p) / n).sum() + 3 * 0.5 * np.sqrt((p * (1 - p) / n).sum())
    assert p.max() / p.min() > 50          # the model is far from uniform, so the test can see a flipped rule


def categorical_test_net():
    """D = 4, C = 3.  Symbols enter as (x - 128)/128, so neighbouring symbols differ by 1/128 at
    the input; the first layer is scaled up (and its bias recentred on the visible inputs) so
    that later positions really depend on earlier symbols."""
    D, C = 4, 3
    net = small_net(D, C, [12], seed=43, gain=1.0, rule="cyclic")
    vis = net.degrees[0][:, None] >= np.arange(1, D + 1)[None, :]
    net.W[0] = (net.W[0] * 256.0).astype(np.float32)
    net.b[0] = ((net.W[0] * vis).sum(axis=1) + net.b[0]).astype(np.float32)
    return net


def test_sequential_sampler_distribution_gumbel_max():
    net = categorical_test_net()
    D, C = net.D, net.C
    model = _model(net)
    states, p = O.joint_bruteforce(model)
    ref = brute_joint(net)
    assert np.allclose(p, [ref[tuple(int(v) for v in s)] for s in states], rtol=1e-10)
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    # the conditional of the last position moves a lot with the prefix: dependence is exercised
    last = O.conditional_probs(O.logits_all(model, states), C)[:, D - 1, :]
    assert (last.max(axis=0) - last.min(axis=0)).max() > 0.2
    n = 200000
    x, _ = O.sequential_sample(model, S.gumbel_noise(n, D, C, 778))
    code = (x.astype(np.int64) * (C ** np.arange(D - 1, -1, -1))).sum(axis=1)
    counts = np.bincount(code, minlength=C ** D).astype(np.float64)
    assert _chi2(counts, p) > 1e-3
    assert p.max() / p.min() > 20


# ------------------------------------------------------------------ Proposition 1
@pytest.mark.parametrize("name", ["cfg1", "small_f32", "small_cat_f32"])
def test_jacobi_equals_sequential_any_init(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    model = _model(net)
    noise = S.make_noise(w)
    xs, _ = O.sequential_sample(model, noise)
    hi = 2 if w.C == 1 else w.C
    inits = [None, np.full((w.N, w.D), hi - 1, np.uint8),
             np.random.default_rng(0).integers(0, hi, (w.N, w.D)).astype(np.uint8), xs]
    for i, init in enumerate(inits):
        xj, iters, done, traj, _ = O.jacobi_reference(model, noise, init, record=True)
        assert (xj == xs).all() and done.all()
        assert (iters <= w.D).all() and (iters >= 1).all()
        # induction hypothesis in the proof of Prop. 1: after k passes the first k positions are final
        for k, sk in enumerate(traj):
            assert (sk[:, :k] == xs[:, :k]).all()
        if i == 3:
            assert (iters == 1).all()       # started at the solution: one confirming pass
    # the fixed-point certificate accepts the solution and rejects a corrupted one
    ok, _ = O.fixed_point_check(model, xs, noise)
    assert ok.all()
    bad = xs.copy()
    bad[:, 0] = ((bad[:, 0].astype(np.int64) + 1) % hi).astype(np.uint8)
    assert not O.fixed_point_check(model, bad, noise)[0].all()


def test_jacobi_max_iters_reports_unconverged():
    net = S.copy_chain_network(12)
    model = _model(net)
    u = S.uniform_noise(3, 12, 5) * 0.98 + 0.01
    x, iters, done, _, _ = O.jacobi_reference(model, u, None, max_iters=5)
    assert (iters == 5).all() and not done.any()
    assert (x[:, :5] == 1).all() and (x[:, 5:] == 0).all()


# ------------------------------------------------------------------ Section 4.1 examples
def _golden_examples():
    rows = {}
    with open(os.path.join(GOLDEN, "section4_1_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            rows[parts[0]] = parts[-1]
    return rows


def _first_exact(traj, xs):
    return [min(k for k, sk in enumerate(traj) if (sk[n] == xs[n]).all()) for n in range(xs.shape[0])]


def test_example1_independent_one_iteration():
    assert _golden_examples()["example1"] == "1"
    net = S.independent_network(20, 33, seed=9)
    model = _model(net)
    u = S.uniform_noise(6, 20, 1)
    xs, _ = O.sequential_sample(model, u)
    init = 1 - xs                                     # start everywhere wrong
    xj, iters, done, traj, _ = O.jacobi_reference(model, u, init, record=True)
    assert (xj == xs).all() and _first_exact(traj, xs) == [1] * 6
    assert (iters == 2).all()                         # one pass to reach it + one to confirm


def test_example2_skip_to_first_two_iterations():
    assert _golden_examples()["example2"] == "2"
    net = S.first_only_network(20, 40, seed=10)
    model = _model(net)
    u = S.uniform_noise(16, 20, 2)
    xs, _ = O.sequential_sample(model, u)
    assert (xs[:, 0] == 1).all()
    xj, iters, done, traj, _ = O.jacobi_reference(model, u, None, record=True)
    fe = _first_exact(traj, xs)
    assert (xj == xs).all() and max(fe) == 2 and (iters <= 3).all()
    assert (np.array(fe) + 1 == iters).all()


def test_example3_markov_chain_needs_T_iterations():
    assert _golden_examples()["example3"] == "T"
    T = 17
    net = S.copy_chain_network(T)
    model = _model(net)
    u = S.uniform_noise(4, T, 3) * 0.98 + 0.01
    xs, _ = O.sequential_sample(model, u)
    assert (xs == 1).all()
    xj, iters, done, traj, _ = O.jacobi_reference(model, u, None, record=True)
    assert (xj == xs).all() and (iters == T).all() and done.all()
    assert _first_exact(traj, xs) == [T] * 4
    for k in range(T + 1):                            # the 1 walks one position per pass
        assert (traj[k][:, :k] == 1).all() and (traj[k][:, k:] == 0).all()


@pytest.mark.parametrize("skip", [3, 5, 16])
def test_critical_path_bound(skip):
    D = 32
    net = S.skip_network(D, 64, skip, seed=11)
    model = _model(net)
    u = S.uniform_noise(32, D, 4)
    xs, _ = O.sequential_sample(model, u)
    xj, iters, done, traj, _ = O.jacobi_reference(model, u, 1 - xs, record=True)
    assert (xj == xs).all()
    assert max(_first_exact(traj, xs)) <= math.ceil(D / skip)


# ------------------------------------------------------------------ Proposition 2 / Algorithm 3
@pytest.mark.parametrize("name", ["cfg1", "small_f32", "small_cat_f32"])
def test_gs_jacobi_exact_for_every_block_size(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    model = _model(net)
    noise = S.make_noise(w)
    xs, _ = O.sequential_sample(model, noise)
    xj, it_j, _, _, _ = O.jacobi_reference(model, noise)
    for B in [1, 2, 7, 16, w.D - 1, w.D, w.D + 5]:
        xg, iters, per_block, _ = O.gs_jacobi_reference(model, noise, B)
        parts = O.block_partition(w.D, B)
        assert parts[0][0] == 0 and parts[-1][1] == w.D
        assert all(p[1] == q[0] for p, q in zip(parts, parts[1:]))
        assert (xg == xs).all()
        sizes = np.array([b - a for a, b in parts])
        assert (per_block <= sizes[None, :]).all() and (per_block >= 1).all()
        if B == 1:
            assert (iters == w.D).all()               # one GS sweep = feedforward computation
        if B >= w.D:
            assert (iters == it_j).all()              # a single block is Algorithm 1 itself
    # any initial guess gives the same answer
    init = np.random.default_rng(5).integers(0, 2 if w.C == 1 else w.C, (w.N, w.D)).astype(np.uint8)
    assert (O.gs_jacobi_reference(model, noise, 7, init)[0] == xs).all()


def test_gs_jacobi_chain_uses_block_size_iterations():
    T = 12
    model = _model(S.copy_chain_network(T))
    u = S.uniform_noise(2, T, 3) * 0.98 + 0.01
    x, iters, per_block, _ = O.gs_jacobi_reference(model, u, 5)
    assert (x == 1).all() and (per_block == np.array([5, 5, 2])[None, :]).all()


# ------------------------------------------------------------------ Proposition 2 / Algorithm 2
@pytest.mark.parametrize("name", ["cfg1", "small_f32", "small_cat_f32"])
def test_jacobi_gs_exact_for_every_block_size(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    model = _model(net)
    noise = S.make_noise(w)
    xs, _ = O.sequential_sample(model, noise)
    xj, it_j, _, _, _ = O.jacobi_reference(model, noise)
    for B in [1, 2, 7, 16, w.D - 1, w.D, w.D + 5]:
        M = len(O.block_partition(w.D, B))
        x, iters, done, _ = O.jacobi_gs_reference(model, noise, B)
        assert (x == xs).all() and done.all()
        assert (iters >= 1).all() and (iters <= M).all()             # Proposition 2: at most M iterations
        if B == 1:
            assert (iters == it_j).all()              # blocks of one position: Algorithm 1 itself
        if B >= w.D:
            assert (iters == 1).all()                 # one block: a single sweep is the feedforward computation
        # proof of Proposition 2: after k iterations the first k blocks are final
        for k in (1, 2, 3):
            if k < M:
                xk = O.jacobi_gs_reference(model, noise, B, max_iters=k)[0]
                assert (xk[:, :k * B] == xs[:, :k * B]).all()
    init = np.random.default_rng(5).integers(0, 2 if w.C == 1 else w.C, (w.N, w.D)).astype(np.uint8)
    assert (O.jacobi_gs_reference(model, noise, 7, init)[0] == xs).all()


def test_jacobi_gs_chain_needs_one_iteration_per_block():
    """A chain that copies its predecessor (Section 4.1, Example 3) started from the wrong symbols: every
    iteration of Algorithm 2 finalises exactly one more block, so M iterations are needed."""
    T = 12
    model = _model(S.copy_chain_network(T))
    u = S.uniform_noise(2, T, 3) * 0.98 + 0.01
    x, iters, done, _ = O.jacobi_gs_reference(model, u, 5)
    assert (x == 1).all() and (iters == 3).all() and done.all()
    x1 = O.jacobi_gs_reference(model, u, 5, max_iters=1)[0]
    assert (x1[:, :5] == 1).all() and not (x1[:, 5:] == 1).all()


def test_jacobi_gs_one_iteration_by_hand():
    """One iteration of Algorithm 2 written out with the scalar evaluator: position j of block [a, b) sees the
    previous iterate before a and this iteration's symbols in a .. j-1."""
    net = small_net(7, 1, [9], seed=21)
    model = _model(net)
    u = S.uniform_noise(3, 7, 8)
    prev = np.random.default_rng(2).integers(0, 2, (3, 7)).astype(np.uint8)
    expect = prev.copy()
    for n in range(3):
        for (a, b) in [(0, 3), (3, 6), (6, 7)]:
            mixed = [int(v) for v in prev[n]]
            for j in range(a, b):
                z = scalar_logits(net, mixed, j)[0]
                mixed[j] = 1 if u[n, j] < 1.0 / (1.0 + math.exp(-z)) else 0
            expect[n, a:b] = mixed[a:b]
    got = O.jacobi_gs_reference(model, u, 3, prev, max_iters=1)[0]
    assert (got == expect).all()


# ------------------------------------------------------------------ bf16-activation mode
def test_bf16_activation_mode_rounds_hidden_units_only():
    w = S.workload("small_bf16")
    net = S.make_network(w)
    exact, rounded = _model(net), _model(net, "bf16")
    x = np.random.default_rng(0).integers(0, 2, (4, w.D)).astype(np.uint8)
    h = O.last_hidden(rounded, x)
    assert (O.round_to_bf16(h) == h).all()
    z0, z1 = O.logits_all(exact, x), O.logits_all(rounded, x)
    assert np.abs(z0 - z1).max() < 2e-2 * z0.std() and (z0 != z1).any()
    noise = S.make_noise(w)
    xs, _ = O.sequential_sample(rounded, noise)
    assert (O.jacobi_reference(rounded, noise)[0] == xs).all()


# ------------------------------------------------------------------ one-hot categorical input
def test_onehot_masks_by_hand():
    # D = 3, C = 2, hidden degrees [1, 2]: unit of degree m reads the C inputs of every position d <= m
    masks = O.masks_from_degrees(3, 2, [np.array([1, 2])], onehot=True)
    m1 = np.array([[1, 1, 0, 0, 0, 0], [1, 1, 1, 1, 0, 0]], bool)
    assert (masks[0] == m1).all() and masks[1].shape == (6, 2)
    e = O.encode(np.array([[1, 0, 1]]), 2, onehot=True)
    assert (e == np.array([[0, 1, 1, 0, 0, 1]])).all()


def test_onehot_logits_match_scalar_definition_and_are_autoregressive():
    net = small_net(6, 4, [9, 7], seed=61, onehot=True)
    model = _model(net)
    rng = np.random.default_rng(0)
    x = rng.integers(0, 4, size=(5, 6)).astype(np.uint8)
    z = O.logits_all(model, x)
    for n in range(5):
        for t in range(6):
            assert np.allclose(z[n, t], scalar_logits(net, x[n], t), rtol=1e-12, atol=1e-12)
    # position t reads x_{<t} only; and it does read them (every symbol value gives different logits somewhere)
    for t in range(6):
        y = x.copy()
        y[:, t:] = rng.integers(0, 4, size=(5, 6 - t))
        assert np.array_equal(O.logits_all(model, y)[:, :t + 1], z[:, :t + 1])
    y = x.copy()
    y[:, 0] = (y[:, 0] + 1) % 4
    assert np.abs(O.logits_all(model, y)[:, 1:] - z[:, 1:]).max() > 1e-3
    # the first layer is a sum of one weight column per position: h1 = relu(b + sum_t W[:, t*C + x_t] * mask)
    vis = net.degrees[0][:, None] >= np.arange(1, 7)[None, :]
    for n in range(5):
        pre = net.b[0].astype(np.float64) + sum(net.W[0][:, t * 4 + int(x[n, t])].astype(np.float64) * vis[:, t] for t in range(6))
        h1 = np.maximum(pre, 0.0)
        assert np.allclose(O.affine(O.encode(x[n:n + 1], 4, True), model.WM[0], model.b[0])[0], pre, rtol=1e-12, atol=1e-14)
        assert np.allclose(np.maximum(O.affine(O.encode(x[n:n + 1], 4, True), model.WM[0], model.b[0])[0], 0.0), h1)


def test_onehot_sequential_sampler_distribution():
    D, C = 4, 3
    net = small_net(D, C, [12], seed=63, gain=2.5, rule="cyclic", onehot=True)
    model = _model(net)
    states, p = O.joint_bruteforce(model)
    ref = brute_joint(net)
    assert np.allclose(p, [ref[tuple(int(v) for v in s)] for s in states], rtol=1e-10)
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    n = 200000
    x, _ = O.sequential_sample(model, S.gumbel_noise(n, D, C, 779))
    code = (x.astype(np.int64) * (C ** np.arange(D - 1, -1, -1))).sum(axis=1)
    counts = np.bincount(code, minlength=C ** D).astype(np.float64)
    assert _chi2(counts, p) > 1e-3
    assert p.max() / p.min() > 20


@pytest.mark.parametrize("name", ["small_cat_onehot_f32", "mid_cat_onehot"])
def test_onehot_jacobi_and_gs_jacobi_equal_sequential(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    model = _model(net)
    noise = S.make_noise(w)
    xs, _ = O.sequential_sample(model, noise)
    xj, it, done, _, _ = O.jacobi_reference(model, noise)
    assert (xj == xs).all() and done.all() and (it <= w.D).all()
    xg, _, _, _ = O.gs_jacobi_reference(model, noise, 5)
    assert (xg == xs).all()
