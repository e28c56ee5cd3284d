"""CPU pins of the masked-convolution oracle: hand-written masks, a scalar loop evaluator, the exact
autoregressive property, normalisation of the chain-rule joint, the sampler's distribution, Proposition 1."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

from oracle import conv_oracle as CO
from oracle import made_oracle as O
from paper_2002_03629_amd import synth as S


def tiny(H, W, C, F, k, n_conv, seed, gain=3.0, bias=True):
    w = S.ConvWorkload("t", H, W, C, F, k, n_conv, "f32", 2, seed, gain)
    return S.make_conv_network(w, with_bias=bias)


def model_of(net, act_round=None):
    return CO.build_conv_model(net.H, net.W, net.C, net.F, net.k, net.W_, net.b, act_round)


def test_group_sizes_and_masks_by_hand():
    assert CO.group_sizes(128) == (43, 43, 42) and CO.group_sizes(64) == (22, 21, 21) and CO.group_sizes(3) == (1, 1, 1)
    g = np.array([0, 1, 2])
    a = CO.conv_mask(g, g, 3, "A")
    b = CO.conv_mask(g, g, 3, "B")
    for m in (a, b):
        assert m[:, 0, :, :].all() and m[:, 1, 0, :].all()            # row above, left neighbour: visible
        assert not m[:, 1, 2, :].any() and not m[:, 2, :, :].any()    # right neighbour, row below: invisible
    assert (a[:, 1, 1, :] == np.array([[0, 0, 0], [1, 0, 0], [1, 1, 0]], bool)).all()   # centre, type A: strictly earlier
    assert (b[:, 1, 1, :] == np.array([[1, 0, 0], [1, 1, 0], [1, 1, 1]], bool)).all()   # centre, type B: earlier or same


def scalar_conv_logits(net, x, t):
    """Logits of state t for one image from the definition, with Python loops and its own mask rule."""
    H, W, C, F, k = net.H, net.W, net.C, net.F, net.k
    mid = k // 2
    s0 = -(-F // 3)
    s1 = -(-(F - s0) // 2)
    grp = [0] * s0 + [1] * s1 + [2] * (F - s0 - s1)
    a = [[[(float(x[(y * W + xx) * 3 + c]) - 128.0) / 128.0 for c in range(3)] for xx in range(W)] for y in range(H)]
    in_grp = [0, 1, 2]
    n = len(net.W_)
    for l in range(n - 1):
        Wl, bl = net.W_[l], net.b[l]
        out = [[[0.0] * F for _ in range(W)] for _ in range(H)]
        for y in range(H):
            for xx in range(W):
                for f in range(F):
                    acc = 0.0 if bl is None else float(bl[f])
                    for ky in range(k):
                        for kx in range(k):
                            yy, xs = y + ky - mid, xx + kx - mid
                            if not (0 <= yy < H and 0 <= xs < W):
                                continue
                            earlier = ky < mid or (ky == mid and kx < mid)
                            centre = ky == mid and kx == mid
                            for ci in range(len(in_grp)):
                                vis = earlier or (centre and (in_grp[ci] < grp[f] if l == 0 else in_grp[ci] <= grp[f]))
                                if vis:
                                    acc += float(Wl[f, ky, kx, ci]) * a[yy][xs][ci]
                    out[y][xx][f] = max(acc, 0.0)
        a, in_grp = out, grp
    y, xx, c = t // (3 * W), (t // 3) % W, t % 3
    Wl, bl = net.W_[-1], net.b[-1]
    z = []
    for cls in range(C):
        row = c * C + cls
        acc = 0.0 if bl is None else float(bl[row])
        for f in range(F):
            if grp[f] <= c:
                acc += float(Wl[row, 0, 0, f]) * a[y][xx][f]
        z.append(acc)
    return z


def test_logits_match_scalar_definition():
    net = tiny(2, 3, 4, 5, 3, 2, seed=3)
    model = model_of(net)
    rng = np.random.default_rng(0)
    x = rng.integers(0, 256, size=(2, net.D)).astype(np.uint8)
    z = CO.conv_logits_all(model, x)
    for n in range(2):
        for t in range(net.D):
            assert np.allclose(z[n, t], scalar_conv_logits(net, x[n], t), rtol=1e-11, atol=1e-11)


def test_autoregressive_property_exact():
    net = tiny(3, 4, 3, 6, 5, 3, seed=4)
    model = model_of(net)
    rng = np.random.default_rng(1)
    x = rng.integers(0, 256, size=(3, net.D)).astype(np.uint8)
    z = CO.conv_logits_all(model, x)
    seen = 0
    for t in range(net.D):
        y = x.copy()
        y[:, t:] = rng.integers(0, 256, size=(3, net.D - t))
        assert (CO.conv_logits_all(model, y)[:, t] == z[:, t]).all()
        if t > 0:
            y = x.copy()
            y[:, t - 1] = ((y[:, t - 1].astype(int) + 97) % 256).astype(np.uint8)
            seen += bool((CO.conv_logits_all(model, y)[:, t] != z[:, t]).any())
    assert seen >= (net.D - 1) // 2


def conv_joint(net, model):
    """All C^D states and their chain-rule probability (Appendix A.3), tiny models only."""
    C, D = net.C, net.D
    states = np.array(list(itertools.product(range(C), repeat=D)), dtype=np.uint8)
    z = CO.conv_logits_all(model, states)
    p = O.conditional_probs(z, C)
    chosen = np.take_along_axis(p, states[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    return states, chosen.prod(axis=1)


def test_joint_normalised_and_sampler_distribution():
    net = tiny(1, 2, 3, 3, 3, 2, seed=8, gain=1.0)
    # symbols 0..2 enter as (v - 128)/128, i.e. -1 plus a little: scale layer 1 up and recentre it (bias = sum
    # of its weights, exact for the centre and left taps that exist in a 1 x 2 image) so that states really
    # depend on earlier ones
    net.W_[0] = (net.W_[0] * 100.0).astype(np.float32)
    net.b[0] = (net.W_[0][:, 1, 0:2, :].sum(axis=(1, 2)) * 0.75 + net.b[0]).astype(np.float32)
    net.W_[1] = (net.W_[1] * 2.0).astype(np.float32)
    model = model_of(net)
    states, p = conv_joint(net, model)
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    cond = O.conditional_probs(CO.conv_logits_all(model, states), net.C)
    assert max((cond[:, t].max(axis=0) - cond[:, t].min(axis=0)).max() for t in range(1, net.D)) > 0.05
    n = 150000
    xs, _ = CO.conv_sequential_sample(model, S.gumbel_noise(n, net.D, net.C, 99))
    code = (xs.astype(np.int64) * (net.C ** np.arange(net.D - 1, -1, -1))).sum(axis=1)
    counts = np.bincount(code, minlength=net.C ** net.D).astype(np.float64)
    exp = p * n
    keep = exp > 5
    chi = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert stats.chi2.sf(chi, int(keep.sum()) - 1) > 1e-3
    # a leaky centre tap (type B in the first layer) breaks the normalisation
    leaky = model_of(net)
    leaky.WM[0] = np.where(CO.conv_mask(CO.group_of_feature(net.F), np.arange(3), net.k, "B"),
                           net.W_[0].astype(np.float64), 0.0)
    assert abs(conv_joint(net, leaky)[1].sum() - 1.0) > 1e-4


@pytest.mark.parametrize("act_round", [None, "bf16"])
def test_jacobi_equals_sequential(act_round):
    w = S.ConvWorkload("t", 2, 5, 256, 6, 3, 3, "f32", 3, 7, 3.0)
    net = S.make_conv_network(w, with_bias=True)
    model = model_of(net, act_round)
    noise = S.make_conv_noise(w)
    xs, margins = CO.conv_sequential_sample(model, noise)
    for init in (None, np.full((w.N, net.D), 255, np.uint8), xs):
        x, iters, done, _ = CO.conv_jacobi_reference(model, noise, init)
        assert (x == xs).all() and done.all() and (iters <= net.D).all()
    assert (CO.conv_jacobi_reference(model, noise, xs)[1] == 1).all()
    ok, _ = CO.conv_fixed_point_check(model, xs, noise)
    assert ok.all()
    bad = xs.copy()
    bad[:, 0] ^= 1
    assert not CO.conv_fixed_point_check(model, bad, noise)[0].all()


def test_conv_jacobi_gs_equals_sequential_and_one_iteration_by_hand():
    """Algorithm 2 on the convolutional model: exact in at most M iterations for every block size (Proposition 2),
    one block = the sequential sampler in one iteration, and one iteration written out with the scalar evaluator."""
    net = tiny(2, 2, 3, 4, 3, 2, seed=12)
    model = model_of(net)
    N, D, C = 2, net.D, net.C
    noise = S.gumbel_noise(N, D, C, 91)
    xs, _ = CO.conv_sequential_sample(model, noise)
    for block in (1, 2, 3, 5, D, D + 4):
        x, iters, done, _ = CO.conv_jacobi_gs_reference(model, noise, block)
        M = -(-D // min(block, D))
        assert (x == xs).all() and done.all() and (iters >= 1).all() and (iters <= M).all(), block
        if block >= D:
            assert (iters == 1).all()
    # one iteration from a random iterate, by hand: state j of block [a, b) sees the previous iterate before a and
    # this iteration's states in a .. j-1
    prev = np.random.default_rng(4).integers(0, C, (N, D)).astype(np.uint8)
    expect = prev.copy()
    block = 5
    for n in range(N):
        for a in range(0, D, block):
            mixed = [int(v) for v in prev[n]]
            for j in range(a, min(a + block, D)):
                z = scalar_conv_logits(net, mixed, j)
                s = [z[c] + float(noise[n, j, c]) for c in range(C)]
                mixed[j] = s.index(max(s))
            expect[n, a:a + block] = mixed[a:a + block]
    got = CO.conv_jacobi_gs_reference(model, noise, block, prev, max_iters=1)[0]
    assert (got == expect).all()
    # an iteration limit below M leaves the image unconverged and says so
    lim = CO.conv_jacobi_gs_reference(model, noise, 2, None, max_iters=1)
    assert (lim[1] == 1).all() and not lim[2].all()
