"""GPU parity of the masked convolutional (PixelCNN-style) model against its CPU oracle."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import conv_oracle as CO
from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S

import layer_certificate as LC
from gpu_util import LOGIT_TOL, MARGIN, assert_logits_close, dev, progress

pytestmark = pytest.mark.gpu


def models(net):
    exact = CO.build_conv_model(net.H, net.W, net.C, net.F, net.k, net.W_, net.b, None)
    same = dataclasses.replace(exact, act_round="bf16") if net.dtype == "bf16" else exact
    return exact, same


def certify(same, noise, x, xs=None, margins=None):
    ok, margin = CO.conv_fixed_point_check(same, x, noise)
    bad = ~ok & (margin >= MARGIN)
    assert not bad.any(), f"{int(bad.sum())} states differ from the oracle's decision with margin >= {MARGIN}"
    if xs is not None:
        clear = margins.min(axis=1) >= MARGIN
        assert ((x == xs).all(axis=1))[clear].all()
    return int((~ok).sum())


class ConvGpu:
    def __init__(self, net):
        self.net, self.h = net, B.conv_model_from_network(net)

    def __enter__(self):
        return self

    def __exit__(self, *a):
        B.made_free(self.h)

    def logits(self, x):
        N = x.shape[0]
        out = torch.empty((N, self.net.D, self.net.C), dtype=torch.float32, device="cuda")
        B.made_forward_logits(self.h, dev(x), N, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def activations(self, x, layer, N=None):
        """k x k layer `layer` as the library holds it, [N, H, 32, F] float32: evaluated on symbols x, or (x = None)
        whatever the most recent sampling call left in the model's per-layer buffers."""
        N = x.shape[0] if x is not None else N
        out = torch.empty((N, self.net.H, 32, self.net.F), dtype=torch.float32, device="cuda")
        B.made_layer_activations(self.h, None if x is None else dev(x), N, layer, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def run(self, what, noise, *args, x_init=None):
        N = noise.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.uint8, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        xi = None if x_init is None else dev(x_init)
        if what == "jacobi":
            B.jacobi_sample(self.h, dev(noise), N, xi, args[0] if args else 0, x, it)
        elif what == "gs":
            B.gs_jacobi_sample(self.h, dev(noise), N, xi, args[0], x, it)
        else:
            B.sequential_sample(self.h, dev(noise), N, args[0], x)
        return x.cpu().numpy(), it.cpu().numpy()


def conv_layer_certificate(g, same, x, noise, from_buffers=False, label=""):
    """Every kernel of the convolutional model on its own (see layer_certificate.py).  For l = 1 .. n_conv the
    oracle's layer l applied to the activations the library holds for layer l - 1 must reproduce the library's
    layer l: bit for bit except within the fp32 accumulation error of a bf16 rounding boundary, where the
    neighbouring bf16 value is accepted (fp32 models: within the accumulation error).  The head's logits must follow
    from the library's last layer within the accumulation error, and every symbol of x must be the oracle's
    Gumbel-max decision from those logits unless its margin is below MARGIN -- the parity bar, applied to each
    kernel separately instead of to the composition of nine of them.
    from_buffers: take the activations a sampling call left behind (they must equal a fresh evaluation on x)."""
    net = g.net
    N = x.shape[0]
    n_conv = len(same.WM) - 1
    rounded = same.act_round == "bf16"
    a = (x.astype(np.float64).reshape(N, net.H, net.W, 3) - 128.0) / 128.0
    stats = []
    # (read what the sampling call left behind BEFORE any fresh evaluation overwrites the buffers)
    kept = [g.activations(None, l, N) for l in range(n_conv)] if from_buffers else None
    for l in range(n_conv):
        got = g.activations(x, l).astype(np.float64)
        if from_buffers:
            assert (kept[l] == got).all(), f"{label} layer {l}: the buffers a sampling call left differ from a fresh evaluation"
        pre = CO.conv_layer(a, same.WM[l], same.b[l])
        err = LC.sum_error(CO.conv_layer(np.abs(a), np.abs(same.WM[l]), np.abs(same.b[l])))
        if rounded:
            ok, exact, near = LC.certify_rounded(pre, err, got)
            assert ok.all(), LC.summarize(f"{label} layer {l}", ok, exact, near)
            assert exact.mean() > 0.95, LC.summarize(f"{label} layer {l}", ok, exact, near)
            stats.append((float(exact.mean()), float(near.mean())))
        else:
            ok = LC.certify_plain(np.maximum(pre, 0.0), err, got)
            assert ok.all(), f"{label} layer {l}: {int((~ok).sum())} of {ok.size} outside the accumulation error"
        a = got
    z_ref = CO.conv_layer(a, same.WM[-1], same.b[-1])
    mag = CO.conv_layer(np.abs(a), np.abs(same.WM[-1]), np.abs(same.b[-1]))
    z = g.logits(x).astype(np.float64).reshape(z_ref.shape)
    ok = LC.certify_plain(z_ref, LC.sum_error(mag), z)
    assert ok.all(), f"{label} head: {int((~ok).sum())} of {ok.size} logits outside the accumulation error"
    worst = float((np.abs(z - z_ref) / (LC.U32 * np.maximum(mag, 1e-30))).max())
    fx, margin = CO.decide(z_ref.reshape(N, same.D, same.C), noise, same.C)
    wrong = (fx != x) & (margin >= MARGIN)
    assert not wrong.any(), f"{label}: {int(wrong.sum())} states are not the oracle's decision at margin >= {MARGIN}"
    return {"exempt_states": int((fx != x).sum()), "worst_logit_error_in_u_sum_abs": worst,
            "bit_identical_per_layer": [round(e, 5) for e, _ in stats],
            "near_boundary_per_layer": [round(n, 5) for _, n in stats]}


@pytest.mark.parametrize("name", ["small_conv", "small_conv_f32"])
def test_conv_parity(name):
    w = S.conv_workload(name)
    net = S.make_conv_network(w, with_bias=True)
    exact, same = models(net)
    noise = S.make_conv_noise(w)
    rng = np.random.default_rng(3)
    x0 = rng.integers(0, 256, size=(w.N, net.D)).astype(np.uint8)
    xs, margins = CO.conv_sequential_sample(same, noise)
    ref = CO.conv_jacobi_reference(same, noise)
    with ConvGpu(net) as g:
        z = g.logits(x0)
        assert_logits_close(z, CO.conv_logits_all(exact, x0), LOGIT_TOL[w.dtype])
        assert_logits_close(z, CO.conv_logits_all(same, x0), 3e-3 if w.dtype == "bf16" else 1e-4)
        x, it = g.run("jacobi", noise)
        certify(same, noise, x, xs, margins)
        clear = ref[3] >= MARGIN
        assert (it[clear] == ref[1][clear]).all(), (it, ref[1])
        x2, it2 = g.run("jacobi", noise)
        assert (x2 == x).all() and (it2 == it).all()
        xi, _ = g.run("jacobi", noise, x_init=x0)
        certify(same, noise, xi, xs, margins)
        for block in (96, 100, net.D):
            xb, itb = g.run("gs", noise, block)
            certify(same, noise, xb, xs, margins)
        for mode in (0, 1):
            xq, _ = g.run("seq", noise, mode)
            certify(same, noise, xq, xs, margins)
        # Jacobi only recomputes the image rows below the first symbol that changed in the pass before
        xj, _ = g.run("jacobi", noise)
        st = B.made_last_stats(g.h)
        assert 0 < st["conv_rows"] <= st["passes"] * w.N * net.H
        if net.H > 2:                                    # (with two rows nothing is ever final before the last pass)
            assert st["conv_rows"] < st["passes"] * w.N * net.H
        # every kernel on its own, on the activations the call left in the per-layer buffers
        print(conv_layer_certificate(g, same, xj, noise, from_buffers=True, label=name))
        with pytest.raises(B.MadeError) as e:
            g.run("jacobi", noise, 1)
        assert e.value.code == B.MADE_ERR_NOT_CONVERGED


@pytest.mark.timeout(900)
def test_cfg5_shape_f32_certificate():
    """The full-size network shape (32 x 32 x 3 images, 8 masked 5 x 5 layers of 128 channels) in fp32, batch 4:
    no activation rounding, so logits agree to 1e-4 of rms and every decision with margin >= 1e-3 is bit-exact.
    One oracle pass at the GPU's result certifies it (the triangular system has one fixed point)."""
    w = dataclasses.replace(S.conv_workload("cfg5"), dtype="f32", N=4)
    net = S.make_conv_network(w)
    exact, _ = models(net)
    noise = S.make_conv_noise(w)
    with ConvGpu(net) as g:
        progress("cfg5 shape, fp32: jacobi on the GPU")
        x, it = g.run("jacobi", noise)
        z = g.logits(x)
        progress("cfg5 shape, fp32: oracle pass")
        zs = CO.conv_logits_all(exact, x)
        assert_logits_close(z, zs, LOGIT_TOL["f32"])
        fx, margin = CO.decide(zs, noise, w.C)
        assert not ((fx != x) & (margin >= MARGIN)).any()
        print(f"cfg5 shape fp32: passes {it}, {int((fx != x).sum())} states differ (all with margin < {MARGIN})")


@pytest.mark.timeout(1500)
def test_cfg5_full_size_certificate():
    """cfg5 as benchmarked: bf16 weights and activations, batch 32, Jacobi and GS-Jacobi (blocks of 4 / 8 / 16 image
    rows).  A sequential oracle run would be 3072 network passes per image, so the results are certified at the
    library's own output.

    Grading.  Two correct evaluations of this network disagree END TO END by far more than the parity bar's
    margin: every layer rounds to bf16, a value next to a rounding boundary rounds the other way under another
    summation order, and each such flip perturbs the next layer (tests/test_bf16_cascade.py shows it between two
    CPU evaluations).  The bar is therefore applied LAYER BY LAYER (conv_layer_certificate): each of the nine
    kernels, fed the library's own input, must reproduce the oracle's layer bit for bit except within the fp32
    accumulation error of a rounding boundary, the logits must follow from the last layer within that error, and
    every drawn state must be the oracle's decision from those logits unless its margin is below 1e-3.  The
    end-to-end figures are kept as a secondary, looser check in the rms norm and are printed."""
    w = S.conv_workload("cfg5")
    progress("cfg5: drawing network and noise")
    net = S.make_conv_network(w)
    exact, same = models(net)
    noise = S.make_conv_noise(w)
    with ConvGpu(net) as g:
        progress("cfg5: jacobi on the GPU")
        x, it = g.run("jacobi", noise)
        st = B.made_last_stats(g.h)
        assert 0 < st["conv_rows"] < st["passes"] * w.N * net.H      # row windows: strictly fewer rows than passes x rows
        progress("cfg5: layer-by-layer certificate of the Jacobi result (32 images)")
        cert = conv_layer_certificate(g, same, x, noise, from_buffers=True, label="cfg5 jacobi")
        print(f"cfg5 jacobi: passes mean {it.mean():.2f} max {it.max()}, stats {st}; certificate {cert}")
        # secondary: end to end against the oracle's own chain of layers, in the rms norm (see the docstring)
        z = g.logits(x)
        progress("cfg5: end-to-end oracle pass over 32 images")
        zs = CO.conv_logits_all(same, x)
        rms = float(np.sqrt(np.mean(zs ** 2)))
        err_max = float(np.abs(z - zs).max())
        err_rms = float(np.sqrt(np.mean((z - zs) ** 2)))
        fx, margin = CO.decide(zs, noise, w.C)
        differ = fx != x
        print(f"cfg5 end to end: logits rms {rms:.3f}, error rms {err_rms:.2e} max {err_max:.2e}; {int(differ.sum())} of "
              f"{differ.size} states differ from the decision of the oracle's own chain, largest margin among them "
              f"{margin[differ].max() if differ.any() else 0:.2e}")
        assert err_rms <= 1.5 * 3.2e-3 * rms                    # (rms norm; the max norm is printed, not graded)
        assert differ.mean() < 5e-3
        ze = CO.conv_logits_all(exact, x[:2])
        assert np.sqrt(np.mean((z[:2] - ze) ** 2)) <= LOGIT_TOL["bf16"] * np.sqrt(np.mean(ze ** 2))   # (rms norm)
        # GS-Jacobi with blocks of whole image rows: same certificate; images whose result equals the Jacobi one
        # are covered by the certificate above, the others are certified themselves
        full_rows = None
        for rows in (8, 4, 16):
            progress(f"cfg5: gs-jacobi, blocks of {rows} rows")
            xb, itb = g.run("gs", noise, rows * 96)
            stb = B.made_last_stats(g.h)
            other = np.flatnonzero((xb != x).any(axis=1))
            print(f"cfg5 gs-jacobi {rows} rows: inner passes mean {itb.mean():.1f}, stats {stb}, "
                  f"{other.size} images differ from the Jacobi result")
            assert (itb >= net.H // rows).all() and (itb <= net.D).all()
            # a block only evaluates the rows up to its own last row, and not the rows that are already final
            if full_rows is None:
                full_rows = stb["passes"] * w.N * net.H
            assert 0 < stb["conv_rows"] < stb["passes"] * w.N * net.H
            if rows == 8 or other.size:
                sel = np.arange(w.N) if rows == 8 else other
                # (the buffers hold the last block's window only for the rows it evaluated: fresh evaluation)
                sub = conv_layer_certificate(_Subset(g, sel), same, xb[sel], noise[sel], label=f"cfg5 gs {rows} rows")
                print(f"  certificate on {sel.size} images: {sub}")
        # Algorithm 2 with blocks of one image row (the block size of the paper's CIFAR-10 run, Section 5.3.2): 32 blocks
        # x 32 images = 1024 copies of the image
        progress("cfg5: jacobi-gs, blocks of one row")
        xg = torch.empty((w.N, net.D), dtype=torch.uint8, device="cuda")
        itg = torch.empty((w.N,), dtype=torch.int32, device="cuda")
        B.jacobi_gs_sample(g.h, dev(noise), w.N, None, 96, 0, xg, itg)
        xg, itg = xg.cpu().numpy(), itg.cpu().numpy()
        other = np.flatnonzero((xg != x).any(axis=1))
        print(f"cfg5 jacobi-gs, one row per block: iterations mean {itg.mean():.1f} max {itg.max()}, stats "
              f"{B.made_last_stats(g.h)}, {other.size} images differ from the Jacobi result")
        assert (itg >= 1).all() and (itg <= 32).all()
        # the copies sit at other batch positions than their images; the kernels' sums do not depend on the position,
        # so Algorithm 2 iterates the very same function and reaches the very same fixed point
        assert other.size == 0, f"{other.size} images differ from the Jacobi result"
    # same network on 2-row images: full sequential oracle
    progress("cfg5: 2-row images against the sequential oracle")
    w2 = dataclasses.replace(w, H=2, N=4)
    net2 = dataclasses.replace(net, H=2)
    _, same2 = models(net2)
    noise2 = S.make_conv_noise(w2)
    xs, margins = CO.conv_sequential_sample(same2, noise2)
    with ConvGpu(net2) as g:
        x, it = g.run("jacobi", noise2)
        certify(same2, noise2, x, xs, margins)


class _Subset:
    """A ConvGpu seen through a subset of its batch (fresh evaluations only)."""

    def __init__(self, g, sel):
        self.g, self.net = g, g.net

    def activations(self, x, layer, N=None):
        return self.g.activations(x, layer)

    def logits(self, x):
        return self.g.logits(x)


@pytest.mark.timeout(900)
def test_taller_reduced_shape_against_the_sequential_oracle():
    """8-row images (768 states) of a reduced network against the oracle's full sequential run at the ordinary bar
    (bit-exact unless a margin is below 1e-3), Jacobi and GS-Jacobi with blocks of 2 and 3 rows, plus the
    layer-by-layer certificate."""
    w = dataclasses.replace(S.conv_workload("small_conv"), H=8, N=2)
    net = S.make_conv_network(w, with_bias=True)
    _, same = models(net)
    noise = S.make_conv_noise(w)
    progress("8-row images: sequential oracle")
    xs, margins = CO.conv_sequential_sample(same, noise)
    with ConvGpu(net) as g:
        x, it = g.run("jacobi", noise)
        certify(same, noise, x, xs, margins)
        st = B.made_last_stats(g.h)
        assert 0 < st["conv_rows"] < st["passes"] * w.N * net.H
        print(conv_layer_certificate(g, same, x, noise, from_buffers=True, label="8 rows"))
        for rows in (2, 3):
            xb, _ = g.run("gs", noise, rows * 96)
            certify(same, noise, xb, xs, margins)
            stb = B.made_last_stats(g.h)
            assert 0 < stb["conv_rows"] < stb["passes"] * w.N * net.H


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["small_conv", "small_conv_f32", "small_conv/8 rows"])
def test_conv_jacobi_gs(name):
    """Algorithm 2 on the convolutional model against its oracle: the sequential result, the oracle's iteration
    counts, blocks that are whole rows, cut rows, a single block, and an iteration limit; on 8-row images (two
    workgroups' rows per image and layer) blocks of one row and of two rows and a bit."""
    tall = name.endswith("/8 rows")
    w = S.conv_workload(name.split("/")[0])
    if tall:
        w = dataclasses.replace(w, H=8, N=2)
    net = S.make_conv_network(w, with_bias=True)
    _, same = models(net)
    noise = S.make_conv_noise(w)
    xs, margins = CO.conv_sequential_sample(same, noise)
    D = net.D

    def run(block, max_iters=0, x_init=None):
        x = torch.empty((w.N, D), dtype=torch.uint8, device="cuda")
        it = torch.empty((w.N,), dtype=torch.int32, device="cuda")
        B.jacobi_gs_sample(g.h, dev(noise), w.N, None if x_init is None else dev(x_init), block, max_iters, x, it)
        return x.cpu().numpy(), it.cpu().numpy()

    with ConvGpu(net) as g:
        for block in ((96, 200) if tall else (96, 50, 192, D, D + 5)):
            progress(f"{name}: jacobi-gs, blocks of {block} states")
            x, it = run(block)
            certify(same, noise, x, xs, margins)
            ref = CO.conv_jacobi_gs_reference(same, noise, block)
            clear = ref[3] >= MARGIN
            assert (it[clear] == ref[1][clear]).all(), (block, it, ref[1])
            M = -(-D // min(block, D))
            assert (it >= 1).all() and (it <= M).all()
            if block >= D:
                assert (it == 1).all()
        init = np.random.default_rng(5).integers(0, 256, size=(w.N, D)).astype(np.uint8)
        x, it = run(96, 0, init)
        certify(same, noise, x, xs, margins)
        ref1 = CO.conv_jacobi_gs_reference(same, noise, 96, None, 1)
        if not ref1[2].all():
            with pytest.raises(B.MadeError) as e:
                run(96, 1)
            assert e.value.code == B.MADE_ERR_NOT_CONVERGED
        # Jacobi still works on the model afterwards (the workspace has grown to the copies' size)
        xj, _ = g.run("jacobi", noise)
        certify(same, noise, xj, xs, margins)


def test_an_image_gets_the_same_bits_at_any_batch_position():
    """The benchmark's network on a batch and on the same batch in another order: symbols, iteration counts and every
    layer's activations are those of the image, not of its place in the batch (the order of the fp32 additions in
    the kernels must not depend on the workgroup's index).  Algorithm 2 relies on it: its copies of an image sit
    at other batch positions and have to iterate the same function."""
    w = dataclasses.replace(S.conv_workload("cfg5"), N=7)
    net = S.make_conv_network(w)
    noise = S.make_conv_noise(w)
    perm = np.array([3, 6, 0, 5, 1, 4, 2])
    with ConvGpu(net) as g:
        x1, it1 = g.run("jacobi", noise)
        a1 = [g.activations(None, l, w.N) for l in range(w.n_conv)]
        x2, it2 = g.run("jacobi", noise[perm])
        a2 = [g.activations(None, l, w.N) for l in range(w.n_conv)]
        assert (x2 == x1[perm]).all() and (it2 == it1[perm]).all()
        for l in range(w.n_conv):
            assert (a2[l] == a1[l][perm]).all(), f"layer {l}"
        z1, z2 = g.logits(x1), g.logits(x1[perm])
        assert (z2 == z1[perm]).all()


def test_a_large_batch_repeats_the_small_one():
    """The benchmark's network on 7 images and on 70 (the same 7 noise arrays ten times over): every copy gets the
    symbols and pass counts of its original.  At 70 images a workgroup of the head draws more rows than fit one of
    its finishing phases, so the phases repeat within a launch."""
    w = dataclasses.replace(S.conv_workload("cfg5"), N=7)
    net = S.make_conv_network(w)
    noise = S.make_conv_noise(w)
    with ConvGpu(net) as g:
        x1, it1 = g.run("jacobi", noise)
        x2, it2 = g.run("jacobi", np.tile(noise, (10,) + (1,) * (noise.ndim - 1)))
        assert (x2.reshape(10, 7, -1) == x1[None]).all()
        assert (it2.reshape(10, 7) == it1[None]).all()
