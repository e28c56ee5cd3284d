"""CPU-only: what two correct evaluations of the deep bf16 convolutional network may differ by, and why the
full-size parity test grades it layer by layer.

Two evaluations of the SAME network (the benchmark's 8 masked 5 x 5 layers of 128 channels, weights and noise
recipe of the cfg5 workload, on images of 4 rows) that differ only in the precision of their sums -- fp64 (the
oracle) against fp32 (numpy's float32 products, standing in for any fp32-accumulating implementation):

* end to end they drift apart: each layer rounds to bf16, an activation next to a rounding boundary rounds the
  other way, and the share of activations that differ by one bf16 step grows with depth, so that the logits of
  the two evaluations differ by far more than the 1e-3 decision margin of the parity bar;
* layer by layer they agree to the accumulation error: the oracle's layer l + 1 applied to the fp32 side's
  layer-l activations reproduces the fp32 side's layer l + 1 bit for bit, except within the accumulation
  error of a rounding boundary, where the neighbouring bf16 value is the only other outcome
  (tests/layer_certificate.py).  The GPU tests hold every kernel of the network to that certificate."""
import dataclasses

import numpy as np

from oracle import conv_oracle as CO
from oracle import made_oracle as O
from paper_2002_03629_amd import synth as S

import layer_certificate as LC


def conv_layer_f32(a, WM, b):
    """The masked convolution with every product and sum in float32 (same taps, same zero padding)."""
    N, H, W, _ = a.shape
    k = WM.shape[1]
    mid = k // 2
    pad = np.zeros((N, H + 2 * mid, W + 2 * mid, a.shape[3]), np.float32)
    pad[:, mid:mid + H, mid:mid + W, :] = a
    out = np.zeros((N, H, W, WM.shape[0]), np.float32) + b.astype(np.float32)
    for ky in range(k):
        for kx in range(k):
            w = WM[:, ky, kx, :].astype(np.float32)
            if w.any():
                out += pad[:, ky:ky + H, kx:kx + W, :] @ w.T
    return out


def _network():
    w = dataclasses.replace(S.conv_workload("cfg5"), H=4, N=2)
    net = S.make_conv_network(w)
    model = CO.build_conv_model(net.H, net.W, net.C, net.F, net.k, net.W_, net.b, "bf16")
    x = np.random.default_rng(11).integers(0, 256, size=(w.N, net.D)).astype(np.uint8)
    a0 = (x.astype(np.float64).reshape(w.N, net.H, net.W, 3) - 128.0) / 128.0
    return w, net, model, a0


def test_two_summation_precisions_drift_apart_end_to_end_but_agree_layer_by_layer():
    w, net, model, a0 = _network()
    n_conv = len(model.WM) - 1
    a64, a32 = a0, a0.astype(np.float32)
    differing = []
    for l in range(n_conv):
        # the fp32 side's layer l + 1 from its own layer l
        nxt32 = O.round_to_bf16(np.maximum(conv_layer_f32(a32, model.WM[l], model.b[l]), 0.0)).astype(np.float32)
        # layer-by-layer certificate: the oracle's layer l + 1 on the fp32 side's layer l
        pre = CO.conv_layer(a32.astype(np.float64), model.WM[l], model.b[l])
        err = LC.sum_error(CO.conv_layer(np.abs(a32.astype(np.float64)), np.abs(model.WM[l]), np.abs(model.b[l])))
        ok, exact, near = LC.certify_rounded(pre, err, nxt32)
        assert ok.all(), LC.summarize(f"layer {l}", ok, exact, near)
        assert exact.mean() > 0.97 and (exact | near).all()
        # end to end: the oracle's own chain
        a64 = O.round_to_bf16(np.maximum(CO.conv_layer(a64, model.WM[l], model.b[l]), 0.0))
        d = a64 != nxt32
        differing.append(float(d.mean()))
        a32 = nxt32
    # the share of differing activations grows with depth, from none to a sizeable fraction
    assert differing[0] < 0.02 and differing[-1] > 5 * max(differing[0], 1e-3), differing
    assert 0.01 < differing[-1] < 0.5, differing
    z64 = CO.conv_layer(a64, model.WM[-1], model.b[-1])
    z32 = conv_layer_f32(a32, model.WM[-1], model.b[-1]).astype(np.float64)
    rms = float(np.sqrt(np.mean(z64 ** 2)))
    err_rms = float(np.sqrt(np.mean((z64 - z32) ** 2))) / rms
    err_max = float(np.abs(z64 - z32).max()) / rms
    print(f"differing activations per layer {['%.3f' % v for v in differing]}; logits: error rms {err_rms:.2e}, "
          f"max {err_max:.2e} of rms {rms:.2f}")
    # rounding noise of relative size 2^-9 / sqrt(3) per layer, in quadrature over the layers: ~3e-3 of rms; the
    # largest element is several times that, i.e. far above the parity bar's decision margin of 1e-3 / rms
    assert 5e-4 < err_rms < 1e-2
    assert err_max > 3e-3


def test_the_certificate_rejects_a_wrong_layer():
    """Teeth: a dropped tap, a missing bias and a shifted channel are all rejected."""
    w, net, model, a0 = _network()
    l = 1
    a1 = O.round_to_bf16(np.maximum(CO.conv_layer(a0, model.WM[0], model.b[0]), 0.0))
    pre = CO.conv_layer(a1, model.WM[l], model.b[l])
    err = LC.sum_error(CO.conv_layer(np.abs(a1), np.abs(model.WM[l]), np.abs(model.b[l])))
    good = O.round_to_bf16(np.maximum(pre, 0.0))
    assert LC.certify_rounded(pre, err, good)[0].all()
    dropped = model.WM[l].copy()
    dropped[:, 0, 0, :] = 0.0                                   # one tap missing
    bad = O.round_to_bf16(np.maximum(CO.conv_layer(a1, dropped, model.b[l]), 0.0))
    assert not LC.certify_rounded(pre, err, bad)[0].all()
    assert not LC.certify_rounded(pre, err, np.roll(good, 1, axis=3))[0].all()      # channels shifted by one
    one_step = good * (1.0 + 2.0 ** -7)                         # every value one bf16 step too large
    assert LC.certify_rounded(pre, err, O.round_to_bf16(one_step))[0].mean() < 0.6
