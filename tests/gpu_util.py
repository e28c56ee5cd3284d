"""Helpers shared by the GPU parity tests (test code; may import both the binding and the oracle)."""
import dataclasses
import time

import numpy as np
import torch

from oracle import made_oracle as O
from paper_2002_03629_amd import binding as B

MARGIN = 1e-3          # positions whose oracle decision margin is below this are exempt from bit-exactness
CLEAR_FLOOR = 0.25     # iteration counts are compared for samples none of whose decisions came within MARGIN of a
                       # tie; on the reduced workloads at least this share of the batch must be such samples
LOGIT_TOL = {"f32": 1e-4, "bf16": 2e-2}


def progress(msg):
    """Long tests say where they are (visible with `pytest -s`; the output of a failing test is shown anyway)."""
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def oracle_models(net):
    """(exact fp64 model, model whose hidden activations are rounded like the library's)."""
    exact = O.build_model(net.D, net.C, net.degrees, net.W, net.b, None, getattr(net, "onehot", False))
    # the two differ only in the activation-rounding switch; share the (possibly multi-GiB) arrays
    same = dataclasses.replace(exact, act_round="bf16") if net.dtype == "bf16" else exact
    return exact, same


PERSISTENT = False     # execution path the models below are switched to (the tests run both)
RESIDENT = 0           # sample-resident kernel: 0 never, 1 whenever the model fits it (2, the library's default, = where it pays)
FUSED_CATEGORICAL = True
CHAINS = 4
RETIRE_SPLIT = None   # None: the library's default; 1: the stop test always runs as a kernel of its own
LAZY = None           # stop test without a tail (Jacobi, Bernoulli, one chain of up to 256 samples): None = library default (on)
XCD = 0               # whole-call kernel with one share of the batch per XCD: 0 never, 2 whenever the batch fits, None: library default


class GpuModel:
    def __init__(self, net, persistent=None, big_tile_batch=None, mid_tile_batch=None):
        self.net = net
        self.h = B.model_from_network(net)
        B.made_set_option(self.h, B.MADE_OPT_PERSISTENT, int(PERSISTENT if persistent is None else persistent))
        B.made_set_option(self.h, B.MADE_OPT_RESIDENT, int(RESIDENT))
        B.made_set_option(self.h, B.MADE_OPT_FUSED_CATEGORICAL, int(FUSED_CATEGORICAL))
        B.made_set_option(self.h, B.MADE_OPT_CHAINS, CHAINS)
        if RETIRE_SPLIT is not None:
            B.made_set_option(self.h, B.MADE_OPT_RETIRE_SPLIT, RETIRE_SPLIT)
        if XCD is not None:
            B.made_set_option(self.h, B.MADE_OPT_XCD_RESIDENT, XCD)
        if LAZY is not None:
            B.made_set_option(self.h, B.MADE_OPT_LAZY_STOP_TEST, LAZY)
        if big_tile_batch is not None:
            B.made_set_option(self.h, B.MADE_OPT_BIG_TILE_BATCH, big_tile_batch)
        if mid_tile_batch is not None:
            B.made_set_option(self.h, B.MADE_OPT_MID_TILE_BATCH, mid_tile_batch)

    def close(self):
        if self.h:
            B.made_free(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def logits(self, x):
        N = x.shape[0]
        out = torch.empty((N, self.net.D, self.net.C), dtype=torch.float32, device="cuda")
        B.made_forward_logits(self.h, dev(x), N, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def jacobi(self, noise, x_init=None, max_iters=0):
        N = noise.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.uint8, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        B.jacobi_sample(self.h, dev(noise), N, None if x_init is None else dev(x_init), max_iters, x, it)
        return x.cpu().numpy(), it.cpu().numpy()

    def gs_jacobi(self, noise, block, x_init=None):
        N = noise.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.uint8, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        B.gs_jacobi_sample(self.h, dev(noise), N, None if x_init is None else dev(x_init), block, x, it)
        return x.cpu().numpy(), it.cpu().numpy()

    def jacobi_gs(self, noise, block, x_init=None, max_iters=0):
        N = noise.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.uint8, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        B.jacobi_gs_sample(self.h, dev(noise), N, None if x_init is None else dev(x_init), block, max_iters, x, it)
        return x.cpu().numpy(), it.cpu().numpy()

    def activations(self, x, layer):
        """Hidden layer `layer` evaluated on symbols x, as the library holds it, [N, width] float32."""
        N = x.shape[0]
        out = torch.empty((N, self.net.hidden[layer]), dtype=torch.float32, device="cuda")
        B.made_layer_activations(self.h, dev(x), N, layer, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def sequential(self, noise, mode):
        N = noise.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.uint8, device="cuda")
        B.sequential_sample(self.h, dev(noise), N, mode, x)
        return x.cpu().numpy()

    def stats(self):
        return B.made_last_stats(self.h)


def assert_logits_close(z_gpu, z_ref, tol):
    """max |z_gpu - z_ref| <= tol * rms(z_ref) (the logits of a random network are centred on 0, so
    the error is scaled by the tensor's own size rather than element by element)."""
    rms = max(1e-6, float(np.sqrt(np.mean(z_ref ** 2))))
    err = float(np.abs(z_gpu - z_ref).max())
    assert err <= tol * rms, f"logit error {err:.3e} > {tol} * rms {rms:.3e}"
    return err / rms


def assert_sample_parity(model_same, noise, x_gpu, x_oracle=None, margin_oracle=None):
    """The library's symbols against the oracle.

    1. Fixed-point certificate: at the library's own output x, every position must equal the
       oracle's decision from x, unless the oracle's margin there is below MARGIN.
    2. Wherever the oracle's own sequential run never came within MARGIN of a decision boundary,
       the symbols must be identical.
    Returns (exempt positions, fraction of samples that are bit-identical or None).
    """
    ok, margin = O.fixed_point_check(model_same, x_gpu, noise)
    bad = ~ok & (margin >= MARGIN)
    assert not bad.any(), f"{int(bad.sum())} positions differ from the oracle's decision with margin >= {MARGIN}"
    exempt = int((~ok).sum())
    frac = None
    if x_oracle is not None:
        same = (x_gpu == x_oracle).all(axis=1)
        frac = float(same.mean())
        if margin_oracle is not None:
            clear = margin_oracle.min(axis=1) >= MARGIN
            assert same[clear].all(), "a sample with every margin >= 1e-3 differs from the sequential oracle"
    return exempt, frac


def assert_counts_match(it, it_ref, min_margin, floor=CLEAR_FLOOR):
    """Iteration counts against the oracle's for every sample whose decisions all stayed clear of a tie, and
    there must be enough such samples for the comparison to mean something."""
    clear = min_margin >= MARGIN
    assert clear.mean() >= floor, f"only {clear.mean():.2f} of the samples have all margins >= {MARGIN}"
    assert (it[clear] == it_ref[clear]).all(), (it, it_ref)
    return float(clear.mean())


def mlp_layer_certificate(g, model_same, x, noise=None):
    """Every layer of the masked MLP on its own (see layer_certificate.py): the oracle's layer l + 1 applied to
    the activations the library produced for layer l must reproduce the library's layer l + 1 -- bit for bit
    except within the fp32 accumulation error of a bf16 rounding boundary (bf16 model), resp. within that error
    (fp32 model) -- and the logits must follow from the library's last hidden layer within the accumulation
    error.  With `noise`, x is also checked to be the oracle's decision from those logits wherever its margin is
    at least MARGIN.  Prints the worst accumulation error seen in units of 2^-24 sum|a_i w_i|."""
    import layer_certificate as LC
    net = g.net
    L = len(net.hidden)
    h = O.encode(x, model_same.C, model_same.onehot)
    rounded = model_same.act_round == "bf16"
    worst = 0.0
    for l in range(L + 1):
        pre = O.affine(h, model_same.WM[l], model_same.b[l])
        mag = O.affine(np.abs(h), np.abs(model_same.WM[l]), np.abs(model_same.b[l]))
        err = LC.sum_error(mag)
        if l == L:
            got = g.logits(x).reshape(x.shape[0], -1).astype(np.float64)
            ok = LC.certify_plain(pre, err, got)
            assert ok.all(), f"logits: {int((~ok).sum())} of {ok.size} outside the accumulation error"
            worst = max(worst, float((np.abs(got - pre) / (LC.U32 * np.maximum(mag, 1e-30))).max()))
            if noise is not None:
                fx, margin = O.decide(pre.reshape(x.shape[0], model_same.D, model_same.C), noise, model_same.C)
                assert not ((fx != x) & (margin >= MARGIN)).any()
            break
        got = g.activations(x, l).astype(np.float64)
        if rounded:
            ok, exact, near = LC.certify_rounded(pre, err, got)
            assert ok.all(), LC.summarize(f"hidden layer {l}", ok, exact, near)
            assert exact.mean() > 0.95, LC.summarize(f"hidden layer {l}", ok, exact, near)
        else:
            ok = LC.certify_plain(np.maximum(pre, 0.0), err, got)
            assert ok.all(), f"hidden layer {l}: {int((~ok).sum())} of {ok.size} outside the accumulation error"
            worst = max(worst, float((np.abs(got - np.maximum(pre, 0.0)) / (LC.U32 * np.maximum(mag, 1e-30))).max()))
        h = got
    return worst
