"""GPU parity of the MADE with real states and logistic conditionals (tolerance-based Jacobi stopping)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import logistic_oracle as L
from oracle import made_oracle as O
from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S

from gpu_util import dev, progress

pytestmark = pytest.mark.gpu

# |x_gpu - x_oracle| <= X_TOL * rms(x): fp32 differs from the fp64 oracle by summation rounding only; with bf16
# the states are rounded to bf16 where they enter the network, and a state next to a rounding boundary can
# round the other way on the two sides (one step = 2^-8 relative), which later positions inherit: the bound is
# that of the bf16 logits (2e-2 of rms), the rms error is an order of magnitude below it.
X_TOL = {"f32": 1e-4, "bf16": 2e-2}
# network outputs at given states: against the oracle in the same arithmetic (bf16 states and activations) only
# summation order differs; against the exact oracle three roundings (states, two hidden layers) instead of the
# two of the discrete models compound: 2e-2 * sqrt(3/2) -> 3e-2
P_TOL_SAME = {"f32": 1e-4, "bf16": 3e-3}
P_TOL_EXACT = {"f32": 1e-4, "bf16": 3e-2}


def models(net):
    exact = O.build_model(net.D, net.C, net.degrees, net.W, net.b, None)
    same = dataclasses.replace(exact, act_round="bf16") if net.dtype == "bf16" else exact
    return exact, same


class RealGpu:
    def __init__(self, net):
        self.net, self.h = net, B.model_from_network(net)

    def __enter__(self):
        return self

    def __exit__(self, *a):
        B.made_free(self.h)

    def params(self, x):
        N = x.shape[0]
        out = torch.empty((N, self.net.D, 2), dtype=torch.float32, device="cuda")
        B.made_forward_params(self.h, dev(x.astype(np.float32)), N, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def jacobi(self, l, eps, x_init=None, max_iters=0):
        N = l.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.float32, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        xi = None if x_init is None else dev(x_init.astype(np.float32))
        B.jacobi_sample_real(self.h, dev(l), N, xi, eps, max_iters, x, it)
        return x.cpu().numpy().astype(np.float64), it.cpu().numpy()

    def gs_jacobi(self, l, block, eps):
        N = l.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.float32, device="cuda")
        it = torch.empty((N,), dtype=torch.int32, device="cuda")
        B.gs_jacobi_sample_real(self.h, dev(l), N, None, block, eps, x, it)
        return x.cpu().numpy().astype(np.float64), it.cpu().numpy()

    def sequential(self, l, mode):
        N = l.shape[0]
        x = torch.empty((N, self.net.D), dtype=torch.float32, device="cuda")
        B.sequential_sample_real(self.h, dev(l), N, mode, x)
        return x.cpu().numpy().astype(np.float64)


def close(x, ref, tol, what):
    rms = float(np.sqrt(np.mean(ref ** 2)))
    err = float(np.abs(x - ref).max())
    assert err <= tol * rms, f"{what}: max error {err:.3e} > {tol} * rms {rms:.3e}"
    return err / rms


@pytest.mark.parametrize("name", ["small_real_f32", "small_real_bf16"])
def test_logistic_parity(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    exact, same = models(net)
    l = S.make_noise(w)
    xs = L.sequential_sample_real(same, l)
    tol = X_TOL[w.dtype]
    with RealGpu(net) as g:
        # network outputs at given states
        x0 = np.random.default_rng(3).normal(size=xs.shape) * 2.0
        x0 = x0.astype(np.float32).astype(np.float64)
        p = g.params(x0)
        for model, ptol in ((same, P_TOL_SAME[w.dtype]), (exact, P_TOL_EXACT[w.dtype])):
            mu, a = L.params_all(model, x0)
            close(p[:, :, 0], mu, ptol, "mu")
            close(p[:, :, 1], a, ptol, "a")
        # sequential sampling, both modes
        xq0 = g.sequential(l, 0)
        close(xq0, xs, tol, "sequential whole network")
        close(g.sequential(l, 1), xs, tol, "sequential lean")
        # Jacobi with eps = 0 reproduces the sequential result of the same arithmetic bit for bit
        xj, it = g.jacobi(l, 0.0)
        assert (xj == xq0).all() and (it <= w.D).all()
        # the fixed-point residual measured by the oracle at the GPU's result
        assert np.abs(L.jacobi_pass_real(same, xj, l) - xj).max() <= tol * np.sqrt(np.mean(xs ** 2))
        # any start
        xi, _ = g.jacobi(l, 0.0, x0)
        assert (xi == xq0).all()
        # tolerance: stops where the oracle stops, except for samples one of whose forward differences lies so
        # close to eps that arithmetic noise (of relative size `band`) decides; the result stays within tol
        band = 0.02 if w.dtype == "f32" else 0.3
        for eps in (1e-1, 1e-2):
            xr, it_ref, done, traj = L.jacobi_reference_real(same, l, eps, record=True)
            xe, ite = g.jacobi(l, eps)
            clear = np.ones(w.N, dtype=bool)
            for n in range(w.N):
                for k in range(1, it_ref[n] + 1):
                    fd = np.abs(traj[k][n] - traj[k - 1][n]).max()
                    if eps * (1 - band) <= fd <= eps * (1 + band):
                        clear[n] = False
            print(f"{name} eps {eps}: {int(clear.sum())} of {w.N} samples clear, iterations gpu {ite.mean():.2f} "
                  f"oracle {it_ref.mean():.2f}, mismatches among clear {int((ite[clear] != it_ref[clear]).sum())}")
            assert clear.sum() >= w.N // 2
            assert (ite[clear] == it_ref[clear]).all(), (eps, ite, it_ref)
            assert np.abs(xe - xr)[clear].max() <= tol * np.sqrt(np.mean(xs ** 2)) + 1e-6
            assert (ite <= it).all()
        # GS-Jacobi (Algorithm 3) with real states
        for block in (7, 32, w.D):
            xb, itb = g.gs_jacobi(l, block, 0.0)
            close(xb, xs, tol, f"gs-jacobi block {block}")
        # iteration limit
        with pytest.raises(B.MadeError) as e:
            g.jacobi(l, 0.0, None, 1)
        assert e.value.code == B.MADE_ERR_NOT_CONVERGED
        # the discrete entry points refuse this model
        with pytest.raises(B.MadeError) as e:
            B.jacobi_sample(g.h, dev(l), w.N, None, 0, torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda"), None)
        assert e.value.code == B.MADE_ERR_ARG


@pytest.mark.timeout(600)
def test_made_logistic_full_size():
    """The paper's own MADE shape (T = 784, 2 x 512 hidden, 100 samples, logistic conditionals), bf16."""
    w = S.workload("made_logistic")
    net = S.make_network(w)
    exact, same = models(net)
    l = S.make_noise(w)
    sub = 8
    progress("made_logistic: oracle sequential run on a sub-batch")
    xs = L.sequential_sample_real(same, l[:sub])
    rms = float(np.sqrt(np.mean(xs ** 2)))
    with RealGpu(net) as g:
        xq = g.sequential(l, 0)
        xj, it = g.jacobi(l, 0.0)
        assert (xj == xq).all()
        e = close(xj[:sub], xs, X_TOL["bf16"], "jacobi eps=0 vs oracle sequential")
        resid = np.abs(L.jacobi_pass_real(same, xj, l) - xj).max()
        assert resid <= X_TOL["bf16"] * rms
        xe, ite = g.jacobi(l, 1e-2)
        print(f"made_logistic: eps=0 iterations mean {it.mean():.2f} max {it.max()}; eps=1e-2 iterations mean "
              f"{ite.mean():.2f} max {ite.max()}, max deviation from eps=0 {np.abs(xe - xj).max():.2e}; "
              f"error vs oracle {e:.2e} of rms {rms:.2f}, oracle residual {resid:.2e}")
        assert (ite <= it).all() and np.abs(xe - xj).max() <= 0.1
