"""GPU parity of the recurrent-network entry points (include/jacobi_rnn.h) against oracle/rnn_oracle.py on the
same seeded inputs.  Tolerances, relative to the largest entry of the compared tensor: 1e-5 where the GPU
computes in fp32 (forward pass, standard backward pass), 1e-4 where a matrix product takes its operands as two
bf16 parts each (Jacobi passes: ~2^-16 per product) or sums tens of thousands of fp32 terms (parameter gradients)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import rnn_oracle as R
from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S

from gpu_util import dev, progress

pytestmark = pytest.mark.gpu

F32_TOL, SPLIT_TOL = 1e-5, 1e-4


def rel_err(a, ref):
    return float(np.abs(np.asarray(a, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


class Case:
    """Parameters and inputs of one workload; the backward pass gets the oracle's forward results rounded to fp32,
    and the oracle continues from those same fp32 values."""

    def __init__(self, w, rep=0):
        self.w = w
        W, U, b = S.make_rnn_params(w)
        b = (b + 0.05 * np.arange(w.H, dtype=np.float32) / w.H).astype(np.float32)
        x, y = S.make_rnn_inputs(w, rep)
        self.W, self.U, self.b, self.x, self.y = W, U, b, x, y
        z, h = R.rnn_forward(W.astype(np.float64), U.astype(np.float64), b.astype(np.float64), x)
        self.z_ref, self.h_ref = z, h
        self.z32, self.h32 = z.astype(np.float32), h.astype(np.float32)
        self.g32 = (h - y).astype(np.float32)
        self.W64 = W.astype(np.float64)

    def oracle_jacobi(self, n=0, eps=0.0, init=None):
        return R.jacobi_reference(self.W64, self.z32.astype(np.float64), self.g32.astype(np.float64), n, eps, init)

    def oracle_backprop(self):
        return R.backprop_sequential(self.W64, self.z32.astype(np.float64), self.g32.astype(np.float64))

    def gpu_jacobi(self, n=0, eps=0.0, init=None):
        w = self.w
        d = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device="cuda")
        it = torch.full((w.B,), -1, dtype=torch.int32, device="cuda")
        cv = torch.full((w.B,), -1, dtype=torch.int32, device="cuda")
        B.rnn_backward_jacobi(dev(self.W), dev(self.z32), dev(self.g32), None if init is None else dev(init), w.B, w.T, w.H, n,
                              eps, d, it, cv)
        torch.cuda.synchronize()
        return d.cpu().numpy(), it.cpu().numpy(), cv.cpu().numpy()


@pytest.mark.parametrize("name", ["rnn_small", "rnn_wide", "rnn_paper"])
def test_rnn_parity(name):
    w = S.rnn_workload(name)
    c = Case(w)
    progress(f"rnn parity {name}: forward")
    z = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device="cuda")
    h = torch.empty_like(z)
    B.rnn_forward(dev(c.W), dev(c.U), dev(c.b), dev(c.x), None, w.B, w.T, w.H, w.I, z, h)
    torch.cuda.synchronize()
    assert rel_err(z.cpu().numpy(), c.z_ref) <= F32_TOL and rel_err(h.cpu().numpy(), c.h_ref) <= F32_TOL
    h0 = np.random.default_rng(5).uniform(0, 1, (w.B, w.H)).astype(np.float32)
    B.rnn_forward(dev(c.W), dev(c.U), dev(c.b), dev(c.x), dev(h0), w.B, w.T, w.H, w.I, z, h)
    torch.cuda.synchronize()
    z0, h0_ref = R.rnn_forward(c.W64, c.U.astype(np.float64), c.b.astype(np.float64), c.x, h0)
    assert rel_err(z.cpu().numpy(), z0) <= F32_TOL and rel_err(h.cpu().numpy(), h0_ref) <= F32_TOL

    progress(f"rnn parity {name}: standard backward pass")
    d_ref = c.oracle_backprop()
    d = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device="cuda")
    B.rnn_backward_sequential(dev(c.W), dev(c.z32), dev(c.g32), w.B, w.T, w.H, d)
    torch.cuda.synchronize()
    assert rel_err(d.cpu().numpy(), d_ref) <= F32_TOL

    progress(f"rnn parity {name}: Jacobi_n")
    for n in (1, 2, 7, w.T // 2, w.T, 0):
        dj, it, cv = c.gpu_jacobi(n)
        ref, it_ref, cv_ref, _ = c.oracle_jacobi(n)
        assert rel_err(dj, ref) <= SPLIT_TOL, (n, rel_err(dj, ref))
        assert (it == it_ref).all() and (it == (w.T if n in (0, w.T) else n)).all()
        assert (cv == 0).all() or n in (0, w.T)      # eps = 0 is only met if a pass changes nothing at all
    # T passes reproduce the standard backward pass (Proposition 1), and truncation approaches it (Section 5.1)
    dj, _, _ = c.gpu_jacobi(0)
    assert rel_err(dj, d_ref) <= SPLIT_TOL
    errs = [rel_err(c.gpu_jacobi(n)[0], d_ref) for n in (1, 4, 16)]
    assert errs[0] > errs[1] > errs[2]

    progress(f"rnn parity {name}: forward-difference stop, initial iterate")
    scale = np.abs(d_ref).max()
    for eps in (1e-2 * scale, 1e-4 * scale):
        dj, it, cv = c.gpu_jacobi(0, float(eps))
        ref, it_ref, cv_ref, diffs = c.oracle_jacobi(0, float(eps))
        # a sequence whose forward differences all stay clear of eps must stop at the oracle's pass
        clear = np.ones(w.B, dtype=bool)
        for dk in diffs:
            clear &= ~(np.abs(dk - eps) <= 0.05 * eps)
        assert clear.any()
        assert (it[clear] == it_ref[clear]).all() and (cv[clear] == cv_ref[clear]).all(), (eps, it, it_ref)
        assert np.abs(it - it_ref).max() <= 1
        for bi in np.nonzero(clear)[0]:
            assert rel_err(dj[bi], ref[bi]) <= SPLIT_TOL
    init = np.random.default_rng(6).standard_normal((w.B, w.T, w.H)).astype(np.float32)
    for n in (1, 3, 0):
        dj, it, cv = c.gpu_jacobi(n, 0.0, init)
        ref, it_ref, _, _ = c.oracle_jacobi(n, 0.0, init.astype(np.float64))
        assert rel_err(dj, ref) <= SPLIT_TOL * max(1.0, np.abs(init).max() / np.abs(ref).max()) and (it == it_ref).all()

    progress(f"rnn parity {name}: parameter gradients")
    dW = torch.empty((w.H, w.H), dtype=torch.float32, device="cuda")
    dU = torch.empty((w.H, w.I), dtype=torch.float32, device="cuda")
    db = torch.empty((w.H,), dtype=torch.float32, device="cuda")
    d32 = d_ref.astype(np.float32)
    B.rnn_param_grads(dev(c.z32), dev(c.h32), dev(c.x), dev(d32), None, w.B, w.T, w.H, w.I, dW, dU, db)
    torch.cuda.synchronize()
    rW, rU, rb = R.param_grads(c.z32.astype(np.float64), c.h32.astype(np.float64), c.x, d32.astype(np.float64))
    assert rel_err(dW.cpu().numpy(), rW) <= SPLIT_TOL and rel_err(dU.cpu().numpy(), rU) <= SPLIT_TOL
    assert rel_err(db.cpu().numpy(), rb) <= SPLIT_TOL
    B.rnn_param_grads(dev(c.z32), dev(c.h32), dev(c.x), dev(d32), dev(h0), w.B, w.T, w.H, w.I, dW, dU, db)
    torch.cuda.synchronize()
    rW0, _, _ = R.param_grads(c.z32.astype(np.float64), c.h32.astype(np.float64), c.x, d32.astype(np.float64), h0)
    assert rel_err(dW.cpu().numpy(), rW0) <= SPLIT_TOL


def test_rnn_edge_cases():
    # largest shape of the Jacobi call at H = 128, a single step, an empty batch, and the argument errors
    for (Bn, T, H, I) in ((2, 128, 128, 1), (3, 1, 40, 2), (2, 256, 64, 1), (1, 33, 1, 1), (2, 97, 65, 1)):
        progress(f"rnn edge case B={Bn} T={T} H={H}")
        w = dataclasses.replace(S.rnn_workload("rnn_small"), B=Bn, T=T, H=H, I=I, w_std=min(0.2, 1.2 / np.sqrt(H)))
        c = Case(w)
        for n in (0, 3):
            dj, it, cv = c.gpu_jacobi(n)
            ref, it_ref, _, _ = c.oracle_jacobi(n)
            assert rel_err(dj, ref) <= SPLIT_TOL
            # with eps = 0 a sequence ends before the pass limit only if a pass changed nothing at all, and when
            # that happens depends on the arithmetic (fp64 there, fp32 with split products here)
            assert ((it == it_ref) | ((cv == 1) & (it <= it_ref))).all(), (it, it_ref, cv)
        d = torch.empty((Bn, T, H), dtype=torch.float32, device="cuda")
        B.rnn_backward_sequential(dev(c.W), dev(c.z32), dev(c.g32), Bn, T, H, d)
        torch.cuda.synchronize()
        assert rel_err(d.cpu().numpy(), c.oracle_backprop()) <= F32_TOL
    w = S.rnn_workload("rnn_small")
    c = Case(w)
    empty = torch.empty((0, w.T, w.H), dtype=torch.float32, device="cuda")
    B.rnn_backward_jacobi(dev(c.W), empty, empty, None, 0, w.T, w.H, 0, 0.0, empty)
    B.rnn_backward_sequential(dev(c.W), empty, empty, 0, w.T, w.H, empty)
    d = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device="cuda")
    for call in (lambda: B.rnn_backward_jacobi(dev(c.W), dev(c.z32), dev(c.g32), None, w.B, 200, 100, 0, 0.0, d),
                 lambda: B.rnn_backward_jacobi(dev(c.W), dev(c.z32), dev(c.g32), None, w.B, w.T, w.H, 0, -1.0, d),
                 lambda: B.rnn_backward_jacobi(dev(c.W), dev(c.z32), dev(c.g32), None, w.B, w.T, 129, 0, 0.0, d),
                 lambda: B.rnn_backward_sequential(dev(c.W), None, dev(c.g32), w.B, w.T, w.H, d)):
        with pytest.raises(B.MadeError) as e:
            call()
        assert e.value.code == B.MADE_ERR_ARG


def test_rnn_full_batch():
    """256 sequences of the paper's shape in one call (the launch bench.py times); the oracle checks a sample of them."""
    w = S.rnn_workload("rnn_batch")
    c = Case(w)
    progress("rnn full batch: Jacobi_10, Jacobi_T, standard backward pass")
    d_ref = c.oracle_backprop()
    for n in (10, 0):
        dj, it, cv = c.gpu_jacobi(n)
        ref, it_ref, _, _ = c.oracle_jacobi(n)
        assert rel_err(dj, ref) <= SPLIT_TOL and (it == it_ref).all()
    d = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device="cuda")
    B.rnn_backward_sequential(dev(c.W), dev(c.z32), dev(c.g32), w.B, w.T, w.H, d)
    torch.cuda.synchronize()
    assert rel_err(d.cpu().numpy(), d_ref) <= F32_TOL
