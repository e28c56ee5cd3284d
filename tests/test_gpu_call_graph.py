"""MADE_OPT_CALL_GRAPH: a Jacobi call recorded as a HIP graph gives, on every replay, what the launch-by-launch call
gives (whose parity with the oracle the other GPU tests establish): symbols, per-sample pass counts, return code and
the call's pass statistics -- with other contents in the same buffers, with more passes needed than were recorded,
with the pass limit cutting the call short, and with unrelated work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S
from gpu_util import GpuModel, progress

pytestmark = pytest.mark.gpu


def _call(g, w, noise_d, x0_d, limit, x_d, it_d, stream):
    code = 0
    try:
        B.jacobi_sample(g.h, noise_d, w.N, x0_d, limit, x_d, it_d, stream=stream)
    except B.MadeError as e:
        code = e.code
    stream.synchronize()
    return x_d.cpu().numpy().copy(), it_d.cpu().numpy().copy(), code, g.stats()


@pytest.mark.parametrize("name", ["mid_bf16", "small_f32", "cfg1", "cfg2"])
def test_recorded_calls_replay_to_the_results_of_single_launches(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    rng = np.random.default_rng(31)
    hi = 2 if w.C == 1 else w.C
    # contents the same buffers take in turn: noise rep 0 from zeros-like start, rep 1 from a random start (more or
    # fewer passes), rep 2 from a start that is already the solution of rep 0 (one pass)
    contents = [(S.make_noise(w, rep=r), rng.integers(0, hi, size=(w.N, w.D)).astype(np.uint8)) for r in range(3)]
    stream = torch.cuda.Stream()
    with GpuModel(net) as g:
        B.made_set_option(g.h, B.MADE_OPT_CHAINS, 1)
        B.made_set_option(g.h, B.MADE_OPT_XCD_RESIDENT, 0)
        B.made_set_option(g.h, B.MADE_OPT_RESIDENT, 0)
        B.made_set_option(g.h, B.MADE_OPT_PERSISTENT, 0)
        B.made_set_option(g.h, B.MADE_OPT_LAZY_STOP_TEST, 1)
        noise_d = torch.empty((w.N, w.D), dtype=torch.float32, device="cuda")
        x0_d = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
        x_d = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
        it_d = torch.empty((w.N,), dtype=torch.int32, device="cuda")
        junk = torch.randn(1 << 20, device="cuda")

        def load(c):
            with torch.cuda.stream(stream):
                noise_d.copy_(torch.from_numpy(contents[c][0]), non_blocking=False)
                x0_d.copy_(torch.from_numpy(contents[c][1]), non_blocking=False)
                x_d.fill_(7)
                it_d.fill_(-7)
            stream.synchronize()

        for with_init, limit in ((False, 0), (True, 0), (True, 3)):
            # launch by launch
            B.made_set_option(g.h, B.MADE_OPT_CALL_GRAPH, 0)
            want = []
            for c in range(3):
                load(c)
                want.append(_call(g, w, noise_d, x0_d if with_init else None, limit, x_d, it_d, stream))
            if with_init and limit == 0:   # content 2: start at content 0's solution under content 0's noise
                contents[2] = (contents[0][0], want[0][0])
                load(2)
                want[2] = _call(g, w, noise_d, x0_d, limit, x_d, it_d, stream)
                assert want[2][3]["passes"] == 1
            # recorded: both halves of the pass log see every content several times, in changing order
            B.made_set_option(g.h, B.MADE_OPT_CALL_GRAPH, 1)
            order = [0, 0, 0, 0, 1, 1, 1, 1, 2, 2, 0, 1, 2, 0, 0, 1, 1, 1]
            replays = 0
            for i, c in enumerate(order):
                load(c)
                (junk * 1.0001).sum().item()                      # unrelated work and a synchronisation in between
                x, it, code, st = _call(g, w, noise_d, x0_d if with_init else None, limit, x_d, it_d, stream)
                ex, eit, ecode, est = want[c]
                assert code == ecode, (name, with_init, limit, i, c)
                assert (x == ex).all() and (it == eit).all(), (name, with_init, limit, i, c)
                assert st["passes"] == est["passes"] and st["sample_passes"] == est["sample_passes"], (i, c, st, est)
                # (a recorded call's last pass keeps its tail: one tail-less pass fewer than passes recorded)
                if st["tail_less_passes"] < est["tail_less_passes"]:
                    replays += 1
            progress(f"{name} init={with_init} limit={limit}: {replays} of {len(order)} calls took the recorded form")
            if limit == 0:   # (under a pass limit the launch-by-launch call's last pass has a tail as well)
                assert replays >= 8
        B.made_set_option(g.h, B.MADE_OPT_CALL_GRAPH, 0)


def test_a_prepared_call_is_the_plain_call():
    """binding.PreparedJacobi marshals the arguments once; every call of the object is jacobi_sample on them."""
    w = S.workload("mid_bf16")
    net = S.make_network(w, with_bias=True)
    stream = torch.cuda.Stream()
    with GpuModel(net) as g:
        noise_d = torch.from_numpy(S.make_noise(w)).cuda()
        x_a = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
        it_a = torch.empty((w.N,), dtype=torch.int32, device="cuda")
        x_b, it_b = torch.empty_like(x_a), torch.empty_like(it_a)
        torch.cuda.synchronize()
        B.jacobi_sample(g.h, noise_d, w.N, None, 0, x_a, it_a, stream=stream)
        call = B.PreparedJacobi(g.h, noise_d, w.N, None, 0, x_b, it_b, stream=stream)
        for rep in range(3):
            x_b.fill_(9)
            torch.cuda.synchronize()
            call()
            stream.synchronize()
            assert (x_a == x_b).all() and (it_a == it_b).all(), rep
            noise_d.copy_(torch.from_numpy(S.make_noise(w, rep=rep + 1)))     # (contents may change between calls)
            torch.cuda.synchronize()
            B.jacobi_sample(g.h, noise_d, w.N, None, 0, x_a, it_a, stream=stream)
            stream.synchronize()
        limited = B.PreparedJacobi(g.h, noise_d, w.N, None, 1, x_b, it_b, stream=stream)
        with pytest.raises(B.MadeError) as e:
            limited()
        assert e.value.code == B.MADE_ERR_NOT_CONVERGED
