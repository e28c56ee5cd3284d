"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Symbols must be bit-exact except where the oracle's decision margin is below 1e-3;
logits agree to 1e-4 (fp32 path) / 2e-2 (bf16 path) of the tensor's rms."""
import numpy as np
import pytest
import torch

from oracle import made_oracle as O
from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S

from gpu_util import (LOGIT_TOL, MARGIN, GpuModel, assert_counts_match, assert_logits_close, assert_sample_parity, dev,
                      mlp_layer_certificate, oracle_models, progress)

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["per-layer launches", "single chain", "persistent", "sample-resident",
                                      "library defaults", "unfused categorical", "xcd-resident", "tail-less stop test"])
def execution_path(request):
    """Every test runs on every execution path of the library (they must all agree with the oracle)."""
    import gpu_util
    if request.param == "unfused categorical":
        name = getattr(request.node, "callspec", None) and request.node.callspec.params.get("name")
        if name not in ("small_cat", "small_cat_onehot"):
            pytest.skip("only the 256-class workloads have a fused and an unfused output path")
    if request.param in ("sample-resident", "xcd-resident", "tail-less stop test"):
        name = getattr(request.node, "callspec", None) and request.node.callspec.params.get("name")
        if name is not None and "cat" in name:
            pytest.skip("the sample-resident and XCD-resident kernels and the tail-less stop test serve Bernoulli models only")
    gpu_util.PERSISTENT = request.param == "persistent"
    gpu_util.RESIDENT = 1 if request.param == "sample-resident" else (2 if request.param == "library defaults" else 0)
    gpu_util.FUSED_CATEGORICAL = request.param != "unfused categorical"
    gpu_util.CHAINS = 1 if request.param in ("single chain", "library defaults", "tail-less stop test") else 4
    # (the list of a pass derived by its own first kernel: Jacobi on one chain of per-layer launches)
    gpu_util.LAZY = 1 if request.param == "tail-less stop test" else (None if request.param == "library defaults" else 0)
    gpu_util.RETIRE_SPLIT = 1 if request.param == "single chain" else None   # (the stop test as its own kernel)
    gpu_util.XCD = 2 if request.param == "xcd-resident" else (None if request.param == "library defaults" else 0)
    yield
    gpu_util.LAZY = None
    gpu_util.XCD = 0
    gpu_util.RETIRE_SPLIT = None
    gpu_util.PERSISTENT = False
    gpu_util.RESIDENT = 0
    gpu_util.FUSED_CATEGORICAL = True
    gpu_util.CHAINS = 4


SMALL = ["cfg1", "small_f32", "small_bf16", "mid_bf16", "small_cat", "small_cat_f32", "small_cat_onehot",
         "small_cat_onehot_f32", "mid_cat_onehot", "wide_cat_onehot", "wide_cat_onehot_f32"]


def _symbols(w, rng, N):
    hi = 2 if w.C == 1 else w.C
    return rng.integers(0, hi, size=(N, w.D)).astype(np.uint8)


@pytest.mark.parametrize("name", SMALL)
def test_forward_logits(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    exact, same = oracle_models(net)
    x = _symbols(w, np.random.default_rng(1), w.N)
    with GpuModel(net) as g:
        z = g.logits(x)
    assert_logits_close(z, O.logits_all(exact, x), LOGIT_TOL[w.dtype])
    # against the oracle that rounds hidden activations the same way only fp32 summation order remains
    assert_logits_close(z, O.logits_all(same, x), 2e-3 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("name", SMALL)
def test_every_layer_on_its_own(name):
    """The layer-by-layer certificate: each masked layer, fed the library's own previous layer, against the oracle's
    layer -- bit-exact bf16 activations except within the fp32 accumulation error of a rounding boundary."""
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    x = _symbols(w, np.random.default_rng(7), w.N)
    with GpuModel(net) as g:
        worst = mlp_layer_certificate(g, same, x)
    print(f"{name}: worst accumulation error {worst:.2f} x 2^-24 sum|a w|")


@pytest.mark.parametrize("name", SMALL)
def test_jacobi_matches_sequential_oracle(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    noise = S.make_noise(w)
    xs, margins = O.sequential_sample(same, noise)
    xr, it_ref, _, _, mm = O.jacobi_reference(same, noise)
    with GpuModel(net) as g:
        x, it = g.jacobi(noise)
        st = g.stats()
        x2, it2 = g.jacobi(noise)                       # determinism: same symbols and same counts
        assert (x2 == x).all() and (it2 == it).all()
        hi = 2 if w.C == 1 else w.C
        for init in (np.full((w.N, w.D), hi - 1, np.uint8), _symbols(w, np.random.default_rng(2), w.N), xs):
            xi, iti = g.jacobi(noise, init)
            assert_sample_parity(same, noise, xi, xs, margins)
            ref_i = O.jacobi_reference(same, noise, init)
            assert_counts_match(iti, ref_i[1], ref_i[4])
    assert_sample_parity(same, noise, x, xs, margins)
    assert (it >= 1).all() and (it <= w.D).all()
    assert_counts_match(it, it_ref, mm)
    assert st["passes"] == it.max() and st["sample_passes"] == it.sum()


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("mode", [0, 1])
def test_sequential_matches_oracle(name, mode):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    noise = S.make_noise(w)
    xs, margins = O.sequential_sample(same, noise)
    with GpuModel(net) as g:
        x = g.sequential(noise, mode)
    assert_sample_parity(same, noise, x, xs, margins)


@pytest.mark.parametrize("name", SMALL)
def test_gs_jacobi_every_block_size(name):
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    noise = S.make_noise(w)
    xs, margins = O.sequential_sample(same, noise)
    with GpuModel(net) as g:
        for block in [1, 5, 16, 33, w.D - 1, w.D, w.D + 7]:
            x, it = g.gs_jacobi(noise, block)
            assert_sample_parity(same, noise, x, xs, margins)
            xr, it_ref, per_block, mm = O.gs_jacobi_reference(same, noise, block)
            assert_counts_match(it, it_ref, mm)
            if block == 1:
                assert (it == w.D).all()
        init = _symbols(w, np.random.default_rng(3), w.N)
        x, it = g.gs_jacobi(noise, 7, init)
        assert_sample_parity(same, noise, x, xs, margins)
        ref = O.gs_jacobi_reference(same, noise, 7, init)
        assert_counts_match(it, ref[1], ref[3])
        # the frozen-prefix reuse changes no bit: same symbols and pass counts with it switched off
        B.made_set_option(g.h, B.MADE_OPT_PREFIX_CACHE, 1)
        x_on, it_on = g.gs_jacobi(noise, 16)
        B.made_set_option(g.h, B.MADE_OPT_PREFIX_CACHE, 0)
        x_off, it_off = g.gs_jacobi(noise, 16)
        assert (x_on == x_off).all() and (it_on == it_off).all()
        # the partial-sum cache (forced on at this small batch) re-orders fp32 sums: same parity bar as every path
        if w.C == 1:
            B.made_set_option(g.h, B.MADE_OPT_PREFIX_CACHE, 2)
            B.made_set_option(g.h, B.MADE_OPT_PARTIAL_SUM_BATCH, 1)
            for block in (5, 16, 33, w.D - 1):
                x, it = g.gs_jacobi(noise, block)
                assert_sample_parity(same, noise, x, xs, margins)
                ref = O.gs_jacobi_reference(same, noise, block)
                assert_counts_match(it, ref[1], ref[3])
            xi, iti = g.gs_jacobi(noise, 7, init)
            assert_sample_parity(same, noise, xi, xs, margins)


@pytest.mark.parametrize("name", ["cfg1", "small_f32", "small_bf16", "mid_bf16"])
def test_jacobi_gs_every_block_size(name):
    """Algorithm 2 against its oracle: same result as the sequential sampler, same iteration counts."""
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    noise = S.make_noise(w)
    xs, margins = O.sequential_sample(same, noise)
    with GpuModel(net) as g:
        for block in [1, 5, 16, 33, w.D - 1, w.D, w.D + 7]:
            progress(f"jacobi_gs {name} block {block}")
            x, it = g.jacobi_gs(noise, block)
            assert_sample_parity(same, noise, x, xs, margins)
            xr, it_ref, done, mm = O.jacobi_gs_reference(same, noise, block)
            assert_counts_match(it, it_ref, mm)
            M = -(-w.D // min(block, w.D))
            assert (it >= 1).all() and (it <= M).all()
            if block >= w.D:
                assert (it == 1).all()
        init = _symbols(w, np.random.default_rng(3), w.N)
        x, it = g.jacobi_gs(noise, 7, init)
        assert_sample_parity(same, noise, x, xs, margins)
        ref = O.jacobi_gs_reference(same, noise, 7, init)
        assert_counts_match(it, ref[1], ref[3])
        # an iteration limit below M: the iterate after one iteration, and the not-converged status
        ref1 = O.jacobi_gs_reference(same, noise, 7, None, 1)
        if not ref1[2].all() and (ref1[3] >= MARGIN).all():
            with pytest.raises(B.MadeError) as e:
                g.jacobi_gs(noise, 7, None, 1)
            assert e.value.code == B.MADE_ERR_NOT_CONVERGED


def test_jacobi_gs_rejects_unsupported_models():
    w = S.workload("small_cat_f32")
    net = S.make_network(w)
    with GpuModel(net) as g:
        with pytest.raises(B.MadeError) as e:
            g.jacobi_gs(S.make_noise(w), 4)
        assert e.value.code == B.MADE_ERR_ARG


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_section4_1_examples_on_gpu(dtype):
    # Example 1: independent positions -> right after one pass, confirmed by the second
    net = S.independent_network(40, 70, seed=9, dtype=dtype)
    _, same = oracle_models(net)
    u = S.uniform_noise(33, 40, 1)
    xs, mg = O.sequential_sample(same, u)
    with GpuModel(net) as g:
        x, it = g.jacobi(u, 1 - xs)
    assert_sample_parity(same, u, x, xs, mg)
    assert (it[mg.min(axis=1) >= MARGIN] == 2).all()
    # Example 2: everything hangs on position 1 -> right after two passes
    net = S.first_only_network(40, 70, seed=10, dtype=dtype)
    _, same = oracle_models(net)
    xs, mg = O.sequential_sample(same, u)
    ref = O.jacobi_reference(same, u)
    with GpuModel(net) as g:
        x, it = g.jacobi(u)
    assert_sample_parity(same, u, x, xs, mg)
    clear = ref[4] >= MARGIN
    assert (it[clear] == ref[1][clear]).all() and it.max() <= 3
    # Example 3: Markov chain -> exactly T passes, ended by the k = T clause
    T = 45
    net = S.copy_chain_network(T, dtype=dtype)
    u = S.uniform_noise(5, T, 3) * 0.98 + 0.01
    with GpuModel(net) as g:
        x, it = g.jacobi(u)
        assert (x == 1).all() and (it == T).all()
        with pytest.raises(B.MadeError) as e:
            g.jacobi(u, None, 10)
        assert e.value.code == B.MADE_ERR_NOT_CONVERGED
        x, it = g.gs_jacobi(u, 8)
        assert (x == 1).all() and (it == T).all()
        assert (g.sequential(u, 0) == 1).all() and (g.sequential(u, 1) == 1).all()


def test_edge_cases():
    w = S.workload("small_bf16")
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    with GpuModel(net) as g:
        # empty batch: nothing to do, nothing touched
        empty = torch.empty((0, w.D), dtype=torch.uint8, device="cuda")
        B.jacobi_sample(g.h, torch.empty((0, w.D), device="cuda"), 0, None, 0, empty, None)
        B.gs_jacobi_sample(g.h, torch.empty((0, w.D), device="cuda"), 0, None, 4, empty, None)
        B.sequential_sample(g.h, torch.empty((0, w.D), device="cuda"), 0, 0, empty)
        # batch sizes around the 32-row tile, growing and shrinking (workspace reuse)
        for N in (1, 31, 32, 33, 97, 5):
            noise = S.make_noise(w, rep=N, N=N)
            xs, mg = O.sequential_sample(same, noise)
            x, it = g.jacobi(noise)
            assert_sample_parity(same, noise, x, xs, mg)
        # argument errors come back as status codes
        noise = dev(S.make_noise(w))
        x = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
        for call in (lambda: B.gs_jacobi_sample(g.h, noise, w.N, None, 0, x, None),
                     lambda: B.sequential_sample(g.h, noise, w.N, 2, x),
                     lambda: B.jacobi_sample(g.h, None, w.N, None, 0, x, None),
                     lambda: B.jacobi_sample(g.h, noise, -1, None, 0, x, None)):
            with pytest.raises(B.MadeError) as e:
                call()
            assert e.value.code == B.MADE_ERR_ARG
        # x_out may alias x_init
        init = dev(np.random.default_rng(0).integers(0, 2, (w.N, w.D)).astype(np.uint8))
        B.jacobi_sample(g.h, noise, w.N, init, 0, init, None)
        xs, mg = O.sequential_sample(same, S.make_noise(w))
        assert_sample_parity(same, S.make_noise(w), init.cpu().numpy(), xs, mg)
    with pytest.raises(B.MadeError):
        B.made_init(1, 1, [4], B.MADE_F32, [np.ones(4, np.int32)], [np.zeros((4, 1)), np.zeros((1, 4))])
    with pytest.raises(B.MadeError):     # degree outside [1, D-1]
        B.made_init(4, 1, [3], B.MADE_F32, [np.array([1, 2, 4], np.int32)], [np.zeros((3, 4)), np.zeros((4, 3))])


@pytest.mark.parametrize("tile", [256, 128])
@pytest.mark.parametrize("name,N", [("mid_bf16", 700), ("small_f32", 300), ("small_bf16", 515)])
def test_large_batch_uses_big_tiles(name, N, tile):
    """Large batches run the layers with 256 x 256 (or, below that threshold, 128 x 128) workgroup tiles (the
    thresholds are lowered to 256 / 128 samples here so that the oracle stays cheap); same parity bar."""
    import dataclasses
    w = dataclasses.replace(S.workload(name), N=N)
    net = S.make_network(w, with_bias=True)
    exact, same = oracle_models(net)
    noise = S.make_noise(w)
    x0 = _symbols(w, np.random.default_rng(4), N)
    xs, margins = O.sequential_sample(same, noise)
    ref = O.jacobi_reference(same, noise)
    with GpuModel(net, big_tile_batch=256 if tile == 256 else 1 << 30, mid_tile_batch=128 if tile == 128 else None) as g:
        z = g.logits(x0)
        assert_logits_close(z, O.logits_all(exact, x0), LOGIT_TOL[w.dtype])
        x, it = g.jacobi(noise)
        assert_sample_parity(same, noise, x, xs, margins)
        assert_counts_match(it, ref[1], ref[4])
        xb, itb = g.gs_jacobi(noise, 33)
        assert_sample_parity(same, noise, xb, xs, margins)
        xq = g.sequential(noise, 1)
        assert_sample_parity(same, noise, xq, xs, margins)


@pytest.mark.parametrize("name", ["small_bf16", "mid_bf16", "small_cat_f32"])
def test_back_to_back_calls_without_synchronisation(name):
    """The sampling calls return before the stream has drained (a speculative, empty pass may still be queued).
    Many calls in a row, on one stream and alternating between two, with different noise, batch sizes and initial
    iterates and no synchronisation in between, must each give the result they give on their own."""
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    _, same = oracle_models(net)
    hi = 2 if w.C == 1 else w.C
    cases = []
    for r in range(12):
        N = [w.N, 5, 33, w.N, 1, 64][r % 6]
        noise = S.make_noise(w, rep=r, N=N)
        init = None if r % 3 else np.random.default_rng(r).integers(0, hi, (N, w.D)).astype(np.uint8)
        cases.append((N, noise, init))
    with GpuModel(net) as g:
        alone = []
        for N, noise, init in cases:                      # every call on its own, synchronised
            x, it = g.jacobi(noise, init)
            assert_sample_parity(same, noise, x)
            alone.append((x, it))
        side = torch.cuda.Stream()
        for streams in ([None] * len(cases), [None if i % 2 else side for i in range(len(cases))]):
            outs = []
            for (N, noise, init), st in zip(cases, streams):
                un, xin = dev(noise), (None if init is None else dev(init))
                x = torch.empty((N, w.D), dtype=torch.uint8, device="cuda")
                it = torch.empty((N,), dtype=torch.int32, device="cuda")
                if st is not None:
                    st.wait_stream(torch.cuda.current_stream())      # the inputs were uploaded on the current stream
                B.jacobi_sample(g.h, un, N, xin, 0, x, it, st)
                outs.append((x, it, un, xin))
            torch.cuda.synchronize()
            for (x, it, _, _), (xa, ita) in zip(outs, alone):
                assert (x.cpu().numpy() == xa).all() and (it.cpu().numpy() == ita).all()
        # GS-Jacobi and the sequential sampler interleaved with Jacobi, same stream, one synchronisation at the end
        N, noise, _ = cases[0]
        un = dev(noise)
        res = []
        for call in ("gs", "jacobi", "seq", "gs", "jacobi"):
            x = torch.empty((N, w.D), dtype=torch.uint8, device="cuda")
            it = torch.zeros((N,), dtype=torch.int32, device="cuda")
            if call == "gs":
                B.gs_jacobi_sample(g.h, un, N, None, 7, x, it)
            elif call == "jacobi":
                B.jacobi_sample(g.h, un, N, None, 0, x, it)
            else:
                B.sequential_sample(g.h, un, N, 1, x)
            res.append(x)
        torch.cuda.synchronize()
        for x in res:
            assert (x.cpu().numpy() == alone[0][0]).all()


def test_xcd_resident_kernel_serves_the_call():
    """With MADE_OPT_XCD_RESIDENT = 2 a Bernoulli call is ONE launch, not three launches per pass: the kernel did not back out, and its results are those of the per-layer launches bit for bit."""
    import gpu_util
    if gpu_util.XCD != 2:
        pytest.skip("runs once, on the XCD-resident execution path")
    for name in ("mid_bf16", "small_f32", "cfg1"):
        w = S.workload(name)
        net = S.make_network(w, with_bias=True)
        noise = S.make_noise(w)
        with GpuModel(net) as g:
            x, it = g.jacobi(noise)
            st = g.stats()
            assert st["kernels"] == 1, (st, B.made_last_error())
            xb, itb = g.gs_jacobi(noise, 16)
            assert g.stats()["kernels"] == 1
            B.made_set_option(g.h, B.MADE_OPT_XCD_RESIDENT, 0)
            B.made_set_option(g.h, B.MADE_OPT_RESIDENT, 0)
            x2, it2 = g.jacobi(noise)
            assert g.stats()["kernels"] > 1
            xb2, itb2 = g.gs_jacobi(noise, 16)
            assert (x == x2).all() and (it == it2).all() and st["passes"] == it.max() and st["sample_passes"] == it.sum()
            assert (xb == xb2).all() and (itb == itb2).all()


def test_tail_less_stop_test_serves_the_call_and_changes_nothing():
    """MADE_OPT_LAZY_STOP_TEST = 1: every pass but a call's last allowed one has no tail (the next pass derives its
    list), and symbols, per-sample pass counts and the call's statistics are those of the tail, bit for bit -- from
    zeros, from a random start, and when the pass limit cuts the call short."""
    import gpu_util
    if gpu_util.LAZY != 1:
        pytest.skip("runs once, on the tail-less execution path")
    for name in ("mid_bf16", "small_f32", "small_bf16", "cfg1"):
        w = S.workload(name)
        net = S.make_network(w, with_bias=True)
        noise = S.make_noise(w)
        x0 = _symbols(w, np.random.default_rng(9), w.N)
        with GpuModel(net) as g:
            for init, limit in ((None, 0), (x0, 0), (None, 2), (x0, 3)):
                res = {}
                for lazy in (1, 0):
                    B.made_set_option(g.h, B.MADE_OPT_LAZY_STOP_TEST, lazy)
                    x = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
                    it = torch.full((w.N,), -7, dtype=torch.int32, device="cuda")
                    code = 0
                    try:
                        B.jacobi_sample(g.h, dev(noise), w.N, None if init is None else dev(init), limit, x, it)
                    except B.MadeError as e:
                        code = e.code
                    torch.cuda.synchronize()
                    st = g.stats()
                    res[lazy] = (x.cpu().numpy(), it.cpu().numpy(), code, st)
                    if lazy and limit == 0:
                        assert st["tail_less_passes"] >= st["passes"] >= 1, st     # (every pass, the speculative one included)
                    elif lazy:
                        assert 0 < st["tail_less_passes"] <= limit - 1, st        # (the last allowed pass keeps its tail)
                    else:
                        assert st["tail_less_passes"] == 0
                a, b = res[1], res[0]
                assert (a[0] == b[0]).all() and (a[1] == b[1]).all() and a[2] == b[2], (name, limit)
                assert a[3]["passes"] == b[3]["passes"] and a[3]["sample_passes"] == b[3]["sample_passes"]
                if limit:
                    assert a[2] in (0, B.MADE_ERR_NOT_CONVERGED)


def test_zero_start_saves_a_launch_and_changes_nothing():
    """MADE_OPT_ZERO_START: started from zeros, the first pass's first hidden layer is ReLU(bias) for every sample and
    the set-up kernel writes it.  Symbols, pass counts and statistics are those of the launched layer, bit for bit
    (with and without bias, one and several hidden layers), with one kernel less; a call with an
    x_init launches the layer as before."""
    import gpu_util
    if gpu_util.CHAINS != 1 or gpu_util.PERSISTENT or gpu_util.RESIDENT or gpu_util.XCD != 0:
        pytest.skip("runs once, on one chain of per-layer launches")
    cases = [("small_f32", None, True), ("small_bf16", None, True), ("mid_bf16", None, False), ("cfg1", None, True),
             ("cfg2", None, True), ("small_bf16", 32, True)]
    for name, big, with_bias in cases:
        w = S.workload(name)
        net = S.make_network(w, with_bias=with_bias)
        noise = S.make_noise(w)
        x0 = _symbols(w, np.random.default_rng(5), w.N)
        kw = {} if big is None else {"big_tile_batch": big, "mid_tile_batch": big}
        with GpuModel(net, **kw) as g:
            res = {}
            for fill in (1, 0):
                B.made_set_option(g.h, B.MADE_OPT_ZERO_START, fill)
                x, it = g.jacobi(noise)
                torch.cuda.synchronize()
                st = g.stats()
                xl, itl = g.jacobi(noise, max_iters=w.D)
                xi, iti = g.jacobi(noise, x_init=x0)
                torch.cuda.synchronize()
                sti = g.stats()
                # a call of exactly one pass (nothing speculative): its kernel count is fixed
                x1 = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
                try:
                    B.jacobi_sample(g.h, dev(noise), w.N, None, 1, x1, None)
                except B.MadeError as e:
                    assert e.code == B.MADE_ERR_NOT_CONVERGED
                torch.cuda.synchronize()
                res[fill] = (x, it, st, xl, itl, xi, iti, sti, x1.cpu().numpy(), g.stats()["kernels"])
            a, b = res[1], res[0]
            for i in (0, 1, 3, 4, 5, 6, 8):
                assert (a[i] == b[i]).all(), (name, big, i)
            assert a[2]["passes"] == b[2]["passes"] and a[2]["sample_passes"] == b[2]["sample_passes"]
            assert a[7]["passes"] == b[7]["passes"] and a[7]["sample_passes"] == b[7]["sample_passes"]
            # (batches that the large tile kernels serve launch the layer: writing its activations costs as much)
            assert a[9] == b[9] - (0 if big else 1), (name, big, a[9], b[9])


@pytest.mark.parametrize("name", ["small_cat", "small_cat_onehot", "mid_cat_onehot"])
def test_frozen_positions_change_nothing_but_the_work(name):
    """MADE_OPT_FROZEN_POSITIONS: a pass of the 256-class output kernel skips the positions below the first one the
    pass before changed.  Symbols and pass counts are those of full passes, for Jacobi (zeros and a random start)
    and GS-Jacobi; the weights the passes multiply are fewer."""
    import gpu_util
    if gpu_util.CHAINS != 1 or not gpu_util.FUSED_CATEGORICAL or gpu_util.RETIRE_SPLIT is not None:
        pytest.skip("runs on the single-chain paths with the fused output kernel")
    w = S.workload(name)
    net = S.make_network(w, with_bias=True)
    noise = S.make_noise(w)
    x0 = _symbols(w, np.random.default_rng(12), w.N)
    with GpuModel(net) as g:
        res = {}
        for frozen in (1, 0):
            B.made_set_option(g.h, B.MADE_OPT_FROZEN_POSITIONS, frozen)
            x, it = g.jacobi(noise)
            torch.cuda.synchronize()
            st = g.stats()
            xi, iti = g.jacobi(noise, x_init=x0)
            xb, itb = g.gs_jacobi(noise, 5)
            res[frozen] = (x, it, st, xi, iti, xb, itb)
        a, b = res[1], res[0]
        for i in (0, 1, 3, 4, 5, 6):
            assert (a[i] == b[i]).all(), i
        assert a[2]["passes"] == b[2]["passes"] and a[2]["sample_passes"] == b[2]["sample_passes"]
        if w.C != 256:            # (other class counts take the unfused path: nothing to skip, nothing counted)
            assert a[2]["output_weights_evaluated"] == 0
            return
        assert 0 < a[2]["output_weights_evaluated"] <= b[2]["output_weights_evaluated"]
        if a[2]["passes"] >= 3:
            assert a[2]["output_weights_evaluated"] < b[2]["output_weights_evaluated"], (a[2], b[2])
