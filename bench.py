#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: Jacobi sampling (Algorithm 1) of the MNIST-shaped
binary MADE (D = 784, 2 x 2000 hidden, bf16, batch 128), synthetic seeded weights and noise.

One "step" = one jacobi_sample call on one batch whose noise is already resident in HBM: every
pass of the whole masked network, the sampling epilogue, the per-sample stop test and the final
synchronisation are inside the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3


def cpu_baseline(w, net, noises, budget_s=12.0, single_thread_s=0.0):
    """The numpy oracle's sequential sampler, as it stands, on a bounded sample of the workload: whole batches
    (different noise each) until about budget_s seconds of CPU work are done, at least one batch."""
    from oracle import made_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    model = O.build_model(net.D, net.C, net.degrees, net.W, net.b, "bf16" if net.dtype == "bf16" else None,
                          getattr(net, "onehot", False))
    sub = noises[0].shape[0] if net.D * net.C < (1 << 16) else min(8, noises[0].shape[0])   # huge models: 8 samples
    O.sequential_sample(model, noises[0][:1])              # warm the BLAS threads
    done, xs0 = 0, None
    t0 = time.perf_counter()
    for r in range(len(noises)):
        xs, _ = O.sequential_sample(model, noises[r][:sub])
        if r == 0:
            xs0 = xs
        done += sub
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    base = {"value": done / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle sequential_sample (numpy fp64, activations rounded as on the GPU) on {done} samples "
                      f"({done // sub} x {sub} of a batch of {noises[0].shape[0]}), {dt:.1f} s"}
    if single_thread_s > 0:
        # the same oracle held to one thread (the other mode a CPU baseline is usually quoted in), on a smaller sample
        try:
            from threadpoolctl import threadpool_limits
            n1 = max(1, min(sub, 16))
            with threadpool_limits(limits=1):
                t1 = time.perf_counter()
                reps1 = 0
                while reps1 == 0 or time.perf_counter() - t1 < single_thread_s:
                    O.sequential_sample(model, noises[0][:n1])
                    reps1 += 1
                d1 = time.perf_counter() - t1
            base["single_thread"] = {"value": reps1 * n1 / d1, "unit": "samples/s", "cores": 1,
                                     "sample": f"{reps1} x {n1} samples, {d1:.1f} s"}
        except Exception as e:   # (threadpoolctl missing: the figure is left out)
            base["single_thread"] = {"error": str(e)}
    return base, xs0, sub



def own_stream(torch):
    """The benchmark runs on a stream of its own (default priority), made current so that torch's work is ordered with the
    library's.  Measured on the MI355X boxes: back-to-back calls of the launch-bound configurations take 1-3 % less on
    such a stream than on the default stream (0.095 against 0.0975 ms per call on cfg2)."""
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    return stream

def coupling_sweep(w, torch, B, S, stream):
    """Supplementary (not a benchmark configuration): how the number of Jacobi passes, and with it the speed-up over
    the sequential sampler, depends on how strongly the states are coupled (Section 4.1: learned weights leave few
    long dependency chains; these random ones are scaled up instead).  The workload's network with every weight
    multiplied by gamma, and the Markov copy chain of Section 4.1's third example (exactly T passes) at T = D."""
    import dataclasses
    out = {}
    cases = [(f"gamma{g:g}", dataclasses.replace(w, gain=w.gain * g), None) for g in (1.0, 4.0, 16.0, 64.0)]
    cases.append(("copy_chain_T%d" % w.D, None, S.copy_chain_network(w.D, dtype=w.dtype)))
    for name, wg, net in cases:
        if net is None:
            net = S.make_network(wg)
            u = torch.from_numpy(S.make_noise(wg)).cuda()
        else:
            u = torch.from_numpy(S.uniform_noise(w.N, w.D, w.seed + 2) * 0.98 + 0.01).cuda()
        h = B.model_from_network(net)
        try:
            x = torch.empty((w.N, w.D), dtype=torch.uint8, device="cuda")
            xq = torch.empty_like(x)
            it = torch.empty((w.N,), dtype=torch.int32, device="cuda")
            B.jacobi_sample(h, u, w.N, None, 0, x, it, stream)
            torch.cuda.synchronize()
            reps = 5
            t0 = time.perf_counter()
            for _ in range(reps):
                B.jacobi_sample(h, u, w.N, None, 0, x, it, stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            B.sequential_sample(h, u, w.N, 1, xq, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.sequential_sample(h, u, w.N, 1, xq, stream)
            torch.cuda.synchronize()
            ds = time.perf_counter() - t0
            itc = it.cpu().numpy()
            out[name] = {"jacobi_ms": dt * 1e3, "iters_mean": float(itc.mean()), "iters_max": int(itc.max()),
                         "sequential_lean_ms": ds * 1e3, "jacobi_speedup_vs_lean_sequential": ds / dt,
                         "same_output_as_sequential": bool(torch.equal(x, xq))}
        finally:
            B.made_free(h)
    return out


def cpu_baseline_real(w, net, noises, budget_s=12.0):
    """The logistic oracle's sequential sampler (Eq. 1) on whole batches until about budget_s seconds are spent."""
    from oracle import logistic_oracle as LO
    from oracle import made_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    model = O.build_model(net.D, net.C, net.degrees, net.W, net.b, "bf16" if net.dtype == "bf16" else None)
    LO.sequential_sample_real(model, noises[0][:1])
    done, xs0 = 0, None
    t0 = time.perf_counter()
    for r in range(len(noises)):
        xs = LO.sequential_sample_real(model, noises[r])
        if r == 0:
            xs0 = xs
        done += noises[r].shape[0]
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle sequential_sample_real (numpy fp64, states and activations rounded as on the GPU) on "
                      f"{done} samples, {dt:.1f} s"}, xs0, noises[0].shape[0]


def cpu_baseline_conv(w, net, noise, budget_s=12.0):
    """The conv oracle's sequential sampler (Eq. 1) on a bounded sample: the first states of ONE image, one network
    evaluation per state exactly as conv_sequential_sample does it; every state costs the same, so the time per
    state scales to the D states of a whole image."""
    from oracle import conv_oracle as CO
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    model = CO.build_conv_model(net.H, net.W, net.C, net.F, net.k, net.W_, net.b,
                                "bf16" if net.dtype == "bf16" else None)
    x = np.zeros((1, model.D), dtype=np.uint8)
    CO.conv_logits_all(model, x)                              # warm the BLAS threads
    t0 = time.perf_counter()
    t = 0
    while t < model.D and time.perf_counter() - t0 < budget_s:
        z_t = CO.conv_logits_all(model, x)[:, t]
        x[:, t], _ = CO.decide(z_t, noise[:1, t], model.C)
        t += 1
    dt = time.perf_counter() - t0
    return {"value": 1.0 / (dt / t * model.D), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle conv_sequential_sample steps (numpy fp64, activations rounded as on the GPU): the first "
                      f"{t} of {model.D} states of one image in {dt:.1f} s, scaled to a whole image"}, x[:, :t], t


def measured_traffic(workload: str, path: str, dom_is_output: bool):
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 PMC counters in a separate run
    (counters cannot be read from inside this process); the summary under profiles/ holds the figure."""
    if workload not in ("cfg2", "cfg4") or path == "persistent" or not dom_is_output:
        return None
    fn = os.path.join(ROOT, "profiles", f"{workload}_jacobi_pmc_traffic.txt")
    try:
        for line in open(fn):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.rsplit(":", 1)[1])
    except OSError:
        pass
    return None


def measured_mfma(workload: str):
    """MFMA counters of the workload's kernels from a separate `rocprofv3 --pmc` run, as summarised under profiles/
    (lines `name: value` after the marker `bench_fields:`); None when no such summary exists."""
    fn = os.path.join(ROOT, "profiles", f"{workload}_pmc_mfma.txt")
    try:
        lines = open(fn).read().splitlines()
    except OSError:
        return None
    out, on = {"source": f"profiles/{workload}_pmc_mfma.txt"}, False
    for line in lines:
        if line.startswith("bench_fields:"):
            on = True
            continue
        if on and ":" in line:
            k, v = line.split(":", 1)
            try:
                out[k.strip()] = float(v)
            except ValueError:
                out[k.strip()] = v.strip()
    return out if len(out) > 1 else None


def bench_rnn(args, torch, B, S) -> int:
    """Backward pass of the paper's RNN (Section 5.1) by Jacobi_n: one step = one rnn_backward_jacobi call on a
    resident batch of sequences; side measurements: the standard backward pass, other n, the truncation error."""
    import dataclasses
    w = S.rnn_workload(args.workload)
    if args.batch > 0:
        w = dataclasses.replace(w, B=args.batch)
    Bn, T, H, I = w.B, w.T, w.H, w.I
    Wh, Uh, bh = S.make_rnn_params(w)
    W, U, b = (torch.from_numpy(a).cuda() for a in (Wh, Uh, bh))
    n_in = 4
    stream = own_stream(torch)
    zs, gs = [], []
    for r in range(n_in):          # forward pass on the GPU; the loss is 0.5 |h_t - y_t|^2, so g = h - y
        xh, yh = S.make_rnn_inputs(w, r)
        x, y = torch.from_numpy(xh).cuda(), torch.from_numpy(yh).cuda()
        z = torch.empty((Bn, T, H), dtype=torch.float32, device="cuda")
        h = torch.empty_like(z)
        B.rnn_forward(W, U, b, x, None, Bn, T, H, I, z, h, stream)
        zs.append(z)
        gs.append(h - y)
    d = torch.empty((Bn, T, H), dtype=torch.float32, device="cuda")
    d_seq = torch.empty_like(d)
    iters = torch.empty((Bn,), dtype=torch.int32, device="cuda")
    n = args.jacobi_n if 0 < args.jacobi_n <= T else T

    def timed(fn, steps, warmup):
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(steps):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, e0.elapsed_time(e1) * 1e-3 / steps

    jac = lambda i: B.rnn_backward_jacobi(W, zs[i % n_in], gs[i % n_in], None, Bn, T, H, n, 0.0, d, iters, None, stream)
    seq = lambda i: B.rnn_backward_sequential(W, zs[i % n_in], gs[i % n_in], Bn, T, H, d_seq, stream)
    wall, dev_s = timed(jac, args.steps, args.warmup)
    result = {
        "metric": "sequences/s (backward pass of the RNN by Jacobi_n, Section 5.1)", "value": Bn / wall, "unit": "sequences/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 (matrix products as three bf16 MFMAs on split operands)",
        "data": "synthetic", "config": {"workload": w.name, "sequences": Bn, "steps_T": T, "hidden": H, "jacobi_n": n},
    }
    # the one kernel of a call does n passes of a [T, H] x [H, H] product per sequence (algorithmic flops: one
    # product per pass; the split into bf16 parts makes the hardware do three)
    flops = 2.0 * T * H * H * n * Bn
    ach = flops / dev_s / 1e12
    result["roofline"] = {"bound": "mfma", "achieved": ach, "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0, "traffic": None,
                          "kernel": "rnn_jacobi_kernel (all passes of a call)", "avg_launch_us": dev_s * 1e6, "launches": args.steps}
    if not args.no_extras:
        extras = {}
        sw, sd = timed(seq, args.steps, args.warmup)
        extras["standard_backward_ms"] = sw * 1e3
        extras["speedup_vs_standard_backward"] = sw / wall
        seq(0)
        torch.cuda.synchronize()
        ref_scale = float(d_seq.abs().max())
        sweep = {}
        for nn in sorted({1, 2, 5, 10, 20, 50, T}):
            f = lambda i, nn=nn: B.rnn_backward_jacobi(W, zs[0], gs[0], None, Bn, T, H, nn, 0.0, d, iters, None, stream)
            ww, _ = timed(f, max(10, args.steps // 4), 3)
            sweep[str(nn)] = {"ms": ww * 1e3, "rel_err_vs_standard": float((d - d_seq).abs().max()) / ref_scale}
        extras["jacobi_n_sweep"] = sweep
        result["extras"] = extras
    if not args.no_cpu_baseline:
        from oracle import rnn_oracle as R
        z64, g64 = zs[0].cpu().numpy().astype(np.float64), gs[0].cpu().numpy().astype(np.float64)
        W64 = Wh.astype(np.float64)
        reps, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < 10.0:
            R.backprop_sequential(W64, z64, g64)
            reps += 1
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        result["cpu_baseline"] = {"value": reps * Bn / dt, "unit": "sequences/s", "cores": int(cores), "kind": "oracle",
                                  "sample": f"{reps} standard backward passes (numpy fp64) over the same {Bn} sequences, {dt:.1f} s"}
    print(json.dumps(result))
    return 0


def parse_args(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip sequential / GS-Jacobi side measurements")
    ap.add_argument("--path", choices=["persistent", "layers", "default"], default="default",
                    help="persistent: one cooperative launch per call; layers: one launch per layer and pass; default: "
                         "the library's own choice (small Bernoulli batches: one launch per call, XCD by XCD)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (supplementary sweeps)")
    ap.add_argument("--big-tile-batch", type=int, default=0,
                    help="batch size from which the 256 x 256 tile kernels are used (0 = library default)")
    ap.add_argument("--mid-tile-batch", type=int, default=0,
                    help="batch size from which the 128 x 128 tile kernels are used (0 = library default)")
    ap.add_argument("--frozen-positions", type=int, default=-1, choices=[-1, 0, 1],
                    help="MADE_OPT_FROZEN_POSITIONS (-1 = library default)")
    ap.add_argument("--call-graph", type=int, default=0, choices=[0, 1],
                    help="MADE_OPT_CALL_GRAPH (library default 0): replay each call's launches as one HIP graph where the "
                         "library supports it (Jacobi, Bernoulli MLP, per-layer launches, up to 256 samples); recorded "
                         "before the warm-up.  cfg2: 0.098 ms per call whatever the host's launch cost, against "
                         "0.091 / 0.104-0.108 ms launch by launch")
    ap.add_argument("--zero-start", type=int, default=1, choices=[0, 1],
                    help="MADE_OPT_ZERO_START (library default 1): a Bernoulli MLP's call started from zeros gets the first "
                         "hidden layer of its first pass (ReLU of the bias) from the set-up kernel; 0 launches the layer")
    ap.add_argument("--lazy-stop-test", type=int, default=-1, choices=[-1, 0, 1],
                    help="MADE_OPT_LAZY_STOP_TEST (-1 = library default)")
    ap.add_argument("--retire-split", type=int, default=0,
                    help="active-list length from which the stop test runs as a kernel of its own (0 = library default)")
    ap.add_argument("--conv-rows", type=int, default=0,
                    help="image rows per workgroup of the conv model's k x k layers (0 = library default)")
    ap.add_argument("--eps", type=float, default=0.0,
                    help="forward-difference tolerance of Algorithm 1 (workloads with real states only)")
    ap.add_argument("--chains", type=int, default=0, help="sub-batches on separate streams (0 = library default)")
    ap.add_argument("--jacobi-n", type=int, default=10,
                    help="pass limit n of Jacobi_n (Section 5.1; workloads rnn_paper / rnn_batch only)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="no timing: run 20 device copies of 64 MiB (calibration of FETCH_SIZE / WRITE_SIZE), then "
                         "20 steps; meant to run under `rocprofv3 --pmc ...`")
    ap.add_argument("--single", action="store_true",
                    help="time only --workload (default: the cfg2 run also times cfg1, cfg4 and cfg5 and reports all "
                         "five configurations in the one JSON line)")
    ap.add_argument("--gain", type=float, default=0.0,
                    help="scale every weight of the workload by this factor (coupling-strength sweeps; 0 = as defined)")
    return ap.parse_args(argv)


def run_one(args, torch, B, S, light=False):
    """Time one workload; returns the result dict of the JSON line.  light: the short form used for the other
    configurations of the default run (no Jacobi-GS, no batch sweep, a shorter CPU baseline)."""
    import dataclasses
    conv = args.workload in ("cfg5", "small_conv", "small_conv_f32")
    w = S.conv_workload(args.workload) if conv else S.workload(args.workload)
    if args.batch > 0:
        w = dataclasses.replace(w, N=args.batch)
    if args.gain > 0:
        w = dataclasses.replace(w, gain=w.gain * args.gain)
    if conv:
        net = S.make_conv_network(w)
        model = B.conv_model_from_network(net)
    else:
        net = S.make_network(w)
        model = B.model_from_network(net)
    B.made_set_option(model, B.MADE_OPT_PERSISTENT, int(args.path == "persistent"))
    if args.path == "layers":
        B.made_set_option(model, B.MADE_OPT_XCD_RESIDENT, 0)
    if args.chains > 0:
        B.made_set_option(model, B.MADE_OPT_CHAINS, args.chains)
    if args.conv_rows > 0:
        B.made_set_option(model, B.MADE_OPT_CONV_ROWS, args.conv_rows)
    if args.big_tile_batch > 0:
        B.made_set_option(model, B.MADE_OPT_BIG_TILE_BATCH, args.big_tile_batch)
    if args.mid_tile_batch > 0:
        B.made_set_option(model, B.MADE_OPT_MID_TILE_BATCH, args.mid_tile_batch)
    if args.retire_split > 0:
        B.made_set_option(model, B.MADE_OPT_RETIRE_SPLIT, args.retire_split)
    if args.frozen_positions >= 0 and not conv:
        B.made_set_option(model, B.MADE_OPT_FROZEN_POSITIONS, args.frozen_positions)
    if args.lazy_stop_test >= 0 and not conv:
        B.made_set_option(model, B.MADE_OPT_LAZY_STOP_TEST, args.lazy_stop_test)
    if not conv:
        B.made_set_option(model, B.MADE_OPT_CALL_GRAPH, args.call_graph)
        B.made_set_option(model, B.MADE_OPT_ZERO_START, args.zero_start)
    n_layers = (w.n_conv if conv else len(net.hidden)) + 1
    nnz = B.made_layer_nnz(model, n_layers)
    n_slots = n_layers + 1                     # per-layer kernels + the persistent whole-call kernel
    flops_per_sample_pass = 2.0 * np.array(list(nnz) + [sum(nnz)], dtype=np.float64)
    N, D = w.N, net.D

    n_noise = min(args.steps, 4 if conv else 32)
    noises_host = [S.make_conv_noise(w, rep=r) if conv else S.make_noise(w, rep=r) for r in range(n_noise)]
    noises = [torch.from_numpy(a).cuda() for a in noises_host]
    real = (not conv) and w.real
    x = torch.empty((N, D), dtype=torch.float32 if real else torch.uint8, device="cuda")
    iters = torch.empty((N,), dtype=torch.int32, device="cuda")
    stream = own_stream(torch)

    # (the timed loop calls the library on the same buffers again and again: arguments marshalled once)
    prepared = None if real else [B.PreparedJacobi(model, noises[r], N, None, 0, x, iters, stream) for r in range(n_noise)]

    def step(i):
        if real:
            B.jacobi_sample_real(model, noises[i % n_noise], N, None, args.eps, 0, x, iters, stream)
        else:
            prepared[i % n_noise]()

    if args.pmc_probe:
        src = torch.ones((16 << 20,), dtype=torch.float32, device="cuda")     # 64 MiB read + 64 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        for i in range(20):
            step(i)
        torch.cuda.synchronize()
        B.made_free(model)
        return {"pmc_probe": True, "copy_bytes_read": 64 << 20, "copy_bytes_written": 64 << 20}

    # (recorded calls: the library runs the first call with given buffers launch by launch and records the second,
    # for each half of its pass log, which alternates from call to call: four calls per noise buffer, all untimed)
    call_graph = False
    if (not conv) and (not real) and args.call_graph == 1:
        step(0)
        call_graph = B.made_last_stats(model)["tail_less_passes"] > 0     # (the calls the option covers)
    if call_graph:
        for r in range(n_noise):
            for _ in range(4):
                step(r)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region (events off): whole-call throughput
    it_sum, it_max, sample_passes, passes, conv_rows = 0.0, 0, 0, 0, 0
    out_weights, out_draws = 0, 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- same region again with per-layer HIP events on the launch stream (roofline of the dominant kernel)
    B.made_set_profiling(model, True)
    layer_ms = np.zeros(n_slots)
    layer_launches = np.zeros(n_slots, dtype=np.int64)
    layer_flops = np.zeros(n_slots)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
        ms, cnt = B.made_last_profile(model, n_slots)
        st = B.made_last_stats(model)
        layer_ms += ms
        layer_launches += np.array(cnt)
        # (the convolutional trunk recomputes, per image, the rows below the first symbol that changed)
        work = st["conv_rows"] / w.H if conv else st["sample_passes"]       # in whole-sample evaluations
        layer_flops += flops_per_sample_pass * work * (np.array(cnt) > 0)
        conv_rows += st.get("conv_rows", 0)
        sample_passes += st["sample_passes"]
        passes += st["passes"]
        out_weights += st.get("output_weights_evaluated", 0)
        out_draws += st.get("output_draws_evaluated", 0)
        itc = iters.cpu().numpy()
        it_sum += itc.mean()
        it_max = max(it_max, int(itc.max()))
    torch.cuda.synchronize()
    elapsed_prof = time.perf_counter() - t0
    B.made_set_profiling(model, False)

    # ---- one pass on the FULL batch (pass limit 1) with events: the launch a kernel's roofline is best quoted on
    # (later passes of a call run on fewer samples or fewer image rows, and the last launch finds an empty list)
    first_ms = np.zeros(n_slots)
    first_launches = np.zeros(n_slots, dtype=np.int64)
    if not real:
        B.made_set_profiling(model, True)
        for i in range(5):
            try:
                B.jacobi_sample(model, noises[i % n_noise], N, None, 1, x, iters, stream)
            except B.MadeError as e:                       # one pass does not converge: that is the point
                if e.code != B.MADE_ERR_NOT_CONVERGED:
                    raise
            ms, cnt = B.made_last_profile(model, n_slots)
            first_ms += ms
            first_launches += np.array(cnt)
        B.made_set_profiling(model, False)

    if conv:
        # the k x k layers are launches of one kernel on one shape: fold their slots into slot 1
        for arr in (layer_ms, layer_launches, layer_flops, first_ms, first_launches):
            arr[1] = arr[1:n_layers - 1].sum()
            arr[2:n_layers - 1] = 0
    dom = int(np.argmax(layer_ms))
    dom_avg_us = layer_ms[dom] / max(1, layer_launches[dom]) * 1e3
    es = 2 if w.dtype == "bf16" else 4
    # A layer whose visible weights exceed the chip's caches (32 MB L2 + 256 MB Infinity Cache) must be
    # streamed from HBM once per pass; at batch <= 128 that puts it far below the MFMA ridge: HBM-bound.
    hbm_bound = (not conv) and dom < n_layers and nnz[dom] * es > 288e6
    if hbm_bound:
        noise_bytes = 4.0 * D * w.C * (w.C > 1) + 4.0 * D * (w.C == 1)       # per active sample
        act_bytes = es * (w.hidden[-1] if dom == n_layers - 1 else 0)
        # weights are charged only to launches that found a non-empty list (`passes`); the speculative launch behind
        # the converged pass reads nothing, but its duration stays in the denominator (it is a launch of this kernel)
        dom_bytes = passes * nnz[dom] * es + sample_passes * (noise_bytes + act_bytes)
        if dom == n_layers - 1 and out_weights > 0:
            # the 256-class output kernel skips the positions that cannot change: charge what the passes did read
            # (visible weights of the evaluated positions, 1 KB of noise per evaluated (sample, position))
            dom_bytes = out_weights * es + out_draws * 4.0 * w.C + sample_passes * act_bytes
        achieved = dom_bytes / (layer_ms[dom] * 1e-3) / 1e9
        peak, unit, bound = 8000.0, "GB/s", "hbm"
    else:
        achieved = layer_flops[dom] / (layer_ms[dom] * 1e-3) / 1e12 if layer_ms[dom] > 0 else 0.0
        peak, unit, bound = (PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS), "TFLOP/s", "mfma"
    if conv:
        layer_name = ("conv_first_kernel" if dom == 0 else
                      f"conv_layer_kernel (k x k masked convolution as implicit GEMM, all {n_layers - 2} such layers)"
                      if dom < n_layers - 1 else "conv_head_kernel (1 x 1 head + Gumbel-max)")
    elif dom == n_layers:
        layer_name = ("persistent_sampler_kernel" if args.path == "persistent" else "xcd_sampler_kernel") + \
                     " (all passes of a call in one launch: hidden layers, output layer + sampling, stop test)"
    else:
        if dom == n_layers - 1 and w.C == 256:
            layer_name = "categorical_output_kernel (output layer + Gumbel-max draw + stop test)"
        else:
            layer_name = (f"masked_layer_kernel layer {dom} "
                          f"({'output+sampling epilogue' if dom == n_layers - 1 else 'hidden'})")

    # the dominant kernel on a full batch
    full = None
    if first_launches[dom] > 0 and dom < n_layers:
        full_us = first_ms[dom] / first_launches[dom] * 1e3
        if hbm_bound:
            full_ach = (nnz[dom] * es + N * (noise_bytes + act_bytes)) / (full_us * 1e-6) / 1e9
        else:
            # (for the convolutional model slot 1 holds the launches of all k x k layers: one layer's work each)
            full_ach = flops_per_sample_pass[dom] * N / (full_us * 1e-6) / 1e12
        full = {"avg_launch_us": full_us, "achieved": full_ach, "frac": full_ach / peak,
                "launches": int(first_launches[dom]),
                "what": "the same kernel on a pass over the full batch (first pass of a call with pass limit 1)"}
    pmc = measured_mfma(w.name)

    result = {
        "metric": "samples/s (Jacobi vs sequential, same output); iters to converge; MFMA util",
        "value": N * args.steps / elapsed,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": (f"{w.name}: masked conv net {w.H}x{w.W}x3 states, {w.n_conv} masked {w.k}x{w.k} layers of "
                                f"{w.F} channels + 1x1 head, C={w.C}, batch={N}, Jacobi (Algorithm 1), seeded weights, "
                                f"fixed Gumbel noise") if conv else
                               (f"{w.name}: MADE D={D} hidden={w.hidden} real states, logistic conditionals, batch={N}, "
                                f"Jacobi (Algorithm 1) with tolerance eps={args.eps}, seeded N(0,1/fan_in) weights, "
                                f"random degrees, fixed logistic noise") if real else
                               (f"{w.name}: MADE D={D} hidden={w.hidden} C={w.C} batch={N} Jacobi (Algorithm 1), "
                                f"seeded N(0,1/fan_in) weights, random degrees, fixed U(0,1) noise"),
                   "path": args.path, **({"call_graph": 1} if call_graph else {}),
                   **({"zero_start": args.zero_start} if (not conv and not real and w.C == 1) else {})},
        "iters_mean": it_sum / args.steps,
        "iters_max": it_max,
        "passes_per_step": passes / args.steps,
        **({"image_evaluations_per_step": conv_rows / w.H / args.steps} if conv else {}),
        "roofline": {
            "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
            "traffic": measured_traffic(w.name, args.path, dom == n_layers - 1), "kernel": layer_name, "avg_launch_us": dom_avg_us,
            "launches": int(layer_launches[dom]),
            "per_slot_avg_us": [float(m / max(1, c) * 1e3) for m, c in zip(layer_ms, layer_launches)],
            "mfma_tflops": layer_flops[dom] / (layer_ms[dom] * 1e-3) / 1e12 if layer_ms[dom] > 0 else 0.0,
            "full_batch_launch": full,
            "traffic_source": "profiles/%s_jacobi_pmc_traffic.txt (two separate rocprofv3 --pmc runs)" % w.name,
            "rocprof": pmc,
            "note": "frac uses durations from HIP events around each launch on the launch stream, measured live in a "
                    "second pass over the same steps, averaged over ALL launches of the kernel in a call (late "
                    "passes on few samples and the final launch on an empty list included); full_batch_launch is "
                    "the same kernel on a whole batch.  algorithmic flops = 2*nnz(W*mask) per active sample per pass; "
                    "algorithmic bytes (hbm bound) = visible weights once per launch on a non-empty list + noise and "
                    "last-hidden activations per active sample; the 256-class output kernel is charged what its passes "
                    "read after skipping the positions that cannot change (made_last_stats).  rocprof: figures of separate rocprofv3 runs "
                    "(kernel-trace duration, MFMA counters) read from the named summaries under profiles/",
        },
        "whole_call_tflops": 2.0 * sum(nnz) * (conv_rows / w.H if conv else sample_passes) / elapsed_prof / 1e12,
        "ms_per_step_with_events": elapsed_prof / args.steps * 1e3,
    }

    # ---- side measurements: on-GPU sequential sampler (speedup denominator) and GS-Jacobi
    x_jac = None
    if not args.no_extras and real:
        xq = torch.empty_like(x)
        B.jacobi_sample_real(model, noises[0], N, None, 0.0, 0, x, iters, stream)
        torch.cuda.synchronize()
        x_jac = x.clone()
        extras = {}
        for mode, name in ((0, "sequential_whole_network"), (1, "sequential_lean")):
            B.sequential_sample_real(model, noises[0], N, mode, xq, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 3
            for _ in range(reps):
                B.sequential_sample_real(model, noises[0], N, mode, xq, stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            extras[name] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                            "max_abs_difference_to_jacobi_eps0": float((xq - x_jac).abs().max()),
                            "jacobi_speedup": (N * args.steps / elapsed) / (N / dt)}
        for eps in (0.0, 1e-3, 1e-2, 1e-1):               # the paper's trade of accuracy for iterations
            B.jacobi_sample_real(model, noises[0], N, None, eps, 0, xq, iters, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 20
            for _ in range(reps):
                B.jacobi_sample_real(model, noises[0], N, None, eps, 0, xq, iters, stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            itc = iters.cpu().numpy()
            extras[f"jacobi_eps{eps:g}"] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                                           "iters_mean": float(itc.mean()), "iters_max": int(itc.max()),
                                           "max_abs_difference_to_eps0": float((xq - x_jac).abs().max())}
        result["extras"] = extras
    elif not args.no_extras:
        xq = torch.empty_like(x)
        B.jacobi_sample(model, noises[0], N, None, 0, x, iters, stream)
        torch.cuda.synchronize()
        x_jac = x.clone()
        extras = {}
        for mode, name in ((0, "sequential_whole_network"), (1, "sequential_lean")):
            B.sequential_sample(model, noises[0], N, mode, xq, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 1 if conv else 3
            for _ in range(reps):
                B.sequential_sample(model, noises[0], N, mode, xq, stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            extras[name] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                            "same_output_as_jacobi": bool(torch.equal(xq, x_jac)),
                            "jacobi_speedup": (N * args.steps / elapsed) / (N / dt)}
        # conv model: GS-Jacobi with blocks of whole image rows (4 / 8 / 16 rows of 96 states)
        for blk in ([4 * 96, 8 * 96, 16 * 96] if conv else (w.block_sizes or [])):
            B.gs_jacobi_sample(model, noises[0], N, None, blk, xq, iters, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            reps = 5
            for _ in range(reps):
                B.gs_jacobi_sample(model, noises[0], N, None, blk, xq, iters, stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / reps
            itc = iters.cpu().numpy()
            st = B.made_last_stats(model)
            extras[f"gs_jacobi_B{blk}"] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                                           "iters_mean": float(itc.mean()), "iters_max": int(itc.max()),
                                           "batch_passes": int(st["passes"]),
                                           "same_output_as_jacobi": bool(torch.equal(xq, x_jac))}
        if conv:
            for rows in (1, 2):                         # Algorithm 2 with blocks of whole image rows: one timed call each
                blk = rows * 96
                B.jacobi_gs_sample(model, noises[0], N, None, blk, 0, xq, iters, stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                B.jacobi_gs_sample(model, noises[0], N, None, blk, 0, xq, iters, stream)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                itc = iters.cpu().numpy()
                extras[f"jacobi_gs_B{blk}"] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                                               "iters_mean": float(itc.mean()), "iters_max": int(itc.max()),
                                               "same_output_as_jacobi": bool(torch.equal(xq, x_jac))}
        if not conv and w.C == 1 and not light:
            for blk in (w.block_sizes or []):           # Algorithm 2: one timed call per block size (it is slow)
                B.jacobi_gs_sample(model, noises[0], N, None, blk, 0, xq, iters, stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                B.jacobi_gs_sample(model, noises[0], N, None, blk, 0, xq, iters, stream)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                itc = iters.cpu().numpy()
                extras[f"jacobi_gs_B{blk}"] = {"samples_per_s": N / dt, "ms_per_batch": dt * 1e3,
                                               "iters_mean": float(itc.mean()), "iters_max": int(itc.max()),
                                               "same_output_as_jacobi": bool(torch.equal(xq, x_jac))}
        if not conv and w.C == 1 and not light and not args.batch and not args.gain and w.name == "cfg2":
            extras["coupling_sweep"] = coupling_sweep(w, torch, B, S, stream)
        if not conv and w.C == 1 and not getattr(net, "onehot", False) and not args.batch and not light:
            # the same network on larger batches (supplementary: throughput once the layers are real GEMMs); the
            # noise recipe is the workload's, so the first N samples are the headline batch again
            sweep = {}
            for nb in (2048, 8192, 32768):
                wb = dataclasses.replace(w, N=nb)
                ub = torch.from_numpy(S.make_noise(wb, rep=0)).cuda()
                xb = torch.empty((nb, w.D), dtype=torch.uint8, device="cuda")
                ib = torch.empty((nb,), dtype=torch.int32, device="cuda")
                for _ in range(2):
                    B.jacobi_sample(model, ub, nb, None, 0, xb, ib, stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                reps = 5
                for _ in range(reps):
                    B.jacobi_sample(model, ub, nb, None, 0, xb, ib, stream)
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t0) / reps
                same_noise = bool(torch.equal(ub[:N], noises[0]))
                stb = B.made_last_stats(model)
                tfl = 2.0 * sum(nnz) * stb["sample_passes"] / dt / 1e12      # algorithmic: masked weights, active samples
                sweep[str(nb)] = {"samples_per_s": nb / dt, "ms_per_batch": dt * 1e3,
                                  "iters_mean": float(ib.float().mean().item()),
                                  "algorithmic_tflops": tfl, "frac_of_bf16_mfma_peak": tfl / 2500.0,
                                  "positions_differing_from_headline_batch":
                                      int((xb[:N] != x_jac).sum().item()) if same_noise else None}
                del ub, xb, ib
            extras["batch_sweep"] = sweep
        result["extras"] = extras

    if not args.no_cpu_baseline and conv:
        base, xs, n2 = cpu_baseline_conv(w, net, noises_host[0], 6.0 if light else 12.0)
        result["cpu_baseline"] = base
        if x_jac is not None:
            # early states depend on early states only: the oracle's first states are final
            result["cpu_baseline"]["gpu_matches_oracle_on_sample"] = bool(
                np.array_equal(x_jac[:1, :n2].cpu().numpy(), xs))
    elif not args.no_cpu_baseline and real:
        base, xs, n2 = cpu_baseline_real(w, net, noises_host)
        result["cpu_baseline"] = base
        if x_jac is not None:
            result["cpu_baseline"]["max_abs_difference_gpu_to_oracle_on_sample"] = float(
                np.abs(x_jac[:n2].cpu().numpy() - xs).max())
    elif not args.no_cpu_baseline and getattr(net, "onehot", False) and net.D * net.C >= (1 << 16):
        # a sequential oracle run multiplies a [., D*C] one-hot matrix with the 4 GB first layer at every position:
        # hours, not seconds; the scalar-input workload of the same shape (cfg4) carries the CPU baseline
        result["cpu_baseline"] = None
    elif not args.no_cpu_baseline:
        base, xs, n2 = cpu_baseline(w, net, noises_host, 6.0 if light else 12.0, 0.0 if light else 4.0)
        result["cpu_baseline"] = base
        if x_jac is not None:
            result["cpu_baseline"]["gpu_matches_oracle_on_sample"] = bool(
                np.array_equal(x_jac[:n2].cpu().numpy(), xs))
    else:
        result["cpu_baseline"] = None

    B.made_free(model)
    return result


def summary_of(r):
    """The figures of one configuration that go into the multi-configuration line."""
    ex = r.get("extras") or {}
    out = {"workload": r["config"]["workload"], "dtype": r["dtype"], "steps": r["steps"],
           "samples_per_s": r["value"], "ms_per_step": r["ms_per_step"],
           "iters_mean": r["iters_mean"], "iters_max": r["iters_max"], "passes_per_step": r["passes_per_step"]}
    for key in ("sequential_whole_network", "sequential_lean"):
        if key in ex:
            out[key] = {"ms_per_batch": ex[key]["ms_per_batch"], "jacobi_speedup": ex[key]["jacobi_speedup"],
                        "same_output_as_jacobi": ex[key].get("same_output_as_jacobi")}
    gs = {k: v for k, v in ex.items() if k.startswith("gs_jacobi_B")}
    if gs:
        out["gs_jacobi"] = gs
    rf = r["roofline"]
    out["roofline"] = {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel",
                                          "avg_launch_us", "launches", "full_batch_launch", "rocprof")}
    out["whole_call_tflops"] = r["whole_call_tflops"]
    out["cpu_baseline"] = r.get("cpu_baseline")
    return out


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (samples are independent systems, so a batch would "
              "shard without any exchange). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2002_03629_amd import binding as B
    from paper_2002_03629_amd import synth as S

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.workload.startswith("rnn"):
        return bench_rnn(args, torch, B, S)
    result = run_one(args, torch, B, S)
    multi = (args.workload == "cfg2" and not args.single and not args.pmc_probe and not args.batch and not args.gain
             and args.path == "default" and not args.no_extras)
    if multi:
        # The headline (`value`, `roofline`, `cpu_baseline`) is cfg2, the configuration of the paper's MADE
        # experiment; the other benchmark configurations are timed in the same run, each as its own model.
        import copy
        configs = {"cfg1": None, "cfg2": summary_of(result)}
        gs = configs["cfg2"].pop("gs_jacobi", {})
        seq = configs["cfg2"].get("sequential_whole_network", {}).get("ms_per_batch")
        configs["cfg3"] = {"workload": "cfg2's network, GS-Jacobi (Algorithm 3) with blocks of 16 / 64 / 196 positions, batch 128",
                           **{k: dict(v, speedup_vs_sequential_whole_network=(seq / v["ms_per_batch"] if seq else None))
                              for k, v in gs.items()}}
        for name in ("cfg1", "cfg4", "cfg5"):
            sub = copy.copy(args)
            sub.workload = name
            sub.steps = args.steps if name == "cfg1" else min(args.steps, 20)
            sub.warmup = min(args.warmup, 5) if name != "cfg1" else args.warmup
            sub.no_cpu_baseline = args.no_cpu_baseline
            t0 = time.perf_counter()
            r = run_one(sub, torch, B, S, light=True)
            configs[name] = summary_of(r)
            configs[name]["bench_wall_s"] = time.perf_counter() - t0
            torch.cuda.empty_cache()
        result["configs"] = configs
        # flat copies of the main figures (scalars survive any truncation of nested values)
        flat = {}
        for name, c in configs.items():
            if name == "cfg3":
                for k, v in c.items():
                    if isinstance(v, dict):
                        flat[f"cfg3_{k}_samples_per_s"] = v["samples_per_s"]
                        flat[f"cfg3_{k}_iters_mean"] = v["iters_mean"]
                continue
            flat[f"{name}_samples_per_s"] = c["samples_per_s"]
            flat[f"{name}_ms_per_step"] = c["ms_per_step"]
            flat[f"{name}_iters_mean"] = c["iters_mean"]
            flat[f"{name}_speedup_vs_seq"] = (c.get("sequential_whole_network") or {}).get("jacobi_speedup")
            flat[f"{name}_roofline_bound"] = c["roofline"]["bound"]
            flat[f"{name}_roofline_frac"] = c["roofline"]["frac"]
            fb = c["roofline"].get("full_batch_launch")
            flat[f"{name}_full_batch_frac"] = fb["frac"] if fb else None
            flat[f"{name}_cpu_oracle_samples_per_s"] = (c.get("cpu_baseline") or {}).get("value")
        result["config"].update(flat)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
