"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

from paper_2002_03629_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_symbols_are_exported():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2002_03629_amd import build
        build.build_library(verbose=False)
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS), names
    L = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_argument_errors_need_no_gpu():
    L = binding.lib()
    assert L.made_free(None) == binding.MADE_OK
    assert L.made_init(None, None, None, None, None) == binding.MADE_ERR_ARG
    out = ctypes.c_void_p()
    assert L.made_init(None, None, None, None, ctypes.byref(out)) == binding.MADE_ERR_ARG
    assert "NULL" in binding.made_last_error()
    assert L.jacobi_sample(None, None, 4, None, 0, None, None, None) == binding.MADE_ERR_ARG
    assert L.gs_jacobi_sample(None, None, 4, None, 0, None, None, None) == binding.MADE_ERR_ARG
    assert L.sequential_sample(None, None, 4, 0, None, None) == binding.MADE_ERR_ARG
    assert L.made_forward_logits(None, None, 4, None, None) == binding.MADE_ERR_ARG
    with pytest.raises(binding.MadeError):
        binding._check(L.made_last_stats(None, None, 4))
    # recurrent-network entry points: shape and NULL checks come before any device work
    assert L.rnn_backward_jacobi(None, None, None, None, 1, 10, 16, 0, 0.0, None, None, None, None) == binding.MADE_ERR_ARG
    assert L.rnn_backward_sequential(None, None, None, 1, 10, 200, None, None) == binding.MADE_ERR_ARG
    assert "128" in binding.made_last_error()
    assert L.rnn_forward(None, None, None, None, None, 1, 0, 16, 1, None, None, None) == binding.MADE_ERR_ARG
    assert L.rnn_param_grads(None, None, None, None, None, 1, 10, 16, 1, None, None, None, None) == binding.MADE_ERR_ARG
    assert binding.rnn_jacobi_max_steps(128) == 128 and binding.rnn_jacobi_max_steps(64) == 256
    assert binding.rnn_jacobi_max_steps(20) == 512 and binding.rnn_jacobi_max_steps(129) == 0


def test_header_constants_match_the_binding():
    """Every enumerator the headers define (status codes, dtypes, options) has the same value in the binding."""
    inc = os.path.join(ROOT, "include")
    found = {}
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, fn)).read(), flags=re.S)
        for body in re.findall(r"enum\s*\w*\s*\{(.*?)\}", text, flags=re.S):
            for name, value in re.findall(r"(\w+)\s*=\s*(-?\d+)", body):
                found[name] = int(value)
    assert found, "no enumerators parsed"
    missing = [n for n in found if not hasattr(binding, n)]
    assert not missing, missing
    for name, value in found.items():
        assert getattr(binding, name) == value, name
    # an option the library does not know is an argument error, also without a GPU
    L = binding.lib()
    assert L.made_set_option(None, binding.MADE_OPT_RETIRE_SPLIT, 1) == binding.MADE_ERR_ARG


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits (before it touches any GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
