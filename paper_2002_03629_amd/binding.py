"""ctypes binding of libjacobi_made.so: argument marshalling only.

Function names and argument order follow include/jacobi_made.h.  Device buffers are torch
tensors (torch is used for device memory and streams, nothing else); host arrays are numpy.
There is no fallback: if the shared library is missing, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libjacobi_made.so")

MADE_OK, MADE_ERR_ARG, MADE_ERR_NOMEM, MADE_ERR_HIP, MADE_ERR_NOT_CONVERGED = 0, -1, -2, -3, -4
MADE_F32, MADE_BF16 = 0, 1

EXPORTS = ["made_init", "made_conv_init", "made_free", "made_forward_logits", "made_forward_logits_noalloc", "made_layer_activations", "sequential_sample", "jacobi_sample",
           "gs_jacobi_sample", "jacobi_gs_sample", "made_forward_params", "sequential_sample_real",
           "jacobi_sample_real", "gs_jacobi_sample_real", "made_last_stats", "made_set_profiling", "made_last_profile", "made_set_option",
           "made_layer_nnz",
           "rnn_forward", "rnn_backward_sequential", "rnn_backward_jacobi", "rnn_jacobi_max_steps", "rnn_param_grads",
           "made_last_error"]


class MadeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libjacobi_made status {code}: {message}")
        self.code = code


class made_config(C.Structure):
    _fields_ = [("D", C.c_int32), ("C", C.c_int32), ("n_hidden", C.c_int32),
                ("hidden", C.POINTER(C.c_int32)), ("dtype", C.c_int32), ("real", C.c_int32), ("onehot", C.c_int32)]


class made_conv_config(C.Structure):
    _fields_ = [("H", C.c_int32), ("W", C.c_int32), ("C", C.c_int32), ("F", C.c_int32), ("k", C.c_int32),
                ("n_conv", C.c_int32), ("dtype", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2002_03629_amd.build` "
                               "(there is no CPU fallback)")
        # Device pointers and streams come from torch, so the library must run on the very HIP runtime
        # torch has loaded: import torch first, then the loader resolves libamdhip64.so.7 to that copy.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int64)
        L.made_init.argtypes = [C.POINTER(made_config), C.POINTER(C.POINTER(C.c_int32)),
                                C.POINTER(C.POINTER(C.c_float)), C.POINTER(C.POINTER(C.c_float)), C.POINTER(vp)]
        L.made_conv_init.argtypes = [C.POINTER(made_conv_config), C.POINTER(C.POINTER(C.c_float)),
                                     C.POINTER(C.POINTER(C.c_float)), C.POINTER(vp)]
        L.made_free.argtypes = [vp]
        L.made_forward_logits.argtypes = [vp, vp, i32, vp, vp]
        L.made_forward_logits_noalloc.argtypes = [vp, vp, i32, vp, vp]
        L.made_layer_activations.argtypes = [vp, vp, i32, i32, vp, vp]
        L.sequential_sample.argtypes = [vp, vp, i32, i32, vp, vp]
        L.jacobi_sample.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp]
        L.gs_jacobi_sample.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp]
        L.jacobi_gs_sample.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp]
        L.made_forward_params.argtypes = [vp, vp, i32, vp, vp]
        L.sequential_sample_real.argtypes = [vp, vp, i32, i32, vp, vp]
        L.jacobi_sample_real.argtypes = [vp, vp, i32, vp, C.c_float, i32, vp, vp, vp]
        L.gs_jacobi_sample_real.argtypes = [vp, vp, i32, vp, i32, C.c_float, vp, vp, vp]
        L.made_last_stats.argtypes = [vp, i64p, i32]
        L.made_set_profiling.argtypes = [vp, i32]
        L.made_last_profile.argtypes = [vp, C.POINTER(C.c_double), i64p, i32]
        L.made_layer_nnz.argtypes = [vp, i64p, i32]
        L.made_set_option.argtypes = [vp, i32, i32]
        L.rnn_forward.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
        L.rnn_backward_sequential.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        L.rnn_backward_jacobi.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, C.c_float, vp, vp, vp, vp]
        L.rnn_jacobi_max_steps.argtypes = [i32]
        L.rnn_param_grads.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        L.made_last_error.argtypes = []
        L.made_last_error.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def made_last_error() -> str:
    return lib().made_last_error().decode()


def _check(code: int) -> None:
    if code != MADE_OK:
        raise MadeError(code, made_last_error())


def _ptr(t, dtype=None) -> Optional[int]:
    """Device pointer of a contiguous torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("device tensors must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def made_init(D: int, Cn: int, hidden: Sequence[int], dtype: int, degrees: Sequence[np.ndarray],
              W: Sequence[np.ndarray], b: Optional[Sequence[Optional[np.ndarray]]] = None, real: bool = False,
              onehot: bool = False) -> int:
    """Returns the opaque model handle (an integer address)."""
    L = len(hidden)
    hid = np.ascontiguousarray(hidden, dtype=np.int32)
    cfg = made_config(int(D), int(Cn), L, hid.ctypes.data_as(C.POINTER(C.c_int32)), int(dtype), 1 if real else 0,
                      1 if onehot else 0)
    keep = []
    deg_arr = (C.POINTER(C.c_int32) * L)()
    for l in range(L):
        a = np.ascontiguousarray(degrees[l], dtype=np.int32)
        if a.shape != (hidden[l],):
            raise ValueError("degrees[%d] has shape %s" % (l, a.shape))
        keep.append(a)
        deg_arr[l] = a.ctypes.data_as(C.POINTER(C.c_int32))
    dims = [D * Cn if onehot else D] + list(hidden) + [D * Cn]
    W_arr = (C.POINTER(C.c_float) * (L + 1))()
    b_arr = (C.POINTER(C.c_float) * (L + 1))()
    for l in range(L + 1):
        a = np.ascontiguousarray(W[l], dtype=np.float32)
        if a.shape != (dims[l + 1], dims[l]):
            raise ValueError("W[%d] has shape %s, expected %s" % (l, a.shape, (dims[l + 1], dims[l])))
        keep.append(a)
        W_arr[l] = a.ctypes.data_as(C.POINTER(C.c_float))
        bl = None if b is None else b[l]
        if bl is not None:
            bb = np.ascontiguousarray(bl, dtype=np.float32)
            if bb.shape != (dims[l + 1],):
                raise ValueError("b[%d] has shape %s" % (l, bb.shape))
            keep.append(bb)
            b_arr[l] = bb.ctypes.data_as(C.POINTER(C.c_float))
    out = C.c_void_p()
    _check(lib().made_init(C.byref(cfg), deg_arr, W_arr, b_arr, C.byref(out)))
    return out.value


def made_conv_init(H: int, W: int, Cn: int, F: int, k: int, n_conv: int, dtype: int, Wts: Sequence[np.ndarray],
                   b: Optional[Sequence[Optional[np.ndarray]]] = None) -> int:
    """Returns the opaque handle of a masked convolutional model (see include/jacobi_made.h)."""
    cfg = made_conv_config(int(H), int(W), int(Cn), int(F), int(k), int(n_conv), int(dtype))
    shapes = [(F, k, k, 3)] + [(F, k, k, F)] * (n_conv - 1) + [(3 * Cn, 1, 1, F)]
    keep = []
    W_arr = (C.POINTER(C.c_float) * (n_conv + 1))()
    b_arr = (C.POINTER(C.c_float) * (n_conv + 1))()
    for l, shp in enumerate(shapes):
        a = np.ascontiguousarray(Wts[l], dtype=np.float32)
        if a.shape != shp and a.shape != (shp[0], shp[3]):
            raise ValueError("W[%d] has shape %s, expected %s" % (l, a.shape, shp))
        keep.append(a)
        W_arr[l] = a.ctypes.data_as(C.POINTER(C.c_float))
        bl = None if b is None else b[l]
        if bl is not None:
            bb = np.ascontiguousarray(bl, dtype=np.float32)
            if bb.shape != (shp[0],):
                raise ValueError("b[%d] has shape %s" % (l, bb.shape))
            keep.append(bb)
            b_arr[l] = bb.ctypes.data_as(C.POINTER(C.c_float))
    out = C.c_void_p()
    _check(lib().made_conv_init(C.byref(cfg), W_arr, b_arr, C.byref(out)))
    return out.value


def conv_model_from_network(net) -> int:
    """made_conv_init from a synth.ConvNetwork description."""
    n_conv = len(net.W_) - 1
    return made_conv_init(net.H, net.W, net.C, net.F, net.k, n_conv, MADE_BF16 if net.dtype == "bf16" else MADE_F32,
                          net.W_, net.b)


def made_free(model: Optional[int]) -> None:
    _check(lib().made_free(model))


def made_forward_logits(model: int, x, N: int, logits, stream=None) -> None:
    import torch
    _check(lib().made_forward_logits(model, _ptr(x, torch.uint8), N, _ptr(logits, torch.float32), _stream(stream)))


def made_forward_logits_noalloc(model: int, x, N: int, logits, stream=None) -> None:
    import torch
    _check(lib().made_forward_logits_noalloc(model, _ptr(x, torch.uint8), N, _ptr(logits, torch.float32),
                                             _stream(stream)))


def made_layer_activations(model: int, x, N: int, layer: int, out, stream=None) -> None:
    import torch
    _check(lib().made_layer_activations(model, _ptr(x, torch.uint8), N, layer, _ptr(out, torch.float32),
                                        _stream(stream)))


def sequential_sample(model: int, noise, N: int, mode: int, x_out, stream=None) -> None:
    import torch
    _check(lib().sequential_sample(model, _ptr(noise, torch.float32), N, mode, _ptr(x_out, torch.uint8),
                                   _stream(stream)))


def jacobi_sample(model: int, noise, N: int, x_init, max_iters: int, x_out, iters_out=None, stream=None) -> None:
    import torch
    _check(lib().jacobi_sample(model, _ptr(noise, torch.float32), N, _ptr(x_init, torch.uint8), max_iters,
                               _ptr(x_out, torch.uint8), _ptr(iters_out, torch.int32), _stream(stream)))


class PreparedJacobi:
    """jacobi_sample with its arguments marshalled once, for loops that call it again and again on the same buffers
    (a call of cfg2's size takes ~90 us, of which checking and converting eight arguments costs ~2.5): calling the
    object runs the call.  The tensors are kept alive; their contents may change between calls."""

    def __init__(self, model: int, noise, N: int, x_init, max_iters: int, x_out, iters_out=None, stream=None):
        import torch
        self._keep = (noise, x_init, x_out, iters_out, stream)
        self._fn = lib().jacobi_sample
        self._args = (C.c_void_p(model), C.c_void_p(_ptr(noise, torch.float32)), C.c_int32(N),
                      C.c_void_p(_ptr(x_init, torch.uint8)), C.c_int32(max_iters), C.c_void_p(_ptr(x_out, torch.uint8)),
                      C.c_void_p(_ptr(iters_out, torch.int32)), C.c_void_p(_stream(stream)))

    def __call__(self) -> None:
        code = self._fn(*self._args)
        if code != MADE_OK:
            raise MadeError(code, made_last_error())


def gs_jacobi_sample(model: int, noise, N: int, x_init, block: int, x_out, iters_out=None, stream=None) -> None:
    import torch
    _check(lib().gs_jacobi_sample(model, _ptr(noise, torch.float32), N, _ptr(x_init, torch.uint8), block,
                                  _ptr(x_out, torch.uint8), _ptr(iters_out, torch.int32), _stream(stream)))


def jacobi_gs_sample(model: int, noise, N: int, x_init, block: int, max_iters: int, x_out, iters_out=None,
                     stream=None) -> None:
    import torch
    _check(lib().jacobi_gs_sample(model, _ptr(noise, torch.float32), N, _ptr(x_init, torch.uint8), block, max_iters,
                                  _ptr(x_out, torch.uint8), _ptr(iters_out, torch.int32), _stream(stream)))


def made_forward_params(model: int, x, N: int, params, stream=None) -> None:
    import torch
    _check(lib().made_forward_params(model, _ptr(x, torch.float32), N, _ptr(params, torch.float32), _stream(stream)))


def sequential_sample_real(model: int, noise, N: int, mode: int, x_out, stream=None) -> None:
    import torch
    _check(lib().sequential_sample_real(model, _ptr(noise, torch.float32), N, mode, _ptr(x_out, torch.float32),
                                        _stream(stream)))


def jacobi_sample_real(model: int, noise, N: int, x_init, eps: float, max_iters: int, x_out, iters_out=None,
                       stream=None) -> None:
    import torch
    _check(lib().jacobi_sample_real(model, _ptr(noise, torch.float32), N, _ptr(x_init, torch.float32), float(eps),
                                    max_iters, _ptr(x_out, torch.float32), _ptr(iters_out, torch.int32),
                                    _stream(stream)))


def gs_jacobi_sample_real(model: int, noise, N: int, x_init, block: int, eps: float, x_out, iters_out=None,
                          stream=None) -> None:
    import torch
    _check(lib().gs_jacobi_sample_real(model, _ptr(noise, torch.float32), N, _ptr(x_init, torch.float32), block,
                                       float(eps), _ptr(x_out, torch.float32), _ptr(iters_out, torch.int32),
                                       _stream(stream)))


def made_last_stats(model: int) -> dict:
    buf = (C.c_int64 * 8)()
    _check(lib().made_last_stats(model, buf, 8))
    return {"passes": buf[0], "sample_passes": buf[1], "kernels": buf[2], "host_waits": buf[3],
            "conv_rows": buf[4], "tail_less_passes": buf[5], "output_weights_evaluated": buf[6],
            "output_draws_evaluated": buf[7]}


def made_set_profiling(model: int, enable: bool) -> None:
    _check(lib().made_set_profiling(model, 1 if enable else 0))


MADE_OPT_PERSISTENT = 1
MADE_OPT_FUSED_CATEGORICAL = 2
MADE_OPT_CHAINS = 3
MADE_OPT_BIG_TILE_BATCH = 4
MADE_OPT_CONV_ROWS = 5
MADE_OPT_PREFIX_CACHE = 6
MADE_OPT_RESIDENT = 7
MADE_OPT_RETIRE_SPLIT = 8
MADE_OPT_MID_TILE_BATCH = 9
MADE_OPT_PARTIAL_SUM_BATCH = 10
MADE_OPT_XCD_RESIDENT = 11
MADE_OPT_LAZY_STOP_TEST = 12
MADE_OPT_CALL_GRAPH = 14
MADE_OPT_ZERO_START = 15
MADE_OPT_FROZEN_POSITIONS = 13


def made_set_option(model: int, option: int, value: int) -> None:
    _check(lib().made_set_option(model, option, value))


def made_last_profile(model: int, n_slots: int):
    """(ms[n_slots], launches[n_slots]) of the most recent *_sample call; n_slots = L + 2."""
    ms = (C.c_double * n_slots)()
    cnt = (C.c_int64 * n_slots)()
    _check(lib().made_last_profile(model, ms, cnt, n_slots))
    return list(ms), list(cnt)


def made_layer_nnz(model: int, n_layers: int) -> List[int]:
    buf = (C.c_int64 * n_layers)()
    _check(lib().made_layer_nnz(model, buf, n_layers))
    return list(buf)


def model_from_network(net) -> int:
    """made_init from a synth.Network description."""
    return made_init(net.D, net.C, net.hidden, MADE_BF16 if net.dtype == "bf16" else MADE_F32, net.degrees, net.W,
                     net.b, getattr(net, "real", False), getattr(net, "onehot", False))


# ------------------------------------------------------------------------------------------------
# recurrent network: backward pass by Jacobi iteration (include/jacobi_rnn.h); all tensors are float32 on the device
# ------------------------------------------------------------------------------------------------
def rnn_forward(W, U, b, x, h0, B: int, T: int, H: int, I: int, z, h, stream=None) -> None:
    import torch
    f = torch.float32
    _check(lib().rnn_forward(_ptr(W, f), _ptr(U, f), _ptr(b, f), _ptr(x, f), _ptr(h0, f), B, T, H, I, _ptr(z, f), _ptr(h, f),
                             _stream(stream)))


def rnn_backward_sequential(W, z, g, B: int, T: int, H: int, d, stream=None) -> None:
    import torch
    f = torch.float32
    _check(lib().rnn_backward_sequential(_ptr(W, f), _ptr(z, f), _ptr(g, f), B, T, H, _ptr(d, f), _stream(stream)))


def rnn_backward_jacobi(W, z, g, d_init, B: int, T: int, H: int, n_iters: int, eps: float, d, iters_out=None,
                        converged_out=None, stream=None) -> None:
    import torch
    f = torch.float32
    _check(lib().rnn_backward_jacobi(_ptr(W, f), _ptr(z, f), _ptr(g, f), _ptr(d_init, f), B, T, H, int(n_iters), float(eps),
                                     _ptr(d, f), _ptr(iters_out, torch.int32), _ptr(converged_out, torch.int32),
                                     _stream(stream)))


def rnn_jacobi_max_steps(H: int) -> int:
    return int(lib().rnn_jacobi_max_steps(int(H)))


def rnn_param_grads(z, h, x, d, h0, B: int, T: int, H: int, I: int, dW, dU, db, stream=None) -> None:
    import torch
    f = torch.float32
    _check(lib().rnn_param_grads(_ptr(z, f), _ptr(h, f), _ptr(x, f), _ptr(d, f), _ptr(h0, f), B, T, H, I, _ptr(dW, f),
                                 _ptr(dU, f), _ptr(db, f), _stream(stream)))
