"""Thin ctypes binding of libtardis (include/tardis.h).

Argument marshalling only: every step of the method runs in the library's HIP
kernels.  Tensors are torch CUDA tensors used as plain device buffers; the
current torch stream is passed unless one is given.  The library must have been
built (``python -m paper_2501_10054_amd.build``); there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("TARDIS_LIB") or os.path.join(_HERE, "libtardis.so")

OK, ERR_INVALID_ARG, ERR_SHAPE, ERR_DTYPE, ERR_STATE, ERR_OOM, ERR_HIP = range(7)
ACT = {"gelu_erf": 0, "gelu_tanh": 1, "relu": 2, "identity": 3}
F32, BF16, FP8_E4M3 = 0, 1, 2
_TORCH_DTYPE = {F32: torch.float32, BF16: torch.bfloat16}
_DTYPE_CODE = {torch.float32: F32, torch.bfloat16: BF16}

EXPORTS = (
    "tardis_calibrate", "tardis_calibrate_search", "tardis_estimate_errors", "tardis_assign_thresholds", "tardis_fold", "tardis_ffn_forward", "tardis_ffn_forward_batched",
    "tardis_ffn_forward_static", "tardis_stack_forward", "tardis_dense_forward", "tardis_get_folded", "tardis_get_predictor_state",
    "tardis_get_sketch_groups", "tardis_get_last_outliers", "tardis_get_last_union", "tardis_get_handover", "tardis_set_next_layer",
    "tardis_destroy", "tardis_status_string", "tardis_version",
)


class TardisError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class tardis_ffn_desc(C.Structure):
    _fields_ = [("d", C.c_int64), ("h", C.c_int64), ("dtype", C.c_int32), ("act", C.c_int32),
                ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p)]


class tardis_fold_opts(C.Structure):
    _fields_ = [("sketch_bits", C.c_int32), ("folded_dtype", C.c_int32), ("max_batch", C.c_int64),
                ("deterministic", C.c_int32), ("margin", C.c_float)]


_lib_handle = None


def lib() -> C.CDLL:
    """The loaded shared library (loaded on first use)."""
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_10054_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, f32 = C.c_void_p, C.c_int64, C.c_float
        L.tardis_calibrate.argtypes = [C.POINTER(tardis_ffn_desc), vp, i64, f32, vp, vp, vp, vp, vp, vp]
        L.tardis_calibrate_search.argtypes = [C.POINTER(tardis_ffn_desc), vp, i64, f32, vp, f32, vp, vp, vp, vp, vp]
        L.tardis_estimate_errors.argtypes = [C.POINTER(tardis_ffn_desc), vp, i64, vp, vp, vp, vp, vp, vp, vp]
        L.tardis_assign_thresholds.argtypes = [vp, i64, f32, f32, f32, vp, vp]
        L.tardis_fold.argtypes = [C.POINTER(tardis_ffn_desc), vp, vp, vp, vp, C.POINTER(tardis_fold_opts), vp,
                                  C.POINTER(vp)]
        L.tardis_ffn_forward.argtypes = [vp, vp, vp, vp]
        L.tardis_ffn_forward_batched.argtypes = [vp, vp, i64, vp, vp]
        L.tardis_ffn_forward_static.argtypes = [vp, vp, i64, vp, vp, vp]
        L.tardis_dense_forward.argtypes = [vp, vp, i64, vp, vp]
        L.tardis_stack_forward.argtypes = [C.POINTER(vp), C.c_int32, vp, i64, vp, vp]
        L.tardis_set_next_layer.argtypes = [vp, vp]
        L.tardis_get_folded.argtypes = [vp, vp, vp, vp]
        L.tardis_get_predictor_state.argtypes = [vp, vp, vp, vp, vp]
        L.tardis_get_sketch_groups.argtypes = [vp, vp, vp]
        L.tardis_get_last_outliers.argtypes = [vp, i64, vp, vp, vp, vp]
        L.tardis_get_last_union.argtypes = [vp, i64, vp, vp, vp]
        L.tardis_get_handover.argtypes = [vp, i64, vp, vp]
        L.tardis_destroy.argtypes = [vp]
        L.tardis_status_string.argtypes = [C.c_int]
        L.tardis_status_string.restype = C.c_char_p
        L.tardis_version.argtypes = []
        L.tardis_version.restype = C.c_int32
        for name in EXPORTS:
            if name not in ("tardis_status_string", "tardis_version"):
                getattr(L, name).restype = C.c_int
        _lib_handle = L
    return _lib_handle


def status_string(status: int) -> str:
    return lib().tardis_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise TardisError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class FFN:
    """Device tensors of one FFN layer plus the matching C descriptor."""

    def __init__(self, W1, W2, b1=None, b2=None, act: str = "gelu_erf"):
        h, d = W1.shape
        assert W2.shape == (d, h)
        for t in (W1, W2, b1, b2):
            assert t is None or (t.is_cuda and t.is_contiguous() and t.dtype == W1.dtype)
        self.W1, self.W2, self.b1, self.b2 = W1, W2, b1, b2
        self.d, self.h, self.act = d, h, act
        self.dtype = _DTYPE_CODE[W1.dtype]
        self.desc = tardis_ffn_desc(d, h, self.dtype, ACT[act], W1.data_ptr(),
                                    b1.data_ptr() if b1 is not None else None, W2.data_ptr(),
                                    b2.data_ptr() if b2 is not None else None)


def tardis_calibrate(ffn: FFN, X_cal, coverage: float = 0.95, coverage_per_neuron=None, stream=None):
    """-> (lo, hi, a, c), four float32 device tensors of length h."""
    assert X_cal.is_cuda and X_cal.is_contiguous() and X_cal.dtype == ffn.W1.dtype and X_cal.shape[1] == ffn.d
    out = [torch.empty(ffn.h, dtype=torch.float32, device=X_cal.device) for _ in range(4)]
    st = lib().tardis_calibrate(C.byref(ffn.desc), _ptr(X_cal), X_cal.shape[0], float(coverage),
                                _ptr(coverage_per_neuron), *[_ptr(t) for t in out], _stream(stream))
    _check(st, "tardis_calibrate")
    return tuple(out)


def tardis_calibrate_search(ffn: FFN, X_cal, coverage: float = 0.95, step: float = 0.05, coverage_per_neuron=None,
                            stream=None):
    """-> (lo, hi, a, c) with greedily searched ranges."""
    assert X_cal.is_cuda and X_cal.is_contiguous() and X_cal.dtype == ffn.W1.dtype and X_cal.shape[1] == ffn.d
    out = [torch.empty(ffn.h, dtype=torch.float32, device=X_cal.device) for _ in range(4)]
    st = lib().tardis_calibrate_search(C.byref(ffn.desc), _ptr(X_cal), X_cal.shape[0], float(coverage),
                                       _ptr(coverage_per_neuron), float(step), *[_ptr(t) for t in out],
                                       _stream(stream))
    _check(st, "tardis_calibrate_search")
    return tuple(out)


def tardis_estimate_errors(ffn: FFN, X_cal, lo, hi, a, c, stream=None):
    """-> (err_neurons float32[h], err_layer float32[1]): empirical approximation error over X_cal."""
    err = torch.empty(ffn.h, dtype=torch.float32, device=X_cal.device)
    tot = torch.empty(1, dtype=torch.float32, device=X_cal.device)
    st = lib().tardis_estimate_errors(C.byref(ffn.desc), _ptr(X_cal), X_cal.shape[0], _ptr(lo), _ptr(hi), _ptr(a), _ptr(c),
                                      _ptr(err), _ptr(tot), _stream(stream))
    _check(st, "tardis_estimate_errors")
    return err, tot


def tardis_assign_thresholds(err, t: float, t_min: float, t_max: float, stream=None):
    """-> float32[n] thresholds: minimise sum err_i t_i with mean t and the given bounds."""
    out = torch.empty_like(err)
    _check(lib().tardis_assign_thresholds(_ptr(err), err.numel(), float(t), float(t_min), float(t_max), _ptr(out),
                                          _stream(stream)), "tardis_assign_thresholds")
    return out


class Layer:
    """Owner of a tardis_handle_t.  Keeps the borrowed weight tensors alive."""

    def __init__(self, handle, ffn: FFN, max_batch: int):
        self.handle, self.ffn, self.max_batch = handle, ffn, max_batch
        self.d, self.h = ffn.d, ffn.h
        self.torch_dtype = ffn.W1.dtype
        self.device = ffn.W1.device

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            lib().tardis_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tardis_fold(ffn: FFN, lo, hi, a, c, max_batch: int = 1, sketch_bits: int = 8, deterministic: bool = False,
                margin: float = 0.0, folded_fp8: bool = False, stream=None) -> Layer:
    for t in (lo, hi, a, c):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and t.numel() == ffn.h
    opts = tardis_fold_opts(sketch_bits, FP8_E4M3 if folded_fp8 else ffn.dtype, max_batch, 1 if deterministic else 0,
                            float(margin))
    handle = C.c_void_p()
    st = lib().tardis_fold(C.byref(ffn.desc), _ptr(lo), _ptr(hi), _ptr(a), _ptr(c), C.byref(opts),
                           _stream(stream), C.byref(handle))
    _check(st, "tardis_fold")
    return Layer(handle, ffn, max_batch)


def tardis_ffn_forward(L: Layer, x, y=None, stream=None):
    if y is None:
        y = torch.empty_like(x)
    _check(lib().tardis_ffn_forward(L.handle, _ptr(x), _ptr(y), _stream(stream)), "tardis_ffn_forward")
    return y


def tardis_ffn_forward_batched(L: Layer, x, y=None, stream=None):
    if y is None:
        y = torch.empty_like(x)
    _check(lib().tardis_ffn_forward_batched(L.handle, _ptr(x), x.shape[0], _ptr(y), _stream(stream)),
           "tardis_ffn_forward_batched")
    return y


def tardis_ffn_forward_static(L: Layer, x, y=None, mask_out=None, stream=None):
    """n <= 16 tokens with the library's static working memory (the call allocates nothing)."""
    if y is None:
        y = torch.empty_like(x)
    n = 1 if x.dim() == 1 else x.shape[0]
    _check(lib().tardis_ffn_forward_static(L.handle, _ptr(x), n, _ptr(y), _ptr(mask_out), _stream(stream)),
           "tardis_ffn_forward_static")
    return y


def tardis_stack_forward(layers, x, y=None, stream=None):
    """x: n x d through every layer in turn (RMS-normalised between layers)."""
    if y is None:
        y = torch.empty_like(x)
    arr = (C.c_void_p * len(layers))(*[L.handle for L in layers])
    n = 1 if x.dim() == 1 else x.shape[0]
    _check(lib().tardis_stack_forward(arr, len(layers), _ptr(x), n, _ptr(y), _stream(stream)), "tardis_stack_forward")
    return y


def tardis_set_next_layer(L: Layer, nxt):
    """Hint: `nxt` (a Layer or None) is the layer whose call follows L's."""
    _check(lib().tardis_set_next_layer(L.handle, nxt.handle if nxt is not None else None), "tardis_set_next_layer")


def tardis_dense_forward(L: Layer, x, y=None, stream=None):
    if y is None:
        y = torch.empty_like(x)
    n = 1 if x.dim() == 1 else x.shape[0]
    _check(lib().tardis_dense_forward(L.handle, _ptr(x), n, _ptr(y), _stream(stream)), "tardis_dense_forward")
    return y


def tardis_get_folded(L: Layer, stream=None):
    Wp = torch.empty(L.d, L.d, dtype=L.torch_dtype, device=L.device)
    bp = torch.empty(L.d, dtype=torch.float32, device=L.device)
    _check(lib().tardis_get_folded(L.handle, _ptr(Wp), _ptr(bp), _stream(stream)), "tardis_get_folded")
    return Wp, bp


def tardis_get_predictor_state(L: Layer, stream=None):
    Q = torch.empty(L.h, L.d, dtype=torch.int8, device=L.device)
    tlo = torch.empty(L.h, dtype=torch.float32, device=L.device)
    thi = torch.empty(L.h, dtype=torch.float32, device=L.device)
    _check(lib().tardis_get_predictor_state(L.handle, _ptr(Q), _ptr(tlo), _ptr(thi), _stream(stream)),
           "tardis_get_predictor_state")
    return Q, tlo, thi


def tardis_get_sketch_groups(L: Layer, stream=None):
    M = torch.empty(L.h, (L.d + 31) // 32, dtype=torch.uint8, device=L.device)
    _check(lib().tardis_get_sketch_groups(L.handle, _ptr(M), _stream(stream)), "tardis_get_sketch_groups")
    return M


def tardis_get_handover(L: Layer, n: int, stream=None):
    out = torch.empty(n, L.d, dtype=L.torch_dtype, device=L.device)
    _check(lib().tardis_get_handover(L.handle, n, _ptr(out), _stream(stream)), "tardis_get_handover")
    return out


def tardis_get_last_outliers(L: Layer, n: int, want_list: bool = True, stream=None):
    """-> (mask int32[n, ceil(h/32)] holding the uint32 words, counts int32[n], list int32[n, h] or None)."""
    words = (L.h + 31) // 32
    mask = torch.empty(n, words, dtype=torch.int32, device=L.device)
    counts = torch.empty(n, dtype=torch.int32, device=L.device)
    lst = torch.empty(n, L.h, dtype=torch.int32, device=L.device) if want_list else None
    _check(lib().tardis_get_last_outliers(L.handle, n, _ptr(mask), _ptr(counts), _ptr(lst), _stream(stream)),
           "tardis_get_last_outliers")
    return mask, counts, lst


def tardis_get_last_union(L: Layer, n: int, want_mask: bool = False, stream=None):
    """-> (union_count int32[1] on the device, union mask int32[ceil(h/32)] or None)."""
    cnt = torch.empty(1, dtype=torch.int32, device=L.device)
    um = torch.empty((L.h + 31) // 32, dtype=torch.int32, device=L.device) if want_mask else None
    _check(lib().tardis_get_last_union(L.handle, n, _ptr(um), _ptr(cnt), _stream(stream)), "tardis_get_last_union")
    return cnt, um
