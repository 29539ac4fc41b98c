"""Host-only checks of the C ABI: the library loads, exports every function the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2501_10054_amd import tardis as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "tardis.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tardis_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_function():
    lib = T.lib()
    names = _declared()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(T.EXPORTS) == names


def test_version_and_status_strings():
    assert T.lib().tardis_version() == 1
    seen = {T.status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert T.status_string(99) == "unknown status"


def _desc(**kw):
    base = dict(d=64, h=256, dtype=T.F32, act=0, W1=0x1000, b1=None, W2=0x2000, b2=None)
    base.update(kw)
    return T.tardis_ffn_desc(**base)


def test_fold_rejects_bad_arguments_without_a_gpu():
    lib = T.lib()
    h = C.c_void_p()
    p = C.c_void_p(0x4000)
    ok_opts = T.tardis_fold_opts(8, T.F32, 1, 0, 0)

    def fold(desc, lo=p, opts=ok_opts, out=h):
        return lib.tardis_fold(C.byref(desc) if desc is not None else None, lo, p, p, p,
                               C.byref(opts) if opts is not None else None, None,
                               C.byref(out) if out is not None else None)

    assert fold(None) == T.ERR_INVALID_ARG
    assert fold(_desc(), out=None) == T.ERR_INVALID_ARG
    assert fold(_desc(W1=None)) == T.ERR_INVALID_ARG
    assert fold(_desc(W2=None)) == T.ERR_INVALID_ARG
    assert fold(_desc(W1=0x1004)) == T.ERR_INVALID_ARG          # misaligned
    assert fold(_desc(d=0)) == T.ERR_SHAPE
    assert fold(_desc(h=-3)) == T.ERR_SHAPE
    assert fold(_desc(d=1 << 20)) == T.ERR_SHAPE
    assert fold(_desc(dtype=7)) == T.ERR_DTYPE
    assert fold(_desc(act=9)) == T.ERR_INVALID_ARG
    assert fold(_desc(), lo=None) == T.ERR_INVALID_ARG
    assert fold(_desc(), opts=T.tardis_fold_opts(5, T.F32, 1, 0, 0)) == T.ERR_INVALID_ARG       # 8, 4, 3, 2 only
    assert fold(_desc(), opts=T.tardis_fold_opts(1, T.F32, 1, 0, 0)) == T.ERR_INVALID_ARG
    assert fold(_desc(), opts=T.tardis_fold_opts(4, T.F32, 1, 0, 0.5)) == T.ERR_INVALID_ARG     # margin in [0, 0.5)
    assert fold(_desc(), opts=T.tardis_fold_opts(4, T.F32, 1, 0, -0.1)) == T.ERR_INVALID_ARG
    assert fold(_desc(), opts=T.tardis_fold_opts(4, T.F32, 1, 0, float('nan'))) == T.ERR_INVALID_ARG
    assert fold(_desc(), opts=T.tardis_fold_opts(16, T.F32, 1, 0, 0)) == T.ERR_INVALID_ARG
    assert fold(_desc(), opts=T.tardis_fold_opts(8, T.BF16, 1, 0, 0)) == T.ERR_DTYPE
    assert fold(_desc(), opts=T.tardis_fold_opts(8, T.FP8_E4M3, 1, 0, 0)) == T.ERR_DTYPE       # 8-bit W' needs a bf16 layer
    assert fold(_desc(), opts=T.tardis_fold_opts(8, T.F32, 0, 0, 0)) == T.ERR_SHAPE
    assert fold(_desc(), opts=T.tardis_fold_opts(8, T.F32, 1, 2, 0)) == T.ERR_INVALID_ARG       # deterministic is 0 or 1
    assert h.value is None


def test_calibrate_rejects_bad_arguments_without_a_gpu():
    lib = T.lib()
    p = C.c_void_p(0x4000)

    def cal(desc, X=p, n=16, t=0.9, lo=p):
        return lib.tardis_calibrate(C.byref(desc), X, n, t, None, lo, p, p, p, None)

    assert cal(_desc(), X=None) == T.ERR_INVALID_ARG
    assert cal(_desc(), lo=None) == T.ERR_INVALID_ARG
    assert cal(_desc(), n=0) == T.ERR_SHAPE
    assert cal(_desc(), n=1 << 20) == T.ERR_SHAPE
    assert cal(_desc(), t=0.0) == T.ERR_INVALID_ARG
    assert cal(_desc(), t=1.5) == T.ERR_INVALID_ARG
    assert cal(_desc(h=0)) == T.ERR_SHAPE

    def search(desc, X=p, n=16, t=0.9, step=0.1, lo=p):
        return lib.tardis_calibrate_search(C.byref(desc), X, n, t, None, step, lo, p, p, p, None)

    assert search(_desc(), X=None) == T.ERR_INVALID_ARG
    assert search(_desc(), lo=None) == T.ERR_INVALID_ARG
    assert search(_desc(), n=0) == T.ERR_SHAPE
    assert search(_desc(), n=8193) == T.ERR_SHAPE                # the search keeps more per sample in LDS
    assert search(_desc(), t=1.5) == T.ERR_INVALID_ARG
    assert search(_desc(), step=0.0) == T.ERR_INVALID_ARG
    assert search(_desc(), step=-1.0) == T.ERR_INVALID_ARG
    assert search(_desc(), step=float("inf")) == T.ERR_INVALID_ARG
    assert search(_desc(), step=float("nan")) == T.ERR_INVALID_ARG


def test_threshold_calls_reject_bad_arguments_without_a_gpu():
    lib = T.lib()
    p = C.c_void_p(0x4000)
    assert lib.tardis_assign_thresholds(None, 4, 0.9, 0.8, 1.0, p, None) == T.ERR_INVALID_ARG
    assert lib.tardis_assign_thresholds(p, 4, 0.9, 0.8, 1.0, None, None) == T.ERR_INVALID_ARG
    assert lib.tardis_assign_thresholds(p, 0, 0.9, 0.8, 1.0, p, None) == T.ERR_SHAPE
    assert lib.tardis_assign_thresholds(p, 4, 0.7, 0.8, 1.0, p, None) == T.ERR_INVALID_ARG      # t below t_min
    assert lib.tardis_assign_thresholds(p, 4, 0.95, 0.8, 0.9, p, None) == T.ERR_INVALID_ARG     # t above t_max
    assert lib.tardis_assign_thresholds(p, 4, 0.9, -0.1, 1.0, p, None) == T.ERR_INVALID_ARG
    assert lib.tardis_assign_thresholds(p, 4, 0.9, 0.8, 1.5, p, None) == T.ERR_INVALID_ARG
    assert lib.tardis_assign_thresholds(p, 4, float("nan"), 0.8, 1.0, p, None) == T.ERR_INVALID_ARG

    def est(desc, X=p, n=16, lo=p, err=p):
        return lib.tardis_estimate_errors(C.byref(desc), X, n, lo, p, p, p, err, None, None)

    assert est(_desc(), X=None) == T.ERR_INVALID_ARG
    assert est(_desc(), lo=None) == T.ERR_INVALID_ARG
    assert est(_desc(), err=None) == T.ERR_INVALID_ARG
    assert est(_desc(), n=0) == T.ERR_SHAPE
    assert est(_desc(d=0)) == T.ERR_SHAPE


def test_online_calls_reject_null_handle():
    lib = T.lib()
    p = C.c_void_p(0x4000)
    assert lib.tardis_ffn_forward(None, p, p, None) == T.ERR_STATE
    assert lib.tardis_ffn_forward_batched(None, p, 1, p, None) == T.ERR_STATE
    assert lib.tardis_dense_forward(None, p, 1, p, None) == T.ERR_STATE
    assert lib.tardis_get_folded(None, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_predictor_state(None, p, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_last_outliers(None, 1, p, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_handover(None, 1, p, None) == T.ERR_STATE
    assert lib.tardis_get_sketch_groups(None, p, None) == T.ERR_STATE
    arr = (C.c_void_p * 2)(None, None)
    assert lib.tardis_stack_forward(arr, 2, p, 1, C.c_void_p(0x8000), None) == T.ERR_STATE
    assert lib.tardis_stack_forward(None, 2, p, 1, C.c_void_p(0x8000), None) == T.ERR_INVALID_ARG
    assert lib.tardis_stack_forward(arr, 0, p, 1, C.c_void_p(0x8000), None) == T.ERR_INVALID_ARG
    assert lib.tardis_get_last_union(None, 1, p, p, None) == T.ERR_STATE
    assert lib.tardis_ffn_forward_static(None, p, 1, C.c_void_p(0x8000), None, None) == T.ERR_STATE
    assert lib.tardis_set_next_layer(None, None) == T.ERR_STATE
    assert lib.tardis_set_next_layer(p, None) == T.ERR_STATE     # not a handle this library made
    assert lib.tardis_destroy(None) == T.OK


def test_calls_reject_a_pointer_that_is_not_a_live_handle():
    """Every entry point looks the handle up in the table of live layers before touching it: a
    stale or foreign pointer is an error, never a dereference (0x4000 is not mapped)."""
    lib = T.lib()
    bogus = C.c_void_p(0x4000)
    p, q = C.c_void_p(0x10000), C.c_void_p(0x20000)
    assert lib.tardis_ffn_forward(bogus, p, q, None) == T.ERR_STATE
    assert lib.tardis_ffn_forward_batched(bogus, p, 1, q, None) == T.ERR_STATE
    assert lib.tardis_ffn_forward_static(bogus, p, 1, q, None, None) == T.ERR_STATE
    assert lib.tardis_dense_forward(bogus, p, 1, q, None) == T.ERR_STATE
    assert lib.tardis_get_folded(bogus, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_predictor_state(bogus, p, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_sketch_groups(bogus, p, None) == T.ERR_STATE
    assert lib.tardis_get_last_outliers(bogus, 1, p, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_last_union(bogus, 1, p, p, None) == T.ERR_STATE
    assert lib.tardis_get_handover(bogus, 1, p, None) == T.ERR_STATE
    arr = (C.c_void_p * 1)(bogus)
    assert lib.tardis_stack_forward(arr, 1, p, 1, q, None) == T.ERR_STATE
    assert lib.tardis_destroy(bogus) == T.ERR_STATE


def test_error_type_carries_status():
    with pytest.raises(T.TardisError) as e:
        T._check(T.ERR_SHAPE, "x")
    assert e.value.status == T.ERR_SHAPE and "shape" in str(e.value)
