"""numpy-facing wrapper of the CPU oracle (oracle/floe_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke run and the benchmark's cpu_baseline leg.
The HIP library and its Python binding never import this package, and this package imports nothing
from them.  All fp16 data crosses as numpy float16 arrays (bit patterns are passed through).
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build())

_u16p = C.POINTER(C.c_uint16)
_u32p = C.POINTER(C.c_uint32)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)


class _Expert(C.Structure):
    _fields_ = [("codes", _u32p), ("scale", _u16p), ("zero", _u16p), ("gd", _u16p)]


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


def _h(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


_lib.floe_oracle_half_to_float.restype = C.c_float
_lib.floe_oracle_half_to_float.argtypes = [C.c_uint16]
_lib.floe_oracle_float_to_half.restype = C.c_uint16
_lib.floe_oracle_float_to_half.argtypes = [C.c_float]
_lib.floe_oracle_double_to_half.restype = C.c_uint16
_lib.floe_oracle_double_to_half.argtypes = [C.c_double]
_lib.floe_oracle_threshold_for_sparsity.restype = C.c_float
_lib.floe_oracle_threshold_for_sparsity.argtypes = [_f32p, C.c_int, C.c_int]
_lib.floe_oracle_select.argtypes = [_f32p, C.c_int, C.c_float, _i32p]
_lib.floe_oracle_masked_dense_ffn.argtypes = [_f32p, _u16p, C.c_int, C.c_int, _u16p, C.c_float, _f64p]
_lib.floe_oracle_sparsified_ffn.argtypes = [C.c_int, _u16p, C.c_int, C.c_int, _u16p, _f32p, C.c_float, _f64p, _i32p,
                                            C.POINTER(C.c_int32), _f64p]


def set_threads(n: int) -> None:
    _lib.floe_oracle_set_threads(int(n))


def get_threads() -> int:
    return int(_lib.floe_oracle_get_threads())


def half_to_float(bits: int) -> float:
    return float(_lib.floe_oracle_half_to_float(bits))


def float_to_half(x: float) -> int:
    return int(_lib.floe_oracle_float_to_half(x))


def double_to_half(x: float) -> int:
    return int(_lib.floe_oracle_double_to_half(x))


def words_per_channel(d: int, bits: int) -> int:
    return int(_lib.floe_oracle_words_per_channel(d, bits))


def quantize(w_cm: np.ndarray, bits: int, group: int):
    """-> (codes uint32 [f][d*bits/32], scale fp16 [f][d/group], zero fp16 [f][d/group])"""
    w_cm = _h(w_cm)
    f, d = w_cm.shape
    wpc = words_per_channel(d, bits)
    codes = np.zeros((f, wpc), dtype=np.uint32)
    scale = np.zeros((f, d // group), dtype=np.float16)
    zero = np.zeros((f, d // group), dtype=np.float16)
    rc = _lib.floe_oracle_quantize(_p(w_cm, _u16p), f, d, bits, group, _p(codes, _u32p), _p(scale, _u16p), _p(zero, _u16p))
    if rc:
        raise ValueError("floe_oracle_quantize: invalid shape")
    return codes, scale, zero


def dequantize(codes, scale, zero, d: int, bits: int, group: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scale, zero = _h(scale), _h(zero)
    f = codes.shape[0]
    w = np.empty((f, d), dtype=np.float32)
    rc = _lib.floe_oracle_dequantize(_p(codes, _u32p), _p(scale, _u16p), _p(zero, _u16p), f, d, bits, group, _p(w, _f32p))
    if rc:
        raise ValueError("floe_oracle_dequantize: invalid shape")
    return w


def up_gemv(codes, scale, zero, d: int, bits: int, group: int, x) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scale, zero, x = _h(scale), _h(zero), _h(x)
    f = codes.shape[0]
    v = np.empty(f, dtype=np.float32)
    rc = _lib.floe_oracle_up_gemv(_p(codes, _u32p), _p(scale, _u16p), _p(zero, _u16p), f, d, bits, group, _p(x, _u16p), _p(v, _f32p))
    if rc:
        raise ValueError("floe_oracle_up_gemv: invalid shape")
    return v


def select(v, tau: float) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float32)
    idx = np.empty(v.size, dtype=np.int32)
    K = _lib.floe_oracle_select(_p(v, _f32p), v.size, C.c_float(tau), _p(idx, _i32p))
    return idx[:K].copy()


def threshold_for_sparsity(v, pct: int) -> float:
    v = np.ascontiguousarray(v, dtype=np.float32)
    return float(_lib.floe_oracle_threshold_for_sparsity(_p(v, _f32p), v.size, int(pct)))


def sparse_ffn(gd, x, v, idx, staged: bool = False):
    """-> (h float64 [K], y float64 [d])"""
    gd, x = _h(gd), _h(x)
    v = np.ascontiguousarray(v, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    d = gd.shape[-1]
    h = np.empty(idx.size, dtype=np.float64)
    y = np.empty(d, dtype=np.float64)
    rc = _lib.floe_oracle_sparse_ffn(_p(gd, _u16p), int(staged), d, _p(x, _u16p), _p(v, _f32p), _p(idx, _i32p), idx.size, _p(h, _f64p), _p(y, _f64p))
    if rc:
        raise ValueError("floe_oracle_sparse_ffn: invalid argument")
    return h, y


def dense_ffn(w_up_f32, gd, x) -> np.ndarray:
    w_up_f32 = np.ascontiguousarray(w_up_f32, dtype=np.float32)
    gd, x = _h(gd), _h(x)
    f, d = w_up_f32.shape
    y = np.empty(d, dtype=np.float64)
    rc = _lib.floe_oracle_dense_ffn(_p(w_up_f32, _f32p), _p(gd, _u16p), d, f, _p(x, _u16p), _p(y, _f64p))
    if rc:
        raise ValueError("floe_oracle_dense_ffn: invalid argument")
    return y


def masked_dense_ffn(w_up_f32, gd, x, tau: float) -> np.ndarray:
    w_up_f32 = np.ascontiguousarray(w_up_f32, dtype=np.float32)
    gd, x = _h(gd), _h(x)
    f, d = w_up_f32.shape
    y = np.empty(d, dtype=np.float64)
    rc = _lib.floe_oracle_masked_dense_ffn(_p(w_up_f32, _f32p), _p(gd, _u16p), d, f, _p(x, _u16p), C.c_float(tau), _p(y, _f64p))
    if rc:
        raise ValueError("floe_oracle_masked_dense_ffn: invalid argument")
    return y


SPARSIFY_UP, SPARSIFY_GATE, SPARSIFY_DOWN = 0, 1, 2


def sparsified_ffn(which: int, gd, x, a_up, tau: float):
    """Eq. 1 with S_t (Eq. 5) on a_up / a_gate / a_down (Eq. 3-4); returns (y[d], idx[K], act[f])."""
    gd = _h(gd)
    x = _h(x)
    a_up = np.ascontiguousarray(a_up, dtype=np.float32)
    f, _, d = gd.shape
    y = np.empty((d,), np.float64)
    idx = np.empty((f,), np.int32)
    K = C.c_int32(0)
    act = np.empty((f,), np.float64)
    rc = _lib.floe_oracle_sparsified_ffn(int(which), _p(gd, _u16p), d, f, _p(x, _u16p), _p(a_up, _f32p), C.c_float(tau),
                                         _p(y, _f64p), _p(idx, _i32p), C.byref(K), _p(act, _f64p))
    assert rc == 0, rc
    return y, idx[: K.value].copy(), act


def router(router_cm, x, top_k: int, renormalize: bool):
    """-> (ids int32 [top_k], weights float64 [top_k], probs float64 [n_experts])"""
    router_cm, x = _h(router_cm), _h(x)
    n, d = router_cm.shape
    ids = np.empty(top_k, dtype=np.int32)
    w = np.empty(top_k, dtype=np.float64)
    p = np.empty(n, dtype=np.float64)
    rc = _lib.floe_oracle_router(_p(router_cm, _u16p), n, d, _p(x, _u16p), top_k, int(renormalize), _p(ids, _i32p), _p(w, _f64p), _p(p, _f64p))
    if rc:
        raise ValueError("floe_oracle_router: invalid argument")
    return ids, w, p


def moe_layer(experts, n_shared: int, top_k: int, renormalize: bool, router_cm, x, tau, bits: int, group: int):
    """experts: list of (codes, scale, zero, gd) numpy tuples, routed experts first, then shared.

    -> dict(out fp16 [T][d], ids [T][top_k], weights [T][top_k], counts [T][top_k+n_shared], y float64 [T][d])
    """
    x = _h(x)
    T, d = x.shape
    n_all = len(experts)
    n_experts = n_all - n_shared
    keep = []
    arr = (_Expert * n_all)()
    f = experts[0][0].shape[0]
    for e, (codes, scale, zero, gd) in enumerate(experts):
        codes = np.ascontiguousarray(codes, dtype=np.uint32)
        scale, zero, gd = _h(scale), _h(zero), _h(gd)
        keep.append((codes, scale, zero, gd))
        arr[e] = _Expert(_p(codes, _u32p), _p(scale, _u16p), _p(zero, _u16p), _p(gd, _u16p))
    router_cm = _h(router_cm) if top_k > 0 else np.zeros((max(n_experts, 1), d), np.float16)
    tau = np.ascontiguousarray(tau, dtype=np.float32).reshape(T, n_all)
    slots = top_k + n_shared
    out = np.empty((T, d), dtype=np.float16)
    ids = np.empty((T, max(top_k, 1)), dtype=np.int32)
    w = np.empty((T, max(top_k, 1)), dtype=np.float64)
    counts = np.empty((T, slots), dtype=np.int32)
    y = np.empty((T, d), dtype=np.float64)
    rc = _lib.floe_oracle_moe_layer(arr, n_experts, n_shared, top_k, int(renormalize), _p(router_cm, _u16p), d, f, bits, group,
                                    _p(x, _u16p), T, _p(tau, _f32p), _p(out, _u16p), _p(ids, _i32p), _p(w, _f64p), _p(counts, _i32p), _p(y, _f64p))
    if rc:
        raise ValueError("floe_oracle_moe_layer: invalid argument")
    return dict(out=out, ids=ids[:, :top_k], weights=w[:, :top_k], counts=counts, y=y)


def stage_rows(gd, idx) -> np.ndarray:
    gd = _h(gd)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    d = gd.shape[-1]
    dst = np.empty((idx.size, 2, d), dtype=np.float16)
    rc = _lib.floe_oracle_stage_rows(_p(gd, _u16p), d, _p(idx, _i32p), idx.size, _p(dst, _u16p))
    if rc:
        raise ValueError("floe_oracle_stage_rows: invalid argument")
    return dst
