"""ctypes access to the CPU oracle (``rgc_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports this
module and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rgc_oracle.cpp")
_LIB = os.path.join(_HERE, "librgc_oracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
               "-pthread", "-o", _LIB, _SRC]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.rgc_oracle_k_for_density.restype = ctypes.c_int32
        L.rgc_oracle_k_for_density.argtypes = [ctypes.c_int64, ctypes.c_uint32]
        for name in ("rgc_oracle_compress_layer", "rgc_oracle_compress_layer_bruteforce"):
            fn = getattr(L, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float,
                           ctypes.c_int, _i32p, _f32p, _i32p]
        L.rgc_oracle_compress_layers.restype = ctypes.c_int
        L.rgc_oracle_compress_layers.argtypes = [
            ctypes.POINTER(_f32p), ctypes.POINTER(_f32p), ctypes.POINTER(_f32p),
            ctypes.POINTER(ctypes.c_int64), _i32p, ctypes.c_int32, ctypes.c_float, ctypes.c_int,
            ctypes.POINTER(_i32p), ctypes.POINTER(_f32p), _i32p, ctypes.c_int32]
        L.rgc_oracle_compress_layer_ex.restype = ctypes.c_int
        L.rgc_oracle_compress_layer_ex.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int32,
                                                   ctypes.c_float, ctypes.c_int, ctypes.c_int, _f32p,
                                                   _i32p, _f32p, _i32p]
        L.rgc_oracle_compress_layers_ex.restype = ctypes.c_int
        L.rgc_oracle_compress_layers_ex.argtypes = [
            ctypes.POINTER(_f32p), ctypes.POINTER(_f32p), ctypes.POINTER(_f32p),
            ctypes.POINTER(ctypes.c_int64), _i32p, ctypes.c_int32, ctypes.c_float, ctypes.c_int,
            ctypes.c_int, _f32p, ctypes.POINTER(_i32p), ctypes.POINTER(_f32p), _i32p, ctypes.c_int32]
        L.rgc_oracle_clip_coefficient.restype = ctypes.c_float
        L.rgc_oracle_clip_coefficient.argtypes = [ctypes.POINTER(_f32p), ctypes.POINTER(ctypes.c_int64),
                                                  ctypes.c_int32, ctypes.c_float, ctypes.c_int32,
                                                  ctypes.POINTER(ctypes.c_double)]
        L.rgc_oracle_compress_layer_asq.restype = ctypes.c_int
        L.rgc_oracle_compress_layer_asq.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int32,
                                                    ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                    _i32p, _f32p, _i32p]
        L.rgc_oracle_compress_layer_threshold.restype = ctypes.c_int
        L.rgc_oracle_compress_layer_threshold.argtypes = [
            _f32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_int, ctypes.c_int,
            _f32p, ctypes.c_int, _f32p, ctypes.c_int32, _i32p, _f32p, _i32p, ctypes.POINTER(ctypes.c_int64), _f32p]
        L.rgc_oracle_decompress_scalar.restype = ctypes.c_int
        L.rgc_oracle_decompress_scalar.argtypes = [ctypes.POINTER(_i32p), _f32p, _i32p, ctypes.c_int32, _f32p,
                                                   ctypes.c_int64, ctypes.c_float, ctypes.c_int]
        L.rgc_oracle_decompress.restype = ctypes.c_int
        L.rgc_oracle_decompress.argtypes = [
            ctypes.POINTER(_i32p), ctypes.POINTER(_f32p), _i32p, ctypes.c_int32, _f32p,
            ctypes.c_int64, ctypes.c_float, ctypes.c_int]
        L.rgc_oracle_hardware_threads.restype = ctypes.c_int32
        L.rgc_oracle_exact_sum.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int64]
        L.rgc_oracle_exact_sum.restype = ctypes.c_double
        L.rgc_oracle_hardware_threads.argtypes = []
        _lib = L
    return _lib


def _f32(a: np.ndarray) -> "_f32p":
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(_f32p)


def _i32(a: np.ndarray) -> "_i32p":
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(_i32p)


def k_for_density(n: int, ppm: int = 1000) -> int:
    return int(lib().rgc_oracle_k_for_density(int(n), int(ppm)))


def exact_sum(x: np.ndarray) -> float:
    """Sum of fp64 terms rounded once (nearest, ties to even): what the oracle's three long sums are built on."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    return float(lib().rgc_oracle_exact_sum(x.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), x.size))


def hardware_threads() -> int:
    return int(lib().rgc_oracle_hardware_threads())


def _scale_arg(grad_scale):
    """None, or a one-element float32 array holding the clipping coefficient."""
    if grad_scale is None:
        return None, None
    keep = np.array([grad_scale], dtype=np.float32)
    return keep, _f32(keep)


def compress_layer(grad: np.ndarray, residual: np.ndarray, k: int,
                   momentum: Optional[np.ndarray] = None, m: float = 0.0,
                   mask_momentum: bool = True, bruteforce: bool = False,
                   nesterov: bool = False, grad_scale: Optional[float] = None
                   ) -> Tuple[np.ndarray, np.ndarray, int]:
    """Compress one layer IN PLACE (residual, momentum are updated).

    Returns (out_idx int32[k], out_val float32[k], count).
    """
    n = grad.size
    out_idx = np.empty(k, dtype=np.int32)
    out_val = np.empty(k, dtype=np.float32)
    out_cnt = np.zeros(1, dtype=np.int32)
    if nesterov or grad_scale is not None:
        assert not bruteforce
        keep, sp = _scale_arg(grad_scale)
        rc = lib().rgc_oracle_compress_layer_ex(
            _f32(grad), _f32(residual), _f32(momentum) if momentum is not None else None, n, int(k),
            float(m), 1 if mask_momentum else 0, 1 if nesterov else 0, sp, _i32(out_idx),
            _f32(out_val), _i32(out_cnt))
        if rc != 0:
            raise ValueError("oracle rejected the arguments")
        return out_idx, out_val, int(out_cnt[0])
    fn = lib().rgc_oracle_compress_layer_bruteforce if bruteforce else lib().rgc_oracle_compress_layer
    rc = fn(_f32(grad), _f32(residual), _f32(momentum) if momentum is not None else None,
            n, int(k), float(m), 1 if mask_momentum else 0, _i32(out_idx), _f32(out_val),
            _i32(out_cnt))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out_idx, out_val, int(out_cnt[0])


def compress_layers(grads: Sequence[np.ndarray], residuals: Sequence[np.ndarray],
                    ks: Sequence[int], momenta: Optional[Sequence[np.ndarray]] = None,
                    m: float = 0.0, mask_momentum: bool = True, threads: int = 1,
                    nesterov: bool = False, grad_scale: Optional[float] = None
                    ) -> List[Tuple[np.ndarray, np.ndarray, int]]:
    """Compress a whole layer set in place, optionally on several host threads."""
    L = len(grads)
    out_idx = [np.empty(int(k), dtype=np.int32) for k in ks]
    out_val = [np.empty(int(k), dtype=np.float32) for k in ks]
    out_cnt = np.zeros(L, dtype=np.int32)
    g = (_f32p * L)(*[_f32(a) for a in grads])
    r = (_f32p * L)(*[_f32(a) for a in residuals])
    mo = (_f32p * L)(*[_f32(a) for a in momenta]) if momenta is not None else None
    oi = (_i32p * L)(*[_i32(a) for a in out_idx])
    ov = (_f32p * L)(*[_f32(a) for a in out_val])
    n = (ctypes.c_int64 * L)(*[int(a.size) for a in grads])
    kk = (ctypes.c_int32 * L)(*[int(k) for k in ks])
    keep, sp = _scale_arg(grad_scale)
    rc = lib().rgc_oracle_compress_layers_ex(g, r, mo, n, kk, L, float(m),
                                             1 if mask_momentum else 0, 1 if nesterov else 0, sp,
                                             oi, ov, _i32(out_cnt), int(threads))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return [(out_idx[l], out_val[l], int(out_cnt[l])) for l in range(L)]


def compress_layer_asq(grad: np.ndarray, residual: np.ndarray, k: int, sign: int,
                       momentum: Optional[np.ndarray] = None, m: float = 0.0,
                       mask_momentum: bool = True, bruteforce: bool = False
                       ) -> Tuple[np.ndarray, float, int]:
    """Alternating Signs Quantization of one layer IN PLACE: sign = +1 the k largest, -1 the k smallest.

    Returns (out_idx int32[k], mean as float32, count)."""
    out_idx = np.empty(k, dtype=np.int32)
    out_mean = np.zeros(1, dtype=np.float32)
    out_cnt = np.zeros(1, dtype=np.int32)
    rc = lib().rgc_oracle_compress_layer_asq(
        _f32(grad), _f32(residual), _f32(momentum) if momentum is not None else None, grad.size, int(k),
        float(m), 1 if mask_momentum else 0, int(sign), 1 if bruteforce else 0, _i32(out_idx),
        _f32(out_mean), _i32(out_cnt))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out_idx, np.float32(out_mean[0]), int(out_cnt[0])


def compress_layer_threshold(grad: np.ndarray, residual: np.ndarray, k: int, search: bool = True,
                             threshold: float = 0.0, cap: Optional[int] = None,
                             momentum: Optional[np.ndarray] = None, m: float = 0.0,
                             mask_momentum: bool = True, nesterov: bool = False,
                             grad_scale: Optional[float] = None):
    """Threshold binary search selection of one layer IN PLACE (Algorithm 3; search=False applies
    `threshold` as given).  cap defaults to 2k.

    Returns (out_idx int32[count], out_val float32[count], nnz, threshold float32,
    trace = (mean, max, counts taken, last ratio) or None)."""
    if cap is None:
        cap = 2 * int(k)
    out_idx = np.empty(cap, dtype=np.int32)
    out_val = np.empty(cap, dtype=np.float32)
    out_cnt = np.zeros(1, dtype=np.int32)
    nnz = ctypes.c_int64(0)
    thr = np.array([threshold], dtype=np.float32)
    trace = np.zeros(4, dtype=np.float32)
    sc = np.array([grad_scale], dtype=np.float32) if grad_scale is not None else None
    rc = lib().rgc_oracle_compress_layer_threshold(
        _f32(grad), _f32(residual), _f32(momentum) if momentum is not None else None, grad.size, int(k),
        float(m), 1 if mask_momentum else 0, 1 if nesterov else 0, _f32(sc) if sc is not None else None,
        1 if search else 0, _f32(thr), int(cap),
        _i32(out_idx), _f32(out_val), _i32(out_cnt), ctypes.byref(nnz), _f32(trace))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    c = int(out_cnt[0])
    tr = (np.float32(trace[0]), np.float32(trace[1]), int(trace[2]), float(trace[3])) if search else None
    return out_idx[:c].copy(), out_val[:c].copy(), int(nnz.value), np.float32(thr[0]), tr


def decompress_scalar(idx: Sequence[np.ndarray], values: Sequence[float], n: int, scale: float,
                      dense: Optional[np.ndarray] = None) -> np.ndarray:
    """Decompress one layer whose messages carry one value each."""
    N = len(idx)
    add = dense is not None
    if dense is None:
        dense = np.empty(n, dtype=np.float32)
    ip = (_i32p * max(N, 1))(*[_i32(a) for a in idx])
    val = np.array(list(values) if N else [0.0], dtype=np.float32)
    cnt = np.array([a.size for a in idx], dtype=np.int32) if N else np.zeros(1, np.int32)
    rc = lib().rgc_oracle_decompress_scalar(ip, _f32(val), _i32(cnt), N, _f32(dense), int(n), float(scale),
                                            1 if add else 0)
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return dense


def clip_coefficient(grads: Sequence[np.ndarray], max_norm: float, num_workers: int
                     ) -> Tuple[float, float]:
    """-> (coefficient as float32, squared L2 norm over all layers in fp64)."""
    L = len(grads)
    g = (_f32p * L)(*[_f32(a) for a in grads])
    n = (ctypes.c_int64 * L)(*[int(a.size) for a in grads])
    sq = ctypes.c_double(0.0)
    c = lib().rgc_oracle_clip_coefficient(g, n, L, float(max_norm), int(num_workers), ctypes.byref(sq))
    return float(np.float32(c)), float(sq.value)


def decompress(idx: Sequence[np.ndarray], val: Sequence[np.ndarray], n: int, scale: float,
               dense: Optional[np.ndarray] = None) -> np.ndarray:
    """Decompress one layer.  ``dense=None`` overwrites into a fresh buffer, else
    adds into ``dense`` in place (and returns it)."""
    N = len(idx)
    add = dense is not None
    if dense is None:
        dense = np.empty(n, dtype=np.float32)
    ip = (_i32p * max(N, 1))(*[_i32(a) for a in idx])
    vp = (_f32p * max(N, 1))(*[_f32(a) for a in val])
    cnt = np.array([a.size for a in idx], dtype=np.int32) if N else np.zeros(1, np.int32)
    rc = lib().rgc_oracle_decompress(ip, vp, _i32(cnt), N, _f32(dense), int(n), float(scale),
                                     1 if add else 0)
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return dense
