"""CPU oracle for the MMSE scale search -- TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It wraps ``mmse_oracle.c`` (plain C,
built by ``oracle/build.py``) through ctypes and shares nothing with the HIP
library.

Naming follows the C file: ``def_*`` is the fp64 definition of the objective
(Eq. 8, Section 3.4), ``can_*`` the canonical fp32 evaluation whose integer
decisions (argmin index, INT4 codes) the GPU must reproduce bit for bit.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# MMSE_ORACLE_LIB lets the mutation tests point the same Python wrapper at a deliberately broken build
_LIB_PATH = os.environ.get("MMSE_ORACLE_LIB") or os.path.join(_HERE, "libmmse_oracle.so")
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _b
        _b.build()
    lib = C.CDLL(_LIB_PATH)
    f32p, i32p, f64p, u8p = (C.POINTER(C.c_float), C.POINTER(C.c_int32),
                             C.POINTER(C.c_double), C.POINTER(C.c_uint8))
    i64, i32, f32, f64 = C.c_int64, C.c_int, C.c_float, C.c_double
    sig = {
        "def_sse": (f64, [f32p, i64, f64, i32, i32]),
        "def_sse_codes": (f64, [f32p, i32p, i64, f64]),
        "def_sse_dual": (f64, [f32p, i32p, i32p, i64, f64, f64]),
        "can_absmax": (f32, [f32p, i64]),
        "can_grid_alpha": (f32, [f32, i32, i32, i32]),
        "can_sse": (f64, [f32p, i64, f32, i32, i32]),
        "can_search": (i32, [f32p, i64, i32, i32, i32, i32, f32p, i32p, f64p, f64p, f32p]),
        "can_search_kernelwise": (None, [f32p, i64, i64, i32, i32, i32, i32, f32p, i32p, f64p]),
        "can_codes": (None, [f32p, i64, i64, f32p, i32, i32, i32p]),
        "can_pack_int4": (None, [i32p, i64, u8p]),
        "can_unpack_int4": (None, [u8p, i64, i32, i32p]),
        "can_quantize_pack_int4": (None, [f32p, i64, i64, f32p, i32, i32, u8p]),
        "can_residual": (None, [f32p, i64, i64, f32p, i32, i32, f32p]),
        "can_residual_quantize": (None, [f32p, i64, i64, f32p, i32, i32, i32, i32, f32p, i32p, f64p, u8p]),
        "can_dual_alternating_kernelwise": (None, [f32p, i64, i64, i32, i32, i32, i32, f64, i32,
                                                   f32p, f32p, u8p, u8p, f64p, i32p]),
        "def_dual_sse": (f64, [f32p, i64, f64, f64, i32, i32]),
        "can_dual_sse": (f64, [f32p, i64, f32, f32, i32, i32]),
        "can_dual_alpha2": (f32, [f32, i32, i32]),
        "can_dual_codes": (None, [f32p, i64, f32, f32, i32, i32, i32p, i32p]),
        "can_dual_linesearch": (i32, [f32p, i64, i32, i32, i32, i32, f32p, f32p, i32p, i32p, f64p, i32p, i32p, f64p]),
        "can_dual_linesearch_kernelwise": (None, [f32p, i64, i64, i32, i32, i32, i32, f32p, f32p, i32p, i32p, f64p,
                                                  u8p, u8p]),
        "can_act_residual_quantize": (i32, [f32p, i64, f32, i32, i32, i32, i32, i32, i32, f32p, i32p, f64p, u8p]),
        "def_offset_sse": (f64, [f32p, i64, f64, f64, i32]),
        "can_min": (f32, [f32p, i64]),
        "can_offset_search": (i32, [f32p, i64, i32, i32, i32, f32p, f32p, i32p, f64p, u8p]),
        "can_alternating_scale": (i32, [f32p, i64, i32, i32, i32, f32p, f64p, i32p]),
        "can_alternating_scale_kernelwise": (None, [f32p, i64, i64, i32, i32, i32, f32p, f64p, i32p]),
        "oracle_num_threads": (i32, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


# ----------------------------------------------------------------- definition
def def_sse(x, alpha: float, qmin: int, qmax: int) -> float:
    x = _f32(x).ravel()
    return float(_load().def_sse(_p(x, C.c_float), x.size, float(alpha), qmin, qmax))


def def_sse_codes(x, codes, alpha: float) -> float:
    x = _f32(x).ravel()
    q = np.ascontiguousarray(codes, dtype=np.int32).ravel()
    assert q.size == x.size
    return float(_load().def_sse_codes(_p(x, C.c_float), _p(q, C.c_int32), x.size, float(alpha)))


def def_sse_dual(x, q1, q2, a1: float, a2: float) -> float:
    x = _f32(x).ravel()
    q1 = np.ascontiguousarray(q1, dtype=np.int32).ravel()
    q2 = np.ascontiguousarray(q2, dtype=np.int32).ravel()
    assert q1.size == x.size and q2.size == x.size
    return float(_load().def_sse_dual(_p(x, C.c_float), _p(q1, C.c_int32), _p(q2, C.c_int32),
                                      x.size, float(a1), float(a2)))


# ------------------------------------------------------------------ canonical
def can_absmax(x) -> np.float32:
    x = _f32(x).ravel()
    return np.float32(_load().can_absmax(_p(x, C.c_float), x.size))


def can_grid(absmax, qmax: int, G: int) -> np.ndarray:
    lib = _load()
    return np.array([lib.can_grid_alpha(float(np.float32(absmax)), qmax, G, j) for j in range(G)],
                    dtype=np.float32)


def can_sse(x, alpha, qmin: int, qmax: int) -> float:
    x = _f32(x).ravel()
    return float(_load().can_sse(_p(x, C.c_float), x.size, float(np.float32(alpha)), qmin, qmax))


def can_search(x, qmin: int, qmax: int, G: int, iters: int, want_grid: bool = False,
               want_probes: bool = False):
    """One problem.  Returns dict(scale, idx, sse[, grid_sse][, probes], rc)."""
    x = _f32(x).ravel()
    scale = np.zeros(1, np.float32)
    idx = np.zeros(1, np.int32)
    sse = np.zeros(1, np.float64)
    grid = np.zeros(G, np.float64) if want_grid else None
    probes = np.zeros(2 + iters, np.float32) if want_probes else None
    rc = _load().can_search(_p(x, C.c_float), x.size, qmin, qmax, G, iters,
                            _p(scale, C.c_float), _p(idx, C.c_int32), _p(sse, C.c_double),
                            _p(grid, C.c_double) if want_grid else None,
                            _p(probes, C.c_float) if want_probes else None)
    out = {"scale": scale[0], "idx": int(idx[0]), "sse": float(sse[0]), "rc": int(rc)}
    if want_grid:
        out["grid_sse"] = grid
    if want_probes:
        out["probes"] = probes
    return out


def can_search_kernelwise(w, qmin: int, qmax: int, G: int, iters: int
                          ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    w = _f32(w)
    assert w.ndim == 2
    K, n = w.shape
    scale = np.zeros(K, np.float32)
    idx = np.zeros(K, np.int32)
    sse = np.zeros(K, np.float64)
    _load().can_search_kernelwise(_p(w, C.c_float), K, n, qmin, qmax, G, iters,
                                  _p(scale, C.c_float), _p(idx, C.c_int32), _p(sse, C.c_double))
    return scale, idx, sse


def can_codes(x, scale, qmin: int, qmax: int) -> np.ndarray:
    x = _f32(x)
    if x.ndim == 1:
        x = x[None, :]
    K, n = x.shape
    scale = _f32(scale).ravel()
    assert scale.size == K
    codes = np.zeros((K, n), np.int32)
    _load().can_codes(_p(x, C.c_float), K, n, _p(scale, C.c_float), qmin, qmax, _p(codes, C.c_int32))
    return codes


def can_pack_int4(codes) -> np.ndarray:
    q = np.ascontiguousarray(codes, dtype=np.int32).ravel()
    out = np.zeros((q.size + 1) // 2, np.uint8)
    _load().can_pack_int4(_p(q, C.c_int32), q.size, _p(out, C.c_uint8))
    return out


def can_unpack_int4(packed, count: int, signed: bool) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    assert p.size == (count + 1) // 2
    out = np.zeros(count, np.int32)
    _load().can_unpack_int4(_p(p, C.c_uint8), count, int(signed), _p(out, C.c_int32))
    return out


def can_quantize_pack_int4(x, scale, qmin: int, qmax: int) -> np.ndarray:
    x = _f32(x)
    if x.ndim == 1:
        x = x[None, :]
    K, n = x.shape
    scale = _f32(scale).ravel()
    assert scale.size == K
    out = np.zeros((K * n + 1) // 2, np.uint8)
    _load().can_quantize_pack_int4(_p(x, C.c_float), K, n, _p(scale, C.c_float), qmin, qmax,
                                   _p(out, C.c_uint8))
    return out


def can_residual(w, scale1, qmin: int, qmax: int) -> np.ndarray:
    w = _f32(w)
    K, n = w.shape
    scale1 = _f32(scale1).ravel()
    assert scale1.size == K
    out = np.zeros((K, n), np.float32)
    _load().can_residual(_p(w, C.c_float), K, n, _p(scale1, C.c_float), qmin, qmax, _p(out, C.c_float))
    return out


def can_residual_quantize(w, scale1, qmin: int, qmax: int, G: int, iters: int):
    w = _f32(w)
    K, n = w.shape
    scale1 = _f32(scale1).ravel()
    assert scale1.size == K
    scale2 = np.zeros(K, np.float32)
    idx2 = np.zeros(K, np.int32)
    sse2 = np.zeros(K, np.float64)
    packed2 = np.zeros((K * n + 1) // 2, np.uint8)
    _load().can_residual_quantize(_p(w, C.c_float), K, n, _p(scale1, C.c_float), qmin, qmax, G, iters,
                                  _p(scale2, C.c_float), _p(idx2, C.c_int32), _p(sse2, C.c_double),
                                  _p(packed2, C.c_uint8))
    return scale2, idx2, sse2, packed2


def can_dual_alternating(w, qmin: int, qmax: int, G: int, iters: int, eps: float, max_sweeps: int):
    """Algorithm 1 iterated for two tensors, per kernel.  Returns dict(scale1, scale2, packed1, packed2, sse, sweeps)."""
    w = _f32(w)
    K, n = w.shape
    out = {"scale1": np.zeros(K, np.float32), "scale2": np.zeros(K, np.float32),
           "packed1": np.zeros((K * n + 1) // 2, np.uint8), "packed2": np.zeros((K * n + 1) // 2, np.uint8),
           "sse": np.zeros(K, np.float64), "sweeps": np.zeros(K, np.int32)}
    _load().can_dual_alternating_kernelwise(
        _p(w, C.c_float), K, n, qmin, qmax, G, iters, float(eps), int(max_sweeps),
        _p(out["scale1"], C.c_float), _p(out["scale2"], C.c_float), _p(out["packed1"], C.c_uint8),
        _p(out["packed2"], C.c_uint8), _p(out["sse"], C.c_double), _p(out["sweeps"], C.c_int32))
    return out


# ------------------------------------------------------------------ dual line search (Eq. 12)
def def_dual_sse(x, a1: float, a2: float, qmin: int, qmax: int) -> float:
    x = _f32(x).ravel()
    return float(_load().def_dual_sse(_p(x, C.c_float), x.size, float(a1), float(a2), qmin, qmax))


def can_dual_sse(x, a1, a2, qmin: int, qmax: int) -> float:
    x = _f32(x).ravel()
    return float(_load().can_dual_sse(_p(x, C.c_float), x.size, float(np.float32(a1)), float(np.float32(a2)),
                                      qmin, qmax))


def can_dual_alpha2(a1, G2: int, b: int) -> np.float32:
    return np.float32(_load().can_dual_alpha2(float(np.float32(a1)), G2, b))


def can_dual_codes(x, a1, a2, qmin: int, qmax: int):
    x = _f32(x).ravel()
    q1 = np.zeros(x.size, np.int32)
    q2 = np.zeros(x.size, np.int32)
    _load().can_dual_codes(_p(x, C.c_float), x.size, float(np.float32(a1)), float(np.float32(a2)), qmin, qmax,
                           _p(q1, C.c_int32), _p(q2, C.c_int32))
    return q1, q2


def can_dual_linesearch(x, qmin: int, qmax: int, G1: int, G2: int, want_grid: bool = False):
    x = _f32(x).ravel()
    a1, a2 = np.zeros(1, np.float32), np.zeros(1, np.float32)
    ia, ib = np.zeros(1, np.int32), np.zeros(1, np.int32)
    sse = np.zeros(1, np.float64)
    q1, q2 = np.zeros(x.size, np.int32), np.zeros(x.size, np.int32)
    grid = np.zeros((G1, G2), np.float64) if want_grid else None
    rc = _load().can_dual_linesearch(_p(x, C.c_float), x.size, qmin, qmax, G1, G2, _p(a1, C.c_float),
                                     _p(a2, C.c_float), _p(ia, C.c_int32), _p(ib, C.c_int32), _p(sse, C.c_double),
                                     _p(q1, C.c_int32), _p(q2, C.c_int32),
                                     _p(grid, C.c_double) if want_grid else None)
    out = {"scale1": a1[0], "scale2": a2[0], "idx1": int(ia[0]), "idx2": int(ib[0]), "sse": float(sse[0]),
           "q1": q1, "q2": q2, "rc": int(rc)}
    if want_grid:
        out["grid"] = grid
    return out


def can_dual_linesearch_kernelwise(w, qmin: int, qmax: int, G1: int, G2: int):
    w = _f32(w)
    K, n = w.shape
    out = {"scale1": np.zeros(K, np.float32), "scale2": np.zeros(K, np.float32),
           "idx1": np.zeros(K, np.int32), "idx2": np.zeros(K, np.int32), "sse": np.zeros(K, np.float64),
           "packed1": np.zeros((K * n + 1) // 2, np.uint8), "packed2": np.zeros((K * n + 1) // 2, np.uint8)}
    _load().can_dual_linesearch_kernelwise(
        _p(w, C.c_float), K, n, qmin, qmax, G1, G2, _p(out["scale1"], C.c_float), _p(out["scale2"], C.c_float),
        _p(out["idx1"], C.c_int32), _p(out["idx2"], C.c_int32), _p(out["sse"], C.c_double),
        _p(out["packed1"], C.c_uint8), _p(out["packed2"], C.c_uint8))
    return out


def can_act_residual_quantize(x, beta1, q1, q2, G: int, iters: int):
    """Eq. 16: second tensor of an activation.  q1, q2 = (qmin, qmax) of the first and second tensor."""
    x = _f32(x).ravel()
    b2, idx, sse = np.zeros(1, np.float32), np.zeros(1, np.int32), np.zeros(1, np.float64)
    packed = np.zeros((x.size + 1) // 2, np.uint8)
    rc = _load().can_act_residual_quantize(_p(x, C.c_float), x.size, float(beta1), q1[0], q1[1], q2[0], q2[1],
                                           G, iters, _p(b2, C.c_float), _p(idx, C.c_int32), _p(sse, C.c_double),
                                           _p(packed, C.c_uint8))
    return {"scale": b2[0], "idx": int(idx[0]), "sse": float(sse[0]), "packed": packed, "rc": int(rc)}


def def_offset_sse(x, delta: float, alpha: float, qmax: int) -> float:
    x = _f32(x).ravel()
    return float(_load().def_offset_sse(_p(x, C.c_float), x.size, float(delta), float(alpha), qmax))


def can_min(x) -> np.float32:
    x = _f32(x).ravel()
    return np.float32(_load().can_min(_p(x, C.c_float), x.size))


def can_offset_search(x, qmax: int, G: int, iters: int):
    """Eq. 2 with the MMSE scale: dict(delta, scale, idx, sse, packed, rc)."""
    x = _f32(x).ravel()
    d, a = np.zeros(1, np.float32), np.zeros(1, np.float32)
    idx, sse = np.zeros(1, np.int32), np.zeros(1, np.float64)
    packed = np.zeros((x.size + 1) // 2, np.uint8)
    rc = _load().can_offset_search(_p(x, C.c_float), x.size, qmax, G, iters, _p(d, C.c_float), _p(a, C.c_float),
                                   _p(idx, C.c_int32), _p(sse, C.c_double), _p(packed, C.c_uint8))
    return {"delta": d[0], "scale": a[0], "idx": int(idx[0]), "sse": float(sse[0]), "packed": packed, "rc": int(rc)}


def can_alternating_scale(x, qmin: int, qmax: int, max_iters: int):
    """Alternating optimisation of Section 3.4's comparison: dict(scale, sse, updates, rc)."""
    x = _f32(x).ravel()
    a, e, u = np.zeros(1, np.float32), np.zeros(1, np.float64), np.zeros(1, np.int32)
    rc = _load().can_alternating_scale(_p(x, C.c_float), x.size, qmin, qmax, max_iters, _p(a, C.c_float),
                                       _p(e, C.c_double), _p(u, C.c_int32))
    return {"scale": a[0], "sse": float(e[0]), "updates": int(u[0]), "rc": int(rc)}


def can_alternating_scale_kernelwise(w, qmin: int, qmax: int, max_iters: int):
    w = _f32(w)
    K, n = w.shape
    a, e, u = np.zeros(K, np.float32), np.zeros(K, np.float64), np.zeros(K, np.int32)
    _load().can_alternating_scale_kernelwise(_p(w, C.c_float), K, n, qmin, qmax, max_iters, _p(a, C.c_float),
                                             _p(e, C.c_double), _p(u, C.c_int32))
    return a, e, u
