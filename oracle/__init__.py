"""ctypes loader for the CPU oracle (oracle/hsadmm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.

Functions take and return numpy arrays; all arithmetic happens in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hsadmm_oracle.c")
# HSADMM_ORACLE_LIB: load this build of the oracle instead (the sanitizer leg of the tests compiles one with
# -fsanitize=address,undefined into a temporary directory)
_LIB = os.environ.get("HSADMM_ORACLE_LIB") or os.path.join(_HERE, "libhsadmm_oracle.so")
_lib = None
last_call_seconds = 0.0     # wall time of the most recent C call (excludes numpy marshalling)

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a no-op when the library is newer than its source)."""
    if os.environ.get("HSADMM_ORACLE_LIB"):
        return _LIB                      # a build made by the caller: used as it is
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    f32p = ctypes.POINTER(ctypes.c_float)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.oracle_set_threads.argtypes = [ctypes.c_int]
    lib.oracle_set_threads.restype = None
    lib.oracle_get_threads.restype = ctypes.c_int
    lib.oracle_project.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p, i32p, i32p, i32p,
                                   ctypes.POINTER(f32p), ctypes.c_int32, f32p, f32p, f32p, u8p, f64p]
    lib.oracle_project.restype = ctypes.c_int
    lib.oracle_compact.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p, ctypes.c_int32,
                                   f32p, u8p, f32p, i64p, i32p, i64p]
    lib.oracle_compact.restype = ctypes.c_int
    lib.oracle_expand.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p, ctypes.c_int32,
                                  f32p, u8p, f32p]
    lib.oracle_expand.restype = ctypes.c_int
    lib.oracle_project_frozen.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p,
                                          ctypes.POINTER(f32p), ctypes.c_int32, f32p, f32p, f32p, u8p]
    lib.oracle_project_frozen.restype = ctypes.c_int
    f64pp = ctypes.POINTER(ctypes.c_double)
    lib.oracle_node_coefficients.argtypes = [ctypes.c_int32, f64pp, f64pp, ctypes.c_double, ctypes.c_int32,
                                             ctypes.c_int32, f32p, f32p]
    lib.oracle_node_coefficients.restype = ctypes.c_int
    lib.oracle_project_weighted.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p, i32p, i32p, i32p,
                                            ctypes.POINTER(f32p), ctypes.c_int32, f32p, f32p, f32p, f32p, f32p,
                                            f32p, f32p, u8p, f64p]
    lib.oracle_project_weighted.restype = ctypes.c_int
    lib.oracle_project_weighted_frozen.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, i32p,
                                                   ctypes.POINTER(f32p), ctypes.c_int32, f32p, f32p, f32p, f32p,
                                                   f32p, f32p, f32p, u8p]
    lib.oracle_project_weighted_frozen.restype = ctypes.c_int
    lib.oracle_dual_inter.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, f32p, f32p, f32p]
    lib.oracle_dual_inter.restype = ctypes.c_int
    lib.oracle_add_arenas.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, f32p, f32p, f32p]
    lib.oracle_add_arenas.restype = ctypes.c_int
    lib.oracle_residuals.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, ctypes.POINTER(f32p), ctypes.c_int32,
                                     f32p, f32p, f32p, f32p, f64p]
    lib.oracle_residuals.restype = ctypes.c_int
    lib.oracle_average.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(f32p), f32p]
    lib.oracle_average.restype = ctypes.c_int
    lib.oracle_mask_drift.argtypes = [ctypes.c_int32, i32p, i32p, i32p, i32p, u8p, u8p, i32p]
    lib.oracle_mask_drift.restype = ctypes.c_int
    lib.oracle_layer_sqnorms.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, f32p, f64p]
    lib.oracle_layer_sqnorms.restype = ctypes.c_int
    lib.oracle_stopping_test.argtypes = [ctypes.c_int32, i64p, ctypes.c_int32, ctypes.c_int32, f64p, f64p, f64p, f64p,
                                         ctypes.c_double, ctypes.c_double, i32p, i32p]
    lib.oracle_stopping_test.restype = ctypes.c_int
    lib.oracle_adapt_penalties.argtypes = [ctypes.c_int32, f64pp, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                           f64pp, f64pp, f32p, f32p]
    lib.oracle_adapt_penalties.restype = ctypes.c_int
    lib.oracle_scale_layers.argtypes = [ctypes.c_int32, i64p, i32p, i32p, i32p, f32p, f32p]
    lib.oracle_scale_layers.restype = ctypes.c_int
    lib.oracle_mask_or.argtypes = [ctypes.c_int64, ctypes.POINTER(u8p), ctypes.c_int32, u8p]
    lib.oracle_mask_or.restype = ctypes.c_int
    _lib = lib
    return lib


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def get_threads() -> int:
    return int(_load().oracle_get_threads())


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _cols(table):
    out = {}
    for name, dt in (("elem_off", np.int64), ("c_out", np.int32), ("c_in", np.int32),
                     ("khw", np.int32), ("mode", np.int32), ("k", np.int32)):
        out[name] = np.ascontiguousarray(table[name], dtype=dt)
    # channels kept by a layer under both constraints (mode 3); tables without such layers may omit it
    out["k_in"] = (np.ascontiguousarray(table["k_in"], dtype=np.int32) if "k_in" in table
                   else np.zeros(len(out["k"]), dtype=np.int32))
    # shape groups kept by a layer of mode 5 or 6 (after its channels); tables without such layers may omit it
    out["k_kern"] = (np.ascontiguousarray(table["k_kern"], dtype=np.int32) if "k_kern" in table
                     else np.zeros(len(out["k"]), dtype=np.int32))
    return out


def _poisoned_arena(t, n_arena):
    """Output arena pre-filled with NaN inside layers (so a write the C code forgets shows) and +0 in padding."""
    a = np.zeros(int(n_arena), dtype=np.float32)
    n = t["c_out"].astype(np.int64) * t["c_in"] * t["khw"]
    for off, cnt in zip(t["elem_off"], n):
        a[int(off):int(off) + int(cnt)] = np.nan
    return a


def groups_total(table) -> int:
    t = _cols(table)
    g = np.where(t["mode"] == 2, t["c_in"], t["c_out"]) + np.where(t["mode"] == 3, t["c_in"], 0)
    g = np.where(t["mode"] == 4, t["c_in"] * t["khw"], g)
    g = np.where(t["mode"] == 5, t["c_in"] + t["c_in"] * t["khw"], g)
    g = np.where(t["mode"] == 6, t["c_out"] + t["c_in"] + t["c_in"] * t["khw"], g)
    return int(g.sum())


def project(table, W, U, want_wbar: bool = False):
    """Steps (a)-(d).  W: [R, n_arena] float32; U: [n_arena] float32 (not modified).

    Returns dict(U=new U, Z, mask uint8[groups_total], key float64[groups_total], Wbar or None).
    """
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    W = np.ascontiguousarray(W, dtype=np.float32)
    assert W.ndim == 2
    R, n_arena = W.shape
    U_new = np.array(U, dtype=np.float32, copy=True, order="C")
    assert U_new.shape == (n_arena,)
    Z = _poisoned_arena(t, n_arena)
    Wbar = _poisoned_arena(t, n_arena) if want_wbar else None
    gt = groups_total(t)
    mask = np.zeros(gt, dtype=np.uint8)
    key = np.zeros(gt, dtype=np.float64)
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * R)(*[_p(W[r], ctypes.c_float) for r in range(R)])
    global last_call_seconds
    _t0 = time.perf_counter()
    rc = lib.oracle_project(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                            _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                            _p(t["mode"], ctypes.c_int32), _p(t["k"], ctypes.c_int32),
                            _p(t["k_in"], ctypes.c_int32), _p(t["k_kern"], ctypes.c_int32),
                            ptrs, R, _p(U_new, ctypes.c_float), _p(Z, ctypes.c_float),
                            _p(Wbar, ctypes.c_float) if want_wbar else None,
                            _p(mask, ctypes.c_uint8), _p(key, ctypes.c_double))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_project failed with code %d" % rc)
    return {"U": U_new, "Z": Z, "mask": mask, "key": key, "Wbar": Wbar}


def packed_capacity(table) -> int:
    t = _cols(table)
    return int((t["c_out"].astype(np.int64) * t["c_in"] * t["khw"]).sum())


def compact(table, src, mask, pack_align: int = 1):
    """Step (e1).  Returns dict(packed (trimmed to its used length), layer_off int64[L+1], kept_idx int32)."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    src = np.ascontiguousarray(src, dtype=np.float32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    gt = groups_total(t)
    assert mask.shape == (gt,)
    cap = packed_capacity(t) + L * (pack_align - 1)
    packed = np.zeros(cap, dtype=np.float32)
    layer_off = np.zeros(L + 1, dtype=np.int64)
    kept_idx = np.zeros(gt, dtype=np.int32)
    nk = ctypes.c_int64(0)
    global last_call_seconds
    _t0 = time.perf_counter()
    rc = lib.oracle_compact(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                            _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                            _p(t["mode"], ctypes.c_int32), int(pack_align),
                            _p(src, ctypes.c_float), _p(mask, ctypes.c_uint8),
                            _p(packed, ctypes.c_float), _p(layer_off, ctypes.c_int64),
                            _p(kept_idx, ctypes.c_int32), ctypes.byref(nk))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_compact failed with code %d" % rc)
    return {"packed": packed[:int(layer_off[L])], "layer_off": layer_off,
            "kept_idx": kept_idx[:nk.value]}


def expand(table, packed, mask, n_arena: int, pack_align: int = 1):
    """Step (e2).  Returns dst float32[n_arena] (padding between layers stays +0)."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    packed = np.ascontiguousarray(packed, dtype=np.float32)
    if packed.size == 0:
        packed = np.zeros(1, dtype=np.float32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    dst = _poisoned_arena(t, n_arena)
    global last_call_seconds
    _t0 = time.perf_counter()
    rc = lib.oracle_expand(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                           _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                           _p(t["mode"], ctypes.c_int32), int(pack_align),
                           _p(packed, ctypes.c_float), _p(mask, ctypes.c_uint8),
                           _p(dst, ctypes.c_float))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_expand failed with code %d" % rc)
    return dst


def project_frozen(table, W, U, mask, want_wbar: bool = False):
    """Frozen-mask branch: Z = (Wbar + U) under a given mask, dual update.  Returns dict(U, Z, Wbar or None)."""
    global last_call_seconds
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    W = np.ascontiguousarray(W, dtype=np.float32)
    R, n_arena = W.shape
    U_new = np.array(U, dtype=np.float32, copy=True, order="C")
    Z = _poisoned_arena(t, n_arena)
    Wbar = _poisoned_arena(t, n_arena) if want_wbar else None
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.shape == (groups_total(t),)
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * R)(*[_p(W[r], ctypes.c_float) for r in range(R)])
    _t0 = time.perf_counter()
    rc = lib.oracle_project_frozen(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                                   _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                                   _p(t["mode"], ctypes.c_int32), ptrs, R, _p(U_new, ctypes.c_float),
                                   _p(Z, ctypes.c_float), _p(Wbar, ctypes.c_float) if want_wbar else None,
                                   _p(mask, ctypes.c_uint8))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_project_frozen failed with code %d" % rc)
    return {"U": U_new, "Z": Z, "Wbar": Wbar}


def mask_or(masks):
    """Eq. (14): union of M masks (list of uint8 arrays of equal length)."""
    lib = _load()
    ms = [np.ascontiguousarray(m, dtype=np.uint8) for m in masks]
    n = ms[0].size
    assert all(m.shape == (n,) for m in ms)
    out = np.full(n, 255, dtype=np.uint8)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    ptrs = (u8p * len(ms))(*[_p(m, ctypes.c_uint8) for m in ms])
    rc = lib.oracle_mask_or(n, ptrs, len(ms), _p(out, ctypes.c_uint8))
    if rc != 0:
        raise ValueError("oracle_mask_or failed with code %d" % rc)
    return out


def mask_drift(table, mask_a, mask_b):
    """Section 4.5: per layer, the number of groups whose kept flag differs between the two masks (int32[L])."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    a = np.ascontiguousarray(mask_a, dtype=np.uint8)
    b = np.ascontiguousarray(mask_b, dtype=np.uint8)
    assert a.shape == b.shape == (groups_total(t),)
    out = np.full(L, -1, dtype=np.int32)
    rc = lib.oracle_mask_drift(L, _p(t["c_out"], ctypes.c_int32), _p(t["c_in"], ctypes.c_int32),
                               _p(t["khw"], ctypes.c_int32), _p(t["mode"], ctypes.c_int32),
                               _p(a, ctypes.c_uint8), _p(b, ctypes.c_uint8), _p(out, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_mask_drift failed with code %d" % rc)
    return out


def average(bufs):
    """Eq. (11): mean of M equally long float32 buffers (left-to-right sum in node order, times fl32(1/M))."""
    lib = _load()
    bs = [np.ascontiguousarray(b, dtype=np.float32) for b in bufs]
    n = bs[0].size
    assert all(b.shape == (n,) for b in bs)
    out = np.full(max(n, 1), np.nan, dtype=np.float32)
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * len(bs))(*[_p(b, ctypes.c_float) for b in bs])
    rc = lib.oracle_average(len(bs), n, ptrs, _p(out, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_average failed with code %d" % rc)
    return out[:n]


def node_coefficients(rho1, rho2, lam: float, M: int, P: int):
    """Eq. (9): a_l = P rho_1 / gamma_l, b_l = rho_2 / gamma_l with gamma_l = lambda/M + P rho_1 + rho_2 (fp32 arrays)."""
    lib = _load()
    r1 = np.ascontiguousarray(rho1, dtype=np.float64)
    r2 = np.ascontiguousarray(rho2, dtype=np.float64)
    L = r1.size
    a = np.zeros(L, dtype=np.float32)
    b = np.zeros(L, dtype=np.float32)
    rc = lib.oracle_node_coefficients(L, _p(r1, ctypes.c_double), _p(r2, ctypes.c_double), float(lam), int(M), int(P),
                                      _p(a, ctypes.c_float), _p(b, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_node_coefficients failed with code %d" % rc)
    return a, b


def project_weighted(table, W, U, Zg, Vd, a, b, want_wbar: bool = False):
    """Steps (a)-(d) with the full candidate of Eq. (9).  Returns dict(U, Z, mask, key, Wbar or None)."""
    global last_call_seconds
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    W = np.ascontiguousarray(W, dtype=np.float32)
    R, n_arena = W.shape
    U_new = np.array(U, dtype=np.float32, copy=True, order="C")
    Zg = np.ascontiguousarray(Zg, dtype=np.float32)
    Vd = np.ascontiguousarray(Vd, dtype=np.float32)
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.shape == (L,) and b.shape == (L,) and Zg.shape == (n_arena,) and Vd.shape == (n_arena,)
    Z = _poisoned_arena(t, n_arena)
    Wbar = _poisoned_arena(t, n_arena) if want_wbar else None
    gt = groups_total(t)
    mask = np.zeros(gt, dtype=np.uint8)
    key = np.zeros(gt, dtype=np.float64)
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * R)(*[_p(W[r], ctypes.c_float) for r in range(R)])
    _t0 = time.perf_counter()
    rc = lib.oracle_project_weighted(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                                     _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                                     _p(t["mode"], ctypes.c_int32), _p(t["k"], ctypes.c_int32),
                                     _p(t["k_in"], ctypes.c_int32), _p(t["k_kern"], ctypes.c_int32), ptrs, R,
                                     _p(U_new, ctypes.c_float), _p(Zg, ctypes.c_float), _p(Vd, ctypes.c_float),
                                     _p(a, ctypes.c_float), _p(b, ctypes.c_float), _p(Z, ctypes.c_float),
                                     _p(Wbar, ctypes.c_float) if want_wbar else None,
                                     _p(mask, ctypes.c_uint8), _p(key, ctypes.c_double))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_project_weighted failed with code %d" % rc)
    return {"U": U_new, "Z": Z, "mask": mask, "key": key, "Wbar": Wbar}


def project_weighted_frozen(table, W, U, Zg, Vd, a, b, mask, want_wbar: bool = False):
    """Retraining branch with the full candidate of Eq. (9): Z = z~ under a given mask, dual update.
    Returns dict(U, Z, Wbar or None)."""
    global last_call_seconds
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    W = np.ascontiguousarray(W, dtype=np.float32)
    R, n_arena = W.shape
    U_new = np.array(U, dtype=np.float32, copy=True, order="C")
    Zg = np.ascontiguousarray(Zg, dtype=np.float32)
    Vd = np.ascontiguousarray(Vd, dtype=np.float32)
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert a.shape == (L,) and b.shape == (L,) and Zg.shape == (n_arena,) and Vd.shape == (n_arena,)
    assert mask.shape == (groups_total(t),)
    Z = _poisoned_arena(t, n_arena)
    Wbar = _poisoned_arena(t, n_arena) if want_wbar else None
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * R)(*[_p(W[r], ctypes.c_float) for r in range(R)])
    _t0 = time.perf_counter()
    rc = lib.oracle_project_weighted_frozen(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                                            _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                                            _p(t["mode"], ctypes.c_int32), ptrs, R, _p(U_new, ctypes.c_float),
                                            _p(Zg, ctypes.c_float), _p(Vd, ctypes.c_float), _p(a, ctypes.c_float),
                                            _p(b, ctypes.c_float), _p(Z, ctypes.c_float),
                                            _p(Wbar, ctypes.c_float) if want_wbar else None, _p(mask, ctypes.c_uint8))
    last_call_seconds = time.perf_counter() - _t0
    if rc != 0:
        raise ValueError("oracle_project_weighted_frozen failed with code %d" % rc)
    return {"U": U_new, "Z": Z, "Wbar": Wbar}


def dual_inter(table, Zi, Zg, Vd):
    """Eq. (13): returns v + (z_i - z)."""
    lib = _load()
    t = _cols(table)
    V_new = np.array(Vd, dtype=np.float32, copy=True, order="C")
    Zi = np.ascontiguousarray(Zi, dtype=np.float32)
    Zg = np.ascontiguousarray(Zg, dtype=np.float32)
    rc = lib.oracle_dual_inter(len(t["c_out"]), _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                               _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                               _p(Zi, ctypes.c_float), _p(Zg, ctypes.c_float), _p(V_new, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_dual_inter failed with code %d" % rc)
    return V_new


def add_arenas(table, A, B):
    """c = z_i + v_i of Section 4.4.1 (padding stays +0)."""
    lib = _load()
    t = _cols(table)
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    C = _poisoned_arena(t, A.size)
    rc = lib.oracle_add_arenas(len(t["c_out"]), _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                               _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32),
                               _p(A, ctypes.c_float), _p(B, ctypes.c_float), _p(C, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_add_arenas failed with code %d" % rc)
    return C


def residuals(table, W, Zi, Zi_prev=None, Zg=None, Zg_prev=None):
    """Squared residual norms per layer, float64 array [4, L]: intra primal (summed over replicas), intra dual,
    inter primal, inter dual (the dual ones without their rho factors)."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    W = np.ascontiguousarray(W, dtype=np.float32)
    R = W.shape[0]
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * R)(*[_p(W[r], ctypes.c_float) for r in range(R)])
    arrs = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in (Zi, Zi_prev, Zg, Zg_prev)]
    out = np.full((4, L), np.nan, dtype=np.float64)
    rc = lib.oracle_residuals(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                              _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32), ptrs, R,
                              *[None if a is None else _p(a, ctypes.c_float) for a in arrs],
                              _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_residuals failed with code %d" % rc)
    return out


def adapt_penalties(sq, rho1, rho2, P: int, n_out: int, mu: float, tau_incr: float, tau_decr: float,
                    rho1_max: float, rho2_max: float):
    """Residual balancing per layer and level (Section 3.4; Algorithm 1, Phase 5).  sq: [4, L] squared residual sums
    as residuals() returns them.  Returns (rho1_new, rho2_new, scale_u, scale_v)."""
    lib = _load()
    sq = np.ascontiguousarray(sq, dtype=np.float64)
    r1 = np.array(rho1, dtype=np.float64).ravel().copy()
    r2 = np.array(rho2, dtype=np.float64).ravel().copy()
    L = r1.size
    if sq.size != 4 * L or r2.size != L:
        raise ValueError("adapt_penalties: sizes disagree")
    su = np.zeros(L, dtype=np.float32)
    sv = np.zeros(L, dtype=np.float32)
    rc = lib.oracle_adapt_penalties(L, _p(sq, ctypes.c_double), int(P), int(n_out), float(mu), float(tau_incr),
                                    float(tau_decr), float(rho1_max), float(rho2_max), _p(r1, ctypes.c_double),
                                    _p(r2, ctypes.c_double), _p(su, ctypes.c_float), _p(sv, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_adapt_penalties failed with code %d" % rc)
    return r1, r2, su, sv


def scale_layers(table, X, factor):
    """X * factor[layer] on every layer (a new array; padding copied)."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    out = np.array(X, dtype=np.float32).copy()
    f = np.ascontiguousarray(factor, dtype=np.float32)
    if f.size != L:
        raise ValueError("scale_layers: one factor per layer")
    rc = lib.oracle_scale_layers(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                                 _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32), _p(f, ctypes.c_float),
                                 _p(out, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_scale_layers failed with code %d" % rc)
    return out


def layer_sqnorms(table, X):
    """Squared Frobenius norm of every layer of the arena X, float64[L] (sequential fp64 sums)."""
    lib = _load()
    t = _cols(table)
    L = len(t["c_out"])
    X = np.ascontiguousarray(X, dtype=np.float32)
    out = np.zeros(L, dtype=np.float64)
    rc = lib.oracle_layer_sqnorms(L, _p(t["elem_off"], ctypes.c_int64), _p(t["c_out"], ctypes.c_int32),
                                  _p(t["c_in"], ctypes.c_int32), _p(t["khw"], ctypes.c_int32), _p(X, ctypes.c_float),
                                  _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_layer_sqnorms failed with code %d" % rc)
    return out


def stopping_test(n_elems, P: int, n_out: int, rho1, rho2, sq, mag, eps_abs: float, eps_rel: float):
    """Section 3.4's stopping test per layer.  sq: 4 x L squared residual sums, mag: 5 x L squared magnitudes
    (sum_j ||theta_j||^2, ||z_i||^2, ||z||^2, sum_j ||u_j||^2, ||v_i||^2).  Returns (done int32[L], all_done bool)."""
    lib = _load()
    n_elems = np.ascontiguousarray(n_elems, dtype=np.int64)
    L = n_elems.size
    rho1 = np.ascontiguousarray(rho1, dtype=np.float64)
    rho2 = np.ascontiguousarray(rho2, dtype=np.float64)
    sq = np.ascontiguousarray(sq, dtype=np.float64).reshape(-1)
    mag = np.ascontiguousarray(mag, dtype=np.float64).reshape(-1)
    if rho1.size != L or rho2.size != L or sq.size != 4 * L or mag.size != 5 * L:
        raise ValueError("one rho per layer, 4 residual sums and 5 magnitudes per layer")
    done = np.zeros(L, dtype=np.int32)
    every = ctypes.c_int32(0)
    rc = lib.oracle_stopping_test(L, _p(n_elems, ctypes.c_int64), int(P), int(n_out), _p(rho1, ctypes.c_double),
                                  _p(rho2, ctypes.c_double), _p(sq, ctypes.c_double), _p(mag, ctypes.c_double),
                                  float(eps_abs), float(eps_rel), _p(done, ctypes.c_int32), ctypes.byref(every))
    if rc != 0:
        raise ValueError("oracle_stopping_test failed with code %d" % rc)
    return done, bool(every.value)
