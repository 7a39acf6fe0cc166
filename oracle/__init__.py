"""TEST INFRASTRUCTURE: CPU oracle for the BRA forward pass (ctypes loader).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the HIP library.  Status of its pins: every
function is pinned by tests/test_oracle_*.py (brute force, library routines on the
special cases, closed forms, invariants); nothing here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libbra_oracle.so")
_SRCS = [os.path.join(_HERE, "bra_oracle.c"), os.path.join(_HERE, "bra_oracle_impl.h")]
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP for the timed runs)."""
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRCS)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _SO, _SRCS[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
    return _lib


def default_scale(C: int, heads: int) -> float:
    """1/sqrt(d), d = C/heads: Eq. 1's scaling applied to Eq. 2's per-head operands."""
    return 1.0 / float(np.sqrt(C // heads))


def bra_forward(X, Wqkv, Wo, Wlce, *, S, k, heads, scale=None, Ir_in=None, precision="f64",
                threads=1, want=()):
    """Run the oracle.  X [B,H,W,C]; Wqkv [C,3C]; Wo [C,C]; Wlce [C,5,5].

    Returns a dict with "Y" [B,H,W,C], "Ir" [B,R,k] int32, "Ar" [B,R,R], "macs" (3,)
    and, when named in `want`: "P" [B,heads,R,n,kn], "Oatt" [B,H,W,C], "Lce" [B,H,W,C].
    """
    lib = _load()
    real = {"f32": np.float32, "f64": np.float64}[precision]
    creal = {"f32": ctypes.c_float, "f64": ctypes.c_double}[precision]
    fn = getattr(lib, "oracle_bra_forward_" + precision)
    X = np.ascontiguousarray(X, dtype=real)
    Wqkv = np.ascontiguousarray(Wqkv, dtype=real)
    Wo = np.ascontiguousarray(Wo, dtype=real)
    Wlce = np.ascontiguousarray(Wlce, dtype=real)
    B, H, W, C = X.shape
    assert Wqkv.shape == (C, 3 * C) and Wo.shape == (C, C) and Wlce.shape == (C, 5, 5)
    R = S * S
    n = (H // S) * (W // S)
    if scale is None:
        scale = default_scale(C, heads)
    Y = np.empty_like(X)
    Ir = np.empty((B, R, k), dtype=np.int32)
    Ar = np.empty((B, R, R), dtype=real)
    macs = np.zeros(3, dtype=np.int64)
    P = np.empty((B, heads, R, n, k * n), dtype=real) if "P" in want else None
    Oatt = np.empty_like(X) if "Oatt" in want else None
    Lce = np.empty_like(X) if "Lce" in want else None
    if Ir_in is not None:
        Ir_in = np.ascontiguousarray(Ir_in, dtype=np.int32)
        assert Ir_in.shape == (B, R, k)

    def ptr(a, ct):
        return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None

    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_int] * 7 + [ctypes.c_double] + [ctypes.POINTER(creal)] * 4 + [
        ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(creal), ctypes.POINTER(ctypes.c_int32)
    ] + [ctypes.POINTER(creal)] * 4 + [ctypes.POINTER(ctypes.c_int64), ctypes.c_int]
    rc = fn(B, H, W, C, heads, S, k, float(scale), ptr(X, creal), ptr(Wqkv, creal),
            ptr(Wo, creal), ptr(Wlce, creal), ptr(Ir_in, ctypes.c_int32), ptr(Y, creal),
            ptr(Ir, ctypes.c_int32), ptr(Ar, creal), ptr(P, creal), ptr(Oatt, creal),
            ptr(Lce, creal), ptr(macs, ctypes.c_int64), int(threads))
    if rc != 0:
        raise ValueError("oracle_bra_forward: invalid shape")
    out = {"Y": Y, "Ir": Ir, "Ar": Ar, "macs": macs}
    if P is not None:
        out["P"] = P
    if Oatt is not None:
        out["Oatt"] = Oatt
    if Lce is not None:
        out["Lce"] = Lce
    return out


def bra_forward_padded(X, Wqkv, Wo, Wlce, *, S, k, heads, scale=None, Ir_in=None, precision="f64", threads=1):
    """BRA on a map whose sides S does not divide (appendix on the choice of S and k: other sizes
    than multiples of S are padded).  Reading: zero tokens are appended at the bottom and at the
    right up to the next multiples of S, the layer runs on the padded map, and the top-left
    H x W part of its output is returned; "Ir" and "Ar" refer to the padded map's regions."""
    X = np.asarray(X)
    B, H, W, C = X.shape
    ph, pw = (-H) % S, (-W) % S
    Xp = np.pad(X, ((0, 0), (0, ph), (0, pw), (0, 0)))
    out = bra_forward(Xp, Wqkv, Wo, Wlce, S=S, k=k, heads=heads, scale=scale, Ir_in=Ir_in, precision=precision,
                      threads=threads)
    out["Y"] = np.ascontiguousarray(out["Y"][:, :H, :W, :])
    return out
