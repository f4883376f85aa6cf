"""ctypes front end of the CPU fp64 oracle (oracle/lory_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark; the product path never touches it.  It
shares no code with the HIP library and does not import the GPU package.

Every function takes numpy arrays (converted to float64, an exact widening
for float32 / bf16-representable inputs) and returns float64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lory_oracle.c")
_LIB = os.path.join(_HERE, "liblory_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lg = ctypes.c_long
        lib.lory_oracle_route.argtypes = [lg] * 5 + [dp] * 5
        lib.lory_oracle_ffn_fwd.argtypes = [lg] * 5 + [dp] * 8
        lib.lory_oracle_ffn_bwd.argtypes = [lg] * 5 + [dp] * 11
        lib.lory_oracle_route_bwd.argtypes = [lg] * 5 + [dp] * 5
        for f in (lib.lory_oracle_route, lib.lory_oracle_ffn_fwd, lib.lory_oracle_ffn_bwd,
                  lib.lory_oracle_route_bwd):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    """Threads the OpenMP loops will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    return len(os.sched_getaffinity(0))


def route(X, R, T: int) -> Dict[str, np.ndarray]:
    """X [B,L,d], R [d,E] -> hbar [B*N,d], e [B*N,E] (unshifted), w [B*N,E]."""
    X = _f64(X)
    R = _f64(R)
    B, L, d = X.shape
    E = R.shape[1]
    assert R.shape[0] == d
    if L % T != 0:
        raise ValueError("L must be a multiple of T")
    S = B * (L // T)
    hbar = np.empty((S, d))
    e = np.empty((S, E))
    w = np.empty((S, E))
    rc = _load().lory_oracle_route(B, L, T, d, E, _p(X), _p(R), _p(hbar), _p(e), _p(w))
    if rc:
        raise RuntimeError(f"lory_oracle_route failed ({rc})")
    return {"hbar": hbar, "e": e, "w": w}


def ffn_fwd(X, w, Wg, Wu, Wd, T: int, want_gu: bool = False) -> Dict[str, np.ndarray]:
    """X [..., d] with S*T rows in total, w [S,E] -> Y (same shape as X)."""
    X = _f64(X)
    w, Wg, Wu, Wd = _f64(w), _f64(Wg), _f64(Wu), _f64(Wd)
    E, d, dff = Wg.shape
    assert Wu.shape == (E, d, dff) and Wd.shape == (E, dff, d) and X.shape[-1] == d
    rows = X.size // d
    S = rows // T
    assert S * T == rows and w.shape == (S, E)
    Y = np.empty_like(X)
    G = np.empty((rows, dff)) if want_gu else None
    U = np.empty((rows, dff)) if want_gu else None
    rc = _load().lory_oracle_ffn_fwd(S, T, d, dff, E, _p(X), _p(w), _p(Wg), _p(Wu), _p(Wd),
                                     _p(Y), _p(G), _p(U))
    if rc:
        raise RuntimeError(f"lory_oracle_ffn_fwd failed ({rc})")
    out = {"Y": Y}
    if want_gu:
        out["G"], out["U"] = G, U
    return out


def ffn_bwd(X, w, Wg, Wu, Wd, dY, T: int) -> Dict[str, np.ndarray]:
    """Gradients of <Y, dY> w.r.t. X (FFN path only), the expert stacks and w."""
    X, dY = _f64(X), _f64(dY)
    w, Wg, Wu, Wd = _f64(w), _f64(Wg), _f64(Wu), _f64(Wd)
    E, d, dff = Wg.shape
    assert Wu.shape == (E, d, dff) and Wd.shape == (E, dff, d) and X.shape[-1] == d
    assert dY.shape == X.shape
    rows = X.size // d
    S = rows // T
    assert S * T == rows and w.shape == (S, E)
    dX = np.empty_like(X)
    dWg, dWu, dWd = np.empty_like(Wg), np.empty_like(Wu), np.empty_like(Wd)
    dw = np.empty((S, E))
    rc = _load().lory_oracle_ffn_bwd(S, T, d, dff, E, _p(X), _p(w), _p(Wg), _p(Wu), _p(Wd), _p(dY),
                                     _p(dX), _p(dWg), _p(dWu), _p(dWd), _p(dw))
    if rc:
        raise RuntimeError(f"lory_oracle_ffn_bwd failed ({rc})")
    return {"dX": dX, "dWg": dWg, "dWu": dWu, "dWd": dWd, "dw": dw}


def route_bwd(X, R, dw, T: int) -> Dict[str, np.ndarray]:
    """Router path of the layer's backward (stop gradient on segment 0)."""
    X, R, dw = _f64(X), _f64(R), _f64(dw)
    B, L, d = X.shape
    E = R.shape[1]
    dX_add = np.empty_like(X)
    dR = np.empty_like(R)
    rc = _load().lory_oracle_route_bwd(B, L, T, d, E, _p(X), _p(R), _p(dw), _p(dX_add), _p(dR))
    if rc:
        raise RuntimeError(f"lory_oracle_route_bwd failed ({rc})")
    return {"dX_add": dX_add, "dR": dR}


def layer_fwd(X, R, Wg, Wu, Wd, T: int) -> Dict[str, np.ndarray]:
    """Whole layer: route, then merged FFN (Algorithm 1)."""
    r = route(X, R, T)
    out = ffn_fwd(X, r["w"], Wg, Wu, Wd, T)
    out.update(r)
    return out


def layer_bwd(X, R, Wg, Wu, Wd, dY, T: int) -> Dict[str, np.ndarray]:
    """Whole-layer gradients: FFN backward, then the router backward added."""
    r = route(X, R, T)
    g = ffn_bwd(X, r["w"], Wg, Wu, Wd, dY, T)
    rb = route_bwd(X, R, g["dw"], T)
    g["dX_ffn"] = g["dX"]
    g["dX"] = g["dX"] + rb["dX_add"]
    g["dR"] = rb["dR"]
    g["w"] = r["w"]
    return g
