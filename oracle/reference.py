"""ctypes front end of ``lora_oracle.c`` (fp64 plain-loop definition of the
layer; paper sections 2.2, 4.4 and 5: backbone and adapter products computed
separately and summed).  TEST INFRASTRUCTURE ONLY; shares no code with the HIP
path."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lora_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liblora_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-std=c11", "-Wall", "-Wextra", _SRC, "-o", _LIB + ".tmp"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_lora_linear.restype = ctypes.c_int
        lib.oracle_lora_linear.argtypes = [
            ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64,
        ]
        _lib = lib
    return _lib


def oracle_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def oracle_linear(X: np.ndarray, W0: np.ndarray, req_adapter, req_ntok,
                  A: Sequence[Optional[np.ndarray]], B: Sequence[Optional[np.ndarray]],
                  ranks, scales, rows=None, return_v: bool = False):
    """Y (fp64, [T or len(rows), N]) of the layer for stored tensors.

    X [T,K], W0 [N,K], A[a] [r_a,K], B[a] [N,r_a]; all of one storage dtype,
    uint16 (bf16 bit patterns) or float32.  Entries of A/B may be None for
    adapters the batch does not use."""
    lib = _load()
    X = np.ascontiguousarray(X)
    W0 = np.ascontiguousarray(W0)
    if X.dtype == np.uint16:
        dt = 1
    elif X.dtype == np.float32:
        dt = 0
    else:
        raise TypeError("X must be uint16 (bf16 bits) or float32")
    assert W0.dtype == X.dtype
    T, K = X.shape
    N = W0.shape[0]
    assert W0.shape[1] == K
    req_adapter = np.ascontiguousarray(req_adapter, np.int32)
    req_ntok = np.ascontiguousarray(req_ntok, np.int32)
    ranks = np.ascontiguousarray(ranks, np.int32)
    scales = np.ascontiguousarray(scales, np.float32)
    n_ad = ranks.shape[0]
    keep = []
    Ap = (ctypes.c_void_p * max(n_ad, 1))()
    Bp = (ctypes.c_void_p * max(n_ad, 1))()
    for a in range(n_ad):
        for src, dst, shape in ((A, Ap, (int(ranks[a]), K)), (B, Bp, (N, int(ranks[a])))):
            t = src[a] if a < len(src) else None
            if t is None:
                dst[a] = None
            else:
                t = np.ascontiguousarray(t)
                assert t.dtype == X.dtype and t.shape == shape, (t.dtype, t.shape, shape)
                keep.append(t)
                dst[a] = t.ctypes.data
    if rows is not None:
        rows = np.ascontiguousarray(rows, np.int64)
        n_out = rows.shape[0]
    else:
        n_out = T
    Y = np.empty((n_out, N), np.float64)
    r_cap = int(ranks.max()) if n_ad else 0
    V = np.zeros((n_out, max(r_cap, 1)), np.float64) if return_v else None
    rc = lib.oracle_lora_linear(dt, T, K, N, _ptr(X), K, _ptr(W0), K,
                                req_adapter.shape[0], _ptr(req_adapter), _ptr(req_ntok),
                                n_ad, ctypes.cast(Ap, ctypes.c_void_p), ctypes.cast(Bp, ctypes.c_void_p),
                                _ptr(ranks), _ptr(scales),
                                _ptr(rows), n_out, _ptr(Y), N,
                                _ptr(V), V.shape[1] if V is not None else 0)
    if rc != 0:
        raise ValueError(f"oracle_lora_linear failed with code {rc}")
    return (Y, V) if return_v else Y


def oracle_workload(wl, p: int = 0, rows=None, return_v: bool = False):
    """Run the oracle on projection ``p`` of a ``workloads.Workload``; only the
    adapters the batch uses are materialised."""
    used = set(int(a) for a in wl.used_adapters())
    A = [wl.A(a, p) if a in used else None for a in range(wl.n_adapters)]
    B = [wl.B(a, p) if a in used else None for a in range(wl.n_adapters)]
    return oracle_linear(wl.X(p), wl.W0(p), wl.req_adapter, wl.req_ntok, A, B, wl.ranks, wl.scales,
                         rows=rows, return_v=return_v)
