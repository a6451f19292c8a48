"""CPU fp64 oracle (test infrastructure, NOT part of the product path).

Thin ctypes loader around ``flexsp_oracle.c`` (plain C, fp64, sequential sums).
Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It imports nothing from the HIP library or its binding.

What is computed: paper Sec. 2.1.2 Eq. 3 (attention on complete sequences for the
heads a device holds), per sequence of a packed stream (Sec. 2.2.2, no
cross-contamination), its gradient for L = sum(O * dO), and the local layout
permute either side of the exchanges of Eq. 2 / Eq. 4.

Every function here is pinned by tests/test_oracle_pins.py (brute force through an
independent dense formulation, closed forms, finite differences, invariants); no
function is "parity unpinned".

Array conventions: bf16 tensors are ``numpy.uint16`` bit patterns, widened exactly
to fp64 inside the C code; fp64 inputs are accepted too (needed by the
finite-difference pins).  q, dO, O, dQ are [T, Hq, D]; k, v, dK, dV [T, Hkv, D];
LSE [Hq, T].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "flexsp_oracle.c"
_LIB = _HERE / "_build" / "libflexsp_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (no fast-math: summation order is the source's)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        _LIB.parent.mkdir(exist_ok=True)
        tmp = _LIB.with_suffix(".so.%d.tmp" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O3", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             "-std=c11", "-Wall", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(str(_LIB))
        for name in ("flexsp_oracle_attn", "flexsp_oracle_rows", "flexsp_oracle_dkv_rows",
                     "flexsp_oracle_pack", "flexsp_oracle_unpack"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _in(x):
    """-> (contiguous array, dtype code)"""
    if x is None:
        return None, None
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return np.ascontiguousarray(x), 1
    return np.ascontiguousarray(x, dtype=np.float64), 0


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _prep(q, k, v, dO, cu):
    q, dt = _in(q)
    k, dk = _in(k)
    v, dv = _in(v)
    assert dt == dk == dv, "q, k, v must share a dtype"
    if dO is not None:
        dO, dg = _in(dO)
        assert dg == dt
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    T, Hq, D = q.shape
    Tk, Hkv, Dk = k.shape
    assert v.shape == k.shape and Tk == T and Dk == D and cu[-1] == T
    return q, k, v, dO, dt, cu, T, Hq, Hkv, D


def attn_fwd(q, k, v, cu, causal=True, scale=None):
    """Forward over the packed batch. Returns (O [T,Hq,D] fp64, LSE [Hq,T] fp64)."""
    q, k, v, _, dt, cu, T, Hq, Hkv, D = _prep(q, k, v, None, cu)
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    O = np.zeros((T, Hq, D)); LSE = np.zeros((Hq, T))
    rc = _load().flexsp_oracle_attn(_p(q), _p(k), _p(v), None, dt, _p(cu), len(cu) - 1, Hq, Hkv, D,
                                    int(bool(causal)), ctypes.c_double(scale),
                                    _p(O), _p(LSE), None, None, None)
    if rc:
        raise ValueError("oracle: bad arguments")
    return O, LSE


def attn_fwd_bwd(q, k, v, dO, cu, causal=True, scale=None):
    """Forward and backward. Returns (O, LSE, dQ, dK, dV), all fp64."""
    q, k, v, dO, dt, cu, T, Hq, Hkv, D = _prep(q, k, v, dO, cu)
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    O = np.zeros((T, Hq, D)); LSE = np.zeros((Hq, T))
    dQ = np.zeros((T, Hq, D)); dK = np.zeros((T, Hkv, D)); dV = np.zeros((T, Hkv, D))
    rc = _load().flexsp_oracle_attn(_p(q), _p(k), _p(v), _p(dO), dt, _p(cu), len(cu) - 1, Hq, Hkv, D,
                                    int(bool(causal)), ctypes.c_double(scale),
                                    _p(O), _p(LSE), _p(dQ), _p(dK), _p(dV))
    if rc:
        raise ValueError("oracle: bad arguments")
    return O, LSE, dQ, dK, dV


def rows(q, k, v, dO, cu, tok, head, causal=True, scale=None):
    """Sampled rows: O_rows [N,D], LSE_rows [N], dQ_rows [N,D] (None if dO is None)
    for the (token, query head) samples."""
    q, k, v, dO, dt, cu, T, Hq, Hkv, D = _prep(q, k, v, dO, cu)
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    tok = np.ascontiguousarray(tok, dtype=np.int64)
    head = np.ascontiguousarray(head, dtype=np.int32)
    N = len(tok)
    O = np.zeros((N, D)); LSE = np.zeros(N)
    dQ = np.zeros((N, D)) if dO is not None else None
    rc = _load().flexsp_oracle_rows(_p(q), _p(k), _p(v), _p(dO), dt, _p(cu), len(cu) - 1, Hq, Hkv, D,
                                    int(bool(causal)), ctypes.c_double(scale),
                                    _p(tok), _p(head), N, _p(O), _p(LSE), _p(dQ))
    if rc:
        raise ValueError("oracle: bad arguments")
    return O, LSE, dQ


def dkv_rows(q, k, v, dO, cu, tasks, causal=True, scale=None):
    """Sampled dK/dV rows.  tasks = [(seq, kv_head, [j, ...]), ...] with j positions inside
    the sequence.  Returns (dK_rows, dV_rows), each [sum len(j-list), D], task-major."""
    q, k, v, dO, dt, cu, T, Hq, Hkv, D = _prep(q, k, v, dO, cu)
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    seq = np.array([t[0] for t in tasks], dtype=np.int32)
    kvh = np.array([t[1] for t in tasks], dtype=np.int32)
    joff = np.zeros(len(tasks) + 1, dtype=np.int32)
    joff[1:] = np.cumsum([len(t[2]) for t in tasks])
    jl = np.array([j for t in tasks for j in t[2]], dtype=np.int32)
    dK = np.zeros((int(joff[-1]), D)); dV = np.zeros((int(joff[-1]), D))
    rc = _load().flexsp_oracle_dkv_rows(_p(q), _p(k), _p(v), _p(dO), dt, _p(cu), len(cu) - 1, Hq, Hkv,
                                        D, int(bool(causal)), ctypes.c_double(scale),
                                        _p(seq), _p(kvh), _p(joff), _p(jl), len(tasks), _p(dK), _p(dV))
    if rc:
        raise ValueError("oracle: bad arguments")
    return dK, dV


def pack(x, P):
    """[T,H,D] -> [P,T,H/P,D], any fixed-size element type."""
    x = np.ascontiguousarray(x)
    T, H, D = x.shape
    out = np.empty((P, T, H // max(P, 1) if P > 0 and H % P == 0 else 0, D), dtype=x.dtype)
    rc = _load().flexsp_oracle_pack(_p(x), _p(out), ctypes.c_int64(T), H, D, P, x.dtype.itemsize)
    if rc:
        raise ValueError("oracle: bad arguments")
    return out


def unpack(x, ):
    """[P,T,Hp,D] -> [T,P*Hp,D]."""
    x = np.ascontiguousarray(x)
    P, T, Hp, D = x.shape
    out = np.empty((T, P * Hp, D), dtype=x.dtype)
    rc = _load().flexsp_oracle_unpack(_p(x), _p(out), ctypes.c_int64(T), P * Hp, D, P, x.dtype.itemsize)
    if rc:
        raise ValueError("oracle: bad arguments")
    return out
