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
                     "flexsp_oracle_attn_kvshard", "flexsp_oracle_pack", "flexsp_oracle_unpack"):
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


def attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal=True, scale=None):
    """Attention of each sequence's queries against one shard of its keys (context parallelism,
    paper Sec. 2.1.3, paragraph "Context Parallelism", and the appendix on integrating it): q [Tq,Hq,D]; k, v [Tk,Hkv,D] hold the shard;
    shard key j of sequence b is visible to its query i iff not causal or j <= i + shift[b].
    Returns (O [Tq,Hq,D], LSE [Hq,Tq]); a row that sees no key has O = 0 and LSE = -inf."""
    q, dt = _in(q)
    k, dk = _in(k)
    v, dv = _in(v)
    assert dt == dk == dv
    cu_q = np.ascontiguousarray(cu_q, dtype=np.int32)
    cu_k = np.ascontiguousarray(cu_k, dtype=np.int32)
    shift = np.ascontiguousarray(shift, dtype=np.int32)
    Tq, Hq, D = q.shape
    Tk, Hkv, Dk = k.shape
    assert v.shape == k.shape and Dk == D and cu_q[-1] == Tq and cu_k[-1] == Tk
    assert len(cu_q) == len(cu_k) == len(shift) + 1
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    O = np.zeros((Tq, Hq, D)); LSE = np.zeros((Hq, Tq))
    rc = _load().flexsp_oracle_attn_kvshard(_p(q), _p(k), _p(v), dt, _p(cu_q), _p(cu_k), _p(shift), len(shift), Hq,
                                            Hkv, D, int(bool(causal)), ctypes.c_double(scale), _p(O), _p(LSE))
    if rc:
        raise ValueError("oracle: bad arguments")
    return O, LSE


def attn_bwd_kvshard(q, k, v, dO, lse, delta, cu_q, cu_k, shift, causal=True, scale=None):
    """The backward's share of one key shard (context parallelism, paper Sec. 2.1.3 and the appendix on
    integrating it; gradient of Sec. 2.1.2 Eq. 3).  `lse` [Hq,Tq] is each row's log-sum-exp over ALL its keys
    and `delta` [Hq,Tq] its sum_j P_ij dP_ij over all keys (= dO_i . O_i), both from the complete forward;
    with them the terms of the gradient separate by key:
        P_ij = exp(scale q_i.k_j - lse_i),  dP_ij = dO_i.v_j,  dS_ij = P_ij (dP_ij - delta_i)   (visible j of the shard)
        dQ_i (this shard's part) = scale sum_j dS_ij k_j,   dK_j = scale sum_i dS_ij q_i,   dV_j = sum_i P_ij dO_i.
    Visibility as in attn_fwd_kvshard.  Summed over the shards of a partition of the keys, the dQ parts give dQ
    of the complete attention, and each key's dK / dV are complete by themselves.  A row with lse = -inf (it
    saw no key anywhere) contributes nothing.  Returns (dQ_part [Tq,Hq,D], dK [Tk,Hkv,D], dV [Tk,Hkv,D]), fp64."""
    q, k, v, dO = (bf16_or_f64(x) for x in (q, k, v, dO))
    lse = np.asarray(lse, dtype=np.float64); delta = np.asarray(delta, dtype=np.float64)
    Tq, Hq, D = q.shape
    Tk, Hkv, _ = k.shape
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    dQ = np.zeros((Tq, Hq, D)); dK = np.zeros((Tk, Hkv, D)); dV = np.zeros((Tk, Hkv, D))
    for b in range(len(shift)):
        q0, q1, k0, k1 = int(cu_q[b]), int(cu_q[b + 1]), int(cu_k[b]), int(cu_k[b + 1])
        if q1 == q0 or k1 == k0:
            continue
        i = np.arange(q1 - q0)[:, None]; j = np.arange(k1 - k0)[None, :]
        visible = (j <= i + int(shift[b])) if causal else np.ones((q1 - q0, k1 - k0), dtype=bool)
        for h in range(Hq):
            g = h // G
            S = scale * (q[q0:q1, h] @ k[k0:k1, g].T)
            L = lse[h, q0:q1][:, None]
            with np.errstate(over="ignore", invalid="ignore"):
                P = np.where(visible & np.isfinite(L), np.exp(S - L), 0.0)
            dP = dO[q0:q1, h] @ v[k0:k1, g].T
            dS = P * (dP - delta[h, q0:q1][:, None])
            dQ[q0:q1, h] = scale * (dS @ k[k0:k1, g])
            dK[k0:k1, g] += scale * (dS.T @ q[q0:q1, h])
            dV[k0:k1, g] += P.T @ dO[q0:q1, h]
    return dQ, dK, dV


def bf16_or_f64(x):
    """uint16 bf16 bit patterns widened exactly to fp64; fp64 arrays as they are."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def lse_merge(o_a, lse_a, o_b, lse_b):
    """Two partial attentions of the same queries over disjoint key sets -> attention over the union:
    softmax weights of the union are the partial ones rescaled by exp(LSE_part - LSE_union).
    o [T,H,D], lse [H,T], fp64.  A part with LSE = -inf (no key) has weight 0; both: O = 0, LSE = -inf."""
    o_a, o_b = np.asarray(o_a, dtype=np.float64), np.asarray(o_b, dtype=np.float64)
    lse_a, lse_b = np.asarray(lse_a, dtype=np.float64), np.asarray(lse_b, dtype=np.float64)
    T, H, D = o_a.shape
    out = np.zeros((T, H, D)); lse = np.full((H, T), -np.inf)
    for t in range(T):
        for h in range(H):
            la, lb = lse_a[h, t], lse_b[h, t]
            m = max(la, lb)
            if m == -np.inf:
                continue
            wa, wb = np.exp(la - m), np.exp(lb - m)
            out[t, h] = (wa * o_a[t, h] + wb * o_b[t, h]) / (wa + wb)
            lse[h, t] = m + np.log(wa + wb)
    return out, lse


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
