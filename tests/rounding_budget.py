"""What the GPU path's roundings allow: a per-element error budget for O, dQ, dK, dV.

The kernels compute Eq. 3 (paper Sec. 2.1.2) and its gradient with fp32 scores, statistics and
accumulators; the only roundings coarser than fp32 are, in this order:

  forward   P_ij -> bf16 before O += P V (the row sum l uses the unrounded fp32 P); O -> bf16 (store)
  backward  delta_i = dO_i . O_i is formed from the STORED (bf16) O;
            P_ij -> bf16 before dV += P^T dO;  dS_ij = P_ij (dP_ij - delta_i) -> bf16 before
            dQ += dS K and dK += dS^T Q;  dQ, dK, dV -> bf16 when gradients are stored as bf16.

One round-to-nearest to bf16 (8 significant bits) moves x by at most u|x|, u = 2^-8; modelled as
uniform on its interval it has standard deviation at most u|x|/sqrt(3).  Treating the roundings as
independent and keeping first-order terms:

  var O_id   = r^2 (sum_j P_ij^2 v_jd^2 + O_id^2)                                   r = u/sqrt(3)
  var dlt_i  = r^2 (sum_j P_ij^2 dP_ij^2 + sum_d dO_id^2 O_id^2)    (one P rounding moves every d of O_i)
  var dV_jd  = r^2 sum_{h,i} P_ij^2 dO_id^2                              [+ r^2 dV_jd^2 when stored as bf16]
  var dQ_id  = scale^2 (r^2 sum_j dS_ij^2 k_jd^2 + var dlt_i (sum_j P_ij k_jd)^2)   [+ r^2 dQ_id^2]
  var dK_jd  = scale^2 sum_{h,i} (r^2 dS_ij^2 + var dlt_i P_ij^2) q_id^2            [+ r^2 dK_jd^2]

fp32 accumulation, the hardware exp2 / log and the fp32 log-sum-exp contribute relative errors of
1e-6 and below and are covered by a small floor.  This module is test-side arithmetic in dense
numpy (whole score matrices, small cases only); it shares nothing with the library or the oracle.
"""
import numpy as np

U = 2.0 ** -8                # largest relative move of one round-to-nearest to bf16
R2 = U * U / 3.0             # variance of that move, relative, uniform model
SIGMAS = 8.0                 # tolerance = SIGMAS standard deviations (+ floor)
FLOOR_REL = 2e-5             # everything that is fp32: accumulation order, exp2, log, the stored LSE


def _bf16_f64(bits):
    return (np.asarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _dense(q, k, v, g, causal, scale):
    """One (sequence, head): dense P, dP, delta, dS and the exact results, fp64."""
    s = q.shape[0]
    S = scale * (q @ k.T)
    if causal:
        S = np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    O = P @ v
    dP = g @ v.T
    delta = (P * dP).sum(axis=1)
    dS = P * (dP - delta[:, None])
    return P, O, dP, delta, dS


def budget(q, k, v, dO, cu, causal=True, scale=None, grads_bf16=False):
    """Standard deviations of the rounding error per element: dict O, dQ [T,Hq,D]; dK, dV [T,Hkv,D].
    q, k, v, dO: bf16 bit patterns (uint16) or float arrays."""
    as64 = lambda x: _bf16_f64(x) if np.asarray(x).dtype == np.uint16 else np.asarray(x, dtype=np.float64)
    q, k, v, dO = as64(q), as64(k), as64(v), as64(dO)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    var = {"O": np.zeros((T, Hq, D)), "dQ": np.zeros((T, Hq, D)), "dK": np.zeros((T, Hkv, D)),
           "dV": np.zeros((T, Hkv, D))}
    mag = {n: np.zeros_like(a) for n, a in var.items()}      # |exact value|, for the store term and the floor
    for b in range(len(cu) - 1):
        t0, t1 = int(cu[b]), int(cu[b + 1])
        if t1 == t0:
            continue
        for h in range(Hq):
            kv = h // G
            qq, kk, vv, gg = q[t0:t1, h], k[t0:t1, kv], v[t0:t1, kv], dO[t0:t1, h]
            P, O, dP, delta, dS = _dense(qq, kk, vv, gg, causal, scale)
            P2, dS2 = P * P, dS * dS
            var["O"][t0:t1, h] = R2 * (P2 @ (vv * vv) + O * O)
            mag["O"][t0:t1, h] = np.abs(O)
            vdelta = R2 * ((P2 * dP * dP).sum(axis=1) + (gg * gg * O * O).sum(axis=1))
            var["dQ"][t0:t1, h] = scale ** 2 * (R2 * (dS2 @ (kk * kk)) + vdelta[:, None] * (P @ kk) ** 2)
            mag["dQ"][t0:t1, h] = np.abs(scale * (dS @ kk))
            var["dK"][t0:t1, kv] += scale ** 2 * ((R2 * dS2 + vdelta[:, None] * P2).T @ (qq * qq))
            var["dV"][t0:t1, kv] += R2 * (P2.T @ (gg * gg))
            mag["dK"][t0:t1, kv] += scale * (dS.T @ qq)       # signed sums over the group first
            mag["dV"][t0:t1, kv] += P.T @ gg
    for n in ("dK", "dV"):
        mag[n] = np.abs(mag[n])
    if grads_bf16:
        for n in ("dQ", "dK", "dV"):
            var[n] += R2 * mag[n] ** 2
    return {n: np.sqrt(var[n]) for n in var}, mag


def tolerance(sigma, mag):
    """Per-element tolerance the budget allows: SIGMAS standard deviations plus the fp32 floor."""
    return SIGMAS * sigma + FLOOR_REL * (1.0 + mag)


def emulate(q, k, v, dO, cu, causal=True, scale=None, grads_bf16=False):
    """The same mathematics with exactly the roundings listed above applied (fp64 otherwise): a
    stand-in for the GPU path on the CPU, used to check that the budget covers what those
    roundings do.  Returns O, dQ, dK, dV as fp64 arrays (O holds bf16-representable values)."""
    def rb(x):    # round to nearest even bf16
        x32 = np.ascontiguousarray(x, dtype=np.float32)
        u = x32.view(np.uint32)
        r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
        return r.view(np.float32).astype(np.float64)
    as64 = lambda x: _bf16_f64(x) if np.asarray(x).dtype == np.uint16 else np.asarray(x, dtype=np.float64)
    q, k, v, dO = as64(q), as64(k), as64(v), as64(dO)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    O = np.zeros((T, Hq, D)); dQ = np.zeros((T, Hq, D)); dK = np.zeros((T, Hkv, D)); dV = np.zeros((T, Hkv, D))
    for b in range(len(cu) - 1):
        t0, t1 = int(cu[b]), int(cu[b + 1])
        if t1 == t0:
            continue
        for h in range(Hq):
            kv = h // G
            qq, kk, vv, gg = q[t0:t1, h], k[t0:t1, kv], v[t0:t1, kv], dO[t0:t1, h]
            s = t1 - t0
            S = scale * (qq @ kk.T)
            if causal:
                S = np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf)
            E = np.exp(S - S.max(axis=1, keepdims=True))
            l = E.sum(axis=1, keepdims=True)
            Ost = rb((rb(E) @ vv) / l)
            O[t0:t1, h] = Ost
            P = E / l                                       # = exp(S - LSE), fp32 on the GPU
            dP = gg @ vv.T
            delta = (gg * Ost).sum(axis=1)
            dSr = rb(P * (dP - delta[:, None]))
            dQ[t0:t1, h] = scale * (dSr @ kk)
            dK[t0:t1, kv] += scale * (dSr.T @ qq)
            dV[t0:t1, kv] += rb(P).T @ gg
    if grads_bf16:
        dQ, dK, dV = rb(dQ), rb(dK), rb(dV)
    return O, dQ, dK, dV
