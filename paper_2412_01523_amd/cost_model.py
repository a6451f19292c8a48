"""Computation-cost model of the paper (Sec. 4.1.2 "Cost Estimation", Eq. 12) for one GPU's share:

    T_comp = alpha1 * sum_k s_k^2 + alpha2 * sum_k s_k + beta1

(the 1/d_p of Eq. 12 is folded into the coefficients: they are fitted for the heads one GPU holds).
The paper obtains alpha1, alpha2, beta1 "through profiling" and reports an estimation error below
6 % (below 5 % in its appendix on estimation accuracy).  `fit` is that profiling step for this
library's attention kernels: an ordinary least-squares fit of measured times, weighted by 1/time so
that it is the RELATIVE error that is minimised.  `synthetic_batches` and `profile` produce the
measurements (seeded length lists; the library's own per-kernel HIP-event timing).  No attention
arithmetic here.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def features(lens: Sequence[int]) -> np.ndarray:
    s = np.asarray(lens, dtype=np.float64)
    return np.array([float((s * s).sum()), float(s.sum()), 1.0])


def fit(batches: Sequence[Sequence[int]], times: Sequence[float]) -> Tuple[float, float, float]:
    """(alpha1, alpha2, beta1) minimising sum(((predicted - measured) / measured)^2)."""
    X = np.stack([features(b) for b in batches])
    y = np.asarray(times, dtype=np.float64)
    if len(y) < 3 or (y <= 0).any():
        raise ValueError("need at least 3 positive measurements")
    w = 1.0 / y
    coef, *_ = np.linalg.lstsq(X * w[:, None], y * w, rcond=None)
    return float(coef[0]), float(coef[1]), float(coef[2])


def predict(coef: Tuple[float, float, float], lens: Sequence[int]) -> float:
    return float(np.dot(np.asarray(coef, dtype=np.float64), features(lens)))


def relative_errors(coef, batches, times) -> np.ndarray:
    y = np.asarray(times, dtype=np.float64)
    return np.array([predict(coef, b) for b in batches]) / y - 1.0


def synthetic_batches(totals=(16384, 32768, 65536, 131072), seed: int = 20241201):
    """Seeded length lists to profile on: per token budget a log-normal, a Pareto, a U[64, 1024] and a
    U[2048, 8192] mix (each filled up to the budget, last sequence truncated), four equal sequences
    and one single sequence: short-dominated, long-tailed and homogeneous batches alike."""
    rng = np.random.Generator(np.random.Philox(key=[int(seed), 4242]))

    def fill(draw, total):
        out, left = [], total
        while left > 0:
            s = min(int(draw()), left)
            out.append(s)
            left -= s
        return out

    batches = []
    for total in totals:
        batches.append(fill(lambda: np.clip(np.rint(np.exp(rng.normal(7.0, 1.2))), 128, 32768), total))
        batches.append(fill(lambda: np.clip(np.floor(256.0 * (1.0 - rng.random()) ** (-1 / 1.1)), 256, 65536), total))
        batches.append(fill(lambda: rng.integers(64, 1025), total))
        batches.append(fill(lambda: rng.integers(2048, 8193), total))
        batches.append([total // 4] * 4)
        batches.append([total])
    return batches


def profile(ctx, batches, heads: int = 8, head_dim: int = 128, reps: int = 8):
    """Measured attention fwd+bwd time (ms) of every batch on the context's GPU: after two warm-up
    runs, `reps` runs back to back, and per kernel the mean of the durations the library records
    with HIP events on the stream the kernels run on, summed over the kernels.  (Back to back, as
    the layers of a training step follow one another: a run timed alone, with a synchronisation
    before it, starts on a GPU whose clocks have dropped, and for batches of well under a
    millisecond that ramp is a tenth of the time.)  Inputs are random bf16; their values do not
    affect the time."""
    import torch
    from . import binding as fx
    H, D = heads, head_dim
    times = []
    for lens in batches:
        cu = np.zeros(len(lens) + 1, dtype=np.int32)
        np.cumsum(np.asarray(lens, dtype=np.int64), out=cu[1:])
        T = int(cu[-1])
        q = torch.randn((T, H, D), device="cuda", dtype=torch.float32).to(torch.bfloat16)
        k, v, g = torch.randn_like(q), torch.randn_like(q), torch.randn_like(q)
        o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        lse = torch.empty((H, T), dtype=torch.float32, device="cuda")
        cud = torch.from_numpy(cu).cuda()
        plan = fx.Plan(ctx, cu, H, H, D, True)

        def once():
            fx.flexsp_attn_varlen_fwd(ctx, plan, q, k, v, cud, o, lse)
            fx.flexsp_attn_varlen_bwd(ctx, plan, q, k, v, o, g, lse, cud, dq, dk, dv)

        once(); once()
        ctx.profile_start(4 * reps + 8)
        for _ in range(reps):
            once()
        pr = ctx.profile_stop()
        times.append(float(sum(pr[kk][0] / max(pr[kk][1], 1) for kk in ("fwd", "bwd_delta", "bwd_dkv", "bwd_dq"))))
        plan.close()
        del q, k, v, g, o, dq, dk, dv, lse
    return times
