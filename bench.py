#!/usr/bin/env python3
"""Benchmark of the one-GPU hot path: layout permute + packed causal attention fwd + bwd.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One STEP is one pass of the whole path for one micro-batch of one attention layer on one GPU
of an SP group of degree P (paper Sec. 2.1.2, Eq. 2-4 and their backward):

    plan (host lengths -> tile queues) ->
    pack q, k, v   [T/P, P*Hp, D] -> per-peer slabs            (local half of Eq. 2)
    attention forward on [T, Hp, D]                            (Eq. 3)
    unpack o       slabs -> [T/P, P*Hp, D]                     (local half of Eq. 4)
    pack dO ; attention backward ; unpack dq, dk, dv           (the same exchanges, backward)

The wire exchange itself is out of scope (one GPU): the slabs a GPU packs are fed to its own
attention as if they were what the peers sent, which has the same shapes and byte counts.

Prints ONE JSON line.  `value` = causal-effective attention FLOPs (14*D*Hq*sum_b s_b(s_b+1)/2)
per second over the whole step, inputs resident in HBM.  `roofline` describes the dominant
kernel, timed with HIP events recorded by the library around each of its launches on the
stream they run on.  `cpu_baseline` times the CPU fp64 oracle on a bounded sample of the same
workload (a reported baseline, not a target).

Other legs, each printing one JSON line of its own and nothing else: --cost-model (the paper's Eq. 12 fitted to
these kernels), --kvshard-ring (one device's pass of a context-parallel ring, forward and backward),
--length-sweep (attention by sequence length), --permute-only and --traffic-probe (for counter collection).
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK = 2.5e15     # MI355X dense bf16 MFMA, FLOP/s (256 CU x 4 SIMD x 1024 FLOP/clk x 2.4 GHz)
HBM_PEAK = 8.0e12           # MI355X HBM3E, B/s

# HBM bytes per launch of the attention kernels (FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs,
# each scaled by what the same counter reads for a plain copy of known size; the commands, the raw
# counter values and the algorithmic bytes beside them are in profiles/attention_hbm_traffic.md).
# bench.py cannot run the profiler on itself: these are the figures of that summary.
MEASURED_HBM_TRAFFIC = {
    ("pareto-64k", "fwd"): 1109401063, ("pareto-64k", "bwd_dq"): 1347854523, ("pareto-64k", "bwd_dkv"): 1284704310,
    ("single-128k", "fwd"): 11779112005, ("single-128k", "bwd_dq"): 25981247295, ("single-128k", "bwd_dkv"): 10197784226,
}


def permute_leg(ctx, fx, wl, torch, stream):
    """Achieved HBM bandwidth of pack / unpack on the [32768, 32, 128] bf16, P = 8 shape, rotating
    over 4 distinct buffer pairs (2 GiB) so the 256 MB last-level cache cannot serve the reads;
    then the same kernel with P = 1, which is a plain copy: the ceiling this permute can reach."""
    c1 = wl.CONFIGS[1]
    Tp, Hp_tot, Pp, D = c1.tokens, c1.hq * c1.sp_degree, c1.sp_degree, c1.d
    nbuf = 4
    dev = "cuda"
    srcs = [torch.randn((Tp, Hp_tot, D), device=dev, dtype=torch.float32).to(torch.bfloat16) for _ in range(nbuf)]
    dsts = [torch.empty((Pp, Tp, Hp_tot // Pp, D), dtype=torch.bfloat16, device=dev) for _ in range(nbuf)]
    nbytes = 2 * Tp * Hp_tot * D * 2
    res = {}

    def timed(name, key, run):
        for i in range(10):
            run(i)
        ctx.profile_start(64)
        for i in range(40):
            run(i)
        ms, n = ctx.profile_stop()[key]
        res[name] = {"avg_ms": ms / n, "GBps": nbytes / (ms / n * 1e-3) / 1e9,
                     "frac_of_hbm_peak": nbytes / (ms / n * 1e-3) / HBM_PEAK}

    timed("pack", "pack", lambda i: fx.flexsp_pack(ctx, srcs[i % nbuf], dsts[i % nbuf], Pp, stream))
    timed("unpack", "unpack", lambda i: fx.flexsp_unpack(ctx, dsts[i % nbuf], srcs[i % nbuf], stream))
    timed("plain_copy_same_kernel", "pack",
          lambda i: fx.flexsp_pack(ctx, srcs[i % nbuf], dsts[i % nbuf].view(1, Tp, Hp_tot, D), 1, stream))
    return {"shape": [Tp, Hp_tot, D], "sp_degree": Pp, "dtype": "bf16", "bytes_per_call": nbytes,
            "buffers_rotated": nbuf, "peak_GBps": HBM_PEAK / 1e9, **res}


def cost_model_leg(ctx, fx, wl, torch, np):
    """Paper Sec. 4.1.2, Eq. 12: T_comp = alpha1*sum(s^2) + alpha2*sum(s) + beta1, coefficients
    "obtained through profiling".  Profiles attention fwd+bwd (8 heads, D = 128, causal) on 24 seeded
    synthetic batches of different sizes and length mixes, fits on the even-numbered ones, and
    reports the relative error on every batch (the paper reports < 6 %)."""
    from paper_2412_01523_amd import cost_model as cm
    H, D = 8, 128
    batches = cm.synthetic_batches(seed=wl.BASE_SEED)
    times = cm.profile(ctx, batches, H, D)
    coef = cm.fit(batches[0::2], times[0::2])
    err = cm.relative_errors(coef, batches, times)
    return {"alpha1_ms_per_token2": coef[0], "alpha2_ms_per_token": coef[1], "beta1_ms": coef[2],
            "heads": H, "head_dim": D, "batches": len(batches), "fitted_on": len(batches[0::2]),
            "max_abs_rel_error_fitted": float(np.abs(err[0::2]).max()),
            "max_abs_rel_error_held_out": float(np.abs(err[1::2]).max()),
            "mean_abs_rel_error": float(np.abs(err).mean()),
            "per_batch": [{"tokens": int(sum(b)), "sequences": len(b), "max_len": int(max(b)), "ms": t,
                           "rel_error": float(e)} for b, t, e in zip(batches, times, err)]}


def ring_leg(ctx, fx, wl, torch, np, workload):
    """One device's pass of a context-parallel ring without the wire (paper Sec. 2.1.3, paragraph on context
    parallelism, and the appendix that integrates it): the device holds the LAST 1/P of every sequence's
    query rows (the rank with the most visible keys, which sets the ring's time), the key/value shards come
    by one at a time (its own first, then the earlier ones), each gives a partial attention
    that the shard forward itself folds into the fp32 running result (flexsp_attn_varlen_fwd_kvshard_acc);
    then the backward ring (flexsp_attn_varlen_bwd_kvshard with accumulate, fp32 partial sums).
    Plans are built beforehand (lengths are known on the host); timed with events on the stream."""
    cfg = next(c for c in wl.CONFIGS if c.name == workload)
    lens = [s for s in wl.lengths(cfg)]
    H, Hkv, D = cfg.hq, cfg.hkv, cfg.d
    P = 8 if len(lens) == 1 else 4
    cu = wl.cu_seqlens(lens)
    T = int(cu[-1])
    cut = [[(j * s) // P for j in range(P + 1)] for s in lens]            # shard j of a sequence: positions cut[j] .. cut[j+1]-1
    dev = "cuda"
    k = torch.randn((T, Hkv, D), device=dev).to(torch.bfloat16)
    v = torch.randn((T, Hkv, D), device=dev).to(torch.bfloat16)
    q_full = torch.randn((T, H, D), device=dev).to(torch.bfloat16)

    def rows(x, j):
        return torch.cat([x[int(cu[b]) + c[j]: int(cu[b]) + c[j + 1]] for b, c in enumerate(cut)]).contiguous()

    q = rows(q_full, P - 1)
    cu_q = wl.cu_seqlens([c[P] - c[P - 1] for c in cut])
    Tq = int(cu_q[-1])
    shards = []
    for j in range(P - 1, -1, -1):
        cu_k = wl.cu_seqlens([c[j + 1] - c[j] for c in cut])
        shift = [c[P - 1] - c[j] for c in cut]
        pairs = sum((n * (n + 1)) // 2 if j == P - 1 else n * (c[j + 1] - c[j])
                    for c in cut for n in [c[P] - c[P - 1]])
        shards.append({"plan": fx.ShardPlan(ctx, cu_q, cu_k, shift, H, Hkv, D, True), "k": rows(k, j), "v": rows(v, j),
                       "flops": 4 * D * H * pairs, "shard": j})
    o_acc = torch.empty((Tq, H, D), dtype=torch.bfloat16, device=dev)      # the complete O, rounded to bf16 once
    o_run = torch.empty((Tq, H, D), dtype=torch.float32, device=dev)       # the running result, fp32
    l_acc = torch.empty((H, Tq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    reps = 10
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2 * P)] for _ in range(reps)]

    def one_pass(marks):
        l_acc.fill_(float("-inf"))       # an empty running result (its O may hold anything)
        for n, sh in enumerate(shards):
            fx.flexsp_attn_varlen_fwd_kvshard_acc(ctx, sh["plan"], q, sh["k"], sh["v"], o_run, l_acc,
                                                  o_acc if n == P - 1 else None, stream=stream)
            if marks: marks[2 * n].record(stream)
            if marks: marks[2 * n + 1].record(stream)

    for _ in range(3):
        one_pass(None)
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    start.record(stream)
    for r in range(reps):
        one_pass(ev[r])
    torch.cuda.synchronize()
    total_ms = start.elapsed_time(ev[-1][-1]) / reps
    fwd_ms = np.zeros((reps, P)); mrg_ms = np.zeros((reps, P))
    for r in range(reps):
        prev = start if r == 0 else ev[r - 1][-1]
        for n in range(P):
            fwd_ms[r, n] = prev.elapsed_time(ev[r][2 * n])
            mrg_ms[r, n] = ev[r][2 * n].elapsed_time(ev[r][2 * n + 1])
            prev = ev[r][2 * n + 1]
    fwd_med, mrg_med = np.median(fwd_ms, axis=0), np.median(mrg_ms, axis=0)
    flops = sum(sh["flops"] for sh in shards)
    # the backward ring: every shard's visit adds its part of dQ to one fp32 buffer and this device's part
    # of dK / dV to the fp32 buffers that travel with the shard (o_acc / l_acc are the complete O and LSE)
    g = torch.randn((Tq, H, D), device=dev).to(torch.bfloat16)
    dq = torch.zeros((Tq, H, D), dtype=torch.float32, device=dev)
    for sh in shards:
        sh["dk"] = torch.zeros(sh["k"].shape, dtype=torch.float32, device=dev)
        sh["dv"] = torch.zeros(sh["v"].shape, dtype=torch.float32, device=dev)
    bev = [[torch.cuda.Event(enable_timing=True) for _ in range(P + 1)] for _ in range(reps)]

    def backward_pass(marks):
        if marks: marks[0].record(stream)
        for n, sh in enumerate(shards):
            fx.flexsp_attn_varlen_bwd_kvshard(ctx, sh["plan"], q, sh["k"], sh["v"], o_acc, g, l_acc, dq, sh["dk"], sh["dv"],
                                              accumulate=True, stream=stream)
            if marks: marks[n + 1].record(stream)

    for _ in range(3):
        backward_pass(None)
    torch.cuda.synchronize()
    for r in range(reps):
        backward_pass(bev[r])
    torch.cuda.synchronize()
    bwd_ms = np.array([[bev[r][n].elapsed_time(bev[r][n + 1]) for n in range(P)] for r in range(reps)])
    bwd_med = np.median(bwd_ms, axis=0)
    bwd_total = float(np.median([bev[r][0].elapsed_time(bev[r][P]) for r in range(reps)]))
    # the ordinary forward over the unsplit batch, for the rate the shard kernel is measured against
    plan = fx.Plan(ctx, cu, H, Hkv, D, True)
    o_full = torch.empty_like(q_full)
    l_full = torch.empty((H, T), dtype=torch.float32, device=dev)
    cud = torch.from_numpy(cu).to(dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(6):
        if i == 3: e0.record(stream)
        fx.flexsp_attn_varlen_fwd(ctx, plan, q_full, k, v, cud, o_full, l_full, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    full_ms = e0.elapsed_time(e1) / 3
    full_flops, full_bwd_flops = wl.attn_flops(lens, H, D, True)
    g_full = torch.randn_like(q_full)
    dq_f, dk_f, dv_f = torch.empty_like(q_full), torch.empty_like(k), torch.empty_like(v)
    for i in range(6):
        if i == 3: e0.record(stream)
        fx.flexsp_attn_varlen_bwd(ctx, plan, q_full, k, v, o_full, g_full, l_full, cud, dq_f, dk_f, dv_f, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    full_bwd_ms = e0.elapsed_time(e1) / 3
    plan.close()
    out = {"workload": cfg.name, "ring_degree": P, "query_rows": Tq, "heads": H, "head_dim": D,
           "shards": [{"shard": sh["shard"], "ms": float(fwd_med[n]), "tflops": sh["flops"] / (fwd_med[n] * 1e-3) / 1e12}
                      for n, sh in enumerate(shards)],
           "fold": "inside the shard forward (flexsp_attn_varlen_fwd_kvshard_acc): no merge launches",
           "pass_ms": total_ms, "pass_tflops": flops / (total_ms * 1e-3) / 1e12,
           "shard_forwards_tflops": flops / (fwd_med.sum() * 1e-3) / 1e12,
           "unsplit_forward_ms": full_ms, "unsplit_forward_tflops": full_flops / (full_ms * 1e-3) / 1e12,
           "backward_shards": [{"shard": sh["shard"], "ms": float(bwd_med[n]),
                                "tflops": 2.5 * sh["flops"] / (bwd_med[n] * 1e-3) / 1e12} for n, sh in enumerate(shards)],
           "backward_pass_ms": bwd_total, "backward_pass_tflops": 2.5 * flops / (bwd_total * 1e-3) / 1e12,
           "unsplit_backward_ms": full_bwd_ms, "unsplit_backward_tflops": full_bwd_flops / (full_bwd_ms * 1e-3) / 1e12}
    for sh in shards:
        sh["plan"].close()
    return out


def length_sweep_leg(ctx, fx, wl, torch, np):
    """Attention fwd+bwd (8 heads, D = 128, causal) on batches of 49 152 tokens made of equal sequences of 256 ...
    8 192 tokens, and on the short and the long sequences of the pareto-64k batch by themselves: what the
    per-item costs of short sequences (paper Sec. 3: most sequences of a corpus are short) take from the
    rate long sequences reach.  Per-kernel times from the library's event recorder, 20 steps after 5."""
    H, D = 8, 128
    pareto = wl.lengths(next(c for c in wl.CONFIGS if c.name == "pareto-64k"))
    cases = [(f"{49152 // s} x {s}", [s] * (49152 // s)) for s in (256, 512, 1024, 2048, 4096, 8192)]
    cases += [("pareto-64k, sequences <= 4000", [s for s in pareto if s <= 4000]),
              ("pareto-64k, sequences > 4000", [s for s in pareto if s > 4000]), ("pareto-64k", pareto)]
    out = []
    for name, lens in cases:
        cu = wl.cu_seqlens(lens)
        T = int(cu[-1])
        q = torch.randn((T, H, D), device="cuda").to(torch.bfloat16)
        k, v, g = torch.randn_like(q), torch.randn_like(q), torch.randn_like(q)
        o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
        lse = torch.empty((H, T), dtype=torch.float32, device="cuda")
        cud = torch.from_numpy(cu).cuda()
        plan = fx.Plan(ctx, cu, H, H, D, True)

        def step():
            fx.flexsp_attn_varlen_fwd(ctx, plan, q, k, v, cud, o, lse)
            fx.flexsp_attn_varlen_bwd(ctx, plan, q, k, v, o, g, lse, cud, dq, dk, dv)
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        ctx.profile_start(128)
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        pr = ctx.profile_stop()
        plan.close()
        ms = {n: pr[n][0] / max(pr[n][1], 1) for n in ("fwd", "bwd_dq", "bwd_dkv")}
        f_fwd, f_bwd = wl.attn_flops(lens, H, D, True)
        total = sum(ms.values())
        io = 2 * T * H * D          # bytes of one bf16 [T, H, D] tensor
        out.append({"batch": name, "tokens": T, "sequences": len(lens), "fwd_ms": ms["fwd"], "bwd_dq_ms": ms["bwd_dq"],
                    "bwd_dkv_ms": ms["bwd_dkv"], "tflops": (f_fwd + f_bwd) / (total * 1e-3) / 1e12,
                    "frac_of_bf16_mfma_peak": (f_fwd + f_bwd) / (total * 1e-3) / BF16_MFMA_PEAK,
                    "fwd_flop_per_byte": f_fwd / (4 * io), "fwd_ms_of_its_bytes_at_6TBps": 4 * io / 6e12 * 1e3,
                    "fwd_ms_of_its_flops_at_peak": f_fwd / BF16_MFMA_PEAK * 1e3})
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="pareto-64k",
                    help="lognormal-32k | pareto-64k | single-128k | bimodal-256k-gqa | tiny-436")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-permute-leg", action="store_true")
    ap.add_argument("--reuse-plan", action="store_true",
                    help="build the tile plan once, outside the timed steps (a plan serves every layer of a micro-batch)")
    ap.add_argument("--attention-only", action="store_true", help="step = plan + fwd + bwd (no permutes)")
    ap.add_argument("--no-seed-leg", action="store_true",
                    help="skip the extra leg that times attention on three more length seeds of the same recipe")
    ap.add_argument("--cost-model", action="store_true",
                    help="only the cost-model leg: time attention fwd+bwd on 24 synthetic batches, fit the "
                         "paper's alpha-beta computation model (Eq. 12) on half of them, report the error on all")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for counter collection under rocprofv3 --pmc: 5 plain copies of known size (the permute "
                         "kernel with P = 1 on [32768, 32, 128] bf16: 256 MiB read, 256 MiB written each), then 3 x "
                         "(forward + backward) of the workload with one plan; nothing is timed")
    ap.add_argument("--length-sweep", action="store_true",
                    help="only the sequence-length leg: attention fwd+bwd on batches of equal sequences of 256 ... 8192 "
                         "tokens and on the short and the long sequences of pareto-64k by themselves")
    ap.add_argument("--kvshard-ring", action="store_true",
                    help="only the context-parallel leg: one device's ring pass (forward against one key shard at a "
                         "time + merge, then the backward ring) on single-128k (8 shards) and pareto-64k (4 shards), beside the unsplit forward")
    ap.add_argument("--permute-only", action="store_true",
                    help="only the permute bandwidth leg: 50 pack, 50 unpack, 50 plain copies (pack with P = 1), "
                         "in that order (for counter collection)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2412_01523_amd import binding as fx
    from paper_2412_01523_amd import workloads as wl

    if args.cost_model:
        torch.cuda.set_device(0)
        ctx = fx.Context(0)
        print(json.dumps({"cost_model": cost_model_leg(ctx, fx, wl, torch, np)}))
        return 0

    if args.length_sweep:
        torch.cuda.set_device(0)
        ctx = fx.Context(0)
        print(json.dumps({"length_sweep": length_sweep_leg(ctx, fx, wl, torch, np)}))
        return 0

    if args.kvshard_ring:
        torch.cuda.set_device(0)
        ctx = fx.Context(0)
        names = ("single-128k", "pareto-64k") if args.workload == "pareto-64k" else (args.workload,)
        print(json.dumps({"kvshard_ring": [ring_leg(ctx, fx, wl, torch, np, w) for w in names]}))
        return 0

    if args.traffic_probe:
        torch.cuda.set_device(0)
        ctx = fx.Context(0)
        cfg = next(c for c in wl.CONFIGS if c.name == args.workload)
        lens = wl.lengths(cfg)
        cu = wl.cu_seqlens(lens)
        c1 = wl.CONFIGS[1]
        src = torch.randn((c1.tokens, c1.hq * c1.sp_degree, c1.d), device="cuda").to(torch.bfloat16)
        dst = torch.empty((1,) + tuple(src.shape), dtype=torch.bfloat16, device="cuda")
        for _ in range(5):
            fx.flexsp_pack(ctx, src, dst, 1)
        torch.cuda.synchronize()
        del src, dst
        T, Hq, Hkv, D = cfg.tokens, cfg.hq, cfg.hkv, cfg.d
        q = torch.randn((T, Hq, D), device="cuda").to(torch.bfloat16)
        k = torch.randn((T, Hkv, D), device="cuda").to(torch.bfloat16)
        v, g = torch.randn_like(k), torch.randn_like(q)
        o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(k)
        lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
        cud = torch.from_numpy(cu).cuda()
        plan = fx.Plan(ctx, cu, Hq, Hkv, D, True)
        for _ in range(3):
            fx.flexsp_attn_varlen_fwd(ctx, plan, q, k, v, cud, o, lse)
            fx.flexsp_attn_varlen_bwd(ctx, plan, q, k, v, o, g, lse, cud, dq, dk, dv)
        torch.cuda.synchronize()
        plan.close()
        # algorithmic bytes per launch: every input read once, every output written once
        e = 2
        alg = {"fwd": (T * (2 * Hq + 2 * Hkv) * D) * e + 4 * Hq * T,
               "bwd_dq": (T * (4 * Hq + 2 * Hkv) * D) * e + 3 * 4 * Hq * T,
               "bwd_dkv": (T * (2 * Hq + 4 * Hkv) * D) * e + 2 * 4 * Hq * T}
        print(json.dumps({"traffic_probe": cfg.name, "copy_bytes_each_way": c1.tokens * c1.hq * c1.sp_degree * c1.d * 2,
                          "algorithmic_bytes_per_launch": alg}))
        return 0

    if args.permute_only:
        torch.cuda.set_device(0)
        ctx = fx.Context(0)
        print(json.dumps({"permute": permute_leg(ctx, fx, wl, torch, torch.cuda.current_stream())}))
        return 0

    cfg = next(c for c in wl.CONFIGS if c.name == args.workload)
    lens = wl.lengths(cfg)
    cu = wl.cu_seqlens(lens)
    T, Hq, Hkv, D = cfg.tokens, cfg.hq, cfg.hkv, cfg.d
    P = cfg.sp_degree if cfg.sp_degree else 8
    while T % P:      # the permutes split the token stream into P equal chunks
        P //= 2
    Tl = T // P
    f_fwd, f_bwd = wl.attn_flops(lens, Hq, D, True)
    pairs_heads = wl.causal_pairs(lens) * Hq

    torch.cuda.set_device(0)
    ctx = fx.Context(0)
    dev = "cuda"

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    # sequence-sharded inputs of this GPU: T/P tokens x all heads (synthetic N(0,1), seeded)
    xq = dev_bf16(wl.normal_bf16(cfg.seed, wl.TID_Q, (Tl, P * Hq, D)))
    xk = dev_bf16(wl.normal_bf16(cfg.seed, wl.TID_K, (Tl, P * Hkv, D)))
    xv = dev_bf16(wl.normal_bf16(cfg.seed, wl.TID_V, (Tl, P * Hkv, D)))
    xg = dev_bf16(wl.normal_bf16(cfg.seed, wl.TID_DO, (Tl, P * Hq, D)))
    # head-sharded slabs [P, T/P, Hp, D] == [T, Hp, D]
    new = lambda h: torch.empty((P, Tl, h, D), dtype=torch.bfloat16, device=dev)
    sq, sk, sv, sg, so = new(Hq), new(Hkv), new(Hkv), new(Hq), new(Hq)
    sdq, sdk, sdv = new(Hq), new(Hkv), new(Hkv)
    yo, ydq = torch.empty_like(xq), torch.empty_like(xq)
    ydk, ydv = torch.empty_like(xk), torch.empty_like(xv)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=dev)
    cud = torch.from_numpy(cu).to(dev)
    v3 = lambda t: t.view(T, t.shape[2], D)
    stream = torch.cuda.current_stream()

    shared_plan = fx.Plan(ctx, cu, Hq, Hkv, D, True) if args.reuse_plan else None

    def step():
        plan = shared_plan if args.reuse_plan else fx.Plan(ctx, cu, Hq, Hkv, D, True)
        if not args.attention_only:
            fx.flexsp_pack_many(ctx, [xq, xk, xv], [sq, sk, sv], P, stream)    # q, k, v in one launch
        fx.flexsp_attn_varlen_fwd(ctx, plan, v3(sq), v3(sk), v3(sv), cud, v3(so), lse, stream=stream)
        if not args.attention_only:
            fx.flexsp_unpack(ctx, so, yo, stream)
            fx.flexsp_pack(ctx, xg, sg, P, stream)
        fx.flexsp_attn_varlen_bwd(ctx, plan, v3(sq), v3(sk), v3(sv), v3(so), v3(sg), lse, cud,
                                  v3(sdq), v3(sdk), v3(sdv), stream=stream)
        if not args.attention_only:
            fx.flexsp_unpack_many(ctx, [sdq, sdk, sdv], [ydq, ydk, ydv], stream)  # dq, dk, dv in one launch
        if plan is not shared_plan:
            plan.close()    # hands the plan's memory back to the context (no synchronisation)
        return None

    if args.attention_only:      # the slabs must hold data even when the permutes are skipped
        for x, s in ((xq, sq), (xk, sk), (xv, sv), (xg, sg)):
            fx.flexsp_pack(ctx, x, s, P, stream)

    # (a collection of the interpreter's heap in the middle of a step stalls the host for milliseconds;
    # collected once BEFORE the warm-up, so that nothing but the synchronisation lies between the
    # warm-up and the timed steps: the GPU's clocks drop while it waits for the host)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    gc.collect()
    gc.disable()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- the timed region: K steps, nothing but the path itself between the two synchronisations
    # (the library's per-kernel event recorder is OFF here; one stream marker per step gives the
    # per-step minimum and median)
    t0 = time.perf_counter()
    marks[0].record(stream)
    host_t = [t0]
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
        host_t.append(time.perf_counter())
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    ms_step = (t1 - t0) * 1e3 / max(args.steps, 1)
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]

    # ---- a second pass over the same steps with the per-kernel recorder on (HIP events around every
    # launch, on the stream the kernels run on): the per-kernel split and the roofline object.  Not part
    # of `value` / `ms_per_step`.
    ctx.profile_start(16 * max(args.steps, 1))
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = ctx.profile_stop()

    # plan creation by itself (host time per create + destroy; the upload is asynchronous)
    torch.cuda.synchronize()
    tp0 = time.perf_counter()
    for _ in range(50):
        fx.Plan(ctx, cu, Hq, Hkv, D, True).close()
    plan_ms = (time.perf_counter() - tp0) * 1e3 / 50
    tflops = (f_fwd + f_bwd) / (ms_step * 1e-3) / 1e12

    kern = {}
    for name in fx.KERNELS:
        ms, n = prof[name]
        if n:
            kern[name] = {"avg_ms": ms / n, "launches_per_step": n / max(args.steps, 1)}
    # algorithmic FLOPs per launch, per (query, key) pair and head: fwd 2 GEMMs, dK/dV kernel 4 GEMMs
    # (S, dP, dV, dK), dQ kernel 1 GEMM (its S and dP are recomputation, counted as zero)
    alg = {"fwd": 4 * D * pairs_heads, "bwd_dkv": 8 * D * pairs_heads, "bwd_dq": 2 * D * pairs_heads}
    dom = max((k for k in alg if k in kern), key=lambda k: kern[k]["avg_ms"] * kern[k]["launches_per_step"])
    ach = alg[dom] / (kern[dom]["avg_ms"] * 1e-3) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": BF16_MFMA_PEAK / 1e12,
                "unit": "TFLOP/s", "frac": ach / (BF16_MFMA_PEAK / 1e12),
                "traffic": MEASURED_HBM_TRAFFIC.get((cfg.name, dom)), "avg_ms": kern[dom]["avg_ms"]}
    attn_ms = sum(kern[k]["avg_ms"] * kern[k]["launches_per_step"] for k in ("fwd", "bwd_delta", "bwd_dkv", "bwd_dq") if k in kern)
    out = {
        "metric": "varlen causal attn fwd+bwd TFLOP/s (1 GPU) and % of bf16 MFMA peak",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_step_min": min(per_step) if per_step else None,
        "ms_per_step_median": float(np.median(per_step)) if per_step else None,
        "ms_per_step_max": max(per_step) if per_step else None,
        "plan_create_destroy_host_ms": plan_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "tokens": T, "sequences": len(lens), "max_len": max(lens),
                   "hq": Hq, "hkv": Hkv, "head_dim": D, "causal": True, "sp_degree": P,
                   "step": ("" if args.reuse_plan else "plan+") + ("fwd+bwd" if args.attention_only else "pack(q,k,v)+fwd+unpack(o)+pack(dO)+bwd+unpack(dq,dk,dv)"),
                   "flops_fwd_bwd": f_fwd + f_bwd, "seed": cfg.seed},
        "frac_of_bf16_mfma_peak": tflops * 1e12 / BF16_MFMA_PEAK,
        "attention_kernels_only": {"ms": attn_ms, "tflops": (f_fwd + f_bwd) / (attn_ms * 1e-3) / 1e12,
                                   "frac_of_bf16_mfma_peak": (f_fwd + f_bwd) / (attn_ms * 1e-3) / BF16_MFMA_PEAK},
        "kernels": kern,
        "roofline": roofline,
    }

    if os.environ.get("BENCH_DUMP_STEPS"):
        out["per_step"] = per_step
        out["per_step_host_enqueue_ms"] = [(b - a_) * 1e3 for a_, b in zip(host_t, host_t[1:])]
    if not args.no_permute_leg:
        out["permute"] = permute_leg(ctx, fx, wl, torch, stream)

    # ---- the same recipe with other length seeds (the pareto recipe is seed-sensitive): plan + fwd + bwd
    if not args.no_seed_leg and cfg.name == "pareto-64k":
        legs = []
        for k_ in (1, 2, 3):
            lens_k = wl.lengths(cfg, seed=cfg.seed + k_)
            cu_k = wl.cu_seqlens(lens_k)
            cud_k = torch.from_numpy(cu_k).to(dev)
            fl = sum(wl.attn_flops(lens_k, Hq, D, True))

            def attn_step():
                plan = fx.Plan(ctx, cu_k, Hq, Hkv, D, True)
                fx.flexsp_attn_varlen_fwd(ctx, plan, v3(sq), v3(sk), v3(sv), cud_k, v3(so), lse, stream=stream)
                fx.flexsp_attn_varlen_bwd(ctx, plan, v3(sq), v3(sk), v3(sv), v3(so), v3(sg), lse, cud_k,
                                          v3(sdq), v3(sdk), v3(sdv), stream=stream)
                plan.close()
            n_k = 20
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_k + 1)]
            gc.collect()
            gc.disable()
            for _ in range(10):
                attn_step()
            torch.cuda.synchronize()
            ts0 = time.perf_counter()
            ev[0].record(stream)
            for i in range(n_k):
                attn_step()
                ev[i + 1].record(stream)
            torch.cuda.synchronize()
            ms_k = (time.perf_counter() - ts0) * 1e3 / n_k
            gc.enable()
            each = [ev[i].elapsed_time(ev[i + 1]) for i in range(n_k)]
            med = float(np.median(each))
            legs.append({"length_seed": cfg.seed + k_, "sequences": len(lens_k), "max_len": max(lens_k),
                         "flops_fwd_bwd": fl, "steps": n_k, "ms_per_step": ms_k, "ms_per_step_min": min(each),
                         "ms_per_step_median": med, "ms_per_step_max": max(each),
                         "tflops": fl / (ms_k * 1e-3) / 1e12, "tflops_median_step": fl / (med * 1e-3) / 1e12})
        out["other_length_seeds_attention_only"] = legs

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        budget = 1.4e12          # FLOPs: 10-30 s of plain fp64 loops on 16 cores (all of pareto-64k is 1.31e12)
        per_task_cap = 7e10      # one (sequence, kv head) task runs on one thread: about 20 s
        chosen, used = [], 0.0
        for b in np.argsort(lens)[::-1]:
            s = lens[int(b)]
            per_head = 14 * D * s * (s + 1) // 2
            if per_head * (Hq // Hkv) > per_task_cap or used + per_head * Hq > budget:
                continue
            chosen.append(int(b))
            used += per_head * Hq
        chosen.sort()
        sub_lens = [lens[b] for b in chosen]
        what = f"{len(chosen)} of {len(lens)} sequences of the workload"
        if not chosen:
            # no whole sequence fits: the first n tokens of the longest one (a causal prefix is an attention
            # problem of its own), n from the per-task cap
            n = int(min(max(lens), np.sqrt(2 * per_task_cap / (14 * D * (Hq // Hkv)))))
            sub_lens = [n]
            what = f"the first {n} tokens of the longest sequence"
        idx = np.arange(sum(sub_lens))
        # the same seeded distribution; the oracle gets its own [T, H, D] tensors of the sample's size
        q_, k_, v_, g_ = wl.make_qkvdo(cfg, tokens=len(idx))
        tc0 = time.perf_counter()
        oracle.attn_fwd_bwd(q_, k_, v_, g_, wl.cu_seqlens(sub_lens), True)
        tc1 = time.perf_counter()
        fs = sum(wl.attn_flops(sub_lens, Hq, D, True))
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": fs / (tc1 - tc0) / 1e12, "unit": "TFLOP/s", "cores": threads,
                               "kind": "oracle", "seconds": tc1 - tc0,
                               "sample": f"{what} ({len(idx)} tokens, longest {max(sub_lens)}), all {Hq} heads, fwd+bwd"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
