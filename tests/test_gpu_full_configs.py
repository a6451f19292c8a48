"""GPU parity at the full sizes of benchmark configurations 1..4 (0-based), in the launch
configuration bench.py times.  The oracle cannot run these in full within a test, so the
comparison is on outputs it can compute one by one: sampled rows of O, LSE, dQ; sampled rows of
dK, dV, among them rows of the longest sequences that accumulate over 16 to 64 query steps and,
in the tests at the end of this file, rows that accumulate over a whole sequence from key 0
(256 steps; 64 steps x 8 grouped heads); whole mid-length sequences.  Both gradient modes run:
fp32 gradients are held to the stated bounds, bf16 gradients must be those values rounded once.
Two identities that hold at any size are checked besides, per (sequence, kv head):
    sum_j dV[j] = sum_i dO[i]            (rows of P sum to one)
    <q, dQ> = <k, dK>                    (both equal sum_ij dS_ij S_ij)"""
import sys
import time

import numpy as np
import pytest

import oracle
from paper_2412_01523_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, bf16_f64, errors, to_bits, to_dev

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    from paper_2412_01523_amd import binding as fx
    c = fx.Context(0)
    yield c
    c.close()


def _sample_rows(rng, lens, cu, hq, n_random):
    """(token, head) samples: random ones plus rows on tile edges of the longest sequence and the
    first / last rows of a few sequences."""
    T = int(cu[-1])
    tok = list(rng.integers(0, T, size=n_random))
    b_long = int(np.argmax(lens))
    s = lens[b_long]
    for i in (0, 1, 31, 32, 63, 64, 127, 128, 129, s // 2, s - 129, s - 128, s - 2, s - 1):
        if 0 <= i < s:
            tok.append(int(cu[b_long]) + i)
    for b in rng.integers(0, len(lens), size=6):
        tok += [int(cu[b]), int(cu[b + 1]) - 1]
    tok.append(T - 1)
    tok = np.array(sorted(set(int(t) for t in tok)), dtype=np.int64)
    head = rng.integers(0, hq, size=len(tok)).astype(np.int32)
    return tok, head


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_full_config_sampled_parity(ctx, ci):
    import torch
    from paper_2412_01523_amd import binding as fx
    cfg = wl.CONFIGS[ci]
    lens = wl.lengths(cfg)
    cu = wl.cu_seqlens(lens)
    T, Hq, Hkv, D = cfg.tokens, cfg.hq, cfg.hkv, cfg.d
    G = Hq // Hkv
    t0 = time.time()
    say(f"config {ci} {cfg.name}: T={T} B={len(lens)} max_len={max(lens)} Hq={Hq} Hkv={Hkv} D={D}; generating inputs")
    q, k, v, g = wl.make_qkvdo(cfg)
    say(f"  inputs ready after {time.time() - t0:.1f}s; running the HIP path")
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, True)
    qd, kd, vd, gd = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    cud = torch.from_numpy(cu).cuda()
    o = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
    fx.flexsp_attn_varlen_fwd(ctx, plan, qd, kd, vd, cud, o, lse)
    # backward in both gradient modes: fp32 gradients carry the stated bounds below; the bf16 ones
    # (the default mode) must be exactly those values rounded to bf16 once, over the whole tensors
    grads = {}
    for gdt in (torch.float32, torch.bfloat16):
        gq = torch.full((T, Hq, D), float("nan"), dtype=gdt, device="cuda")
        gk = torch.full((T, Hkv, D), float("nan"), dtype=gdt, device="cuda")
        gv = torch.full((T, Hkv, D), float("nan"), dtype=gdt, device="cuda")
        fx.flexsp_attn_varlen_bwd(ctx, plan, qd, kd, vd, o, gd, lse, cud, gq, gk, gv)
        grads[gdt] = (gq, gk, gv)
    torch.cuda.synchronize()
    say(f"  HIP path done after {time.time() - t0:.1f}s")
    assert torch.isfinite(lse).all() and torch.isfinite(o.float()).all()
    for name, a32, a16 in zip(("dQ", "dK", "dV"), grads[torch.float32], grads[torch.bfloat16]):
        assert torch.isfinite(a32).all(), name
        assert torch.equal(a32.to(torch.bfloat16), a16), f"{name}: bf16 gradients are not the fp32 ones rounded once"
    gq, gk, gv = grads[torch.float32]
    gq16, gk16, gv16 = grads[torch.bfloat16]
    del qd, kd, vd, gd, grads

    def host(t, rows=None):
        """rows of a device tensor as fp64"""
        x = t if rows is None else t[rows]
        if x.dtype == torch.bfloat16:
            return bf16_f64(to_bits(x))
        return x.cpu().numpy().astype(np.float64)

    rng = np.random.Generator(np.random.Philox(key=[cfg.seed, 555]))

    # ---- sampled rows of O, LSE, dQ
    tok, head = _sample_rows(rng, lens, cu, Hq, 48)
    Or, Lr, dQr = oracle.rows(q, k, v, g, cu, tok, head, True)
    tt, hh = torch.from_numpy(tok).cuda(), torch.from_numpy(head.astype(np.int64)).cuda()
    Og = host(o[tt, hh]); Lg = lse[hh, tt].cpu().numpy().astype(np.float64); dQg = host(gq[tt, hh])
    dQg16 = host(gq16[tt, hh])
    eo, eq, eq16 = errors(Og, Or), errors(dQg, dQr), errors(dQg16, dQr)
    say(f"  {len(tok)} sampled rows after {time.time() - t0:.1f}s: O (max_abs, rel_l2)=({eo[0]:.2e},{eo[1]:.2e}) "
        f"dQ fp32=({eq[0]:.2e},{eq[1]:.2e}) bf16=({eq16[0]:.2e},{eq16[1]:.2e}) LSE max_abs={np.abs(Lg - Lr).max():.2e}")
    assert eo[0] <= MAX_ABS and eo[1] <= REL_L2
    assert eq[0] <= MAX_ABS and eq[1] <= REL_L2
    # bf16 store: the value within 2e-2 rounded once more (half a bf16 ulp <= 2^-8 |value|)
    assert (np.abs(dQg16 - dQr) <= MAX_ABS + 2.0 ** -8 * np.abs(dQr)).all() and eq16[1] <= REL_L2
    assert np.abs(Lg - Lr).max() < 1e-3
    # every sampled row on its own, so one bad tile cannot hide in the aggregate
    assert np.abs(Og - Or).max(axis=1).max() <= MAX_ABS

    # ---- sampled rows of dK, dV
    order = np.argsort(lens)
    tasks = []
    b_long = int(order[-1])
    for b in [b_long, int(order[-2]) if len(lens) > 1 else b_long]:
        s = lens[b]
        for kvh in sorted(set([0, Hkv - 1])):
            if s > 10000:
                js = sorted(set([s - 64, s - 63, s - 33, s - 32, s - 2, s - 1]))
            else:
                js = sorted(set(j for j in (0, 1, 127, 128, s // 2, s - 1) if 0 <= j < s))
            tasks.append((b, kvh, js))
    # rows of the longest sequence that accumulate over many 64-query steps (and over all heads of a
    # group): one oracle task per listed depth, each costing depth x s x G score rows on one thread
    s_long = lens[b_long]
    if s_long > 10000:
        deep = [(0, 4096), (Hkv - 1, 1024)] if G == 1 else [(Hkv - 1, 512)]
        for kvh, depth in deep:
            tasks.append((b_long, kvh, [s_long - depth, s_long - depth + 1, s_long - depth + 63]))
            say(f"  deep dK/dV rows: sequence {b_long} (s={s_long}), kv head {kvh}, keys from s-{depth}: "
                f"{depth // 64} steps x {G} heads")
    mids = [int(b) for b in order if 256 <= lens[b] <= 10000]
    if mids:
        b = mids[-1]                      # the longest sequence the oracle can afford from key 0
        s = lens[b]
        tasks.append((b, Hkv // 2, sorted(set(j for j in (0, 1, 63, 64, 127, 128, s // 3, s - 1) if j < s))))
    for b in rng.integers(0, len(lens), size=4):
        s = lens[int(b)]
        if s <= 4096:
            tasks.append((int(b), int(rng.integers(0, Hkv)), sorted(set(int(j) for j in rng.integers(0, s, size=4)))))
    tor = time.time()
    dKr, dVr = oracle.dkv_rows(q, k, v, g, cu, tasks, True)
    say(f"  oracle dK/dV rows: {len(tasks)} tasks in {time.time() - tor:.1f}s")
    rows_t = np.array([int(cu[b]) + j for (b, kvh, js) in tasks for j in js], dtype=np.int64)
    rows_h = np.array([kvh for (b, kvh, js) in tasks for _ in js], dtype=np.int64)
    tt, hh = torch.from_numpy(rows_t).cuda(), torch.from_numpy(rows_h).cuda()
    dKg, dVg = host(gk[tt, hh]), host(gv[tt, hh])
    ek, ev = errors(dKg, dKr), errors(dVg, dVr)
    dKg16, dVg16 = host(gk16[tt, hh]), host(gv16[tt, hh])
    ek16, ev16 = errors(dKg16, dKr), errors(dVg16, dVr)
    say(f"  {len(rows_t)} sampled dK/dV rows after {time.time() - t0:.1f}s: fp32 dK=({ek[0]:.2e},{ek[1]:.2e}) "
        f"dV=({ev[0]:.2e},{ev[1]:.2e}); bf16 dK=({ek16[0]:.2e},{ek16[1]:.2e}) dV=({ev16[0]:.2e},{ev16[1]:.2e}); "
        f"max|ref| dK {np.abs(dKr).max():.1f} dV {np.abs(dVr).max():.1f}")
    assert ek[0] <= MAX_ABS and ek[1] <= REL_L2
    assert ev[0] <= MAX_ABS and ev[1] <= REL_L2
    # every sampled row on its own (a deep row must not hide behind the shallow ones)
    assert np.abs(dKg - dKr).max(axis=1).max() <= MAX_ABS and np.abs(dVg - dVr).max(axis=1).max() <= MAX_ABS
    assert (np.abs(dKg16 - dKr) <= MAX_ABS + 2.0 ** -8 * np.abs(dKr)).all() and ek16[1] <= REL_L2
    assert (np.abs(dVg16 - dVr) <= MAX_ABS + 2.0 ** -8 * np.abs(dVr)).all() and ev16[1] <= REL_L2

    # ---- identities that hold at any size, on the longest sequences and a few others
    qf = lambda x, sl, hs: bf16_f64(x[sl][:, hs])
    for b in sorted(set([int(order[-1]), int(order[-2]) if len(lens) > 1 else 0, int(order[len(order) // 2]), 0])):
        sl = slice(int(cu[b]), int(cu[b + 1]))
        s = lens[b]
        for kvh in sorted(set([0, Hkv - 1])):
            hs = slice(kvh * G, (kvh + 1) * G)
            dv_sum = host(gv[sl, kvh]).sum(0)
            do_sum = qf(g, sl, hs).sum((0, 1))
            # every term of either sum carries an independent rounding error of relative size <= 2^-8
            tol = 2.0 ** -8 * np.sqrt(s * G) * 4 + 1e-3
            assert np.abs(dv_sum - do_sum).max() <= tol, (b, kvh, float(np.abs(dv_sum - do_sum).max()), tol)
            lhs = float((qf(q, sl, hs) * host(gq[sl, hs])).sum())
            rhs = float((bf16_f64(k[sl][:, kvh]) * host(gk[sl, kvh])).sum())
            scale_ = np.sqrt(float((qf(q, sl, hs) ** 2).sum()) * float((host(gq[sl, hs]) ** 2).sum()))
            assert abs(lhs - rhs) <= 5e-3 * scale_ + 1e-3, (b, kvh, lhs, rhs, scale_)
    say(f"  identities hold; config {ci} done after {time.time() - t0:.1f}s")
    plan.close()


def test_mid_length_sequence_of_config2_elementwise(ctx):
    """One whole sequence of the long-tail batch (all heads, every row) against the full oracle."""
    import torch
    from paper_2412_01523_amd import binding as fx
    cfg = wl.CONFIGS[2]
    lens = wl.lengths(cfg)
    cu = wl.cu_seqlens(lens)
    q, k, v, g = wl.make_qkvdo(cfg)
    cand = [b for b in range(len(lens)) if 1500 <= lens[b] <= 3000]
    b = cand[0]
    say(f"config 2, sequence {b} of length {lens[b]}: full batch on the GPU, this sequence against the oracle")
    plan = fx.Plan(ctx, cu, cfg.hq, cfg.hkv, cfg.d, True)
    qd, kd, vd, gd = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    cud = torch.from_numpy(cu).cuda()
    o = torch.zeros_like(qd); lse = torch.zeros((cfg.hq, cfg.tokens), dtype=torch.float32, device="cuda")
    gq, gk, gv = torch.zeros_like(qd), torch.zeros_like(kd), torch.zeros_like(vd)
    fx.flexsp_attn_varlen_fwd(ctx, plan, qd, kd, vd, cud, o, lse)
    fx.flexsp_attn_varlen_bwd(ctx, plan, qd, kd, vd, o, gd, lse, cud, gq, gk, gv)
    torch.cuda.synchronize()
    sl = slice(int(cu[b]), int(cu[b + 1]))
    O, LSE, dQ, dK, dV = oracle.attn_fwd_bwd(q[sl], k[sl], v[sl], g[sl], wl.cu_seqlens([lens[b]]), True)
    for name, got, ref in (("O", o, O), ("dQ", gq, dQ), ("dK", gk, dK), ("dV", gv, dV)):
        ma, rl = errors(bf16_f64(to_bits(got[sl])), ref)
        say(f"  {name}: max_abs={ma:.2e} rel_l2={rl:.2e}")
        assert ma <= MAX_ABS and rl <= REL_L2, name
    assert np.abs(lse[:, sl].cpu().numpy() - LSE).max() < 1e-3
    plan.close()


LONG_ACCUMULATION = [
    # name, sequence length, Hq, Hkv, key rows whose dK/dV the oracle computes (all query rows >= the key contribute)
    ("one-head-16k", 16384, 1, 1, [[0, 1, 63, 64], [8191]]),           # 256 steps of 64 queries into key 0
    ("gqa8-4k", 4096, 8, 1, [[0, 1, 63, 64], [2047], [4032]]),          # 64 steps x 8 heads into key 0
]


@pytest.mark.parametrize("name,s,Hq,Hkv,keys", LONG_ACCUMULATION, ids=[c[0] for c in LONG_ACCUMULATION])
def test_dkv_rows_that_accumulate_over_a_whole_sequence(ctx, name, s, Hq, Hkv, keys):
    """dK/dV rows of the FIRST keys of a long sequence: every query step of the sequence (and every
    head of the group) adds into them, the longest accumulation the dK/dV kernel performs.  Element
    by element against the oracle: fp32 gradients within max-abs 2e-2 / relative L2 5e-3, bf16
    gradients equal to the fp32 ones rounded once."""
    import torch
    from paper_2412_01523_amd import binding as fx
    D = 128
    cu = wl.cu_seqlens([s])
    seed = 6100 + s
    q = wl.normal_bf16(seed, wl.TID_Q, (s, Hq, D)); k = wl.normal_bf16(seed, wl.TID_K, (s, Hkv, D))
    v = wl.normal_bf16(seed, wl.TID_V, (s, Hkv, D)); g = wl.normal_bf16(seed, wl.TID_DO, (s, Hq, D))
    say(f"long accumulation {name}: s={s} Hq={Hq} Hkv={Hkv}, keys {keys}")
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, True)
    qd, kd, vd, gd = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    cud = torch.from_numpy(cu).cuda()
    o = torch.full((s, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((Hq, s), float("nan"), dtype=torch.float32, device="cuda")
    fx.flexsp_attn_varlen_fwd(ctx, plan, qd, kd, vd, cud, o, lse)
    grads = {}
    for gdt in (torch.float32, torch.bfloat16):
        gq = torch.full((s, Hq, D), float("nan"), dtype=gdt, device="cuda")
        gk = torch.full((s, Hkv, D), float("nan"), dtype=gdt, device="cuda")
        gv = torch.full((s, Hkv, D), float("nan"), dtype=gdt, device="cuda")
        fx.flexsp_attn_varlen_bwd(ctx, plan, qd, kd, vd, o, gd, lse, cud, gq, gk, gv)
        grads[gdt] = (gq, gk, gv)
    torch.cuda.synchronize()
    plan.close()
    for a32, a16 in zip(grads[torch.float32], grads[torch.bfloat16]):
        assert torch.isfinite(a32).all() and torch.equal(a32.to(torch.bfloat16), a16)
    tasks = [(0, 0, js) for js in keys]
    t0 = time.time()
    dKr, dVr = oracle.dkv_rows(q, k, v, g, cu, tasks, True)
    say(f"  oracle: {sum(len(j) for j in keys)} rows in {time.time() - t0:.1f}s")
    rows = torch.tensor([j for js in keys for j in js], device="cuda")
    _, gk32, gv32 = grads[torch.float32]
    for nm, got, ref in (("dK", gk32[rows, 0], dKr), ("dV", gv32[rows, 0], dVr)):
        got = got.cpu().numpy().astype(np.float64)
        ma, rl = errors(got, ref)
        say(f"  {nm}: max_abs={ma:.2e} rel_l2={rl:.2e} per row max_abs " +
            " ".join(f"{x:.1e}" for x in np.abs(got - ref).max(axis=1)) + f" max|ref|={np.abs(ref).max():.1f}")
        assert ma <= MAX_ABS and rl <= REL_L2, nm
    # a few rows of O, LSE, dQ of the same run (row s-1 sees every key)
    tok = np.array([0, 63, 64, s // 2, s - 1], dtype=np.int64)
    head = np.array([0, Hq - 1, 0, Hq - 1, Hq // 2], dtype=np.int32)
    Or, Lr, dQr = oracle.rows(q, k, v, g, cu, tok, head, True)
    tt, hh = torch.from_numpy(tok).cuda(), torch.from_numpy(head.astype(np.int64)).cuda()
    eo = errors(bf16_f64(to_bits(o[tt, hh])), Or)
    eq = errors(grads[torch.float32][0][tt, hh].cpu().numpy().astype(np.float64), dQr)
    assert eo[0] <= MAX_ABS and eo[1] <= REL_L2 and eq[0] <= MAX_ABS and eq[1] <= REL_L2
    assert np.abs(lse[hh, tt].cpu().numpy() - Lr).max() < 1e-3
