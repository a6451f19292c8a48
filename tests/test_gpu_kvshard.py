"""GPU parity of the context-parallel pieces (paper Sec. 2.1.3, paragraph "Context Parallelism", and
the appendix on integrating it): attention of packed queries against ONE SHARD of each sequence's keys
(flexsp_attn_varlen_fwd_kvshard) and the log-sum-exp merge of such partial results (flexsp_lse_merge),
through the C ABI, against the CPU fp64 oracle on the same seeded inputs.  Tolerances as for the
forward: O within max-abs 2e-2 and relative L2 5e-3, LSE within 1e-3 where finite; rows that see no
key must come out as O = 0, LSE = -inf exactly."""
import sys

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


def _shard_forward(ctx, q, k, v, cu_q, cu_k, shift, causal):
    """HIP path: (O bits [Tq,Hq,D], LSE [Hq,Tq] fp32) as device tensors."""
    import torch
    from paper_2412_01523_amd import binding as fx
    Tq, Hq, D = q.shape
    Hkv = k.shape[1]
    plan = fx.ShardPlan(ctx, cu_q, cu_k, shift, Hq, Hkv, D, causal)
    qd = to_dev(q)
    kd = to_dev(k) if k.shape[0] else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    vd = to_dev(v) if v.shape[0] else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    o = torch.full((Tq, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((Hq, Tq), float("nan"), dtype=torch.float32, device="cuda")
    fx.flexsp_attn_varlen_fwd_kvshard(ctx, plan, qd, kd, vd, o, lse, causal=causal)
    torch.cuda.synchronize()
    plan.close()
    return o, lse


def _compare(tag, o, lse, O, LSE):
    got = bf16_f64(to_bits(o))
    assert np.isfinite(got).all(), f"{tag}: non-finite O"
    ma, rl = errors(got, O)
    L = lse.cpu().numpy().astype(np.float64)
    dead = np.isneginf(LSE)
    assert (np.isneginf(L) == dead).all(), f"{tag}: rows without a visible key differ"
    assert not got[dead.T].any(), f"{tag}: a row without keys is not zero"
    el = float(np.abs(L[~dead] - LSE[~dead]).max(initial=0.0))
    say(f"  {tag}: O max_abs={ma:.2e} rel_l2={rl:.2e} LSE max_abs={el:.2e} rows without keys={int(dead.sum())}")
    assert ma <= MAX_ABS and rl <= REL_L2 and el < 1e-3, tag


SHARD_CASES = [
    # name, query lengths, key lengths, shift per sequence, Hq, Hkv, D, causal
    ("aligned", [128, 64, 300], [128, 64, 300], [0, 0, 0], 2, 2, 128, True),               # = ordinary causal attention
    ("odd-shifts", [100, 257, 33, 200], [150, 257, 90, 64], [5, -17, 70, 1], 4, 2, 128, True),
    ("late-chunk", [300, 130], [1500, 700], [1200, 570], 2, 2, 128, True),                 # last queries, all keys: many unmasked tiles
    ("early-keys-long", [700], [2000], [1300], 2, 1, 128, True),
    ("nothing-visible", [130, 64, 200], [300, 100, 0], [-400, -64, 0], 2, 2, 128, True),  # keys lie after the queries / empty shard
    ("partly-visible", [200, 129], [128, 300], [-100, -128], 2, 2, 64, True),
    ("noncausal", [70, 300, 1], [129, 64, 500], [0, 0, 0], 4, 2, 64, False),
    ("noncausal-d128", [513, 31], [1000, 257], [-9, 9], 2, 2, 128, False),
    ("ragged-keys", [64, 64, 64], [1, 31, 33], [100, 100, 100], 2, 2, 128, True),
]


@pytest.mark.parametrize("name,lq,lk,shift,Hq,Hkv,D,causal", SHARD_CASES, ids=[c[0] for c in SHARD_CASES])
def test_kvshard_forward_matches_oracle_elementwise(ctx, name, lq, lk, shift, Hq, Hkv, D, causal):
    say(f"key-shard case {name}: queries {lq} keys {lk} shift {shift} Hq={Hq} Hkv={Hkv} D={D} causal={causal}")
    seed = 5200 + len(name)
    q = wl.normal_bf16(seed, wl.TID_Q, (sum(lq), Hq, D))
    k = wl.normal_bf16(seed, wl.TID_K, (sum(lk), Hkv, D))
    v = wl.normal_bf16(seed, wl.TID_V, (sum(lk), Hkv, D))
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    O, LSE = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal)
    o, lse = _shard_forward(ctx, q, k, v, cu_q, cu_k, shift, causal)
    _compare(name, o, lse, O, LSE)


CUT_CASES = [
    # name, query lengths, key lengths, shift, Hq, Hkv, D, causal
    ("diagonal-inside", [700, 60], [5000, 100], [3000, 10], 2, 1, 128, True),    # the diagonal crosses the shard's middle parts
    ("all-visible", [513], [6001], [7000], 1, 1, 128, True),
    ("noncausal-d64", [300, 129], [4500, 64], [0, 0], 2, 2, 64, False),
    ("starts-late", [4000], [4096], [-300], 2, 2, 64, True),                      # the first rows see no key: only later tiles are long
]


@pytest.mark.parametrize("name,lq,lk,shift,Hq,Hkv,D,causal", CUT_CASES, ids=[c[0] for c in CUT_CASES])
def test_long_shard_tiles_cut_into_parts_and_merged(ctx, name, lq, lk, shift, Hq, Hkv, D, causal):
    """Few heads and one long key shard: a query tile's walk over the shard would outlast an even share
    of the pass many times over, so the plan cuts it into parts with their own key ranges; the part
    that finishes last adds the partial results up in part order.  The plan must really contain cut
    tiles; every element against the oracle; three runs give the same bits."""
    import torch
    from paper_2412_01523_amd import binding as fx
    say(f"cut key-shard case {name}: queries {lq} keys {lk} shift {shift} Hq={Hq} Hkv={Hkv} D={D} causal={causal}")
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    plan = fx.ShardPlan(ctx, cu_q, cu_k, shift, Hq, Hkv, D, causal)
    items, _ = plan.items(fx.PASS_FWD)
    plan.close()
    say(f"  {len(items)} items, {int((items['nparts'] > 1).sum())} of them parts of cut tiles, up to {int(items['nparts'].max())} parts")
    assert (items["nparts"] > 2).any()
    seed = 5600 + len(name)
    q = wl.normal_bf16(seed, wl.TID_Q, (sum(lq), Hq, D))
    k = wl.normal_bf16(seed, wl.TID_K, (sum(lk), Hkv, D))
    v = wl.normal_bf16(seed, wl.TID_V, (sum(lk), Hkv, D))
    O, LSE = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal)
    runs = [_shard_forward(ctx, q, k, v, cu_q, cu_k, shift, causal) for _ in range(3)]
    _compare(name, runs[0][0], runs[0][1], O, LSE)
    for o, lse in runs[1:]:
        assert torch.equal(o.view(torch.int16), runs[0][0].view(torch.int16)), "O is not reproducible"
        assert torch.equal(lse.view(torch.int32), runs[0][1].view(torch.int32)), "LSE is not reproducible"


def _complete_statistics(q, k, v, cu_q, cu_k, shift, causal, extra, seed):
    """(O, LSE, delta-free inputs) of a COMPLETE attention that the shard (k, v) is one part of: the other
    part is `extra` more keys per sequence that every row sees (none if extra = 0).  Oracle only."""
    O, LSE = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal)
    if extra:
        B, Hkv, D = len(shift), k.shape[1], k.shape[2]
        k2 = wl.normal_bf16(seed, 11, (extra * B, Hkv, D))
        v2 = wl.normal_bf16(seed, 12, (extra * B, Hkv, D))
        O2, L2 = oracle.attn_fwd_kvshard(q, k2, v2, cu_q, wl.cu_seqlens([extra] * B), [0] * B, False)
        O, LSE = oracle.lse_merge(O, LSE, O2, L2)
    return O, LSE


def _shard_backward(ctx, q, k, v, o_bits, g, lse, cu_q, cu_k, shift, causal, grad_f32, accumulate_onto=None):
    """HIP path: (dQ, dK, dV) as fp64 host arrays.  accumulate_onto: three fp32 host arrays to add to."""
    import torch
    from paper_2412_01523_amd import binding as fx
    Tq, Hq, D = q.shape
    Tk, Hkv = k.shape[0], k.shape[1]
    plan = fx.ShardPlan(ctx, cu_q, cu_k, shift, Hq, Hkv, D, causal)
    kd = to_dev(k) if Tk else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    vd = to_dev(v) if Tk else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    gdt = torch.float32 if grad_f32 else torch.bfloat16
    if accumulate_onto is None:
        dq = torch.full((Tq, Hq, D), float("nan"), dtype=gdt, device="cuda")
        dk = torch.full((max(Tk, 8), Hkv, D), float("nan"), dtype=gdt, device="cuda")
        dv = torch.full((max(Tk, 8), Hkv, D), float("nan"), dtype=gdt, device="cuda")
    else:
        dq, dk, dv = (torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda() for x in accumulate_onto)
    fx.flexsp_attn_varlen_bwd_kvshard(ctx, plan, to_dev(q), kd, vd, to_dev(o_bits), to_dev(g),
                                      torch.from_numpy(np.ascontiguousarray(lse, dtype=np.float32)).cuda(), dq, dk, dv,
                                      causal=causal, accumulate=accumulate_onto is not None)
    torch.cuda.synchronize()
    plan.close()
    host = lambda t: t.cpu().numpy().astype(np.float64) if grad_f32 else bf16_f64(to_bits(t))
    return host(dq), host(dk)[:Tk], host(dv)[:Tk]


def _compare_grads(tag, got, ref, grad_f32, names=("dQ", "dK", "dV"), dq_is_a_part=False):
    """dq_is_a_part: the shard holds only some of the keys the rows see.  Its share of dQ can then be a small
    piece of the rows' gradient, while its error (delta from the rounded O, P rounded to bf16) is that of the
    complete attention: the relative bound belongs to the sum over the shards, the part is held to max-abs."""
    for name, g_, r_ in zip(names, got, ref):
        assert np.isfinite(g_).all(), f"{tag} {name}: non-finite values"
        ma, rl = errors(g_, r_)
        say(f"  {tag} {name}: max_abs={ma:.2e} rel_l2={rl:.2e}")
        # (a gradient stored as bf16 carries its final rounding on top, up to 2^-8 of its value)
        tol = MAX_ABS if grad_f32 else MAX_ABS + np.abs(r_) * 2.0 ** -8
        assert (np.abs(g_ - r_) <= tol).all(), f"{tag} {name}"
        assert rl <= REL_L2 or (name == "dQ" and dq_is_a_part), f"{tag} {name}"


@pytest.mark.parametrize("extra", [0, 37], ids=["shard-is-everything", "one-part-of-more"])
@pytest.mark.parametrize("name,lq,lk,shift,Hq,Hkv,D,causal", SHARD_CASES + CUT_CASES,
                         ids=[c[0] for c in SHARD_CASES + CUT_CASES])
def test_kvshard_backward_matches_oracle_elementwise(ctx, name, lq, lk, shift, Hq, Hkv, D, causal, extra):
    """flexsp_attn_varlen_bwd_kvshard against the oracle's shard backward, every element of dQ (the shard's
    part), dK and dV, fp32 and bf16 gradients.  The rows' log-sum-exp and output are those of a complete
    attention of which the shard is the whole (extra = 0: rows without a visible key then have lse = -inf)
    or one part (37 more keys per sequence that every row sees), computed by the oracle; the HIP path gets
    the output rounded to bf16 and the log-sum-exp rounded to fp32, as the forward ring would leave them."""
    say(f"key-shard backward {name}: queries {lq} keys {lk} shift {shift} Hq={Hq} Hkv={Hkv} D={D} causal={causal} extra={extra}")
    seed = 5700 + len(name)
    q = wl.normal_bf16(seed, wl.TID_Q, (sum(lq), Hq, D))
    k = wl.normal_bf16(seed, wl.TID_K, (sum(lk), Hkv, D))
    v = wl.normal_bf16(seed, wl.TID_V, (sum(lk), Hkv, D))
    g = wl.normal_bf16(seed, wl.TID_DO, (sum(lq), Hq, D))
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    O, LSE = _complete_statistics(q, k, v, cu_q, cu_k, shift, causal, extra, seed)
    delta = np.einsum("thd,thd->ht", bf16_f64(g), O)
    ref = oracle.attn_bwd_kvshard(q, k, v, g, LSE, delta, cu_q, cu_k, shift, causal)
    o_bits = wl.f32_to_bf16_bits(O.astype(np.float32))
    for grad_f32 in (True, False):
        got = _shard_backward(ctx, q, k, v, o_bits, g, LSE, cu_q, cu_k, shift, causal, grad_f32)
        _compare_grads(f"{name} {'fp32' if grad_f32 else 'bf16'}", got, ref, grad_f32, dq_is_a_part=extra > 0)


@pytest.mark.parametrize("causal", [True, False])
def test_backward_ring_accumulates_into_the_full_backward(ctx, causal):
    """One device's backward ring without the wire: it holds ALL query rows here (so dK / dV of a shard
    are complete after its one visit), meets the keys in three shards, ADDS each shard's part of dQ into
    one fp32 buffer and each shard's dK / dV onto a buffer that already holds numbers (what the previous
    device of a ring would have left).  Against the oracle's full backward, and the forward ring's own
    O / LSE feed the backward (nothing here comes from the oracle but the expected values)."""
    import torch
    from paper_2412_01523_amd import binding as fx
    lens, Hq, Hkv, D = [900, 64, 1, 333, 1500], 4, 2, 128
    cu = wl.cu_seqlens(lens)
    T, B = sum(lens), len(lens)
    q = wl.normal_bf16(5800, wl.TID_Q, (T, Hq, D)); g = wl.normal_bf16(5800, wl.TID_DO, (T, Hq, D))
    k = wl.normal_bf16(5800, wl.TID_K, (T, Hkv, D)); v = wl.normal_bf16(5800, wl.TID_V, (T, Hkv, D))
    _, _, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, causal)
    rng = np.random.default_rng(58)
    c1 = [int(rng.integers(0, s + 1)) for s in lens]
    c2 = [int(rng.integers(c, s + 1)) for c, s in zip(c1, lens)]
    say(f"backward ring: lens={lens} key cuts {c1} {c2} causal={causal}")

    def rows(x, lo, hi):
        return np.concatenate([x[int(cu[b]) + lo[b]: int(cu[b]) + hi[b]] for b in range(B)])

    shards = [([0] * B, c1), (c1, c2), (c2, list(lens))]
    # forward ring: partial attentions folded in place
    acc_o = acc_l = None
    for lo, hi in shards:
        o, lse = _shard_forward(ctx, q, rows(k, lo, hi), rows(v, lo, hi), cu, wl.cu_seqlens([h - l for l, h in zip(lo, hi)]),
                                [-l for l in lo], causal)
        if acc_o is None:
            acc_o, acc_l = o, lse
        else:
            fx.flexsp_lse_merge(ctx, acc_o, acc_l, o, lse, acc_o, acc_l)
    torch.cuda.synchronize()
    o_bits, lse_host = to_bits(acc_o), acc_l.cpu().numpy()
    # backward ring
    dq_acc = np.zeros((T, Hq, D), dtype=np.float32)
    for n, (lo, hi) in enumerate(shards):
        ks, vs = rows(k, lo, hi), rows(v, lo, hi)
        before_k = rng.standard_normal(ks.shape).astype(np.float32)
        before_v = rng.standard_normal(vs.shape).astype(np.float32)
        pad = lambda x: np.concatenate([x, np.zeros((max(8 - len(x), 0),) + x.shape[1:], dtype=np.float32)])
        dq_new, dk_s, dv_s = _shard_backward(ctx, q, ks, vs, o_bits, g, lse_host, cu,
                                             wl.cu_seqlens([h - l for l, h in zip(lo, hi)]), [-l for l in lo], causal,
                                             True, accumulate_onto=(dq_acc, pad(before_k), pad(before_v)))
        dq_acc = dq_new.astype(np.float32)
        _compare_grads(f"ring shard {n}", (dk_s - before_k, dv_s - before_v), (rows(dK, lo, hi), rows(dV, lo, hi)), True,
                       names=("dK", "dV"))
    _compare_grads("ring", (dq_acc.astype(np.float64),), (dQ,), True, names=("dQ",))


@pytest.mark.parametrize("seed", range(10))
def test_random_shard_configs_forward_and_backward(ctx, seed):
    """Random sequence counts, query and key lengths (empty ones included), shifts on both sides of the
    diagonal, head counts, head dims and causality, forward and backward against the oracle.  A shard of a
    few keys that hundreds of rows see collects gradients far beyond the N(0,1) magnitudes the stated
    max-abs bound belongs to (2e-2 on values up to about 4): there the bound is the same fraction, 5e-3, of
    the tensor's largest value, i.e. max-abs <= max(2e-2, 5e-3 max|ref|), plus the final rounding (2^-8 of
    the value) for gradients stored as bf16; relative L2 as stated."""
    rng = np.random.default_rng(6100 + seed)

    def rlen():
        kind = rng.integers(0, 8)
        return 0 if kind == 0 else int(rng.integers(1, 5)) if kind == 1 else int(rng.integers(1, 300)) if kind <= 4 \
            else int(rng.integers(300, 2500))

    B = int(rng.integers(1, 6)); Hkv = int(rng.integers(1, 3)); Hq = Hkv * int(rng.choice([1, 2, 4]))
    D = int(rng.choice([64, 128])); causal = bool(rng.integers(0, 4) != 0)
    lq, lk = [rlen() for _ in range(B)], [rlen() for _ in range(B)]
    if sum(lq) == 0:
        lq[0] = 7
    shift = [int(rng.integers(-300, 3000)) if rng.integers(0, 3) else int(rng.integers(-40, 40)) for _ in range(B)]
    extra = int(rng.choice([0, 21]))
    say(f"random shard case {seed}: queries {lq} keys {lk} shift {shift} Hq={Hq} Hkv={Hkv} D={D} causal={causal} extra={extra}")
    q = wl.normal_bf16(6100 + seed, wl.TID_Q, (sum(lq), Hq, D)); g = wl.normal_bf16(6100 + seed, wl.TID_DO, (sum(lq), Hq, D))
    k = wl.normal_bf16(6100 + seed, wl.TID_K, (sum(lk), Hkv, D)); v = wl.normal_bf16(6100 + seed, wl.TID_V, (sum(lk), Hkv, D))
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    O1, L1 = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal)
    o, lse = _shard_forward(ctx, q, k, v, cu_q, cu_k, shift, causal)
    _compare(f"random {seed}", o, lse, O1, L1)
    O, LSE = _complete_statistics(q, k, v, cu_q, cu_k, shift, causal, extra, 6100 + seed)
    delta = np.einsum("thd,thd->ht", bf16_f64(g), O)
    ref = oracle.attn_bwd_kvshard(q, k, v, g, LSE, delta, cu_q, cu_k, shift, causal)
    o_bits = wl.f32_to_bf16_bits(O.astype(np.float32))
    for grad_f32 in (True, False):
        got = _shard_backward(ctx, q, k, v, o_bits, g, LSE, cu_q, cu_k, shift, causal, grad_f32)
        for name, g_, r_ in zip(("dQ", "dK", "dV"), got, ref):
            assert np.isfinite(g_).all(), f"{name}: non-finite values"
            ma, rl = errors(g_, r_)
            top = float(np.abs(r_).max(initial=0.0))
            tol = max(MAX_ABS, REL_L2 * top) + (0.0 if grad_f32 else np.abs(r_) * 2.0 ** -8)
            say(f"  random {seed} {name} {'fp32' if grad_f32 else 'bf16'}: max_abs={ma:.2e} rel_l2={rl:.2e} (largest value {top:.1f})")
            assert (np.abs(g_ - r_) <= tol).all(), name
            assert rl <= REL_L2 or (name == "dQ" and extra > 0), name      # (a part of dQ: see _compare_grads)


def test_four_emulated_devices_ring_forward_and_backward_equal_the_unsplit_attention(ctx):
    """Context parallelism over four devices, all played by the one GPU, without the wire: device r holds the
    r-th quarter of every sequence's rows; in the forward every device meets every key shard (the ones that
    lie after its rows give nothing) and merges; in the backward dq stays with its device and gathers the
    shards' parts, dk / dv belong to a shard and gather the devices' parts (accumulate = 1 onto fp32
    buffers that start at zero).  The pieces put together must be the oracle's attention over the unsplit
    batch, forward and backward, at the stated tolerances."""
    import torch
    from paper_2412_01523_amd import binding as fx
    lens, Hq, Hkv, D, P = [6144, 2048, 333], 2, 1, 128, 4
    cu = wl.cu_seqlens(lens)
    T, B = sum(lens), len(lens)
    q = wl.normal_bf16(5900, wl.TID_Q, (T, Hq, D)); g = wl.normal_bf16(5900, wl.TID_DO, (T, Hq, D))
    k = wl.normal_bf16(5900, wl.TID_K, (T, Hkv, D)); v = wl.normal_bf16(5900, wl.TID_V, (T, Hkv, D))
    O, LSE, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    cut = [[(j * s) // P for j in range(P + 1)] for s in lens]
    say(f"four devices: lens={lens} cuts={cut}")

    def rows(x, j):
        return np.concatenate([x[int(cu[b]) + c[j]: int(cu[b]) + c[j + 1]] for b, c in enumerate(cut)])

    def scatter(parts):   # per-device row blocks -> the packed order
        out = np.zeros((T,) + parts[0].shape[1:], dtype=parts[0].dtype)
        for j, x in enumerate(parts):
            at = 0
            for b, c in enumerate(cut):
                n = c[j + 1] - c[j]
                out[int(cu[b]) + c[j]: int(cu[b]) + c[j + 1]] = x[at: at + n]
                at += n
        return out

    cu_part = [wl.cu_seqlens([c[j + 1] - c[j] for c in cut]) for j in range(P)]
    kd = [to_dev(rows(k, j)) for j in range(P)]
    vd = [to_dev(rows(v, j)) for j in range(P)]
    dk = [torch.zeros(kd[j].shape, dtype=torch.float32, device="cuda") for j in range(P)]
    dv = [torch.zeros(vd[j].shape, dtype=torch.float32, device="cuda") for j in range(P)]
    o_parts, l_parts, dq_parts = [], [], []
    for r in range(P):                                   # device r
        qd, gd = to_dev(rows(q, r)), to_dev(rows(g, r))
        Tq = qd.shape[0]
        plans = [fx.ShardPlan(ctx, cu_part[r], cu_part[j], [c[r] - c[j] for c in cut], Hq, Hkv, D, True) for j in range(P)]
        o_acc = torch.empty((Tq, Hq, D), dtype=torch.bfloat16, device="cuda")       # the complete O, rounded once
        o_run = torch.empty((Tq, Hq, D), dtype=torch.float32, device="cuda")        # the running result
        l_acc = torch.full((Hq, Tq), float("-inf"), dtype=torch.float32, device="cuda")
        o_new = torch.empty_like(o_acc)
        l_new = torch.empty((Hq, Tq), dtype=torch.float32, device="cuda")
        for j in [(r - i) % P for i in range(P)]:                    # its own shard first, then round the ring
            if j % 2:                                                 # (both ways of folding, alternately)
                fx.flexsp_attn_varlen_fwd_kvshard_acc(ctx, plans[j], qd, kd[j], vd[j], o_run, l_acc, o_acc)
            else:
                fx.flexsp_attn_varlen_fwd_kvshard(ctx, plans[j], qd, kd[j], vd[j], o_new, l_new)
                fx.flexsp_lse_merge_acc(ctx, o_run, l_acc, o_new, l_new, o_acc)
        dq = torch.zeros((Tq, Hq, D), dtype=torch.float32, device="cuda")
        for j in [(r - i) % P for i in range(P)]:
            fx.flexsp_attn_varlen_bwd_kvshard(ctx, plans[j], qd, kd[j], vd[j], o_acc, gd, l_acc, dq, dk[j], dv[j],
                                              accumulate=True)
        torch.cuda.synchronize()
        for pl in plans:
            pl.close()
        o_parts.append(bf16_f64(to_bits(o_acc)))
        l_parts.append(l_acc.cpu().numpy().astype(np.float64).T.copy())      # [Tq, Hq] for scatter()
        dq_parts.append(dq.cpu().numpy().astype(np.float64))
    got_o, got_l, got_dq = scatter(o_parts), scatter(l_parts).T, scatter(dq_parts)
    got_dk = scatter([x.cpu().numpy().astype(np.float64) for x in dk])
    got_dv = scatter([x.cpu().numpy().astype(np.float64) for x in dv])
    ma, rl = errors(got_o, O)
    el = float(np.abs(got_l - LSE).max())
    say(f"  ring of four: O max_abs={ma:.2e} rel_l2={rl:.2e} LSE max_abs={el:.2e}")
    assert ma <= MAX_ABS and rl <= REL_L2 and el < 1e-3
    _compare_grads("ring of four", (got_dq, got_dk, got_dv), (dQ, dK, dV), True)


def test_kvshard_backward_error_paths(ctx):
    import torch
    from paper_2412_01523_amd import binding as fx
    Hq, Hkv, D = 2, 2, 128
    sp = fx.ShardPlan(ctx, [0, 64], [0, 64], [0], Hq, Hkv, D, True)
    op = fx.Plan(ctx, [0, 64], Hq, Hkv, D, True)
    t = lambda h, dt=torch.bfloat16: torch.zeros((64, h, D), dtype=dt, device="cuda")
    lse = torch.zeros((Hq, 64), dtype=torch.float32, device="cuda")
    args = (t(Hq), t(Hkv), t(Hkv), t(Hq), t(Hq), lse)
    with pytest.raises(fx.FlexspError) as e:      # partial sums are kept in fp32
        fx.flexsp_attn_varlen_bwd_kvshard(ctx, sp, *args, t(Hq), t(Hkv), t(Hkv), accumulate=True)
    assert e.value.status == fx.UNSUPPORTED
    with pytest.raises(fx.FlexspError) as e:      # an ordinary plan does not serve the shard calls
        fx.flexsp_attn_varlen_bwd_kvshard(ctx, op, *args, t(Hq), t(Hkv), t(Hkv))
    assert e.value.status == fx.PLAN_MISMATCH
    with pytest.raises(fx.FlexspError) as e:      # ... nor a shard plan the ordinary backward
        fx.flexsp_attn_varlen_bwd(ctx, sp, *args, None, t(Hq), t(Hkv), t(Hkv))
    assert e.value.status == fx.PLAN_MISMATCH
    with pytest.raises(fx.FlexspError) as e:
        fx.flexsp_attn_varlen_bwd_kvshard(ctx, sp, *args, t(Hq), t(Hkv), t(Hkv), causal=False)
    assert e.value.status == fx.PLAN_MISMATCH
    fx.flexsp_attn_varlen_bwd_kvshard(ctx, sp, *args, t(Hq, torch.float32), t(Hkv, torch.float32), t(Hkv, torch.float32),
                                      accumulate=True)
    torch.cuda.synchronize()
    sp.close(); op.close()


def test_aligned_shard_equals_the_ordinary_forward_bitwise(ctx):
    """shift = 0 and keys = the whole sequence is ordinary causal attention: same kernel arithmetic,
    so the key-shard call must reproduce flexsp_attn_varlen_fwd bit for bit."""
    import torch
    from paper_2412_01523_amd import binding as fx
    lens, Hq, Hkv, D = [700, 64, 129, 1], 4, 2, 128
    cu = wl.cu_seqlens(lens)
    q, k, v = (wl.normal_bf16(5300, t, (sum(lens), h, D)) for t, h in ((0, Hq), (1, Hkv), (2, Hkv)))
    o, lse = _shard_forward(ctx, q, k, v, cu, cu, [0] * len(lens), True)
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, True)
    o2 = torch.empty_like(o); lse2 = torch.empty_like(lse)
    fx.flexsp_attn_varlen_fwd(ctx, plan, to_dev(q), to_dev(k), to_dev(v), None, o2, lse2)
    torch.cuda.synchronize()
    plan.close()
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16)) and torch.equal(lse, lse2)


@pytest.mark.parametrize("causal", [True, False])
def test_ring_of_three_shards_merges_into_the_full_attention(ctx, causal):
    """One device's view of a context-parallel ring, without the wire: its query chunk of every
    sequence meets the keys in three shards, one after the other, and folds each partial result into
    the running one with flexsp_lse_merge (in place).  The result must be the attention over all
    keys (oracle, and the HIP forward on the unsplit batch)."""
    import torch
    from paper_2412_01523_amd import binding as fx
    lens, Hq, Hkv, D = [900, 64, 1, 333, 1500], 4, 2, 128
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q = wl.normal_bf16(5400, wl.TID_Q, (T, Hq, D))
    k = wl.normal_bf16(5400, wl.TID_K, (T, Hkv, D))
    v = wl.normal_bf16(5400, wl.TID_V, (T, Hkv, D))
    O, LSE = oracle.attn_fwd(q, k, v, cu, causal)
    rng = np.random.default_rng(54)
    a0 = [int(rng.integers(0, max(s // 2, 1))) for s in lens]          # this device's query chunk: rows a0 .. s-1
    c1 = [int(rng.integers(0, s + 1)) for s in lens]
    c2 = [int(rng.integers(c, s + 1)) for c, s in zip(c1, lens)]
    say(f"ring: lens={lens} query chunks start at {a0}, key cuts {c1} {c2}, causal={causal}")

    def rows(x, lo, hi):
        return np.concatenate([x[int(cu[b]) + lo[b]: int(cu[b]) + hi[b]] for b in range(len(lens))])

    qs = rows(q, a0, lens)
    cu_q = wl.cu_seqlens([s - a for s, a in zip(lens, a0)])
    acc_o = acc_l = None
    for lo, hi in (([0] * len(lens), c1), (c1, c2), (c2, list(lens))):
        cu_k = wl.cu_seqlens([h - l for l, h in zip(lo, hi)])
        shift = [a - l for a, l in zip(a0, lo)]
        o, lse = _shard_forward(ctx, qs, rows(k, lo, hi), rows(v, lo, hi), cu_q, cu_k, shift, causal)
        if acc_o is None:
            acc_o, acc_l = o, lse
        else:
            fx.flexsp_lse_merge(ctx, acc_o, acc_l, o, lse, acc_o, acc_l)      # fold in place
    torch.cuda.synchronize()
    Oq = rows(O, a0, lens)
    Lq = np.concatenate([LSE[:, int(cu[b]) + a0[b]: int(cu[b + 1])] for b in range(len(lens))], axis=1)
    _compare(f"ring causal={causal}", acc_o, acc_l, Oq, Lq)
    # and against the HIP forward on the unsplit batch: the same numbers up to the extra roundings of the parts
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, causal)
    o_full = torch.empty((T, Hq, D), dtype=torch.bfloat16, device="cuda")
    l_full = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    fx.flexsp_attn_varlen_fwd(ctx, plan, to_dev(q), to_dev(k), to_dev(v), None, o_full, l_full, causal=causal)
    torch.cuda.synchronize()
    plan.close()
    d = bf16_f64(to_bits(acc_o)) - rows(bf16_f64(to_bits(o_full)), a0, lens)
    assert np.abs(d).max() <= MAX_ABS


def test_lse_merge_matches_oracle_and_ignores_parts_without_keys(ctx):
    import torch
    from paper_2412_01523_amd import binding as fx
    for T, H, D in ((300, 3, 128), (129, 2, 64)):
        rng = np.random.default_rng(T)
        oa = wl.normal_bf16(5500, 0, (T, H, D)); ob = wl.normal_bf16(5500, 1, (T, H, D))
        la = rng.normal(3.0, 2.0, (H, T)).astype(np.float32); lb = rng.normal(3.0, 2.0, (H, T)).astype(np.float32)
        la[0, ::7] = -np.inf                      # part a saw no key on these rows ...
        lb[0, ::5] = -np.inf                      # ... part b on these (every 35th row: neither did)
        oa_f, ob_f = bf16_f64(oa), bf16_f64(ob)
        O, L = oracle.lse_merge(oa_f, la, ob_f, lb)
        oa_dev, ob_dev = to_dev(oa), to_dev(ob)
        oa_dev[::7, 0] = float("nan")             # whatever a part without keys holds must not leak
        la_d, lb_d = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
        out = torch.full((T, H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lo = torch.full((H, T), float("nan"), dtype=torch.float32, device="cuda")
        fx.flexsp_lse_merge(ctx, oa_dev, la_d, ob_dev, lb_d, out, lo)
        torch.cuda.synchronize()
        got, gl = bf16_f64(to_bits(out)), lo.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        dead = np.isneginf(L)
        assert (np.isneginf(gl) == dead).all() and not got[dead.T].any()
        assert np.abs(gl[~dead] - L[~dead]).max() < 1e-5 * (1 + np.abs(L[~dead]).max())
        # one rounding of the result to bf16 plus fp32 arithmetic
        assert (np.abs(got - O) <= 2.0 ** -8 * np.abs(O) + 1e-5).all()
        # strided views (heads 1.. of a wider tensor) and in-place use give the same bits
        wide = torch.zeros((T, H + 2, D), dtype=torch.bfloat16, device="cuda")
        wide[:, 1:H + 1] = oa_dev
        fx.flexsp_lse_merge(ctx, wide[:, 1:H + 1], la_d, ob_dev, lb_d, wide[:, 1:H + 1], la_d)
        torch.cuda.synchronize()
        assert torch.equal(wide[:, 1:H + 1].contiguous().view(torch.int16), out.view(torch.int16))
        assert torch.equal(la_d, lo) and not wide[:, 0].any() and not wide[:, H + 1].any()


def test_lse_merge_acc_keeps_the_running_result_in_fp32(ctx):
    """flexsp_lse_merge_acc against the oracle's merge: the fp32 running result to fp32 accuracy, the optional
    bf16 copy = that result rounded once (bit for bit), a ring started from lse = -inf over rubbish, and the
    reason it exists: sixteen parts folded one by one stay at fp32 accuracy, where the bf16 merge has
    rounded the running result fifteen times."""
    import torch
    from paper_2412_01523_amd import binding as fx
    T, H, D = 300, 3, 128
    rng = np.random.default_rng(77)
    acc = rng.standard_normal((T, H, D)).astype(np.float32)
    ob = wl.normal_bf16(5510, 1, (T, H, D))
    la = rng.normal(3.0, 2.0, (H, T)).astype(np.float32); lb = rng.normal(3.0, 2.0, (H, T)).astype(np.float32)
    la[0, ::7] = -np.inf; lb[0, ::5] = -np.inf
    O, L = oracle.lse_merge(acc.astype(np.float64), la, bf16_f64(ob), lb)
    acc_d = torch.from_numpy(acc).cuda()
    acc_d[::7, 0] = float("nan")                  # whatever a part without keys holds must not leak
    la_d, lb_d = torch.from_numpy(la).cuda(), torch.from_numpy(lb).cuda()
    o16 = torch.full((T, H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    fx.flexsp_lse_merge_acc(ctx, acc_d, la_d, to_dev(ob), lb_d, o16)
    torch.cuda.synchronize()
    got, gl = acc_d.cpu().numpy().astype(np.float64), la_d.cpu().numpy().astype(np.float64)
    dead = np.isneginf(L)
    assert np.isfinite(got).all() and (np.isneginf(gl) == dead).all() and not got[dead.T].any()
    assert np.abs(got - O).max() <= 1e-5 and np.abs(gl[~dead] - L[~dead]).max() <= 1e-5
    assert torch.equal(o16.view(torch.int16), acc_d.to(torch.bfloat16).view(torch.int16))
    # sixteen parts, one by one
    parts = [(wl.normal_bf16(5520 + n, 0, (T, H, D)), rng.normal(0.0, 1.0, (H, T)).astype(np.float32)) for n in range(16)]
    Or, Lr = bf16_f64(parts[0][0]), parts[0][1].astype(np.float64)
    for o_n, l_n in parts[1:]:
        Or, Lr = oracle.lse_merge(Or, Lr, bf16_f64(o_n), l_n)
    acc_d = torch.full((T, H, D), float("nan"), dtype=torch.float32, device="cuda")
    lacc_d = torch.full((H, T), float("-inf"), dtype=torch.float32, device="cuda")
    run16, lrun = to_dev(parts[0][0]).clone(), torch.from_numpy(parts[0][1]).cuda()
    for n, (o_n, l_n) in enumerate(parts):
        fx.flexsp_lse_merge_acc(ctx, acc_d, lacc_d, to_dev(o_n), torch.from_numpy(l_n).cuda())
        if n:
            fx.flexsp_lse_merge(ctx, run16, lrun, to_dev(o_n), torch.from_numpy(l_n).cuda(), run16, lrun)
    torch.cuda.synchronize()
    e32 = errors(acc_d.cpu().numpy().astype(np.float64), Or)
    e16 = errors(bf16_f64(to_bits(run16)), Or)
    say(f"  sixteen parts folded: fp32 running result rel_l2={e32[1]:.2e}, bf16 running result rel_l2={e16[1]:.2e}")
    assert e32[1] <= 1e-5 and e16[1] <= 1e-2 and e32[1] < e16[1] / 50     # (fifteen bf16 roundings: about 5e-3)
    assert np.abs(lacc_d.cpu().numpy() - Lr).max() <= 1e-5


@pytest.mark.parametrize("name,lq,lk,shift,Hq,Hkv,D,causal", SHARD_CASES + CUT_CASES, ids=[c[0] for c in SHARD_CASES + CUT_CASES])
def test_kvshard_forward_folded_into_a_running_result(ctx, name, lq, lk, shift, Hq, Hkv, D, causal):
    """flexsp_attn_varlen_fwd_kvshard_acc = the shard's attention merged into (o_acc, lse_acc), against the
    oracle's shard attention merged by the oracle's merge: from an empty running result (lse = -inf over NaN)
    and from one that holds numbers; the fp32 rows to fp32-with-bf16-operands accuracy (the stated O bounds),
    the bf16 copy = the fp32 rows rounded once, rows that have seen no key anywhere: LSE = -inf, bf16 copy 0."""
    import torch
    from paper_2412_01523_amd import binding as fx
    say(f"folded key-shard case {name}: queries {lq} keys {lk} shift {shift} Hq={Hq} Hkv={Hkv} D={D} causal={causal}")
    seed = 6300 + len(name)
    Tq = sum(lq)
    q = wl.normal_bf16(seed, wl.TID_Q, (Tq, Hq, D))
    k = wl.normal_bf16(seed, wl.TID_K, (sum(lk), Hkv, D))
    v = wl.normal_bf16(seed, wl.TID_V, (sum(lk), Hkv, D))
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    O1, L1 = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, shift, causal)
    rng = np.random.default_rng(seed)
    prev_o = rng.standard_normal((Tq, Hq, D)).astype(np.float32)
    prev_l = rng.normal(2.0, 2.0, (Hq, Tq)).astype(np.float32)
    prev_l[:, ::9] = -np.inf
    plan = fx.ShardPlan(ctx, cu_q, cu_k, shift, Hq, Hkv, D, causal)
    kd = to_dev(k) if len(k) else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    vd = to_dev(v) if len(v) else torch.zeros((8, Hkv, D), dtype=torch.bfloat16, device="cuda")
    for tag, start_o, start_l in (("from nothing", np.full((Tq, Hq, D), np.nan, dtype=np.float32), np.full((Hq, Tq), -np.inf, dtype=np.float32)),
                                  ("onto a result", prev_o, prev_l)):
        want_o, want_l = oracle.lse_merge(np.nan_to_num(start_o.astype(np.float64)), start_l, O1, L1)
        o_acc, l_acc = torch.from_numpy(start_o.copy()).cuda(), torch.from_numpy(start_l.copy()).cuda()
        if tag == "onto a result":
            o_acc[::9] = float("nan")                 # rows whose running result is empty may hold anything
        o16 = torch.full((Tq, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        fx.flexsp_attn_varlen_fwd_kvshard_acc(ctx, plan, to_dev(q), kd, vd, o_acc, l_acc, o16, causal=causal)
        torch.cuda.synchronize()
        got_l = l_acc.cpu().numpy().astype(np.float64)
        dead = np.isneginf(want_l)
        assert (np.isneginf(got_l) == dead).all(), f"{name} {tag}: rows without any key differ"
        live = ~dead.T
        got = o_acc.cpu().numpy().astype(np.float64)
        assert np.isfinite(got[live]).all()
        ma, rl = errors(got[live], want_o[live])
        el = float(np.abs(got_l[~dead] - want_l[~dead]).max(initial=0.0))
        say(f"  {name} {tag}: O max_abs={ma:.2e} rel_l2={rl:.2e} LSE max_abs={el:.2e} rows without any key={int(dead.sum())}")
        assert ma <= MAX_ABS and rl <= REL_L2 and el < 1e-3
        got16 = bf16_f64(to_bits(o16))
        assert not got16[dead.T].any()
        # (rows that stay empty keep whatever o_acc held: only the live rows of the copy are the rounded fp32 rows)
        assert np.array_equal(to_bits(o16)[live], to_bits(o_acc.to(torch.bfloat16))[live])
    plan.close()


def test_kvshard_error_paths(ctx):
    import torch
    from paper_2412_01523_amd import binding as fx
    cu = wl.cu_seqlens([64])
    t = torch.zeros((64, 2, 64), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    shard = fx.ShardPlan(ctx, cu, cu, [0], 2, 2, 64, True)
    plain = fx.Plan(ctx, cu, 2, 2, 64, True)
    with pytest.raises(fx.FlexspError) as e:
        fx.flexsp_attn_varlen_fwd(ctx, shard, t, t, t, None, t, lse)                 # a key-shard plan serves its own call only
    assert e.value.status == fx.PLAN_MISMATCH
    with pytest.raises(fx.FlexspError) as e:
        fx.flexsp_attn_varlen_fwd_kvshard(ctx, plain, t, t, t, t, lse)
    assert e.value.status == fx.PLAN_MISMATCH
    with pytest.raises(fx.FlexspError) as e:
        fx.flexsp_attn_varlen_bwd(ctx, shard, t, t, t, t, t, lse, None, t, t, t)
    assert e.value.status == fx.PLAN_MISMATCH
    shard.close(); plain.close()


def test_ring_at_bench_size_sampled_against_the_oracle(ctx):
    """The configuration `bench.py --kvshard-ring` times: the 131 072-token sequence (8 heads, D = 128) over a
    ring of 8, the device with the last 16 384 query rows, forward ring (8 shard forwards, each folding its
    result into the fp32 running one) and
    backward ring (8 shard backwards, fp32 accumulation).  The oracle cannot run that in full inside a test;
    compared are outputs it computes one by one on the unsplit sequence: sampled rows of O, LSE and dQ (complete
    after the last shard), and late rows of dK / dV of the device's OWN shard, whose keys no other device's
    rows see, so that this device's part is the complete gradient.  Plus, over whole tensors: the ring's O rows
    against the ordinary forward's on the unsplit sequence (HIP against HIP, within the parts' roundings)."""
    import torch
    from paper_2412_01523_amd import binding as fx
    cfg = next(c for c in wl.CONFIGS if c.name == "single-128k")
    S, Hq, Hkv, D, P = cfg.tokens, cfg.hq, cfg.hkv, cfg.d, 8
    C = S // P
    say(f"ring at bench size: S={S} Hq={Hq} D={D} P={P}; generating inputs")
    q, k, v, g = wl.make_qkvdo(cfg)
    cu = wl.cu_seqlens([S])
    first = S - C
    qd, gd = to_dev(q[first:]), to_dev(g[first:])
    kd, vd = to_dev(k), to_dev(v)
    plans = [fx.ShardPlan(ctx, [0, C], [0, C], [first - j * C], Hq, Hkv, D, True) for j in range(P)]
    o_acc = torch.empty((C, Hq, D), dtype=torch.bfloat16, device="cuda")            # the complete O, rounded once
    o_run = torch.empty((C, Hq, D), dtype=torch.float32, device="cuda")             # the running result
    l_acc = torch.full((Hq, C), float("-inf"), dtype=torch.float32, device="cuda")
    o_new = torch.empty_like(o_acc)
    l_new = torch.empty((Hq, C), dtype=torch.float32, device="cuda")
    order = list(range(P - 1, -1, -1))
    for j in order:
        fx.flexsp_attn_varlen_fwd_kvshard_acc(ctx, plans[j], qd, kd[j * C:(j + 1) * C], vd[j * C:(j + 1) * C], o_run, l_acc,
                                              o_acc if j == order[-1] else None)
    dq = torch.zeros((C, Hq, D), dtype=torch.float32, device="cuda")
    dk_own = torch.zeros((C, Hkv, D), dtype=torch.float32, device="cuda")
    dv_own = torch.zeros((C, Hkv, D), dtype=torch.float32, device="cuda")
    dk_other, dv_other = torch.zeros_like(dk_own), torch.zeros_like(dv_own)
    for j in order:
        own = j == P - 1
        fx.flexsp_attn_varlen_bwd_kvshard(ctx, plans[j], qd, kd[j * C:(j + 1) * C], vd[j * C:(j + 1) * C], o_acc, gd, l_acc,
                                          dq, dk_own if own else dk_other, dv_own if own else dv_other, accumulate=True)
    torch.cuda.synchronize()
    for pl in plans:
        pl.close()
    assert torch.isfinite(dq).all() and torch.isfinite(dk_own).all() and torch.isfinite(dv_own).all()
    say("  HIP rings done; sampling the oracle")
    rng = np.random.Generator(np.random.Philox(key=[cfg.seed, 777]))
    rows = sorted(set([0, 1, 31, 32, 127, 128, C // 2, C - 129, C - 2, C - 1] + [int(x) for x in rng.integers(0, C, size=14)]))
    tok = np.array([first + r for r in rows], dtype=np.int64)
    head = rng.integers(0, Hq, size=len(tok)).astype(np.int32)
    Or, Lr, dQr = oracle.rows(q, k, v, g, cu, tok, head, True)
    rr, hh = torch.from_numpy(np.array(rows)).cuda(), torch.from_numpy(head.astype(np.int64)).cuda()
    Og = bf16_f64(to_bits(o_acc[rr, hh])); Lg = l_acc[hh, rr].cpu().numpy().astype(np.float64)
    dQg = dq[rr, hh].cpu().numpy().astype(np.float64)
    eo, eq = errors(Og, Or), errors(dQg, dQr)
    say(f"  {len(tok)} sampled rows: O (max_abs, rel_l2)=({eo[0]:.2e},{eo[1]:.2e}) dQ=({eq[0]:.2e},{eq[1]:.2e}) LSE max_abs={np.abs(Lg - Lr).max():.2e}")
    assert eo[0] <= MAX_ABS and eo[1] <= REL_L2 and eq[0] <= MAX_ABS and eq[1] <= REL_L2 and np.abs(Lg - Lr).max() < 1e-3
    # dK / dV of the own shard: keys first .. S-1, seen by this device's rows only
    # (the oracle needs the complete softmax row of every query that sees a sampled key: keys of the last
    # 1 500 positions, two heads; deeper accumulation is compared at sizes the oracle runs in full, above)
    keys, kv_heads = [C - 1500, C - 701, C - 65, C - 64, C - 1], sorted({0, Hkv - 1})
    dKr, dVr = oracle.dkv_rows(q, k, v, g, cu, [(0, gk, [first + j for j in keys]) for gk in kv_heads], True)
    kk = torch.from_numpy(np.array(keys)).cuda()
    dKg = torch.cat([dk_own[kk, gk] for gk in kv_heads]).cpu().numpy().astype(np.float64)
    dVg = torch.cat([dv_own[kk, gk] for gk in kv_heads]).cpu().numpy().astype(np.float64)
    ek, ev = errors(dKg, dKr), errors(dVg, dVr)
    say(f"  {len(keys)} x {len(kv_heads)} own-shard key rows: dK=({ek[0]:.2e},{ek[1]:.2e}) dV=({ev[0]:.2e},{ev[1]:.2e})")
    assert ek[0] <= MAX_ABS and ek[1] <= REL_L2 and ev[0] <= MAX_ABS and ev[1] <= REL_L2
    # whole tensor: the ring's O against the ordinary forward on the unsplit sequence
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, True)
    o_full = torch.empty((S, Hq, D), dtype=torch.bfloat16, device="cuda")
    l_full = torch.empty((Hq, S), dtype=torch.float32, device="cuda")
    fx.flexsp_attn_varlen_fwd(ctx, plan, to_dev(q), kd, vd, None, o_full, l_full)
    torch.cuda.synchronize()
    plan.close()
    d = (o_acc.float() - o_full[first:].float()).abs().max().item()
    dl = (l_acc - l_full[:, first:]).abs().max().item()
    say(f"  ring vs unsplit forward over all {C} rows: O max_abs={d:.2e} LSE max_abs={dl:.2e}")
    assert d <= MAX_ABS and dl < 1e-3
