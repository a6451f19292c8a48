"""CPU-only tests of the C-ABI library's host logic: it loads, exports every declared symbol,
validates arguments before any launch, and builds longest-first tile plans."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2412_01523_amd import binding as fx
from paper_2412_01523_amd import workloads as wl

ROOT = Path(__file__).resolve().parent.parent


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "flexsp.h").read_text()
    declared = set(re.findall(r"\b(flexsp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(fx.EXPORTS)
    L = fx.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert fx.lib().flexsp_version().decode() == "0.1"
    assert fx.lib().flexsp_strerror(fx.PLAN_MISMATCH).decode() == "arguments do not match the plan"


@pytest.fixture(scope="module")
def host_ctx():
    c = fx.Context(-1)
    yield c
    c.close()


def test_host_only_context_and_bad_devices(host_ctx):
    assert host_ctx.num_cu == 0 and host_ctx.num_xcd == 8
    with pytest.raises(fx.FlexspError) as e:
        fx.Context(-2)
    assert e.value.status == fx.INVALID_ARGUMENT


def test_plan_argument_validation(host_ctx):
    ok = np.array([0, 5, 9], dtype=np.int32)
    for cu, hq, hkv, d, status in [
        (np.array([1, 5], dtype=np.int32), 2, 2, 64, fx.INVALID_ARGUMENT),      # cu[0] != 0
        (np.array([0, 5, 4], dtype=np.int32), 2, 2, 64, fx.INVALID_ARGUMENT),   # decreasing
        (ok, 3, 2, 64, fx.INVALID_ARGUMENT),                                     # Hq % Hkv
        (ok, 0, 1, 64, fx.INVALID_ARGUMENT),
        (ok, 2, 2, 96, fx.UNSUPPORTED),                                          # head dim
    ]:
        with pytest.raises(fx.FlexspError) as e:
            fx.Plan(host_ctx, cu, hq, hkv, d)
        assert e.value.status == status


def _tile_steps(i, which, causal, rows, group=1):
    """Inner-loop steps of the TILE an item belongs to: 64-key steps a query tile walks, or 64-query
    steps (times the heads of the group) a key tile walks."""
    s, t = int(i["seq_len"]), int(i["tile"])
    if which == fx.PASS_BWD_DKV:
        return -(-(s - (t * rows if causal else 0)) // 64) * group
    return -(-(min(s, (t + 1) * rows) if causal else s) // 64)


def _item_steps(i, which, causal, rows, group=1):
    """Steps of the item itself: part p of k of a tile with n steps covers p*n//k .. (p+1)*n//k - 1."""
    n, p, k = _tile_steps(i, which, causal, rows, group), int(i["part"]), int(i["nparts"])
    assert (int(i["step_begin"]), int(i["step_end"])) == (p * n // k, (p + 1) * n // k)
    return (p + 1) * n // k - p * n // k


def _check_pass(plan, which, lens, heads, rows):
    items, offs = plan.items(which)
    cu = wl.cu_seqlens(lens)
    # every (sequence, tile, head) is covered: by one whole item, or by parts 0 .. nparts-1 exactly once,
    # which agree on nparts and on the slot; slots of different tiles do not overlap
    want = set()
    for b, s in enumerate(lens):
        for t in range(-(-s // rows)):
            for h in range(heads):
                want.add((int(cu[b]), s, t, h))
    tiles = {}
    for it in items:
        key = (int(it["seq_start"]), int(it["seq_len"]), int(it["tile"]), int(it["head"]))
        tiles.setdefault(key, []).append((int(it["part"]), int(it["nparts"]), int(it["slot"])))
    assert set(tiles) == want
    used = []
    for key, parts in tiles.items():
        k = parts[0][1]
        assert sorted(p for p, _, _ in parts) == list(range(k)) and all(n == k for _, n, _ in parts), (key, parts)
        if k == 1:
            assert parts[0][2] == -1
        else:
            assert 2 <= k <= 8 and len(set(sl for _, _, sl in parts)) == 1 and parts[0][2] >= 0
            used.append((parts[0][2], parts[0][2] + k))
    used.sort()
    assert all(a[1] <= b[0] for a, b in zip(used, used[1:]))
    assert offs[0] == 0 and offs[-1] == len(items) and (np.diff(offs) >= 0).all()
    return items, offs


@pytest.mark.parametrize("causal", [True, False])
def test_plan_covers_every_tile_once_longest_first(host_ctx, causal):
    lens = [17, 64, 0, 100, 255, 1000, 129, 4000]
    hq, hkv, d = 4, 2, 128
    plan = fx.Plan(host_ctx, wl.cu_seqlens(lens), hq, hkv, d, causal)
    live = [s for s in lens if s > 0]
    for which, heads in ((fx.PASS_FWD, hq), (fx.PASS_BWD_DKV, hkv), (fx.PASS_BWD_DQ, hq)):
        rows = plan.tile_rows(which)
        items, offs = _check_pass(plan, which, live if False else lens, heads, rows)
        # inside a queue: items of long sequences in order of decreasing cost (inner-loop steps); the tiles
        # of a short sequence (none of more than 24 steps) side by side, dearest first, where the dearest
        # of them would stand
        cost = [_item_steps(i, which, causal, rows, hq // hkv) for i in items]
        gmax = {}
        for i, c in zip(items, cost):
            key = (int(i["seq_start"]), int(i["head"]))
            gmax[key] = max(gmax.get(key, 0), c)
        for x in range(len(offs) - 1):
            seg = range(int(offs[x]), int(offs[x + 1]))
            keys = [(int(items[n]["seq_start"]), int(items[n]["head"])) for n in seg]
            rank = [cost[n] if gmax[k] > 24 else gmax[k] for n, k in zip(seg, keys)]
            assert all(a >= b for a, b in zip(rank, rank[1:]))
            seen, prev = set(), None
            for n, k in zip(seg, keys):
                if gmax[k] <= 24:
                    assert k == prev or k not in seen          # a short sequence's tiles are contiguous ...
                    if k == prev:
                        assert cost[n] <= cost[n - 1]          # ... and ordered
                    seen.add(k)
                prev = k
        # tiles are cut when, and only when, they would outlast 3/4 of an even share of the pass over the
        # 512 workgroups a host-only context plans for; no part is shorter than 16 steps
        total = sum(_item_steps(i, which, causal, rows, hq // hkv) for i in items)
        target = max(total // 512 * 3 // 4, 16)
        for i in items:
            n = _tile_steps(i, which, causal, rows, hq // hkv)
            if int(i["nparts"]) > 1:
                assert n > target and n >= 32 and _item_steps(i, which, causal, rows, hq // hkv) >= 16
                assert int(i["nparts"]) == min(-(-n // target), 8, n // 16)
            else:
                assert n <= target or n < 32
        # a (sequence, head) group stays on one queue (one XCD, one L2) unless levelling the queues
        # had to move some of its cheapest tiles: most groups are whole
        owner = {}
        for x in range(len(offs) - 1):
            for i in items[offs[x]:offs[x + 1]]:
                owner.setdefault((int(i["seq_start"]), int(i["head"])), set()).add(x)
        assert sum(1 for v in owner.values() if len(v) == 1) >= 0.6 * len(owner)
    assert plan.workspace_bytes == 2 * sum(lens) * hq * 4      # delta and log2-domain LSE
    plan.close()


def test_plan_balances_queues_on_the_long_tail_config(host_ctx):
    cfg = wl.CONFIGS[2]
    lens = wl.lengths(cfg)
    plan = fx.Plan(host_ctx, wl.cu_seqlens(lens), cfg.hq, cfg.hkv, cfg.d, True)
    items, offs = plan.items(fx.PASS_FWD)
    rows = plan.tile_rows(fx.PASS_FWD)
    load = []
    for x in range(8):
        seg = items[offs[x]:offs[x + 1]]
        load.append(sum(_item_steps(i, fx.PASS_FWD, True, rows) for i in seg))
    assert max(load) <= 1.01 * (sum(load) / 8) + 2
    # the very first item of each queue is one of the longest tiles of the batch
    longest = max(lens)
    assert all(int(items[offs[x]]["seq_len"]) >= 0.2 * longest for x in range(8))
    plan.close()


def test_plan_levels_queues_when_one_sequence_dominates(host_ctx):
    """Config 1: one sequence holds 60 % of the work and there are only 4 heads, so whole
    (sequence, head) groups cannot balance 8 queues; tiles must be moved."""
    cfg = wl.CONFIGS[1]
    lens = wl.lengths(cfg)
    plan = fx.Plan(host_ctx, wl.cu_seqlens(lens), cfg.hq, cfg.hkv, cfg.d, True)
    for which, step in ((fx.PASS_FWD, 64), (fx.PASS_BWD_DQ, 64)):
        items, offs = plan.items(which)
        rows = plan.tile_rows(which)
        load = [sum(_item_steps(i, which, True, rows) for i in items[offs[x]:offs[x + 1]]) for x in range(8)]
        assert max(load) - min(load) <= max(-(-max(lens) // step), 4), load
    plan.close()


def test_plan_with_few_enormous_items_takes_the_comparison_sort_path(host_ctx):
    """One 200 000-token sequence, non-causal, one kv head for sixteen query heads: the dK/dV pass
    has 3 125 items of 50 000 steps each, so a table indexed by cost would be larger than the list
    and the builder sorts by comparison instead; the same invariants hold."""
    lens = [200000, 70, 0, 3]
    plan = fx.Plan(host_ctx, wl.cu_seqlens(lens), 16, 1, 128, False)
    for which, heads in ((fx.PASS_FWD, 16), (fx.PASS_BWD_DKV, 1), (fx.PASS_BWD_DQ, 16)):
        rows = plan.tile_rows(which)
        items, offs = _check_pass(plan, which, lens, heads, rows)
        for x in range(len(offs) - 1):
            seg = [_item_steps(i, which, False, rows, 16) for i in items[offs[x]:offs[x + 1]]]
            assert all(a >= b for a, b in zip(seg, seg[1:]))
        sizes = np.diff(offs)
        assert sizes.max() - sizes.min() <= 2 + len(lens) * heads   # equal-cost items: queues level out
    plan.close()


def test_permute_and_attention_validation_without_a_device(host_ctx):
    L = fx.lib()
    h = host_ctx.handle
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    # shape errors come first, whatever the pointers are
    assert L.flexsp_pack(h, a, a + 2048, 4, 6, 8, 4, 2, None) == fx.INVALID_ARGUMENT    # H % P
    assert L.flexsp_pack(h, a, a + 2048, 4, 4, 8, 2, 3, None) == fx.UNSUPPORTED         # elem size
    assert L.flexsp_pack(h, a, a + 2048, -1, 4, 8, 2, 2, None) == fx.INVALID_ARGUMENT
    assert L.flexsp_pack(None, a, a + 2048, 4, 4, 8, 2, 2, None) == fx.INVALID_ARGUMENT
    assert L.flexsp_pack(h, None, a, 4, 4, 8, 2, 2, None) == fx.INVALID_ARGUMENT
    assert L.flexsp_pack(h, a, a + 64, 4, 4, 8, 2, 2, None) == fx.INVALID_ARGUMENT      # overlap
    assert L.flexsp_unpack(h, a, a + 2048, 0, 4, 8, 2, 2, None) == fx.OK                # empty: no-op
    # well-formed call on a host-only context: refuses to launch, does not crash
    assert L.flexsp_pack(h, a, a + 2048, 4, 4, 8, 2, 2, None) == fx.NO_DEVICE
    # the multi-tensor form: same checks per tensor, and no two of the 2n buffers may overlap
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    def many(fn, srcs, dsts, heads, T=4, D=8, P=2, eb=2, n=None):
        n = len(srcs) if n is None else n
        return fn(h, n, (vp * len(srcs))(*srcs), (vp * len(dsts))(*dsts), T, (i32 * len(heads))(*heads), D, P, eb, None)
    assert many(L.flexsp_pack_many, [a, a + 512], [a + 1024, a + 1536], [4, 4]) == fx.NO_DEVICE
    assert many(L.flexsp_pack_many, [a, a + 512], [a + 1024, a + 1536], [4, 3]) == fx.INVALID_ARGUMENT   # H % P
    assert many(L.flexsp_pack_many, [a, a + 512], [a + 1024, a + 1100], [4, 4]) == fx.INVALID_ARGUMENT   # dst/dst overlap
    assert many(L.flexsp_pack_many, [a, a + 512], [a + 600, a + 1536], [4, 4]) == fx.INVALID_ARGUMENT    # src/dst overlap
    assert many(L.flexsp_unpack_many, [a, None], [a + 1024, a + 1536], [4, 4]) == fx.INVALID_ARGUMENT    # null tensor
    assert many(L.flexsp_unpack_many, [a] * 5, [a] * 5, [4] * 5) == fx.INVALID_ARGUMENT                  # too many
    assert many(L.flexsp_unpack_many, [], [], [], n=0) == fx.OK                                          # none: no-op
    assert many(L.flexsp_pack_many, [a, a + 512], [a + 1024, a + 1536], [4, 4], T=0) == fx.OK            # empty
    plan = fx.Plan(host_ctx, np.array([0, 8], dtype=np.int32), 2, 2, 64, True)
    t = fx.Tensor(a, 128, 64)
    bad = fx.Tensor(a + 2, 128, 64)                                                      # misaligned
    lse = a + 2048
    f = L.flexsp_attn_varlen_fwd
    assert f(h, plan.handle, t, t, t, a, 0, 2, 0, 2, 1, 0.0, t, lse, None) == fx.NO_DEVICE
    assert f(h, plan.handle, bad, t, t, a, 0, 2, 0, 2, 1, 0.0, t, lse, None) == fx.INVALID_ARGUMENT
    assert f(h, plan.handle, t, t, t, a, 0, 4, 0, 2, 1, 0.0, t, lse, None) == fx.PLAN_MISMATCH
    assert f(h, plan.handle, t, t, t, a, 0, 2, 0, 2, 0, 0.0, t, lse, None) == fx.PLAN_MISMATCH
    assert f(h, plan.handle, t, t, t, None, 0, 2, 0, 2, 1, 0.0, t, lse, None) == fx.NO_DEVICE  # cu_seqlens_dev may be NULL: the plan has the lengths
    assert f(h, plan.handle, t, t, t, a, 0, 2, 0, 2, 1, 0.0, t, None, None) == fx.INVALID_ARGUMENT      # lse is required
    assert f(h, None, t, t, t, a, 0, 2, 0, 2, 1, 0.0, t, lse, None) == fx.INVALID_ARGUMENT
    plan.close()


def test_kvshard_plan_lists_every_query_tile_and_validates(host_ctx):
    """Host logic of flexsp_plan_create_kvshard: one item per (sequence with queries, 128-row query
    tile, head), whatever the shard holds; an item names its sequence by index; queues are ordered by
    the key tiles an item can see, most first; bad prefix sums and offsets are refused."""
    import ctypes
    lq, lk, shift = [300, 0, 64, 129], [1000, 50, 0, 129], [700, 0, 0, -64]
    cu_q, cu_k = wl.cu_seqlens(lq), wl.cu_seqlens(lk)
    plan = fx.ShardPlan(host_ctx, cu_q, cu_k, shift, 2, 1, 128, True)
    items, offs = plan.items(fx.PASS_FWD)
    want = sorted((b, t, h) for b, s in enumerate(lq) for t in range((s + 127) // 128) for h in range(2))
    assert sorted(zip(items["seq_start"].tolist(), items["tile"].tolist(), items["head"].tolist())) == want
    assert all(lq[b] == n for b, n in zip(items["seq_start"], items["seq_len"]))
    # the dQ pass lists the same tiles; the dK/dV pass lists every (sequence with shard keys, 64-key tile of
    # the shard, kv head)
    dq_items, _ = plan.items(fx.PASS_BWD_DQ)
    assert sorted(zip(dq_items["seq_start"].tolist(), dq_items["tile"].tolist(), dq_items["head"].tolist())) == want
    dkv_items, _ = plan.items(fx.PASS_BWD_DKV)
    want_k = sorted((b, t, 0) for b, s in enumerate(lk) for t in range((s + 63) // 64))
    assert sorted(zip(dkv_items["seq_start"].tolist(), dkv_items["tile"].tolist(), dkv_items["head"].tolist())) == want_k
    assert all(lk[b] == n for b, n in zip(dkv_items["seq_start"], dkv_items["seq_len"]))
    assert (dkv_items["nparts"] == 1).all()

    def visible_tiles(b, t):
        keys = max(0, min(lk[b], (t + 1) * 128 + shift[b]))
        return (keys + 63) // 64
    for x in range(len(offs) - 1):
        cost = [visible_tiles(int(items["seq_start"][i]), int(items["tile"][i])) for i in range(int(offs[x]), int(offs[x + 1]))]
        assert cost == sorted(cost, reverse=True)
    plan.close()
    L = fx.lib()
    h = ctypes.c_void_p()
    i32 = lambda xs: np.array(xs, dtype=np.int32).ctypes.data_as(ctypes.c_void_p)
    mk = lambda q, k, sh, B=1, D=128: L.flexsp_plan_create_kvshard(host_ctx.handle, i32(q), i32(k), i32(sh), B, 2, 2, D, 1,
                                                                    ctypes.byref(h))
    assert mk([0, 64], [0, 64], [0]) == fx.OK
    L.flexsp_plan_destroy(h)
    assert mk([1, 64], [0, 64], [0]) == fx.INVALID_ARGUMENT          # cu_q[0] != 0
    assert mk([0, 64], [0, -1], [0]) == fx.INVALID_ARGUMENT          # decreasing key prefix sums
    assert mk([0, 64], [0, 64], [2 ** 31 - 1]) == fx.INVALID_ARGUMENT
    assert mk([0, 64], [0, 64], [0], D=96) == fx.UNSUPPORTED
