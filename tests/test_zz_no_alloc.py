"""flexsp_attn_varlen_fwd_static (the forward for callers that cannot allocate: it takes no plan and
builds its work queues on the device in a fixed per-GPU array) against flexsp_attn_varlen_fwd on the
same inputs, on calls in a row, each with a smaller batch than the one before, so that whatever a call
left in the shared array must not leak into the next.  Where the plan walks every tile in one piece
the two must agree bit for bit; where the plan cuts long tiles into parts (which the static call never
does) the partial sums are added in another order, and the results must agree to within the rounding
of fp32 sums and of the final bf16 store (far inside the forward's 2e-2 / 5e-3 against the oracle)."""
import sys

import numpy as np
import pytest

from paper_2412_01523_amd import workloads as wl

from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _both(ctx, lens, Hq, Hkv, D, causal, seed, expect_cut=False):
    import torch
    from paper_2412_01523_amd import binding as fx
    T = sum(lens)
    cu = wl.cu_seqlens(lens)
    q = to_dev(wl.normal_bf16(seed, wl.TID_Q, (T, Hq, D)))
    k = to_dev(wl.normal_bf16(seed, wl.TID_K, (T, Hkv, D)))
    v = to_dev(wl.normal_bf16(seed, wl.TID_V, (T, Hkv, D)))
    cud = torch.from_numpy(cu).cuda()
    o_ref = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse_ref = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, causal)
    fx.flexsp_attn_varlen_fwd(ctx, plan, q, k, v, cud, o_ref, lse_ref, causal=causal)
    torch.cuda.synchronize()
    cut = bool((plan.items(fx.PASS_FWD)[0]["nparts"] > 1).any())
    assert cut == expect_cut, "the test batches are chosen to cover both cases"
    plan.close()
    o = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    fx.flexsp_attn_varlen_fwd_static(ctx, q, k, v, cud, o, lse, causal=causal)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # torch's allocator was not used
    torch.cuda.synchronize()
    assert torch.isfinite(lse_ref).all() and torch.isfinite(o_ref.float()).all()
    if not cut:
        assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), f"O differs (lens={lens})"
        assert torch.equal(lse.view(torch.int32), lse_ref.view(torch.int32)), f"LSE differs (lens={lens})"
    else:
        a, b = o.double(), o_ref.double()
        assert float((a - b).abs().max()) <= 2.0 ** -7 * float(b.abs().max()) + 1e-6         # one bf16 step
        assert float((a - b).norm() / b.norm()) <= 1e-3
        assert float((lse - lse_ref).abs().max()) <= 1e-5 * (1 + float(lse_ref.abs().max()))
        assert float((o.view(torch.int16) != o_ref.view(torch.int16)).double().mean()) < 0.2  # most elements still the same bits


def test_static_forward_matches_the_plan_based_forward_twice_in_a_row():
    from paper_2412_01523_amd import binding as fx
    ctx = fx.Context(0)
    big = [1500, 1, 300, 0, 129, 4096, 64, 777, 128, 33] + [50] * 40     # many levels, several thousand items
    small = [200, 64, 1]
    say(f"static forward, first call: {len(big)} sequences, {sum(big)} tokens, 4 heads")
    _both(ctx, big, 4, 2, 128, True, 7301, expect_cut=True)    # the 4 096-token sequence's last tiles are cut by the plan
    say(f"static forward, second call (smaller): lens={small}, 2 heads")
    _both(ctx, small, 2, 2, 128, True, 7302)
    say("static forward, third call: not causal, head dim 64")
    _both(ctx, [70, 129, 1, 300], 4, 2, 64, False, 7303)
    say("static forward, fourth call: several hundred short sequences")
    _both(ctx, [int(x) for x in np.random.default_rng(5).integers(1, 200, size=300)], 2, 2, 128, True, 7304)
    ctx.close()


def test_static_forward_rejects_what_does_not_fit():
    import torch
    from paper_2412_01523_amd import binding as fx
    ctx = fx.Context(0)
    T = 1024
    t = torch.zeros((T, 2, 64), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((2, T), dtype=torch.float32, device="cuda")
    cud = torch.zeros(70000, dtype=torch.int32, device="cuda")       # 69 999 sequences: more items than the array holds
    with pytest.raises(fx.FlexspError) as e:
        fx.flexsp_attn_varlen_fwd_static(ctx, t, t, t, cud, t, lse)
    assert e.value.status == fx.UNSUPPORTED
    # lengths that are not a prefix-sum list inside [0, T]: checked on the device, nothing is computed
    bad = torch.tensor([0, 700, 600, 1024], dtype=torch.int32, device="cuda")
    o = torch.full((T, 2, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    lse.fill_(7.0)
    fx.flexsp_attn_varlen_fwd_static(ctx, t, t, t, bad, o, lse)
    torch.cuda.synchronize()
    assert bool((o == 7.0).all()) and bool((lse == 7.0).all())
    ctx.close()
