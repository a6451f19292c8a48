"""GPU-side invariants of the packed-stream attention (paper Sec. 2.2.2: sequences packed into one
stream must not see each other), checked on the HIP path's own outputs, bit for bit (the kernels
are deterministic and use no floating-point atomics), plus guard regions around every output."""
import sys

import numpy as np
import pytest

from paper_2412_01523_amd import workloads as wl

from gpu_util import to_bits, to_dev

pytestmark = pytest.mark.gpu

GUARD = 4096          # bytes either side of every output buffer
GUARD_BYTE = 0xA5


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    from paper_2412_01523_amd import binding as fx
    c = fx.Context(0)
    yield c
    c.close()


class Guarded:
    """A tensor carved out of a larger byte buffer with GUARD bytes of a known pattern either side."""

    def __init__(self, shape, dtype):
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        pad = (-n) % 256
        self.raw = torch.full((GUARD + n + pad + GUARD,), GUARD_BYTE, dtype=torch.uint8, device="cuda")
        self.n = n
        self.t = self.raw[GUARD:GUARD + n].view(dtype).view(*shape)
        assert self.t.data_ptr() % 16 == 0

    def guards_intact(self):
        return bool((self.raw[:GUARD] == GUARD_BYTE).all()) and bool((self.raw[GUARD + self.n:] == GUARD_BYTE).all())


def _run(ctx, q, k, v, g, cu, causal=True, grad_f32=False, guarded=False):
    """HIP path on host bit patterns -> dict of host arrays (bf16 outputs as bit patterns)."""
    import torch
    from paper_2412_01523_amd import binding as fx
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    plan = fx.Plan(ctx, cu, Hq, Hkv, D, causal)
    qd, kd, vd, gd = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    cud = torch.from_numpy(np.ascontiguousarray(cu, dtype=np.int32)).cuda()
    gdt = torch.float32 if grad_f32 else torch.bfloat16
    bufs = {"O": Guarded((T, Hq, D), torch.bfloat16), "LSE": Guarded((Hq, T), torch.float32),
            "dQ": Guarded((T, Hq, D), gdt), "dK": Guarded((T, Hkv, D), gdt), "dV": Guarded((T, Hkv, D), gdt)}
    fx.flexsp_attn_varlen_fwd(ctx, plan, qd, kd, vd, cud, bufs["O"].t, bufs["LSE"].t, causal=causal)
    fx.flexsp_attn_varlen_bwd(ctx, plan, qd, kd, vd, bufs["O"].t, gd, bufs["LSE"].t, cud, bufs["dQ"].t,
                              bufs["dK"].t, bufs["dV"].t, causal=causal)
    torch.cuda.synchronize()
    plan.close()
    if guarded:
        for name, b in bufs.items():
            assert b.guards_intact(), f"{name}: bytes outside the tensor were written"
    out = {}
    for name, b in bufs.items():
        out[name] = to_bits(b.t) if b.t.dtype == torch.bfloat16 else b.t.cpu().numpy().copy()
    return out


def _inputs(lens, Hq, Hkv, D, seed):
    T = sum(lens)
    return (wl.normal_bf16(seed, wl.TID_Q, (T, Hq, D)), wl.normal_bf16(seed, wl.TID_K, (T, Hkv, D)),
            wl.normal_bf16(seed, wl.TID_V, (T, Hkv, D)), wl.normal_bf16(seed, wl.TID_DO, (T, Hq, D)))


CASES = [
    # lens (ragged tiles, one-token and empty sequences, one spanning many tiles), Hq, Hkv, D, causal
    ([130, 1, 700, 64, 0, 257, 33, 1500, 5], 4, 2, 128, True),
    ([255, 17, 100, 64, 900], 2, 2, 64, True),
    ([130, 300, 64, 77], 2, 1, 128, False),
]


@pytest.mark.parametrize("lens,Hq,Hkv,D,causal", CASES, ids=["gqa-d128", "mha-d64", "noncausal"])
def test_perturbing_one_sequence_leaves_the_others_bit_identical(ctx, lens, Hq, Hkv, D, causal):
    """Zero leakage across sequence boundaries: new data in ONE sequence (its q, k, v and dO rows)
    must not change a single bit of any other sequence's O, LSE, dQ, dK, dV, and must change its own."""
    cu = wl.cu_seqlens(lens)
    q, k, v, g = _inputs(lens, Hq, Hkv, D, 9101)
    base = _run(ctx, q, k, v, g, cu, causal, guarded=True)
    for victim in (2, len(lens) - 1):
        sl = slice(int(cu[victim]), int(cu[victim + 1]))
        say(f"perturbing sequence {victim} (tokens {sl.start}..{sl.stop - 1}) of lens={lens}")
        q2, k2, v2, g2 = (x.copy() for x in (q, k, v, g))
        other = _inputs(lens, Hq, Hkv, D, 9102 + victim)
        for dst, src in zip((q2, k2, v2, g2), other):
            dst[sl] = src[sl]
        out = _run(ctx, q2, k2, v2, g2, cu, causal)
        keep = np.ones(sum(lens), dtype=bool)
        keep[sl] = False
        for name in ("O", "dQ", "dK", "dV"):
            assert np.array_equal(out[name][keep], base[name][keep]), f"{name}: another sequence changed"
            assert not np.array_equal(out[name][sl], base[name][sl]), f"{name}: the perturbed sequence did not change"
        assert np.array_equal(out["LSE"][:, keep], base["LSE"][:, keep]), "LSE: another sequence changed"


@pytest.mark.parametrize("lens,Hq,Hkv,D,causal", CASES, ids=["gqa-d128", "mha-d64", "noncausal"])
def test_permuting_the_pack_order_permutes_the_outputs(ctx, lens, Hq, Hkv, D, causal):
    """The same sequences packed in another order (other start offsets, other queue positions):
    every sequence's outputs must be the same bits, just moved."""
    cu = wl.cu_seqlens(lens)
    q, k, v, g = _inputs(lens, Hq, Hkv, D, 9201)
    base = _run(ctx, q, k, v, g, cu, causal)
    rng = np.random.default_rng(5)
    for rep in range(2):
        perm = rng.permutation(len(lens))
        say(f"pack order {perm.tolist()} of lens={lens}")
        idx = np.concatenate([np.arange(cu[b], cu[b + 1]) for b in perm]).astype(np.int64)
        lens_p = [lens[b] for b in perm]
        out = _run(ctx, q[idx], k[idx], v[idx], g[idx], wl.cu_seqlens(lens_p), causal, guarded=True)
        for name in ("O", "dQ", "dK", "dV"):
            assert np.array_equal(out[name], base[name][idx]), name
        assert np.array_equal(out["LSE"], base["LSE"][:, idx]), "LSE"


def test_guard_regions_survive_fp32_gradients_and_ragged_tails(ctx):
    """Every output inside a larger buffer with 4 KiB of a known pattern either side: the kernels'
    row clamps and partial tiles must never write past the tensors (fp32 and bf16 gradient stores,
    head dims 64 and 128, lengths that end one row into a tile)."""
    for lens, Hq, Hkv, D in (([1, 65, 129, 257, 31], 2, 1, 128), ([63, 64, 1, 193], 3, 3, 64)):
        cu = wl.cu_seqlens(lens)
        q, k, v, g = _inputs(lens, Hq, Hkv, D, 9301)
        for grad_f32 in (False, True):
            say(f"guards: lens={lens} D={D} grad_f32={grad_f32}")
            _run(ctx, q, k, v, g, cu, True, grad_f32=grad_f32, guarded=True)


def test_guard_regions_around_the_permute(ctx):
    import torch
    from paper_2412_01523_amd import binding as fx
    for T, H, D, P, dt in ((1000, 32, 128, 8, torch.int16), (129, 3, 7, 3, torch.int16), (65, 2, 3, 2, torch.uint8)):
        src = Guarded((T, H, D), dt)
        src.t.copy_(torch.randint(0, 100, (T, H, D), device="cuda").to(dt))
        dst = Guarded((P, T, H // P, D), dt)
        back = Guarded((T, H, D), dt)
        fx.flexsp_pack(ctx, src.t, dst.t, P)
        fx.flexsp_unpack(ctx, dst.t, back.t)
        torch.cuda.synchronize()
        assert dst.guards_intact() and back.guards_intact() and src.guards_intact()
        assert torch.equal(back.t, src.t)
