"""Pins the rounding budget the GPU parity tests assert (tests/rounding_budget.py), on the CPU:
an emulation that applies exactly the roundings the kernels make (P, dS, the stored O and, when
asked, the stored gradients to bf16; everything else fp64) must stay inside the budget against the
fp64 oracle, the budget must be sharper than the stated 2e-2 on ordinary inputs, and a planted
arithmetic mistake of the size of one rounding step per term must fall outside it."""
import numpy as np
import pytest

import oracle
from paper_2412_01523_amd import workloads as wl

import rounding_budget as rb

CASES = [
    # name, lens, Hq, Hkv, D, causal, query multiplier
    ("cfg0", [17, 64, 100, 255], 4, 4, 64, True, 1.0),
    ("gqa", [300, 31, 200], 8, 2, 128, True, 1.0),
    ("noncausal", [17, 64, 100, 130], 2, 2, 128, False, 1.0),
    ("peaky", [400, 129, 64], 2, 2, 128, True, 6.0),
]


def _inputs(lens, Hq, Hkv, D, seed, qmul):
    T = sum(lens)
    q = wl.normal_bf16(seed, wl.TID_Q, (T, Hq, D))
    if qmul != 1.0:
        q = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(q) * np.float32(qmul))
    return (q, wl.normal_bf16(seed, wl.TID_K, (T, Hkv, D)), wl.normal_bf16(seed, wl.TID_V, (T, Hkv, D)),
            wl.normal_bf16(seed, wl.TID_DO, (T, Hq, D)), wl.cu_seqlens(lens))


@pytest.mark.parametrize("name,lens,Hq,Hkv,D,causal,qmul", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("grads_bf16", [False, True])
def test_emulated_roundings_stay_inside_the_budget(name, lens, Hq, Hkv, D, causal, qmul, grads_bf16):
    q, k, v, g, cu = _inputs(lens, Hq, Hkv, D, 611, qmul)
    O, LSE, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, causal)
    sig, mag = rb.budget(q, k, v, g, cu, causal, grads_bf16=grads_bf16)
    em = dict(zip(("O", "dQ", "dK", "dV"), rb.emulate(q, k, v, g, cu, causal, grads_bf16=grads_bf16)))
    for n, ref in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        # the budget's own idea of the exact magnitudes agrees with the oracle
        assert np.allclose(mag[n], np.abs(ref), rtol=1e-9, atol=1e-11), n
        err = np.abs(em[n] - ref)
        tol = rb.tolerance(sig[n], mag[n])
        assert (err <= tol).all(), (n, float((err / tol).max()))
        # 8 standard deviations of an (over-estimated) deviation: the emulation uses less than 5/8 of it
        assert (err / tol).max() < 0.625, (n, float((err / tol).max()))
    if qmul == 1.0:
        # ordinary inputs: for most elements the budget is several times sharper than the stated 2e-2
        for n in ("O", "dQ", "dK", "dV"):
            assert np.median(rb.tolerance(sig[n], mag[n])) < 6e-3, n


def test_a_dropped_delta_or_a_coarser_rounding_falls_outside_the_budget():
    lens, Hq, Hkv, D = [200, 77], 2, 2, 128
    q, k, v, g, cu = _inputs(lens, Hq, Hkv, D, 612, 1.0)
    O, LSE, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    sig, mag = rb.budget(q, k, v, g, cu, True)
    # (a) gradients computed with delta = 0 (a dropped term): far outside
    f = lambda x: wl.bf16_bits_to_f64(x)
    bad_dq = np.zeros_like(dQ)
    for b in range(len(lens)):
        t0, t1 = int(cu[b]), int(cu[b + 1])
        for h in range(Hq):
            P, _, dP, _, _ = rb._dense(f(q)[t0:t1, h], f(k)[t0:t1, h], f(v)[t0:t1, h], f(g)[t0:t1, h], True, D ** -0.5)
            bad_dq[t0:t1, h] = D ** -0.5 * ((P * dP) @ f(k)[t0:t1, h])
    assert (np.abs(bad_dq - dQ) > rb.tolerance(sig["dQ"], mag["dQ"])).mean() > 0.5
    # (b) an error of 2^-5 relative on every element (eight times one bf16 rounding step, still inside
    #     the stated 2e-2 for |x| < 0.6) is caught on most elements of O
    bad_o = O * (1.0 + 2.0 ** -5)
    assert (np.abs(bad_o - O) > rb.tolerance(sig["O"], mag["O"])).mean() > 0.5
