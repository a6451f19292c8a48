"""Pins for the CPU fp64 oracle (no GPU).  Each test checks the oracle against something
other than itself: an independent dense formulation, closed forms, finite differences,
invariants that the definition (paper Sec. 2.1.2 Eq. 3; Sec. 2.2.2 sequence packing) fixes,
a hand-derived rational fixture, and a library cross-check.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2412_01523_amd import workloads as wl

RNG = np.random.default_rng(1234)


def rand(*shape):
    return RNG.standard_normal(shape)


def dense_reference(q, k, v, cu, causal, scale):
    """Independent formulation: one T x T score matrix over the whole packed stream with
    -inf outside the block-diagonal(-causal) support, textbook softmax WITHOUT max
    subtraction, then P @ V.  Returns O and LSE."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    seq_id = np.zeros(T, dtype=np.int64)
    for b in range(len(cu) - 1):
        seq_id[cu[b]:cu[b + 1]] = b
    allowed = seq_id[:, None] == seq_id[None, :]
    if causal:
        allowed &= np.arange(T)[None, :] <= np.arange(T)[:, None]
    O = np.zeros((T, Hq, D))
    LSE = np.zeros((Hq, T))
    for h in range(Hq):
        S = scale * (q[:, h, :] @ k[:, h // G, :].T)
        E = np.where(allowed, np.exp(S), 0.0)
        Z = E.sum(axis=1, keepdims=True)
        O[:, h, :] = (E / Z) @ v[:, h // G, :]
        LSE[h] = np.log(Z[:, 0])
    return O, LSE


CASES = [
    # lens, Hq, Hkv, D, causal
    ([5, 1, 9, 3], 2, 2, 4, True),
    ([5, 1, 9, 3], 2, 2, 4, False),
    ([7, 2, 12], 4, 2, 8, True),
    ([6, 4], 6, 2, 3, False),
    ([1, 1, 1], 2, 1, 5, True),
    ([4, 0, 6], 2, 2, 4, True),       # an empty sequence is a no-op
]


@pytest.mark.parametrize("lens,Hq,Hkv,D,causal", CASES)
def test_forward_brute_force_dense(lens, Hq, Hkv, D, causal):
    cu = wl.cu_seqlens(lens)
    T = int(cu[-1])
    q, k, v = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D)
    scale = 0.37
    O, LSE = oracle.attn_fwd(q, k, v, cu, causal, scale)
    Or, Lr = dense_reference(q, k, v, cu, causal, scale)
    assert np.abs(O - Or).max() < 1e-12
    assert np.abs(LSE - Lr).max() < 1e-12


def test_default_scale_is_inverse_sqrt_head_dim():
    cu = wl.cu_seqlens([6, 3])
    q, k, v = rand(9, 2, 16), rand(9, 2, 16), rand(9, 2, 16)
    O, LSE = oracle.attn_fwd(q, k, v, cu, True)
    Or, Lr = dense_reference(q, k, v, cu, True, 1.0 / math.sqrt(16))
    assert np.abs(O - Or).max() < 1e-12 and np.abs(LSE - Lr).max() < 1e-12


def test_bf16_inputs_are_widened_exactly():
    cu = wl.cu_seqlens([11, 6])
    qb, kb, vb = (wl.normal_bf16(7, i, (17, 2, 8)) for i in range(3))
    O1, L1 = oracle.attn_fwd(qb, kb, vb, cu, True)
    O2, L2 = oracle.attn_fwd(wl.bf16_bits_to_f64(qb), wl.bf16_bits_to_f64(kb), wl.bf16_bits_to_f64(vb), cu, True)
    assert np.array_equal(O1, O2) and np.array_equal(L1, L2)
    # widening itself: 0x3FC0 is 1.5, 0xC000 is -2
    assert wl.bf16_bits_to_f64(np.array([0x3FC0, 0xC000], dtype=np.uint16)).tolist() == [1.5, -2.0]


def test_softmax_rows_sum_to_one():
    # V == 1 everywhere makes O_i = sum_j P_ij
    lens = [33, 1, 70]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k = 3 * rand(T, 2, 8), 3 * rand(T, 2, 8)
    v = np.ones((T, 2, 8))
    for causal in (True, False):
        O, _ = oracle.attn_fwd(q, k, v, cu, causal)
        assert np.abs(O - 1.0).max() <= 1e-14 * max(lens)


def test_length_one_sequence_and_first_rows_return_v():
    lens = [1, 5, 1, 8]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v = rand(T, 4, 8), rand(T, 2, 8), rand(T, 2, 8)
    O, LSE = oracle.attn_fwd(q, k, v, cu, True)
    for b in range(len(lens)):
        t0 = cu[b]
        for h in range(4):
            assert np.array_equal(O[t0, h], v[t0, h // 2])      # exactly, P = 1
            s00 = (q[t0, h] @ k[t0, h // 2]) / math.sqrt(8)
            assert abs(LSE[h, t0] - s00) < 1e-14
    # non-causal length-1 sequences too
    O2, _ = oracle.attn_fwd(q, k, v, cu, False)
    assert np.array_equal(O2[0, 1], v[0, 0]) and np.array_equal(O2[6, 3], v[6, 1])


def test_pack_order_permutation_invariance_bitwise():
    lens = [9, 4, 17, 1, 6]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v, g = rand(T, 4, 8), rand(T, 2, 8), rand(T, 2, 8), rand(T, 4, 8)
    base = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    perm = [3, 0, 4, 2, 1]
    idx = np.concatenate([np.arange(cu[b], cu[b + 1]) for b in perm])
    cu2 = wl.cu_seqlens([lens[b] for b in perm])
    out = oracle.attn_fwd_bwd(q[idx], k[idx], v[idx], g[idx], cu2, True)
    O, LSE, dQ, dK, dV = base
    O2, LSE2, dQ2, dK2, dV2 = out
    assert np.array_equal(O[idx], O2) and np.array_equal(LSE[:, idx], LSE2)
    assert np.array_equal(dQ[idx], dQ2) and np.array_equal(dK[idx], dK2) and np.array_equal(dV[idx], dV2)


def test_zero_leakage_across_sequence_boundaries():
    lens = [9, 4, 17, 6]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v, g = rand(T, 4, 8), rand(T, 2, 8), rand(T, 2, 8), rand(T, 4, 8)
    base = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    q2, k2, v2, g2 = q.copy(), k.copy(), v.copy(), g.copy()
    sl = slice(cu[2], cu[3])                    # perturb sequence 2 only
    for a in (q2, k2, v2, g2):
        a[sl] += 10 * RNG.standard_normal(a[sl].shape)
    pert = oracle.attn_fwd_bwd(q2, k2, v2, g2, cu, True)
    other = np.r_[0:cu[2], cu[3]:T]
    for a, b_ in zip(base, pert):
        if a.shape[0] == T:
            assert np.array_equal(a[other], b_[other])
            assert not np.array_equal(a[sl], b_[sl])
        else:                                   # LSE is [Hq, T]
            assert np.array_equal(a[:, other], b_[:, other])
    # and a mutated boundary (wrong cu) must change results: the test can fail
    cu_bad = cu.copy(); cu_bad[2] += 1
    O_bad, _ = oracle.attn_fwd(q, k, v, cu_bad, True)
    assert not np.array_equal(O_bad, base[0])


def test_closed_form_zero_queries_give_prefix_means():
    lens = [6, 11]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v = np.zeros((T, 2, 4)), rand(T, 2, 4), rand(T, 2, 4)
    O, LSE = oracle.attn_fwd(q, k, v, cu, True)
    On, LSEn = oracle.attn_fwd(q, k, v, cu, False)
    for b, s in enumerate(lens):
        t0 = cu[b]
        for i in range(s):
            assert np.allclose(O[t0 + i], v[t0:t0 + i + 1].mean(axis=0), atol=1e-14, rtol=0)
            assert abs(LSE[0, t0 + i] - math.log(i + 1)) < 1e-14
            assert np.allclose(On[t0 + i], v[t0:t0 + s].mean(axis=0), atol=1e-14, rtol=0)
            assert abs(LSEn[1, t0 + i] - math.log(s)) < 1e-14


def test_closed_form_equal_values_and_key_shift_invariance():
    lens = [13, 7]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k = rand(T, 2, 4), rand(T, 2, 4)
    row = rand(2, 4)
    v = np.broadcast_to(row, (T, 2, 4)).copy()
    O, _ = oracle.attn_fwd(q, k, v, cu, True)
    assert np.abs(O - row[None]).max() < 1e-14
    v = rand(T, 2, 4)
    O1, L1 = oracle.attn_fwd(q, k, v, cu, True)
    u = rand(1, 2, 4)
    O2, L2 = oracle.attn_fwd(q, k + u, v, cu, True)
    assert np.abs(O1 - O2).max() < 1e-12
    shift = np.einsum("thd,hd->ht", q, u[0]) / math.sqrt(4)
    assert np.abs((L2 - L1) - shift).max() < 1e-12


def _load_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "eq3_rational_softmax.txt")
    rows = []
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        seq, tok, q, w, v, oc, on = line.split()
        rows.append((seq, int(tok), float(q), float(w), float(v), Fraction(oc), Fraction(on)))
    return rows


def test_golden_rational_softmax_fixture():
    rows = _load_golden()
    lens = [sum(1 for r in rows if r[0] == "A"), sum(1 for r in rows if r[0] == "B")]
    cu = wl.cu_seqlens(lens)
    q = np.array([r[2] for r in rows]).reshape(-1, 1, 1)
    k = np.log(np.array([r[3] for r in rows])).reshape(-1, 1, 1)
    v = np.array([r[4] for r in rows]).reshape(-1, 1, 1)
    Oc, Lc = oracle.attn_fwd(q, k, v, cu, True, 1.0)
    On, _ = oracle.attn_fwd(q, k, v, cu, False, 1.0)
    assert np.abs(Oc[:, 0, 0] - np.array([float(r[5]) for r in rows])).max() < 1e-14
    assert np.abs(On[:, 0, 0] - np.array([float(r[6]) for r in rows])).max() < 1e-14
    assert np.abs(Lc[0] - np.log([1, 10, 8, 2, 8])).max() < 1e-14


# ----------------------------------------------------------------------------- backward
def loss(q, k, v, g, cu, causal, scale):
    O, _ = oracle.attn_fwd(q, k, v, cu, causal, scale)
    return float((O * g).sum())


@pytest.mark.parametrize("lens,Hq,Hkv,D,causal", [
    ([4, 1, 6], 2, 2, 3, True),
    ([5, 3], 4, 2, 2, True),
    ([5, 3], 2, 1, 3, False),
])
def test_backward_matches_central_finite_differences(lens, Hq, Hkv, D, causal):
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    scale = 0.6
    _, _, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, causal, scale)
    eps = 1e-6
    for name, arr, grad in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + eps
            lp = loss(q, k, v, g, cu, causal, scale)
            arr[i] = old - eps
            lm = loss(q, k, v, g, cu, causal, scale)
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        assert np.abs(num - grad).max() < 2e-8 * max(1.0, np.abs(grad).max()), name


def test_backward_closed_forms():
    lens = [1, 9, 1, 5]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    Hq, Hkv, D = 4, 2, 4
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    _, _, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    for b in (0, 2):                       # length-1 sequences
        t = cu[b]
        assert np.array_equal(dQ[t], np.zeros((Hq, D))) and np.array_equal(dK[t], np.zeros((Hkv, D)))
        for kv in range(Hkv):
            assert np.allclose(dV[t, kv], g[t, 2 * kv] + g[t, 2 * kv + 1], atol=1e-15, rtol=0)
    # all V rows equal inside each sequence -> dP constant per row -> dS = 0 -> dQ = dK = 0
    v2 = v.copy()
    for b in range(len(lens)):
        v2[cu[b]:cu[b + 1]] = v2[cu[b]]
    _, _, dQ2, dK2, _ = oracle.attn_fwd_bwd(q, k, v2, g, cu, True)
    assert np.abs(dQ2).max() < 1e-14 and np.abs(dK2).max() < 1e-14
    # all K rows equal -> dQ_i = scale * (sum_j dS_ij) * k = 0 (rows of dS sum to zero)
    k2 = k.copy()
    for b in range(len(lens)):
        k2[cu[b]:cu[b + 1]] = k2[cu[b]]
    _, _, dQ3, _, _ = oracle.attn_fwd_bwd(q, k2, v, g, cu, True)
    assert np.abs(dQ3).max() < 1e-14
    # q == 0, causal: P_ij = 1/(i+1)  ->  dV[j] = sum over the group and over i >= j of dO_i / (i+1)
    _, _, _, _, dV4 = oracle.attn_fwd_bwd(np.zeros_like(q), k, v, g, cu, True)
    for b, s in enumerate(lens):
        t0 = cu[b]
        for j in range(s):
            for kv in range(Hkv):
                want = sum((g[t0 + i, 2 * kv] + g[t0 + i, 2 * kv + 1]) / (i + 1) for i in range(j, s))
                assert np.allclose(dV4[t0 + j, kv], want, atol=1e-14, rtol=0)


def test_backward_sum_identities():
    lens = [12, 7, 20]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    Hq, Hkv, D = 4, 2, 8
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    for causal in (True, False):
        O, _, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, causal)
        for b in range(len(lens)):
            sl = slice(cu[b], cu[b + 1])
            for kv in range(Hkv):
                hs = slice(2 * kv, 2 * kv + 2)
                # sum_j dV_j = sum_i dO_i (rows of P sum to one)
                assert np.abs(dV[sl, kv].sum(0) - g[sl, hs].sum((0, 1))).max() < 1e-12
                # <q, dQ> = <k, dK>  (both equal sum_ij dS_ij S_ij)
                assert abs((q[sl, hs] * dQ[sl, hs]).sum() - (k[sl, kv] * dK[sl, kv]).sum()) < 1e-11


def test_packed_gradients_equal_unpacked_bitwise():
    # paper Sec. 1 / Sec. 2.2.2: gradients over a packed input equal those of the unpacked sequences
    lens = [9, 4, 17]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    q, k, v, g = rand(T, 4, 8), rand(T, 2, 8), rand(T, 2, 8), rand(T, 4, 8)
    packed = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    for b, s in enumerate(lens):
        sl = slice(cu[b], cu[b + 1])
        alone = oracle.attn_fwd_bwd(q[sl], k[sl], v[sl], g[sl], wl.cu_seqlens([s]), True)
        for a, p in zip(alone, packed):
            assert np.array_equal(a, p[sl] if p.shape[0] == T else p[:, sl])


def test_gqa_equals_mha_with_repeated_kv_heads():
    lens = [10, 6]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    Hq, Hkv, D = 6, 2, 4
    G = Hq // Hkv
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    O, L, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, True)
    kr, vr = np.repeat(k, G, axis=1), np.repeat(v, G, axis=1)
    O2, L2, dQ2, dK2, dV2 = oracle.attn_fwd_bwd(q, kr, vr, g, cu, True)
    assert np.abs(O - O2).max() < 1e-14 and np.abs(L - L2).max() < 1e-14 and np.abs(dQ - dQ2).max() < 1e-14
    assert np.abs(dK - dK2.reshape(T, Hkv, G, D).sum(2)).max() < 1e-13
    assert np.abs(dV - dV2.reshape(T, Hkv, G, D).sum(2)).max() < 1e-13


def test_library_cross_check_torch_autograd():
    torch = pytest.importorskip("torch")
    lens = [14, 3, 9]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    Hq, Hkv, D = 4, 2, 8
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    for causal in (True, False):
        O, _, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, g, cu, causal)
        tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
        outs = []
        for b, s in enumerate(lens):
            sl = slice(int(cu[b]), int(cu[b + 1]))
            qq = tq[sl].transpose(0, 1)                                   # [Hq, s, D]
            kk = tk[sl].transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
            vv = tv[sl].transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
            S = qq @ kk.transpose(1, 2) / math.sqrt(D)
            if causal:
                S = S.masked_fill(torch.ones(s, s, dtype=torch.bool).triu(1), float("-inf"))
            outs.append((torch.softmax(S, -1) @ vv).transpose(0, 1))
        To = torch.cat(outs, 0)
        (To * torch.tensor(g)).sum().backward()
        assert np.abs(O - To.detach().numpy()).max() < 1e-12
        assert np.abs(dQ - tq.grad.numpy()).max() < 1e-12
        assert np.abs(dK - tk.grad.numpy()).max() < 1e-12
        assert np.abs(dV - tv.grad.numpy()).max() < 1e-12


# ------------------------------------------------------------------- sampled-row entry points
@pytest.mark.parametrize("causal", [True, False])
def test_sampled_rows_match_dense_reference_and_finite_differences(causal):
    lens = [7, 1, 12, 5]
    cu = wl.cu_seqlens(lens)
    T = sum(lens)
    Hq, Hkv, D = 4, 2, 4
    q, k, v, g = rand(T, Hq, D), rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
    scale = 0.45
    Or, Lr = dense_reference(q, k, v, cu, causal, scale)
    tok = np.array([0, 6, 7, 8, 19, 20, 24, 13])
    head = np.array([0, 3, 1, 2, 3, 0, 2, 1])
    O, L, dQ = oracle.rows(q, k, v, g, cu, tok, head, causal, scale)
    assert np.abs(O - Or[tok, head]).max() < 1e-12 and np.abs(L - Lr[head, tok]).max() < 1e-12
    # dQ rows against finite differences of the (dense-reference) loss
    eps = 1e-6
    for n in range(len(tok)):
        for d in range(D):
            old = q[tok[n], head[n], d]
            q[tok[n], head[n], d] = old + eps
            lp = (dense_reference(q, k, v, cu, causal, scale)[0] * g).sum()
            q[tok[n], head[n], d] = old - eps
            lm = (dense_reference(q, k, v, cu, causal, scale)[0] * g).sum()
            q[tok[n], head[n], d] = old
            assert abs((lp - lm) / (2 * eps) - dQ[n, d]) < 2e-8
    # dK / dV rows against finite differences too
    tasks = [(0, 0, [0, 3, 6]), (2, 1, [2, 11]), (1, 1, [0]), (3, 0, [4])]
    dKr, dVr = oracle.dkv_rows(q, k, v, g, cu, tasks, causal, scale)
    r = 0
    for (b, kv, js) in tasks:
        for j in js:
            t = cu[b] + j
            for arr, got in ((k, dKr), (v, dVr)):
                for d in range(D):
                    old = arr[t, kv, d]
                    arr[t, kv, d] = old + eps
                    lp = (dense_reference(q, k, v, cu, causal, scale)[0] * g).sum()
                    arr[t, kv, d] = old - eps
                    lm = (dense_reference(q, k, v, cu, causal, scale)[0] * g).sum()
                    arr[t, kv, d] = old
                    assert abs((lp - lm) / (2 * eps) - got[r, d]) < 2e-8
            r += 1


def test_bad_arguments_are_rejected():
    q, k, v = rand(4, 2, 2), rand(4, 2, 2), rand(4, 2, 2)
    with pytest.raises(ValueError):
        oracle.attn_fwd(q, k, v, np.array([1, 4], dtype=np.int32))      # cu[0] != 0
    with pytest.raises(ValueError):
        oracle.attn_fwd(q, k, v, np.array([0, 5, 4], dtype=np.int32))   # decreasing
    with pytest.raises(ValueError):
        oracle.attn_fwd(rand(4, 3, 2), k, v, np.array([0, 4], dtype=np.int32))  # Hq % Hkv


# ------------------------------------------------------------------------------ pack / unpack
@pytest.mark.parametrize("T,H,D,P,dtype", [
    (5, 4, 3, 2, np.uint16), (7, 6, 8, 3, np.uint16), (4, 8, 2, 8, np.uint8),
    (3, 4, 4, 1, np.uint32), (0, 4, 4, 2, np.uint16), (6, 2, 5, 2, np.float64),
])
def test_pack_unpack_index_formula(T, H, D, P, dtype):
    n = T * H * D
    x = (np.arange(n) * 7 + 3).astype(dtype).reshape(T, H, D)      # value encodes (t, h, d)
    Hp = H // P
    y = oracle.pack(x, P)
    assert y.shape == (P, T, Hp, D)
    for r in range(P):
        # slab r is the r-th contiguous head group made contiguous
        assert np.array_equal(y[r], x[:, r * Hp:(r + 1) * Hp, :])
    assert np.array_equal(oracle.unpack(y), x)
    if P == 1:
        assert np.array_equal(y[0], x)


def test_pack_elementwise_loops():
    T, H, D, P = 3, 4, 2, 2
    x = wl.index_pattern_u16((T, H, D))
    y = oracle.pack(x, P)
    for r in range(P):
        for t in range(T):
            for h in range(H // P):
                for d in range(D):
                    assert y[r, t, h, d] == x[t, r * (H // P) + h, d]
    with pytest.raises(ValueError):
        oracle.pack(np.zeros((2, 3, 2), dtype=np.uint16), 2)


# ------------------------------------------------------------------------------ workloads
def test_workload_recipes():
    for cfg in wl.CONFIGS:
        L = wl.lengths(cfg)
        assert sum(L) == cfg.tokens and min(L) >= 1
        assert wl.lengths(cfg) == L                                  # seeded
    assert wl.lengths(wl.CONFIGS[0]) == [17, 64, 100, 255]
    L1 = wl.lengths(wl.CONFIGS[1]); assert all(128 <= s <= 32768 for s in L1[:-1])
    L2 = wl.lengths(wl.CONFIGS[2]); assert all(256 <= s <= 65536 for s in L2[:-1])
    L4 = wl.lengths(wl.CONFIGS[4])
    assert sorted(L4)[-3:] == [32768, 65536, 65536] and all(64 <= s <= 1024 for s in sorted(L4)[:-4])
    assert wl.causal_pairs([17, 64, 100, 255]) == 39923
    assert sum(wl.attn_flops([17, 64, 100, 255], 4, 64)) == 14 * 64 * 4 * 39923
    # bf16 rounding is round-to-nearest-even
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38], dtype=np.float32)
    assert wl.f32_to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x7F62]
    a = wl.normal_bf16(5, 1, (1000,)); b = wl.normal_bf16(5, 1, (1000,))
    assert np.array_equal(a, b) and abs(wl.bf16_bits_to_f32(a).std() - 1) < 0.1


# ----------------------------------------------------------------------------- key shards (context parallelism)
def _shard_inputs(lens, Hq, Hkv, D, seed):
    T = sum(lens)
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)), rng.standard_normal((T, Hkv, D)))


def _split(x, cu, lo, hi):
    """rows lo[b] .. hi[b]-1 of every sequence, concatenated; and their prefix sums"""
    parts = [x[int(cu[b]) + lo[b]: int(cu[b]) + hi[b]] for b in range(len(lo))]
    n = [hi[b] - lo[b] for b in range(len(lo))]
    return np.concatenate(parts) if parts else x[:0], wl.cu_seqlens(n)


@pytest.mark.parametrize("causal", [True, False])
def test_kvshard_parts_merge_into_the_full_attention(causal):
    """Attention over ALL keys (the function pinned above) = the attentions over two or three key
    shards merged by their log-sum-exps; also for a chunk of the queries only, as a device of a
    context-parallel group holds them.  Pins attn_fwd_kvshard and lse_merge together against
    attn_fwd: a wrong mask offset, a wrong weight or a lost normaliser breaks the identity."""
    lens, Hq, Hkv, D = [9, 1, 40, 17, 64], 4, 2, 8
    cu = wl.cu_seqlens(lens)
    q, k, v = _shard_inputs(lens, Hq, Hkv, D, 31)
    O, LSE = oracle.attn_fwd(q, k, v, cu, causal)
    rng = np.random.default_rng(32)
    for trial in range(4):
        c1 = [int(rng.integers(0, s + 1)) for s in lens]                  # first cut: may be 0 or s (an empty shard)
        c2 = [int(rng.integers(c, s + 1)) for c, s in zip(c1, lens)]
        a0 = [int(rng.integers(0, s)) for s in lens]                       # the query chunk starts here ...
        a1 = [int(rng.integers(a + 1, s + 1)) for a, s in zip(a0, lens)]   # ... and ends here
        if trial == 0:
            a0, a1 = [0] * len(lens), list(lens)                           # all queries
        qs, cu_q = _split(q, cu, a0, a1)
        parts = []
        for lo, hi in (([0] * len(lens), c1), (c1, c2), (c2, list(lens))):
            ks, cu_k = _split(k, cu, lo, hi)
            vs, _ = _split(v, cu, lo, hi)
            shift = [a - l for a, l in zip(a0, lo)]                        # first query position - first key position
            parts.append(oracle.attn_fwd_kvshard(qs, ks, vs, cu_q, cu_k, shift, causal))
        o12, l12 = oracle.lse_merge(parts[0][0], parts[0][1], parts[1][0], parts[1][1])
        o, l = oracle.lse_merge(o12, l12, parts[2][0], parts[2][1])
        o_alt, l_alt = oracle.lse_merge(parts[0][0], parts[0][1],
                                        *oracle.lse_merge(parts[1][0], parts[1][1], parts[2][0], parts[2][1]))
        Oq, _ = _split(O, cu, a0, a1)
        Lq = np.concatenate([LSE[:, int(cu[b]) + a0[b]: int(cu[b]) + a1[b]] for b in range(len(lens))], axis=1)
        assert np.abs(o - Oq).max() < 1e-12 and np.abs(l - Lq).max() < 1e-12
        assert np.abs(o_alt - Oq).max() < 1e-12 and np.abs(l_alt - Lq).max() < 1e-12     # merge order is free


def test_kvshard_dense_brute_force_and_closed_forms():
    """(1) Textbook masked softmax over a dense score matrix with the mask j <= i + shift written out.
    (2) q = 0: every visible key weighs the same, so O = mean of the visible V rows, LSE = ln(count).
    (3) Rows that see no key: O = 0, LSE = -inf, and merging them with anything returns the other part."""
    sq, sk, Hq, Hkv, D = 11, 14, 2, 1, 4
    rng = np.random.default_rng(41)
    q, k, v = rng.standard_normal((sq, Hq, D)), rng.standard_normal((sk, Hkv, D)), rng.standard_normal((sk, Hkv, D))
    cu_q, cu_k = wl.cu_seqlens([sq]), wl.cu_seqlens([sk])
    for shift in (-5, -1, 0, 3, 20):
        O, L = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, [shift], True)
        for h in range(Hq):
            S = (q[:, h] @ k[:, 0].T) / np.sqrt(D)
            vis = np.arange(sk)[None, :] <= np.arange(sq)[:, None] + shift
            E = np.where(vis, np.exp(S), 0.0)
            Z = E.sum(1)
            ref = np.where(Z[:, None] > 0, (E @ v[:, 0]) / np.where(Z > 0, Z, 1.0)[:, None], 0.0)
            assert np.abs(O[:, h] - ref).max() < 1e-12
            assert np.abs(L[h][Z > 0] - np.log(Z[Z > 0])).max(initial=0.0) < 1e-12
            assert (np.isneginf(L[h]) == (Z == 0)).all() and (O[:, h][Z == 0] == 0).all()
        O0, L0 = oracle.attn_fwd_kvshard(np.zeros_like(q), k, v, cu_q, cu_k, [shift], True)
        for i in range(sq):
            n = min(max(i + shift + 1, 0), sk)
            if n > 0:
                assert np.abs(O0[i, 0] - v[:n, 0].mean(0)).max() < 1e-13 and abs(L0[0, i] - np.log(n)) < 1e-13
    # not causal: the shift is ignored, every key of the shard counts
    On, Ln = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, [-100], False)
    Of, Lf = oracle.attn_fwd_kvshard(q, k, v, cu_q, cu_k, [100], True)
    assert np.array_equal(On, Of) and np.array_equal(Ln, Lf)
    # a part without keys is the neutral element of the merge
    Oe, Le = oracle.attn_fwd_kvshard(q, k[:0], v[:0], cu_q, wl.cu_seqlens([0]), [0], True)
    assert not Oe.any() and np.isneginf(Le).all()
    Om, Lm = oracle.lse_merge(Oe, Le, On, Ln)
    assert np.array_equal(Om, On) and np.array_equal(Lm, Ln)
    Om, Lm = oracle.lse_merge(Oe, Le, Oe, Le)
    assert not Om.any() and np.isneginf(Lm).all()


@pytest.mark.parametrize("causal", [True, False])
def test_kvshard_backward_parts_add_up_to_the_full_backward(causal):
    """The complete backward (pinned above by finite differences) = the shard backwards of a partition of
    the keys: the dQ parts add up to dQ, every shard's dK / dV are the complete ones of its keys; also
    for a chunk of the queries only (then dK / dV of the chunks add up).  Pins attn_bwd_kvshard: a
    wrong mask offset, a dropped delta, a transposed product or a missing scale breaks the identity."""
    lens, Hq, Hkv, D = [9, 1, 40, 17, 64], 4, 2, 8
    cu = wl.cu_seqlens(lens)
    q, k, v = _shard_inputs(lens, Hq, Hkv, D, 51)
    dO = np.random.default_rng(52).standard_normal(q.shape)
    O, LSE, dQ, dK, dV = oracle.attn_fwd_bwd(q, k, v, dO, cu, causal)
    delta = np.einsum("thd,thd->ht", dO, O)
    rng = np.random.default_rng(53)
    B = len(lens)
    for trial in range(3):
        c1 = [int(rng.integers(0, s + 1)) for s in lens]
        c2 = [int(rng.integers(c, s + 1)) for c, s in zip(c1, lens)]
        a = [int(rng.integers(0, s + 1)) for s in lens]                    # query chunks: rows 0 .. a-1 and a .. s-1
        dq_sum = np.zeros_like(dQ)
        for klo, khi in (([0] * B, c1), (c1, c2), (c2, list(lens))):
            ks, cu_k = _split(k, cu, klo, khi)
            vs, _ = _split(v, cu, klo, khi)
            dk_sum, dv_sum = np.zeros_like(ks), np.zeros_like(vs)
            for qlo, qhi in (([0] * B, a), (a, list(lens))):
                qs, cu_q = _split(q, cu, qlo, qhi)
                gs, _ = _split(dO, cu, qlo, qhi)
                ls = np.concatenate([LSE[:, int(cu[b]) + qlo[b]: int(cu[b]) + qhi[b]] for b in range(B)], axis=1)
                ds = np.concatenate([delta[:, int(cu[b]) + qlo[b]: int(cu[b]) + qhi[b]] for b in range(B)], axis=1)
                shift = [x - l for x, l in zip(qlo, klo)]
                dq_p, dk_p, dv_p = oracle.attn_bwd_kvshard(qs, ks, vs, gs, ls, ds, cu_q, cu_k, shift, causal)
                for b in range(B):
                    dq_sum[int(cu[b]) + qlo[b]: int(cu[b]) + qhi[b]] += dq_p[int(cu_q[b]): int(cu_q[b + 1])]
                dk_sum += dk_p
                dv_sum += dv_p
            assert np.abs(dk_sum - _split(dK, cu, klo, khi)[0]).max(initial=0.0) < 1e-11
            assert np.abs(dv_sum - _split(dV, cu, klo, khi)[0]).max(initial=0.0) < 1e-11
        assert np.abs(dq_sum - dQ).max() < 1e-11


def test_kvshard_backward_closed_forms():
    """(1) One query row that sees exactly one key with the complete softmax's statistics: P = 1, delta = dP,
    so dS = 0: dQ = dK = 0 and dV = dO.  (2) Keys no row sees get dK = dV = 0; rows that see no key of the
    shard get a zero dQ part.  (3) A row whose log-sum-exp is -inf (no key anywhere) contributes nothing."""
    D = 4
    rng = np.random.default_rng(61)
    q, k, v, g = (rng.standard_normal((1, 1, D)) for _ in range(4))
    s = float(q[0, 0] @ k[0, 0]) / np.sqrt(D)
    dq, dk, dv = oracle.attn_bwd_kvshard(q, k, v, g, [[s]], [[float(g[0, 0] @ v[0, 0])]], [0, 1], [0, 1], [0], True)
    assert np.abs(dq).max() < 1e-15 and np.abs(dk).max() < 1e-15 and np.abs(dv - g).max() < 1e-15
    sq, sk = 6, 9
    q, g = rng.standard_normal((sq, 1, D)), rng.standard_normal((sq, 1, D))
    k, v = rng.standard_normal((sk, 1, D)), rng.standard_normal((sk, 1, D))
    lse, delta = rng.standard_normal((1, sq)) + 3.0, rng.standard_normal((1, sq))
    dq, dk, dv = oracle.attn_bwd_kvshard(q, k, v, g, lse, delta, [0, sq], [0, sk], [-2], True)   # key j visible iff j <= i - 2
    assert not dq[:2].any() and dq[2:].any()            # rows 0, 1 see nothing
    assert not dk[4:].any() and not dv[4:].any()        # keys 4 .. 8 are seen by no row (i - 2 <= 3)
    assert dk[:4].any() and dv[:4].any()
    lse[0, 3] = -np.inf
    dq2, dk2, dv2 = oracle.attn_bwd_kvshard(q, k, v, g, lse, delta, [0, sq], [0, sk], [-2], True)
    assert not dq2[3].any() and np.isfinite(dk2).all() and np.isfinite(dv2).all()
    others = [i for i in range(sq) if i != 3]
    dq3, dk3, dv3 = oracle.attn_bwd_kvshard(q[others], k, v, g[others], lse[:, others], delta[:, others],
                                            [0, sq - 1], [0, sk], [-2], False)
    dq4, dk4, dv4 = oracle.attn_bwd_kvshard(q, k, v, g, lse, delta, [0, sq], [0, sk], [-2], False)
    assert np.abs(dk3 - dk4).max() < 1e-13 and np.abs(dv3 - dv4).max() < 1e-13
