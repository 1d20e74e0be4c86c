"""Pins for the oracle's attention forward and backward.

Each check is independent of the oracle's own row-by-row code: a dense
masked-matrix computation written here, closed forms, invariants, finite
differences, or a library routine (PyTorch CPU, fp64) on a single example.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_09105_amd import workloads as wl


def _rand(lengths_rows, hq, hkv, d, seed):
    w = wl.make_custom(lengths_rows, hq, hkv, d, "f32", seed)
    seg = oracle.pack(w.position_ids)
    f = lambda a: a.astype(np.float64)
    return f(w.q), f(w.k), f(w.v), f(w.do), seg


def _dense_mask(seg_id):
    N = len(seg_id)
    i = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    return (seg_id[:, None] == seg_id[None, :]) & (j <= i)


def _dense_fwd(q, k, v, seg_id, scale):
    """softmax(S + log M) V with the full N x N score matrix and an explicit
    block-diagonal causal mask M; numpy, one head at a time."""
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    M = _dense_mask(seg_id)
    O = np.zeros_like(q)
    LSE = np.zeros((Hq, N))
    Ps = []
    for h in range(Hq):
        S = scale * q[:, h, :] @ k[:, h // G, :].T
        S = np.where(M, S, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        Z = E.sum(axis=1, keepdims=True)
        P = E / Z
        O[:, h, :] = P @ v[:, h // G, :]
        LSE[h] = S.max(axis=1) + np.log(Z[:, 0])
        Ps.append(P)
    return O, LSE, Ps


CASES = [
    ([[3, 5, 1, 7]], 2, 2, 16),          # config-1 shape
    ([[4, 8, 5, 11]], 4, 2, 8),          # the paper's worked-example lengths, GQA
    ([[1, 1, 6], [5, 2, 1]], 6, 2, 4),   # two rows, G = 3
    ([[13]], 3, 1, 5),                   # one example, MQA
]


@pytest.mark.parametrize("lengths,hq,hkv,d", CASES)
def test_fwd_matches_dense_masked_attention(lengths, hq, hkv, d):
    q, k, v, do, seg = _rand(lengths, hq, hkv, d, seed=11)
    scale = 1.0 / np.sqrt(d)
    O, LSE = oracle.fwd(q, k, v, seg["cu_seqlens"])
    O2, LSE2, _ = _dense_fwd(q, k, v, seg["seg_id"], scale)
    np.testing.assert_allclose(O, O2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(LSE, LSE2, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("lengths,hq,hkv,d", CASES)
def test_bwd_matches_autograd_of_dense_masked_attention(lengths, hq, hkv, d):
    # library pin: PyTorch CPU autograd (fp64) through a dense masked softmax
    q, k, v, do, seg = _rand(lengths, hq, hkv, d, seed=12)
    G = hq // hkv
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    M = torch.tensor(_dense_mask(seg["seg_id"]))
    kk = tk.repeat_interleave(G, dim=1)
    vv = tv.repeat_interleave(G, dim=1)
    S = torch.einsum("ihc,jhc->hij", tq, kk) / np.sqrt(d)
    S = S.masked_fill(~M[None], float("-inf"))
    O = torch.einsum("hij,jhc->ihc", torch.softmax(S, dim=-1), vv)
    (O * torch.tensor(do)).sum().backward()
    dQ, dK, dV = oracle.bwd(do, q, k, v, seg["cu_seqlens"])
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_single_example_is_library_causal_sdpa():
    # one example, MHA: reduces to the textbook routine
    q, k, v, do, seg = _rand([[29]], 3, 3, 16, seed=5)
    O, _ = oracle.fwd(q, k, v, seg["cu_seqlens"])
    tq, tk, tv = (torch.tensor(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(O, ref[0].permute(1, 0, 2).numpy(), rtol=1e-11, atol=1e-12)


def test_explicit_scale_is_used():
    q, k, v, do, seg = _rand([[6, 3]], 2, 1, 8, seed=6)
    O, LSE = oracle.fwd(q, k, v, seg["cu_seqlens"], scale=0.37)
    O2, LSE2, _ = _dense_fwd(q, k, v, seg["seg_id"], 0.37)
    np.testing.assert_allclose(O, O2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(LSE, LSE2, rtol=1e-12, atol=1e-13)
    dQ, dK, dV = oracle.bwd(do, q, k, v, seg["cu_seqlens"], scale=0.37)
    eps = 1e-6
    qp, qm = q.copy(), q.copy()
    qp[4, 1, 2] += eps
    qm[4, 1, 2] -= eps
    fd = ((oracle.fwd(qp, k, v, seg["cu_seqlens"], scale=0.37)[0] * do).sum()
          - (oracle.fwd(qm, k, v, seg["cu_seqlens"], scale=0.37)[0] * do).sum()) / (2 * eps)
    assert abs(fd - dQ[4, 1, 2]) < 1e-7 * max(1.0, abs(fd))


def test_unpack_invariant():
    # packed result == each example run alone
    lengths = [[3, 5, 1, 7], [9, 2, 4, 1]]
    q, k, v, do, seg = _rand(lengths, 4, 2, 8, seed=21)
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    for s in range(seg["n"]):
        a, b = cu[s], cu[s + 1]
        one = np.array([0, b - a], dtype=np.int32)
        O1, LSE1 = oracle.fwd(q[a:b], k[a:b], v[a:b], one)
        dQ1, dK1, dV1 = oracle.bwd(do[a:b], q[a:b], k[a:b], v[a:b], one)
        assert np.array_equal(O[a:b], O1) and np.array_equal(LSE[:, a:b], LSE1)
        assert np.array_equal(dQ[a:b], dQ1) and np.array_equal(dK[a:b], dK1) and np.array_equal(dV[a:b], dV1)


def test_perturbing_other_examples_changes_nothing():
    lengths = [[4, 6, 3]]
    q, k, v, do, seg = _rand(lengths, 2, 2, 8, seed=22)
    cu = seg["cu_seqlens"]
    base_f = oracle.fwd(q, k, v, cu)
    base_b = oracle.bwd(do, q, k, v, cu)
    rng = np.random.default_rng(0)
    a, b = cu[1], cu[2]     # keep example 1, scramble examples 0 and 2
    q2, k2, v2, do2 = (x.copy() for x in (q, k, v, do))
    for x in (q2, k2, v2, do2):
        x[:a] = rng.standard_normal(x[:a].shape)
        x[b:] = rng.standard_normal(x[b:].shape)
    f2 = oracle.fwd(q2, k2, v2, cu)
    b2 = oracle.bwd(do2, q2, k2, v2, cu)
    assert np.array_equal(base_f[0][a:b], f2[0][a:b]) and np.array_equal(base_f[1][:, a:b], f2[1][:, a:b])
    for x, y in zip(base_b, b2):
        assert np.array_equal(x[a:b], y[a:b])
    # and the scrambled examples did change
    assert not np.array_equal(base_f[0][:a], f2[0][:a])


def test_length_one_example_closed_form():
    # O = V, LSE = scale * q.k, dQ = dK = 0, dV = sum of dO over the heads of the group
    lengths = [[3, 1, 4]]
    q, k, v, do, seg = _rand(lengths, 4, 2, 8, seed=23)
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    t = 3
    for h in range(4):
        np.testing.assert_array_equal(O[t, h], v[t, h // 2])
        assert abs(LSE[h, t] - (q[t, h] @ k[t, h // 2]) / np.sqrt(8)) < 1e-14
    assert np.all(dQ[t] == 0) and np.all(dK[t] == 0)
    np.testing.assert_allclose(dV[t, 0], do[t, 0] + do[t, 1], rtol=0, atol=1e-15)
    np.testing.assert_allclose(dV[t, 1], do[t, 2] + do[t, 3], rtol=0, atol=1e-15)


def test_zero_queries_give_running_means():
    # Q = 0: P_ij = 1/(i-a+1); O_i = mean of v_a..v_i; LSE_i = log(i-a+1); dV_j = sum_{i>=j} dO_i/(i-a+1)
    lengths = [[5, 9]]
    q, k, v, do, seg = _rand(lengths, 2, 1, 4, seed=24)
    q[:] = 0
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    for s in range(2):
        a, b = cu[s], cu[s + 1]
        cnt = np.arange(1, b - a + 1)[:, None]
        mean = np.cumsum(v[a:b, 0], axis=0) / cnt
        for h in range(2):
            np.testing.assert_allclose(O[a:b, h], mean, rtol=1e-13, atol=1e-14)
            np.testing.assert_allclose(LSE[h, a:b], np.log(cnt[:, 0]), rtol=1e-13, atol=1e-14)
        w = (do[a:b, 0] + do[a:b, 1]) / cnt
        expect = np.cumsum(w[::-1], axis=0)[::-1]
        np.testing.assert_allclose(dV[a:b, 0], expect, rtol=1e-13, atol=1e-14)
    assert np.all(dK == 0)          # q = 0 => no gradient reaches K


@pytest.mark.parametrize("lengths,hq,hkv,d", CASES[:3])
def test_finite_differences(lengths, hq, hkv, d):
    q, k, v, do, seg = _rand(lengths, hq, hkv, d, seed=31)
    cu = seg["cu_seqlens"]
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    loss = lambda q_, k_, v_: float((oracle.fwd(q_, k_, v_, cu)[0] * do).sum())
    rng = np.random.default_rng(1)
    eps = 1e-6
    for which, grad in (("q", dQ), ("k", dK), ("v", dV)):
        arrs = {"q": q, "k": k, "v": v}
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in arrs[which].shape)
            plus = {n: a.copy() for n, a in arrs.items()}
            minus = {n: a.copy() for n, a in arrs.items()}
            plus[which][idx] += eps
            minus[which][idx] -= eps
            fd = (loss(plus["q"], plus["k"], plus["v"]) - loss(minus["q"], minus["k"], minus["v"])) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-7 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def test_gqa_equals_mha_on_repeated_kv_heads():
    lengths = [[6, 2, 9]]
    q, k, v, do, seg = _rand(lengths, 6, 2, 8, seed=41)
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    kk, vv = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    O2, LSE2 = oracle.fwd(q, kk, vv, cu)
    dQ2, dK2, dV2 = oracle.bwd(do, q, kk, vv, cu)
    np.testing.assert_array_equal(O, O2)
    np.testing.assert_array_equal(LSE, LSE2)
    np.testing.assert_array_equal(dQ, dQ2)
    np.testing.assert_allclose(dK, dK2.reshape(-1, 2, 3, 8).sum(axis=2), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(dV, dV2.reshape(-1, 2, 3, 8).sum(axis=2), rtol=1e-13, atol=1e-14)


def test_row_identities():
    # rows of P sum to 1 (=> sum_j dS_ij = 0 => dQ.q - dK... check via D_i == dO_i . O_i on the dense P)
    lengths = [[7, 4]]
    q, k, v, do, seg = _rand(lengths, 2, 2, 8, seed=51)
    O, LSE = oracle.fwd(q, k, v, seg["cu_seqlens"])
    _, _, Ps = _dense_fwd(q, k, v, seg["seg_id"], 1 / np.sqrt(8))
    for h in range(2):
        np.testing.assert_allclose(Ps[h].sum(axis=1), 1.0, rtol=1e-14)
        dP = do[:, h] @ v[:, h].T
        D = (Ps[h] * dP).sum(axis=1)
        np.testing.assert_allclose(D, (do[:, h] * O[:, h]).sum(axis=1), rtol=1e-11, atol=1e-13)


def test_padded_batch_equals_packed_at_real_tokens():
    # batch-level padding (Section 3): each example right-padded to the group maximum.  Pads
    # come after the real tokens, so causal attention never sees them.
    lengths = [[3, 5, 1, 7]]
    q, k, v, do, seg = _rand(lengths, 2, 2, 8, seed=61)
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    Lmax = 7
    pads = [np.zeros((4 * Lmax,) + a.shape[1:]) for a in (q, k, v, do)]
    for s in range(4):
        a, b = cu[s], cu[s + 1]
        for dst, src in zip(pads, (q, k, v, do)):
            dst[s * Lmax: s * Lmax + (b - a)] = src[a:b]
    pcu = np.arange(0, 4 * Lmax + 1, Lmax, dtype=np.int32)
    Op, LSEp = oracle.fwd(pads[0], pads[1], pads[2], pcu)
    dQp, dKp, dVp = oracle.bwd(pads[3], pads[0], pads[1], pads[2], pcu)
    for s in range(4):
        a, b = cu[s], cu[s + 1]
        sl = slice(s * Lmax, s * Lmax + (b - a))
        assert np.array_equal(O[a:b], Op[sl]) and np.array_equal(LSE[:, a:b], LSEp[:, sl])
        np.testing.assert_allclose(dQ[a:b], dQp[sl], rtol=0, atol=1e-14)
        np.testing.assert_allclose(dK[a:b], dKp[sl], rtol=0, atol=1e-14)
        np.testing.assert_allclose(dV[a:b], dVp[sl], rtol=0, atol=1e-14)


def test_sampled_rows_equal_full_outputs():
    lengths = [[10, 3, 17], [1, 20, 9]]
    q, k, v, do, seg = _rand(lengths, 4, 2, 8, seed=71)
    cu = seg["cu_seqlens"]
    O, LSE = oracle.fwd(q, k, v, cu)
    dQ, dK, dV = oracle.bwd(do, q, k, v, cu)
    rng = np.random.default_rng(3)
    tok = rng.integers(0, 60, size=25)
    head = rng.integers(0, 4, size=25)
    Or, LSEr, dQr = oracle.rows_q(do, q, k, v, cu, tok, head)
    np.testing.assert_array_equal(Or, O[tok, head])
    np.testing.assert_array_equal(LSEr, LSE[head, tok])
    np.testing.assert_array_equal(dQr, dQ[tok, head])
    kvh = rng.integers(0, 2, size=25)
    dKr, dVr = oracle.rows_kv(do, q, k, v, cu, tok, kvh)
    np.testing.assert_allclose(dKr, dK[tok, kvh], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(dVr, dV[tok, kvh], rtol=1e-13, atol=1e-14)
