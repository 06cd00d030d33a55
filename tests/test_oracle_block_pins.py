"""Pins of the block (context-parallel) oracle against things other than itself.

The packed oracle (oracle/attn_oracle.c, a separate C implementation that is pinned on its own) fixes the
result of whole-sequence attention; any partition of a sequence's rows and keys into blocks must reproduce it
after merging / summing.  Further pins: closed forms of the merge, degenerate blocks, a dense evaluation with
a library softmax and reverse-mode autodiff, brute force over single (row, key) pairs.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import block as ob


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _chunks(total, cuts):
    edges = [0] + sorted(cuts) + [total]
    return [(edges[i], edges[i + 1]) for i in range(len(edges) - 1) if edges[i + 1] >= edges[i]]


def _full(lengths, hq, hkv, d, seed):
    T = sum(lengths)
    q, k, v, do = (_rand((T, h, d), seed + i) for i, h in enumerate((hq, hkv, hkv, hq)))
    s = 1.0 / math.sqrt(d)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    return q, k, v, do, s, o, lse, dq, dk, dv


@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2)])
def test_partition_of_keys_and_rows_reproduces_the_packed_oracle(hq, hkv):
    """One sequence of 37 tokens: rows cut at 11 and 29, keys cut at 5, 20 and 21 (one empty chunk);
    every (row chunk, key chunk) block goes through the block oracle."""
    L, d = 37, 8
    q, k, v, do, s, o, lse, dq, dk, dv = _full([L], hq, hkv, d, 100)
    dsum = ob.row_dot(o, do)
    key_chunks = _chunks(L, [5, 20, 20, 21])
    dk_sum, dv_sum = np.zeros_like(k), np.zeros_like(v)
    for r0, r1 in _chunks(L, [11, 29]):
        acc_o = np.zeros((r1 - r0, hq, d)); acc_l = np.full((hq, r1 - r0), -np.inf)
        dq_sum = np.zeros((r1 - r0, hq, d))
        for k0, k1 in key_chunks:
            args = ([r1 - r0], [k1 - k0], [r0], [k0], s)
            po, pl = ob.block_fwd(q[r0:r1], k[k0:k1], v[k0:k1], *args)
            acc_o, acc_l = ob.merge(acc_o, acc_l, po, pl)
            bdq, bdk, bdv = ob.block_bwd(q[r0:r1], k[k0:k1], v[k0:k1], do[r0:r1], lse[:, r0:r1], dsum[:, r0:r1], *args)
            dq_sum += bdq
            dk_sum[k0:k1] += bdk
            dv_sum[k0:k1] += bdv
        np.testing.assert_allclose(acc_o, o[r0:r1], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(acc_l, lse[:, r0:r1], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dq_sum, dq[r0:r1], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dk_sum, dk, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dv_sum, dv, rtol=1e-11, atol=1e-12)


def test_packed_blocks_equal_per_sequence_blocks():
    """Several sequences in one call == each sequence alone (no leakage across sequences, offsets indexed
    per sequence)."""
    d, hq, hkv = 8, 2, 1
    ql, kl, qp, kp = [5, 0, 9, 3], [7, 4, 2, 6], [3, 0, 10, 0], [0, 2, 11, 1]
    q = _rand((sum(ql), hq, d), 1); k = _rand((sum(kl), hkv, d), 2); v = _rand((sum(kl), hkv, d), 3)
    o, lse = ob.block_fwd(q, k, v, ql, kl, qp, kp, 0.3)
    cq, ck = np.cumsum([0] + ql), np.cumsum([0] + kl)
    for i in range(4):
        oi, li = ob.block_fwd(q[cq[i]:cq[i + 1]], k[ck[i]:ck[i + 1]], v[ck[i]:ck[i + 1]], [ql[i]], [kl[i]], [qp[i]], [kp[i]], 0.3)
        np.testing.assert_array_equal(oi, o[cq[i]:cq[i + 1]])
        np.testing.assert_array_equal(li, lse[:, cq[i]:cq[i + 1]])


def test_brute_force_pairs():
    """Pure-Python loops over (row, key) pairs on a tiny block with a non-trivial offset."""
    d, ql, kl, qp, kp, s = 3, 4, 5, 2, 1, 0.7
    q = _rand((ql, 1, d), 5); k = _rand((kl, 1, d), 6); v = _rand((kl, 1, d), 7); do = _rand((ql, 1, d), 8)
    o, lse = ob.block_fwd(q, k, v, [ql], [kl], [qp], [kp], s)
    for r in range(ql):
        vis = [j for j in range(kl) if kp + j <= qp + r]
        sc = [s * sum(q[r, 0, c] * k[j, 0, c] for c in range(d)) for j in vis]
        z = sum(math.exp(x) for x in sc)
        assert lse[0, r] == pytest.approx(math.log(z), rel=1e-13)
        for c in range(d):
            assert o[r, 0, c] == pytest.approx(sum(math.exp(x) / z * v[j, 0, c] for x, j in zip(sc, vis)), rel=1e-12, abs=1e-14)
    # backward with arbitrary (not self-consistent) row statistics: the formulas must hold term by term
    lse_in = _rand((1, ql), 9); dsum = _rand((1, ql), 10)
    dq, dk, dv = ob.block_bwd(q, k, v, do, lse_in, dsum, [ql], [kl], [qp], [kp], s)
    edq = np.zeros((ql, d)); edk = np.zeros((kl, d)); edv = np.zeros((kl, d))
    for r in range(ql):
        for j in range(kl):
            if kp + j > qp + r:
                continue
            p = math.exp(s * float(q[r, 0] @ k[j, 0]) - lse_in[0, r])
            ds = p * (float(do[r, 0] @ v[j, 0]) - dsum[0, r])
            edq[r] += s * ds * k[j, 0]
            edk[j] += s * ds * q[r, 0]
            edv[j] += p * do[r, 0]
    np.testing.assert_allclose(dq[:, 0], edq, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dk[:, 0], edk, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dv[:, 0], edv, rtol=1e-12, atol=1e-14)


def test_fully_masked_and_empty_blocks():
    d = 4
    q = _rand((6, 2, d), 1); k = _rand((5, 2, d), 2); v = _rand((5, 2, d), 3); do = _rand((6, 2, d), 4)
    # keys start after the last row: nothing visible
    o, lse = ob.block_fwd(q, k, v, [6], [5], [0], [6], 0.5)
    assert np.all(o == 0.0) and np.all(np.isneginf(lse))
    dq, dk, dv = ob.block_bwd(q, k, v, do, np.zeros((2, 6)), np.zeros((2, 6)), [6], [5], [0], [6], 0.5)
    assert np.all(dq == 0.0) and np.all(dk == 0.0) and np.all(dv == 0.0)
    # partly masked rows: rows 0, 1 see nothing, row 2 sees key 0 only -> O = v_0, LSE = s <q, k_0>
    o, lse = ob.block_fwd(q, k, v, [6], [5], [0], [2], 0.5)
    assert np.all(np.isneginf(lse[:, :2])) and np.all(o[:2] == 0.0)
    np.testing.assert_allclose(o[2], v[0], rtol=1e-14)
    np.testing.assert_allclose(lse[:, 2], 0.5 * np.einsum("hc,hc->h", q[2], k[0]), rtol=1e-13)
    # empty key chunk
    o, lse = ob.block_fwd(q, k[:0], v[:0], [6], [0], [0], [0], 0.5)
    assert np.all(o == 0.0) and np.all(np.isneginf(lse))


def test_fully_visible_block_is_plain_softmax_attention():
    torch = pytest.importorskip("torch")
    d, ql, kl = 8, 7, 9
    q = _rand((ql, 2, d), 1); k = _rand((kl, 1, d), 2); v = _rand((kl, 1, d), 3)
    o, lse = ob.block_fwd(q, k, v, [ql], [kl], [100], [0], 0.4)
    for h in range(2):
        s = torch.from_numpy(0.4 * q[:, h] @ k[:, 0].T)
        np.testing.assert_allclose(o[:, h], (torch.softmax(s, dim=1) @ torch.from_numpy(v[:, 0])).numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[h], torch.logsumexp(s, dim=1).numpy(), rtol=1e-13)


def test_offset_block_against_dense_autodiff():
    """Rows [a, b) of a sequence against keys [0, b): the block is the complete attention of those rows, so its own
    LSE and D are the row statistics and reverse-mode autodiff of a dense masked softmax gives its gradients."""
    torch = pytest.importorskip("torch")
    d, a, b, hq, hkv, s = 6, 5, 12, 4, 2, 0.37
    q = _rand((b - a, hq, d), 1); k = _rand((b, hkv, d), 2); v = _rand((b, hkv, d), 3); do = _rand((b - a, hq, d), 4)
    o, lse = ob.block_fwd(q, k, v, [b - a], [b], [a], [0], s)
    dq, dk, dv = ob.block_bwd(q, k, v, do, lse, ob.row_dot(o, do), [b - a], [b], [a], [0], s)
    tq, tk, tv = (torch.from_numpy(x).requires_grad_(True) for x in (q, k, v))
    mask = torch.arange(b)[None, :] <= (torch.arange(b - a)[:, None] + a)
    outs = []
    for h in range(hq):
        sc = s * tq[:, h] @ tk[:, h // 2].T
        outs.append(torch.softmax(sc.masked_fill(~mask, float("-inf")), dim=1) @ tv[:, h // 2])
    to = torch.stack(outs, dim=1)
    to.backward(torch.from_numpy(do))
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_merge_closed_forms():
    o_a = _rand((3, 2, 4), 1); o_b = _rand((3, 2, 4), 2)
    l = _rand((2, 3), 3)
    # equal weights: the mean, LSE + ln 2
    o, lse = ob.merge(o_a, l, o_b, l)
    np.testing.assert_allclose(o, 0.5 * (o_a + o_b), rtol=1e-14)
    np.testing.assert_allclose(lse, l + math.log(2.0), rtol=1e-14)
    # -inf is the neutral element, on either side and on both
    ninf = np.full((2, 3), -np.inf)
    for o1, l1 in (ob.merge(o_a, l, np.zeros_like(o_a), ninf), ob.merge(np.zeros_like(o_a), ninf, o_a, l)):
        np.testing.assert_array_equal(o1, o_a)
        np.testing.assert_array_equal(l1, l)
    o2, l2 = ob.merge(np.zeros_like(o_a), ninf, np.zeros_like(o_a), ninf)
    assert np.all(o2 == 0.0) and np.all(np.isneginf(l2))
    # weights 1/(1+e) and e/(1+e) when the second LSE is larger by 1; commutative; huge LSE values do not overflow
    o, lse = ob.merge(o_a, l + 700.0, o_b, l + 701.0)
    w = 1.0 / (1.0 + math.e)
    np.testing.assert_allclose(o, w * o_a + (1 - w) * o_b, rtol=1e-13)
    np.testing.assert_allclose(lse, l + 700.0 + math.log(1.0 + math.e), rtol=1e-14)
    o_r, lse_r = ob.merge(o_b, l + 701.0, o_a, l + 700.0)
    np.testing.assert_allclose(o_r, o, rtol=1e-15)
    np.testing.assert_allclose(lse_r, lse, rtol=1e-15)


def test_bad_arguments():
    q = _rand((4, 2, 4), 1); k = _rand((4, 2, 4), 2)
    with pytest.raises(ValueError):
        ob.block_fwd(q, k, k, [3], [4], [0], [0], 1.0)        # lengths do not sum to the token count
    with pytest.raises(ValueError):
        ob.block_fwd(q, k, k, [4], [4], [0, 0], [0], 1.0)     # lists differ
    with pytest.raises(ValueError):
        ob.block_fwd(q, k, k, [4], [4], [-1], [0], 1.0)       # negative position
    with pytest.raises(ValueError):
        ob.block_fwd(q, _rand((4, 3, 4), 3), _rand((4, 3, 4), 3), [4], [4], [0], [0], 1.0)   # 2 % 3 != 0
