"""Pins for the fp64 CPU oracle: everything here is fixed by mathematics, not by
the oracle itself.  A dropped term, a wrong sign, an off-by-one in the causal
mask, a transposed operand, a wrong scale or a wrong GQA mapping fails at
least one of these.  The paper prints no worked numeric example of attention,
so there is no golden fixture from it; the closed forms below take its place.
"""
import math

import numpy as np
import pytest

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _inputs(lengths, hq, hkv, d, seed=0):
    T = sum(lengths)
    return (_rand((T, hq, d), seed), _rand((T, hkv, d), seed + 1),
            _rand((T, hkv, d), seed + 2), _rand((T, hq, d), seed + 3))


def test_softmax_rows_sum_to_one_and_mask():
    L, H, d = 37, 3, 8
    q, k, v, _ = _inputs([L], H, H, d, 10)
    o, lse, p = oracle.attn_fwd(q, k, v, [L], 0.3, return_probs=True)
    assert p.shape == (H, L, L)
    assert np.all(p >= 0.0)
    assert np.max(np.abs(p.sum(axis=2) - 1.0)) < 1e-14
    assert np.all(np.triu(p, 1) == 0.0)               # j > r: weight exactly 0
    assert np.all(p[:, np.arange(L), np.arange(L)] > 0)  # diagonal visible
    # P determines O and LSE determines P's normaliser
    for h in range(H):
        np.testing.assert_allclose(o[:, h, :], p[h] @ v[:, h, :], rtol=0, atol=1e-13)
        s = 0.3 * q[:, h, :] @ k[:, h, :].T
        np.testing.assert_allclose(np.tril(p[h]), np.tril(np.exp(s - lse[h][:, None])), rtol=1e-12, atol=1e-15)


def test_length_one_sequences():
    lengths = [1, 1, 1]
    q, k, v, do = _inputs(lengths, 2, 2, 16, 20)
    s = 0.25
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    assert np.array_equal(o, v)
    np.testing.assert_allclose(lse, s * np.einsum("thc,thc->ht", q, k), rtol=1e-15, atol=1e-15)
    assert np.array_equal(dv, do)
    assert np.all(dq == 0.0) and np.all(dk == 0.0)


def test_two_token_closed_form():
    # L = 2, d = 1, one head: everything has a hand-derived closed form.
    a, b, c, e, f, g = 0.7, -1.3, 0.9, 0.4, 2.0, -0.5
    do0, do1, s = 0.3, -1.1, 0.6
    q = np.array([a, b]).reshape(2, 1, 1); k = np.array([c, e]).reshape(2, 1, 1)
    v = np.array([f, g]).reshape(2, 1, 1); do = np.array([do0, do1]).reshape(2, 1, 1)
    o, lse = oracle.attn_fwd(q, k, v, [2], s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, [2], s)
    s10, s11 = s * b * c, s * b * e
    p10 = 1.0 / (1.0 + math.exp(s11 - s10)); p11 = 1.0 - p10
    assert o[0, 0, 0] == f
    assert abs(o[1, 0, 0] - (p10 * f + p11 * g)) < 1e-15
    assert abs(lse[0, 0] - s * a * c) < 1e-15
    assert abs(lse[0, 1] - math.log(math.exp(s10) + math.exp(s11))) < 1e-15
    ds10 = p10 * p11 * do1 * (f - g)
    assert abs(dq[0, 0, 0]) == 0.0
    assert abs(dq[1, 0, 0] - s * ds10 * (c - e)) < 1e-15
    assert abs(dk[0, 0, 0] - s * ds10 * b) < 1e-15
    assert abs(dk[1, 0, 0] + s * ds10 * b) < 1e-15
    assert abs(dv[0, 0, 0] - (do0 + p10 * do1)) < 1e-15
    assert abs(dv[1, 0, 0] - p11 * do1) < 1e-15


def test_zero_query_closed_form():
    # Q = 0: uniform causal weights 1/(r+1).
    lengths, H, d, s = [9, 4], 2, 6, 0.41
    _, k, v, do = _inputs(lengths, H, H, d, 30)
    T = sum(lengths)
    q = np.zeros((T, H, d))
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    t0 = 0
    for L in lengths:
        for h in range(H):
            for r in range(L):
                np.testing.assert_allclose(o[t0 + r, h], v[t0:t0 + r + 1, h].mean(axis=0), rtol=0, atol=1e-14)
                assert abs(lse[h, t0 + r] - math.log(r + 1)) < 1e-14
                dp = v[t0:t0 + r + 1, h] @ do[t0 + r, h]
                ds = (dp - dp.mean()) / (r + 1)
                np.testing.assert_allclose(dq[t0 + r, h], s * ds @ k[t0:t0 + r + 1, h], rtol=0, atol=1e-13)
            for j in range(L):
                want = sum(do[t0 + r, h] / (r + 1) for r in range(j, L))
                np.testing.assert_allclose(dv[t0 + j, h], want, rtol=0, atol=1e-13)
        t0 += L
    assert np.all(dk == 0.0)


def test_one_hot_limit_gathers_the_aligned_value():
    L, d = 12, 16
    k = np.zeros((L, 1, d)); k[np.arange(L), 0, np.arange(L)] = 40.0     # orthogonal, large norm
    v = _rand((L, 1, d), 41)
    target = [0, 0, 1, 3, 2, 5, 0, 7, 4, 9, 10, 6]                     # target[r] <= r
    q = np.zeros((L, 1, d)); q[np.arange(L), 0, target] = 40.0
    o, _ = oracle.attn_fwd(q, k, v, [L], 1.0)
    np.testing.assert_allclose(o[:, 0], v[target, 0], rtol=0, atol=1e-12)


def test_packed_equals_unpacked_and_permutation():
    lengths, hq, hkv, d, s = [5, 1, 13, 8], 4, 2, 8, 0.35
    q, k, v, do = _inputs(lengths, hq, hkv, d, 50)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    for i, L in enumerate(lengths):
        sl = slice(cu[i], cu[i + 1])
        oi, li = oracle.attn_fwd(q[sl], k[sl], v[sl], [L], s)
        dqi, dki, dvi = oracle.attn_bwd(q[sl], k[sl], v[sl], do[sl], [L], s)
        assert np.array_equal(o[sl], oi) and np.array_equal(lse[:, sl], li)
        assert np.array_equal(dq[sl], dqi) and np.array_equal(dk[sl], dki) and np.array_equal(dv[sl], dvi)
    perm = [2, 0, 3, 1]
    tok = np.concatenate([np.arange(cu[i], cu[i + 1]) for i in perm])
    pl = [lengths[i] for i in perm]
    o2, lse2 = oracle.attn_fwd(q[tok], k[tok], v[tok], pl, s)
    dq2, dk2, dv2 = oracle.attn_bwd(q[tok], k[tok], v[tok], do[tok], pl, s)
    assert np.array_equal(o2, o[tok]) and np.array_equal(lse2, lse[:, tok])
    assert np.array_equal(dq2, dq[tok]) and np.array_equal(dk2, dk[tok]) and np.array_equal(dv2, dv[tok])


def test_key_shift_invariance():
    lengths, H, d, s = [11, 6], 2, 8, 0.5
    q, k, v, _ = _inputs(lengths, H, H, d, 60)
    c = _rand((H, d), 61)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    o2, lse2 = oracle.attn_fwd(q, k + c[None], v, lengths, s)
    np.testing.assert_allclose(o2, o, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse2 - lse, s * np.einsum("thc,hc->ht", q, c), rtol=0, atol=1e-13)


def test_softmax_jacobian_and_dv_column_sums():
    lengths, hq, hkv, d, s = [7, 19], 6, 2, 8, 0.3
    q, k, v, do = _inputs(lengths, hq, hkv, d, 70)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    G = hq // hkv
    for i in range(len(lengths)):
        # sum_j dS_rj = 0, so the first row of every sequence (one visible key) has dQ = 0
        assert np.all(dq[cu[i]] == 0.0)
        for g in range(hkv):
            # sum_j dV_j = sum over the group's heads and rows of dO_r  (rows of P sum to 1)
            want = do[cu[i]:cu[i + 1], g * G:(g + 1) * G].sum(axis=(0, 1))
            np.testing.assert_allclose(dv[cu[i]:cu[i + 1], g].sum(axis=0), want, rtol=0, atol=1e-12)
    # constant keys: every <q_r, k_j> equal along j, so dS-weighted sums of k collapse: dQ = s * (sum_j dS_rj) k = 0
    kc = np.broadcast_to(_rand((1, hkv, d), 71), k.shape).copy()
    dq_c, _, _ = oracle.attn_bwd(q, kc, v, do, lengths, s)
    assert np.max(np.abs(dq_c)) < 1e-13


def test_gqa_equals_mha_with_repeated_kv():
    lengths, hq, hkv, d, s = [9, 14], 6, 2, 8, 0.33
    q, k, v, do = _inputs(lengths, hq, hkv, d, 80)
    G = hq // hkv
    kr, vr = np.repeat(k, G, axis=1), np.repeat(v, G, axis=1)     # head h uses kv head h // G
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    o2, lse2 = oracle.attn_fwd(q, kr, vr, lengths, s)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    dq2, dk2, dv2 = oracle.attn_bwd(q, kr, vr, do, lengths, s)
    T = sum(lengths)
    assert np.array_equal(dq, dq2)
    np.testing.assert_allclose(dk, dk2.reshape(T, hkv, G, d).sum(axis=2), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, dv2.reshape(T, hkv, G, d).sum(axis=2), rtol=0, atol=1e-13)
    # and the head mapping is by contiguous groups, not interleaved: perturbing kv head 1
    # must leave the outputs of query heads 0..G-1 untouched
    k3 = k.copy(); k3[:, 1] += 1.0
    o3, _ = oracle.attn_fwd(q, k3, v, lengths, s)
    assert np.array_equal(o3[:, :G], o[:, :G]) and not np.array_equal(o3[:, G:], o[:, G:])


def test_finite_differences_every_element():
    lengths, hq, hkv, d, s = [1, 2, 5], 2, 1, 4, 0.45
    q, k, v, do = _inputs(lengths, hq, hkv, d, 90)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)

    def loss(q_, k_, v_):
        o_, _ = oracle.attn_fwd(q_, k_, v_, lengths, s)
        return float(np.sum(o_ * do))

    eps = 1e-5
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            num[idx] = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
        rel = np.linalg.norm(num - grad) / max(np.linalg.norm(grad), 1e-300)
        assert rel < 1e-6, (name, rel)
        assert np.max(np.abs(num - grad)) < 1e-6 * max(1.0, np.max(np.abs(grad))), name


def test_dense_library_evaluation_with_autodiff():
    """Independent route: dense masked score matrix, library softmax, reverse-mode
    autodiff, per sequence and head, on the tiny benchmark pack's shape."""
    torch = pytest.importorskip("torch")
    lengths, hq, hkv, d = [17, 64, 111], 4, 2, 64
    s = 1.0 / math.sqrt(d)
    q, k, v, do = _inputs(lengths, hq, hkv, d, 100)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    G = hq // hkv
    tq = torch.tensor(q, requires_grad=True); tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True); tdo = torch.tensor(do)
    outs, lses = [], []
    t0 = 0
    for L in lengths:
        mask = torch.ones(L, L, dtype=torch.bool).tril()
        qi = tq[t0:t0 + L].transpose(0, 1)                                  # [Hq, L, d]
        ki = tk[t0:t0 + L].transpose(0, 1).repeat_interleave(G, dim=0)
        vi = tv[t0:t0 + L].transpose(0, 1).repeat_interleave(G, dim=0)
        sc = (qi @ ki.transpose(1, 2)) * s
        sc = sc.masked_fill(~mask, float("-inf"))
        outs.append((torch.softmax(sc, dim=-1) @ vi).transpose(0, 1))
        lses.append(torch.logsumexp(sc, dim=-1))
        t0 += L
    to = torch.cat(outs, dim=0)
    (to * tdo).sum().backward()
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, torch.cat(lses, dim=1).detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-11)


def test_sampled_rows_and_keys_equal_the_full_evaluation():
    lengths, hq, hkv, d, s = [6, 0, 23, 1, 12], 4, 2, 8, 0.37
    q, k, v, do = _inputs(lengths, hq, hkv, d, 130)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    T = sum(lengths)
    tok = np.repeat(np.arange(T), hq); hd = np.tile(np.arange(hq), T)
    o_r, lse_r, dq_r = oracle.attn_rows(q, k, v, do, lengths, s, tok, hd)
    assert np.array_equal(o_r.reshape(T, hq, d), o) and np.array_equal(dq_r.reshape(T, hq, d), dq)
    assert np.array_equal(lse_r.reshape(T, hq).T, lse)
    tok = np.repeat(np.arange(T), hkv); hd = np.tile(np.arange(hkv), T)
    dk_r, dv_r = oracle.attn_keys(q, k, v, do, lengths, s, tok, hd)
    assert np.array_equal(dk_r.reshape(T, hkv, d), dk) and np.array_equal(dv_r.reshape(T, hkv, d), dv)
    # a shuffled subset with repeats: samples that share a (sequence, kv head) share their row statistics, whichever
    # of them comes first
    rng = np.random.default_rng(131)
    pick = rng.integers(0, T * hkv, size=40)
    dk_s, dv_s = oracle.attn_keys(q, k, v, do, lengths, s, tok[pick], hd[pick])
    assert np.array_equal(dk_s, dk[tok[pick], hd[pick]]) and np.array_equal(dv_s, dv[tok[pick], hd[pick]])


def test_zero_length_sequences_and_empty_pack():
    lengths, H, d, s = [0, 4, 0, 3, 0], 2, 4, 0.5
    q, k, v, do = _inputs(lengths, H, H, d, 110)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    o2, lse2 = oracle.attn_fwd(q, k, v, [4, 3], s)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    dq2, dk2, dv2 = oracle.attn_bwd(q, k, v, do, [4, 3], s)
    assert np.array_equal(dq, dq2) and np.array_equal(dk, dk2) and np.array_equal(dv, dv2)
    e = np.zeros((0, H, d))
    oe, lse_e = oracle.attn_fwd(e, e, e, [], s)
    assert oe.shape == (0, H, d) and lse_e.shape == (H, 0)


def test_rejects_bad_arguments():
    q, k, v, _ = _inputs([4], 3, 2, 4, 120)   # 3 query heads on 2 kv heads: not a whole number of groups
    with pytest.raises(RuntimeError):
        oracle.attn_fwd(q, k, v, [4], 0.5)
    with pytest.raises(ValueError):
        oracle.attn_fwd(q[:, :2], k, v, [3], 0.5)
