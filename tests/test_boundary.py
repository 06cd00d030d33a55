"""Host-side tests of the C-ABI boundary: symbol export, cu_seqlens, the cost-sorted work list
and argument validation.  No GPU is touched."""
import ctypes
import os
import re

import numpy as np
import pytest

import hspmd_workloads as w
import paper_2504_20490_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hspmd_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(hspmd_[a-z_0-9]+)\s*\(", header))
    assert {"hspmd_build_cu_seqlens", "hspmd_attn_varlen_fwd", "hspmd_attn_varlen_bwd",
            "hspmd_attn_plan_create", "hspmd_attn_schedule"} <= names
    lib = ctypes.CDLL(A.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert A.load_library().hspmd_last_error() is not None


def test_build_cu_seqlens():
    cu, mx, tot = A.build_cu_seqlens([17, 64, 111])
    assert cu.tolist() == [0, 17, 81, 192] and mx == 111 and tot == 192
    cu, mx, tot = A.build_cu_seqlens([0, 5, 0])
    assert cu.tolist() == [0, 0, 5, 5] and mx == 5 and tot == 5
    cu, mx, tot = A.build_cu_seqlens([])
    assert cu.tolist() == [0] and mx == 0 and tot == 0
    with pytest.raises(A.HspmdError) as e:
        A.build_cu_seqlens([4, -1])
    assert e.value.status == 1 and "negative" in str(e.value)
    with pytest.raises(A.HspmdError):
        A.build_cu_seqlens([2 ** 30, 2 ** 30, 5])      # running sum above INT32_MAX
    cu, _, tot = A.build_cu_seqlens([2 ** 30, 2 ** 30 - 1])
    assert tot == 2 ** 31 - 1 and cu[-1] == 2 ** 31 - 1


def _cost(kind, L, tile, G):
    if kind == A.LIST_DKV:
        return -(-(L - tile * 128) // 64) * G
    return -(-min(L, (tile + 1) * 128) // 64)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
@pytest.mark.parametrize("kind", [A.LIST_FWD, A.LIST_DQ, A.LIST_DKV])
def test_work_list_invariants(name, kind):
    cfg = w.config_by_name(name)
    lengths = w.lengths_for(cfg)
    cu, _, _ = A.build_cu_seqlens(lengths)
    hq, hkv = cfg.q_heads, cfg.kv_heads
    G = hq // hkv
    items = A.schedule(kind, cu, hq, hkv, 8)
    assert items.shape[0] % 8 == 0
    real = items[items[:, 2] >= 0]
    rows = A.tile_rows(kind)
    heads = hkv if kind == A.LIST_DKV else hq
    # every (sequence, tile, head) exactly once; tiles cover [0, L)
    want = set()
    for s, L in enumerate(lengths):
        for t in range(-(-L // rows)):
            for h in range(heads):
                want.add((int(cu[s]), L, t, h))
    got = [tuple(int(x) for x in r) for r in real]
    assert len(got) == len(set(got)) == len(want) and set(got) == want
    # queues (slots with equal p % 8) are balanced by cost
    loads = np.zeros(8)
    for p, r in enumerate(items):
        if r[2] >= 0:
            loads[p % 8] += _cost(kind, int(r[1]), int(r[2]), G)
    biggest = max(_cost(kind, int(r[1]), int(r[2]), G) for r in real)
    if len(real) >= 64:
        assert loads.max() - loads.min() <= max(0.08 * loads.mean(), 2 * biggest), loads
    # items that share K/V (or Q/dO) stay in one queue unless their chain was cut for balance,
    # and inside a queue one chain's items appear most expensive first
    by_chain = {}
    for p, r in enumerate(items):
        if r[2] < 0:
            continue
        kvh = int(r[3]) if kind == A.LIST_DKV else int(r[3]) // G
        by_chain.setdefault((int(r[0]), kvh, p % 8), []).append(_cost(kind, int(r[1]), int(r[2]), G))
    for costs in by_chain.values():
        assert costs == sorted(costs, reverse=True)
    # padding only at the tail of a queue
    for x in range(8):
        tiles = items[x::8, 2]
        pad = np.flatnonzero(tiles < 0)
        if pad.size:
            assert np.all(tiles[pad[0]:] < 0)


def test_work_list_invariants_on_random_packs():
    """The same invariants on packs nobody chose: lengths from 0 up, any number of queues, MHA and GQA."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(lengths=st.lists(st.one_of(st.integers(0, 300), st.integers(0, 5000)), min_size=0, max_size=12),
           hkv=st.integers(1, 4), group=st.sampled_from([1, 2, 4]), queues=st.sampled_from([1, 3, 8]),
           kind=st.sampled_from([A.LIST_FWD, A.LIST_DKV]))
    def check(lengths, hkv, group, queues, kind):
        hq = hkv * group
        cu, _, _ = A.build_cu_seqlens(lengths)
        items = A.schedule(kind, cu, hq, hkv, queues)
        assert items.shape[0] % queues == 0
        real = items[items[:, 2] >= 0]
        rows = A.tile_rows(kind)
        heads = hkv if kind == A.LIST_DKV else hq
        want = {(int(cu[s]), L, t, h) for s, L in enumerate(lengths) for t in range(-(-L // rows)) for h in range(heads)}
        got = [tuple(int(x) for x in r) for r in real]
        assert len(got) == len(want) and set(got) == want
        if not got:
            return
        loads = np.zeros(queues)
        for p, r in enumerate(items):
            if r[2] >= 0:
                loads[p % queues] += max(1, _cost(kind, int(r[1]), int(r[2]), group))
        costs = [max(1, _cost(kind, int(r[1]), int(r[2]), group)) for r in real]
        # longest-processing-time placement of segments no heavier than total / (4 queues) (or one item, if heavier)
        cap = max(max(costs), sum(costs) // (4 * queues) + 1)
        assert loads.max() - loads.min() <= cap, (loads, cap)
        for x in range(queues):
            tiles = items[x::queues, 2]
            pad = np.flatnonzero(tiles < 0)
            if pad.size:
                assert np.all(tiles[pad[0]:] < 0)

    check()


@pytest.mark.parametrize("order", [A.ORDER_NATURAL, A.ORDER_COST])
@pytest.mark.parametrize("kind", [A.LIST_FWD, A.LIST_DKV])
def test_alternative_orders_hold_every_item_once(order, kind):
    cfg = w.config_by_name("C3")
    lengths = w.lengths_for(cfg)
    cu, _, _ = A.build_cu_seqlens(lengths)
    default = A.schedule(kind, cu, cfg.q_heads, cfg.kv_heads, 8)
    other = A.schedule(kind, cu, cfg.q_heads, cfg.kv_heads, 8, order=order)
    assert np.all(other[:, 2] >= 0)                     # no padding without queues
    as_set = lambda a: sorted(tuple(int(x) for x in r) for r in a if r[2] >= 0)
    assert as_set(other) == as_set(default)
    G = cfg.q_heads // cfg.kv_heads
    costs = [_cost(kind, int(r[1]), int(r[2]), G) for r in other]
    if order == A.ORDER_COST:
        assert costs == sorted(costs, reverse=True)
    else:
        assert [int(r[0]) for r in other] == sorted(int(r[0]) for r in other)   # sequence-major
    with pytest.raises(A.HspmdError):
        A.schedule(kind, cu, cfg.q_heads, cfg.kv_heads, 8, order=7)


def test_work_list_gqa_heads_of_one_tile_are_adjacent():
    cu, _, _ = A.build_cu_seqlens([1000, 3000])
    items = A.schedule(A.LIST_FWD, cu, 8, 2, 8)
    for x in range(8):
        q = items[x::8]
        q = q[q[:, 2] >= 0]
        # consecutive items of a queue that share (sequence, tile) walk through the heads of one KV group
        for a, b in zip(q[:-1], q[1:]):
            if a[0] == b[0] and a[2] == b[2]:
                assert a[3] // 4 == b[3] // 4


def test_work_list_single_long_sequence_is_spread():
    # one sequence, one head: the chain must be cut so that all 8 queues get work
    cu, _, _ = A.build_cu_seqlens([32768])
    for kind in (A.LIST_FWD, A.LIST_DKV):
        items = A.schedule(kind, cu, 1, 1, 8)
        loads = np.zeros(8)
        for p, r in enumerate(items):
            if r[2] >= 0:
                loads[p % 8] += _cost(kind, int(r[1]), int(r[2]), 1)
        assert loads.min() > 0.8 * loads.mean(), loads


def test_work_list_empty_and_zero_length():
    assert A.schedule(A.LIST_FWD, [0], 4, 4).shape == (0, 4)
    assert A.schedule(A.LIST_DKV, [0, 0, 0], 4, 2).shape == (0, 4)
    items = A.schedule(A.LIST_FWD, [0, 0, 5, 5], 1, 1, 8)
    real = items[items[:, 2] >= 0]
    assert real.tolist() == [[0, 5, 0, 0]]


def test_schedule_rejects_bad_arguments():
    for bad, frag in ((dict(cu=[0, 4], hq=3, hkv=2), "multiple"), (dict(cu=[1, 4], hq=2, hkv=2), "cu_seqlens[0]"),
                      (dict(cu=[0, 4, 3], hq=2, hkv=2), "non-decreasing"), (dict(cu=[0, 4], hq=0, hkv=1), "positive")):
        with pytest.raises(A.HspmdError) as e:
            A.schedule(A.LIST_FWD, bad["cu"], bad["hq"], bad["hkv"])
        assert e.value.status == 1 and frag in str(e.value)
    with pytest.raises(A.HspmdError):
        A.schedule(7, [0, 4], 2, 2)
    with pytest.raises(A.HspmdError):
        A.schedule(A.LIST_FWD, [0, 4], 2, 2, num_queues=0)
    # capacity too small: nothing written, INVALID_ARG, count still reported
    lib = A.load_library()
    cu = np.array([0, 300], dtype=np.int32)
    n = ctypes.c_int64(0)
    from paper_2504_20490_amd.binding import WorkItem
    buf = (WorkItem * 2)()
    rc = lib.hspmd_attn_schedule(0, cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), 1, 2, 2, 8, buf, 2, ctypes.byref(n))
    assert rc == 1 and n.value == 8


def test_plan_create_validates_before_touching_the_gpu():
    lib = A.load_library()
    cu = np.array([0, 8], dtype=np.int32)
    p = cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    out = ctypes.c_void_p()
    assert lib.hspmd_attn_plan_create(p, 1, 2, 2, 100, None, ctypes.byref(out)) == 2      # head_dim 100: UNSUPPORTED
    assert b"head_dim" in lib.hspmd_last_error()
    assert lib.hspmd_attn_plan_create(p, 1, 3, 2, 128, None, ctypes.byref(out)) == 1      # 3 q heads on 2 kv heads
    assert lib.hspmd_attn_plan_create(p, 1, 2, 2, 128, None, None) == 1
    assert out.value is None
    assert lib.hspmd_attn_plan_destroy(None) == 0
    assert lib.hspmd_attn_varlen_fwd(None, None, None, None, 0, 0, 0.0, None, None, None) == 1
    assert lib.hspmd_attn_plan_total_tokens(None) == -1 and lib.hspmd_attn_bwd_workspace_bytes(None) == 0


# ------------------------------------------------------------------------------ block variant (host logic)
def _block_cost(kind, it, group):
    """Inner steps of a block item, from the definition: key j visible to row r iff j <= r + offset."""
    q_len, k_len, off, tile = int(it[1]), int(it[3]), int(it[4]), int(it[5])
    if kind == A.LIST_DKV:
        rows = [r for r in range(q_len) if r + off >= tile * 128]          # rows that see the tile's first key
        if tile * 128 >= k_len or not rows:
            return 0
        return (-(-q_len // 64) - rows[0] // 64) * group
    last = min(q_len, (tile + 1) * 128) - 1
    keys = max(0, min(k_len, last + off + 1))
    return -(-keys // 64) if tile * 128 < q_len else 0


@pytest.mark.parametrize("kind", [A.LIST_FWD, A.LIST_DQ, A.LIST_DKV])
def test_block_work_list_invariants(kind):
    ql = [300, 129, 64, 200, 0, 77, 1, 2000]
    kl = [200, 257, 130, 128, 90, 0, 300, 1500]
    qp = [100, 0, 700, 0, 5, 9, 299, 1000]
    kp = [0, 64, 0, 200, 0, 0, 0, 0]
    cq, ck = np.concatenate([[0], np.cumsum(ql)]), np.concatenate([[0], np.cumsum(kl)])
    hq, hkv = 4, 2
    items = A.block_schedule(kind, cq, ck, qp, kp, hq, hkv)
    assert items.shape[1] == 8 and items.shape[0] % 8 == 0
    real = items[items[:, 5] >= 0]
    assert np.all(items[items[:, 5] < 0][:, 5] == -1)
    q_pos_of = {(int(cq[i]), ql[i], int(ck[i]), kl[i]): qp[i] for i in range(len(ql))}     # the chunk's position travels with the item
    assert all(int(r[7]) == q_pos_of[(int(r[0]), int(r[1]), int(r[2]), int(r[3]))] for r in real)
    # every tile that owns output rows appears exactly once per head, with its sequence's geometry
    expected = set()
    for i in range(len(ql)):
        rows, per = (kl[i], 128) if kind == A.LIST_DKV else (ql[i], 128)
        heads = hkv if kind == A.LIST_DKV else hq
        for t in range(-(-rows // per)):
            for h in range(heads):
                expected.add((int(cq[i]), ql[i], int(ck[i]), kl[i], qp[i] - kp[i], t, h))
    got = [tuple(int(x) for x in r[:7]) for r in real]
    assert len(got) == len(set(got)) and set(got) == expected
    # queues (slots p % 8) are balanced by the cost from the definition
    group = hq // hkv
    loads = [sum(_block_cost(kind, it, group) for it in items[x::8] if it[5] >= 0) for x in range(8)]
    heaviest = max(_block_cost(kind, it, group) for it in real)
    assert max(loads) - min(loads) <= max(heaviest, sum(loads) // 32 + heaviest)


def test_block_schedule_without_shift_matches_the_packed_schedule():
    lengths = [300, 0, 1000, 64]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    for kind in (A.LIST_FWD, A.LIST_DQ, A.LIST_DKV):
        packed = A.schedule(kind, cu, 4, 2)
        block = A.block_schedule(kind, cu, cu, [0] * 4, [0] * 4, 4, 2)
        assert packed.shape[0] == block.shape[0]
        real = block[:, 5] >= 0
        assert np.array_equal(real, packed[:, 2] >= 0)
        assert np.array_equal(block[real][:, [0, 1, 5, 6]], packed[real])
        assert np.array_equal(block[real][:, [2, 3]], packed[real][:, [0, 1]]) and np.all(block[real][:, 4] == 0)


def test_block_schedule_rejects_bad_arguments():
    ok = ([0, 10], [0, 12], [3], [0], 2, 2)
    A.block_schedule(A.LIST_FWD, *ok)
    for bad in [([0, 10], [0, 12], [-1], [0], 2, 2), ([0, 10], [0, 12], [0], [-2], 2, 2),
                ([1, 10], [0, 12], [0], [0], 2, 2), ([0, 10], [0, 12, 11], [0, 0], [0, 0], 2, 2),
                ([0, 10], [0, 12], [0], [0], 3, 2), ([0, 10], [0, 12], [0], [0], 0, 0),
                ([0, 10], [0, 12], [2 ** 30], [0], 2, 2)]:
        with pytest.raises(A.HspmdError):
            A.block_schedule(A.LIST_FWD, *bad)
    with pytest.raises(A.HspmdError):
        A.block_schedule(A.LIST_FWD, [0, 10], [0, 12], [0, 0], [0], 2, 2)      # arrays differ in length
    with pytest.raises(A.HspmdError):
        A.block_schedule(7, *ok)


def test_block_work_list_of_an_invisible_block_is_spread_over_the_queues():
    """Key chunk wholly in the future: every item only writes zeros (cost 0), and the list must not grow."""
    cq = [0, 3000]
    items = A.block_schedule(A.LIST_FWD, cq, [0, 3000], [0], [5000], 4, 2)
    real = int((items[:, 5] >= 0).sum())
    assert real == 24 * 4 and items.shape[0] <= real + 8


def test_forward_and_dq_lists_are_the_same_list():
    """A plan keeps one device copy for both passes: the two lists must agree slot by slot, in every order."""
    cu = np.concatenate([[0], np.cumsum([700, 0, 3000, 129, 64])])
    for order in (A.ORDER_XCD_COST, A.ORDER_NATURAL, A.ORDER_COST):
        assert np.array_equal(A.schedule(A.LIST_FWD, cu, 6, 2, order=order), A.schedule(A.LIST_DQ, cu, 6, 2, order=order))
    assert np.array_equal(A.block_schedule(A.LIST_FWD, cu, cu[::-1].cumsum() * 0 + cu, [5, 0, 100, 0, 7], [0, 0, 0, 9, 7], 6, 2),
                          A.block_schedule(A.LIST_DQ, cu, cu, [5, 0, 100, 0, 7], [0, 0, 0, 9, 7], 6, 2))


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share on one GPU; asked for more it exits with a message and no JSON line."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_plan_update_rejects_bad_arguments_without_a_gpu():
    lib = A.load_library()
    cu = np.array([0, 5], dtype=np.int32)
    p32 = cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    assert lib.hspmd_attn_plan_update(None, p32, 1) == 1
    assert b"NULL" in lib.hspmd_last_error()
    assert lib.hspmd_attn_block_plan_update(None, p32, p32, p32, p32, 1) == 1
