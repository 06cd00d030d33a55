"""Refilling a plan with the next pack (hspmd_attn_plan_update / hspmd_attn_block_plan_update): the lists are rebuilt on
the host and uploaded into device storage the plan already owns, while launches that read the previous lists may still
be running.  Results must equal those of a freshly created plan bit for bit, and match the oracle; in the steady state
the device's free memory must not move."""
import numpy as np
import pytest

import oracle
import gpu_util
from gpu_util import LSE_ABS, assert_close, default_scale, f64, make_case, to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.contiguous().view(torch.int32 if t.element_size() == 4 else torch.int16).cpu().numpy()


class _Buffers:
    def __init__(self, lengths, hq, hkv, d, seed):
        import torch
        self.lengths = lengths
        T = sum(lengths)
        self.bits = make_case(lengths, hq, hkv, d, seed)
        self.q, self.k, self.v, self.do = (to_dev(x) for x in self.bits)
        self.o = torch.full((T, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.full((hq, T), float("nan"), dtype=torch.float32, device="cuda")
        self.dq = torch.full((T, hq, d), float("nan"), dtype=torch.float32, device="cuda")
        self.dk = torch.full((T, hkv, d), float("nan"), dtype=torch.float32, device="cuda")
        self.dv = torch.full((T, hkv, d), float("nan"), dtype=torch.float32, device="cuda")
        self.ws = torch.empty(2 * hq * T * 4 + 64, dtype=torch.uint8, device="cuda")

    def launch(self, A, plan):
        A.attn_varlen_fwd(plan, self.q, self.k, self.v, self.o, self.lse)
        A.attn_varlen_bwd(plan, self.q, self.k, self.v, self.o, self.lse, self.do, self.dq, self.dk, self.dv, self.ws,
                          grad_dtype=A.GRAD_F32)

    def results(self):
        return {n: _bits(getattr(self, n)) for n in ("o", "lse", "dq", "dk", "dv")}


def test_refilled_plan_equals_fresh_plan_and_oracle():
    import torch
    import paper_2504_20490_amd as A
    hq, hkv, d = 4, 2, 128
    packs = [[300, 41, 1000, 7], [64, 2000, 1, 129], [5], [900, 900, 900, 33, 0, 512], [17, 64, 111], [1500, 300]]
    bufs = [_Buffers(L, hq, hkv, d, 700 + i) for i, L in enumerate(packs)]
    # reference: a fresh plan per pack
    fresh = []
    for b in bufs:
        cu, _, _ = A.build_cu_seqlens(b.lengths)
        plan = A.Plan(cu, hq, hkv, d)
        b.launch(A, plan)
        torch.cuda.synchronize()
        fresh.append(b.results())
        plan.destroy()
        for t in (b.o, b.lse, b.dq, b.dk, b.dv):
            t.fill_(float("nan"))
    # one plan, refilled pack after pack WITHOUT waiting for the launches of the packs before
    cu, _, _ = A.build_cu_seqlens(bufs[0].lengths)
    plan = A.Plan(cu, hq, hkv, d)
    bufs[0].launch(A, plan)
    for b in bufs[1:]:
        cu, _, total = A.build_cu_seqlens(b.lengths)
        plan.update(cu)
        assert plan.total_tokens == total
        b.launch(A, plan)
    torch.cuda.synchronize()
    for i, b in enumerate(bufs):
        got = b.results()
        for n in got:
            assert np.array_equal(got[n], fresh[i][n]), f"pack {i}: {n} differs from the fresh plan's result"
    # and the last refill against the oracle
    b = bufs[-1]
    gpu_util.CONTEXT["case"] = "refilled plan"
    q, k, v, do = (f64(x) for x in b.bits)
    s = default_scale(d)
    ro, rlse = oracle.attn_fwd(q, k, v, b.lengths, s)
    rdq, rdk, rdv = oracle.attn_bwd(q, k, v, do, b.lengths, s)
    assert_close("O", b.o.float().cpu().numpy().astype(np.float64), ro)
    assert np.max(np.abs(b.lse.cpu().numpy() - rlse)) <= LSE_ABS
    assert_close("dQ", b.dq.cpu().numpy().astype(np.float64), rdq)
    assert_close("dK", b.dk.cpu().numpy().astype(np.float64), rdk)
    assert_close("dV", b.dv.cpu().numpy().astype(np.float64), rdv)
    plan.destroy()


def test_steady_state_refills_do_not_allocate():
    import torch
    import paper_2504_20490_amd as A
    hq, hkv, d = 4, 4, 64
    lengths_a, lengths_b = [700, 45, 260, 1, 129], [600, 100, 300, 135]     # similar sizes: b fits the headroom of a
    ba, bb = _Buffers(lengths_a, hq, hkv, d, 801), _Buffers(lengths_b, hq, hkv, d, 802)
    cu_a, _, _ = A.build_cu_seqlens(lengths_a)
    cu_b, _, _ = A.build_cu_seqlens(lengths_b)
    plan = A.Plan(cu_a, hq, hkv, d)
    for i in range(8):                      # every slot of the ring has been sized by now
        plan.update(cu_b if i % 2 == 0 else cu_a)
        (bb if i % 2 == 0 else ba).launch(A, plan)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for i in range(30):
        plan.update(cu_b if i % 2 == 0 else cu_a)
        (bb if i % 2 == 0 else ba).launch(A, plan)
    free_after, _ = torch.cuda.mem_get_info()
    torch.cuda.synchronize()
    assert free_after == free_before, (free_before, free_after)
    # an empty pack and a rejected pack leave the plan usable
    plan.update([0])
    assert plan.total_tokens == 0
    with pytest.raises(A.HspmdError):
        plan.update([0, 5, 3])              # not non-decreasing
    assert plan.total_tokens == 0
    plan.update(cu_a)
    ba.launch(A, plan)
    torch.cuda.synchronize()
    assert not torch.isnan(ba.dk).any()
    plan.destroy()


def test_block_plan_refill_equals_fresh_block_plan():
    import torch
    import paper_2504_20490_amd as A
    hq, hkv, d = 4, 2, 128
    geoms = [([200, 64], [300, 10], [300, 0], [0, 0]), ([128, 1], [128, 500], [0, 499], [0, 0]),
             ([77, 300], [77, 300], [0, 0], [0, 0])]

    def run(plan, ql, kl, seed):
        Tq, Tk = sum(ql), sum(kl)
        q = to_dev(make_case(ql, hq, hkv, d, seed)[0])
        k, v = (to_dev(x) for x in make_case(kl, hq, hkv, d, seed + 1)[1:3])
        o = torch.full((Tq, hq, d), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((hq, Tq), float("nan"), dtype=torch.float32, device="cuda")
        A.attn_block_fwd(plan, q, k, v, o, lse)
        return o, lse

    cuof = lambda ls: np.concatenate([[0], np.cumsum(ls)]).astype(np.int32)
    fresh = []
    for i, (ql, kl, qp, kp) in enumerate(geoms):
        plan = A.BlockPlan(cuof(ql), cuof(kl), qp, kp, hq, hkv, d)
        o, lse = run(plan, ql, kl, 900 + 2 * i)
        torch.cuda.synchronize()
        fresh.append((_bits(o), _bits(lse)))
        plan.destroy()
    ql, kl, qp, kp = geoms[0]
    plan = A.BlockPlan(cuof(ql), cuof(kl), qp, kp, hq, hkv, d)
    outs = [run(plan, ql, kl, 900)]
    for i, (ql, kl, qp, kp) in enumerate(geoms[1:], start=1):
        plan.update(cuof(ql), cuof(kl), qp, kp)
        assert plan.total_tokens == sum(ql) and plan.total_kv_tokens == sum(kl)
        outs.append(run(plan, ql, kl, 900 + 2 * i))
    torch.cuda.synchronize()
    for i, (o, lse) in enumerate(outs):
        assert np.array_equal(_bits(o), fresh[i][0]) and np.array_equal(_bits(lse), fresh[i][1]), f"block geometry {i}"
    plan.destroy()
