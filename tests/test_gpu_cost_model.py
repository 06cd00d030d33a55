"""The cost model's prediction against measured kernel times on the GPU at hand."""
import numpy as np
import pytest

import hspmd_workloads as w

pytestmark = pytest.mark.gpu


def _measured_ms(lengths, hq, hkv, d):
    import torch
    import paper_2504_20490_amd as A
    T = sum(lengths)
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    mk = lambda h: torch.randn(T, h, d, device="cuda", generator=g).to(torch.bfloat16)
    q, k, v, do = mk(hq), mk(hkv), mk(hkv), mk(hq)
    o = torch.empty_like(q)
    lse = torch.empty(hq, T, dtype=torch.float32, device="cuda")
    dq = torch.empty(T, hq, d, dtype=torch.float32, device="cuda")
    dk = torch.empty(T, hkv, d, dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    cu, _, _ = A.build_cu_seqlens(lengths)
    plan = A.Plan(cu, hq, hkv, d)
    ws = torch.empty(plan.bwd_workspace_bytes(), dtype=torch.uint8, device="cuda")

    def step():
        A.attn_varlen_fwd(plan, q, k, v, o, lse)
        A.attn_varlen_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws, grad_dtype=A.GRAD_F32)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    A.profile_enable(True)
    for _ in range(6):
        step()
    torch.cuda.synchronize()
    A.profile_enable(False)
    t = {name: ms / n for name, (ms, n) in A.profile_read().items()}
    return t["fwd_kernel"], t["bwd_dq_kernel"] + t["bwd_dkv_kernel"], cu


@pytest.mark.parametrize("name,tolerance", [("C3", 0.15), ("C4", 0.15), ("C5", 0.15), ("C2", 0.30)])
def test_prediction_matches_measurement(name, tolerance):
    """The long-tailed packs (milliseconds of work) to 15 %, the small uniform one to 30 %."""
    import paper_2504_20490_amd as A
    cfg = w.config_by_name(name)
    fwd, bwd, cu = _measured_ms(w.lengths_for(cfg), cfg.q_heads, cfg.kv_heads, cfg.head_dim)
    pf, pb = A.estimate_ms(cu, cfg.q_heads, cfg.kv_heads, cfg.head_dim)
    assert abs(pf / fwd - 1.0) <= tolerance, (pf, fwd)
    assert abs(pb / bwd - 1.0) <= tolerance, (pb, bwd)


def test_prediction_ranks_packs_like_the_measurement():
    """What a planner needs first: of two candidate packs the one predicted cheaper is the one measured cheaper."""
    import paper_2504_20490_amd as A
    packs = [[8192] * 2, [2048] * 8, [512] * 32, [16384], [1000, 3000, 12000]]
    measured, predicted = [], []
    for lens in packs:
        f, b, cu = _measured_ms(lens, 16, 16, 128)
        pf, pb = A.estimate_ms(cu, 16, 16, 128)
        measured.append(f + b)
        predicted.append(pf + pb)
    assert list(np.argsort(measured)) == list(np.argsort(predicted))
