"""The backward entry point that allocates nothing (hspmd_attn_varlen_bwd_static_ws: the row statistics go into a
fixed device array inside the library) against hspmd_attn_varlen_bwd with a caller's workspace, through the C ABI:
same kernels, so the gradients must agree bit for bit; two calls in a row, the second on a smaller pack (the array
keeps the first call's contents); the device's free memory must not move; the size limit is enforced."""
import numpy as np
import pytest

from gpu_util import make_case, to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.contiguous().view(torch.int32 if t.element_size() == 4 else torch.int16).cpu().numpy()


def _case(A, lengths, hq, hkv, d, seed, grad_dtype):
    import torch
    T = sum(lengths)
    q, k, v, do = (to_dev(x) for x in make_case(lengths, hq, hkv, d, seed))
    cu, _, _ = A.build_cu_seqlens(lengths)
    plan = A.Plan(cu, hq, hkv, d)
    o = torch.empty(T, hq, d, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(hq, T, dtype=torch.float32, device="cuda")
    A.attn_varlen_fwd(plan, q, k, v, o, lse)
    gd = torch.float32 if grad_dtype == A.GRAD_F32 else torch.bfloat16
    grads = lambda: [torch.full(s, float("nan"), dtype=gd, device="cuda") for s in ((T, hq, d), (T, hkv, d), (T, hkv, d))]
    ws = torch.empty(plan.bwd_workspace_bytes(), dtype=torch.uint8, device="cuda")
    return plan, (q, k, v, o, lse, do), grads(), grads(), ws


def test_static_workspace_backward_equals_the_workspace_backward():
    import torch
    import paper_2504_20490_amd as A
    # first call: several tiles, GQA, ragged lengths; second call: a smaller pack, other head counts and head_dim
    cases = [([700, 45, 260, 1, 129, 1500], 4, 2, 128, 41, A.GRAD_F32), ([130, 64, 17], 3, 3, 64, 42, A.GRAD_BF16)]
    prepared = [_case(A, *c) for c in cases]
    for plan, (q, k, v, o, lse, do), ref, _, ws in prepared:
        A.attn_varlen_bwd(plan, q, k, v, o, lse, do, *ref, ws, grad_dtype=(A.GRAD_F32 if ref[0].dtype == torch.float32 else A.GRAD_BF16))
    torch.cuda.synchronize()

    def two_calls():
        for plan, (q, k, v, o, lse, do), _, got, _ in prepared:          # two calls in a row on one stream
            A.attn_varlen_bwd_static_ws(plan, q, k, v, o, lse, do, *got,
                                        grad_dtype=(A.GRAD_F32 if got[0].dtype == torch.float32 else A.GRAD_BF16))

    def check(what):
        for i, (_, _, ref, got, _) in enumerate(prepared):
            for name, a, b in zip(("dq", "dk", "dv"), ref, got):
                assert not torch.isnan(b.float()).any(), f"{what}, call {i}: {name} holds unwritten elements"
                assert np.array_equal(_bits(a), _bits(b)), f"{what}, call {i}: {name} differs from the workspace entry point's"

    two_calls()        # the very first call on the device also looks up the array's address (the runtime may place the
    torch.cuda.synchronize()   # library's device data only then)
    check("first round")
    for _, _, _, got, _ in prepared:
        for t in got:
            t.fill_(float("nan"))
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    two_calls()
    free_after, _ = torch.cuda.mem_get_info()
    torch.cuda.synchronize()
    assert free_after == free_before, (free_before, free_after)      # nothing allocated, nothing freed
    check("second round")


def test_static_workspace_limit_and_validation():
    import torch
    import paper_2504_20490_amd as A
    # 2^21 (head, token) pairs fit exactly; one more token does not
    hq = 32
    fits = A.Plan(np.array([0, 65536], dtype=np.int32), hq, 8, 128)
    assert fits.bwd_workspace_bytes() <= A.STATIC_WORKSPACE_BYTES
    over = A.Plan(np.array([0, 65537], dtype=np.int32), hq, 8, 128)
    assert over.bwd_workspace_bytes() > A.STATIC_WORKSPACE_BYTES
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(A.HspmdError) as e:
        A.attn_varlen_bwd_static_ws(over, dummy, dummy, dummy, dummy, dummy, dummy, dummy, dummy, dummy)
    assert e.value.status == 3 and "HSPMD_STATIC_WORKSPACE_BYTES" in str(e.value)
    plan, (q, k, v, o, lse, do), _, got, _ = _case(A, [40], 2, 2, 128, 43, A.GRAD_F32)
    with pytest.raises(A.HspmdError) as e:
        A.attn_varlen_bwd_static_ws(plan, q.view(-1)[1:], k, v, o, lse, do, *got, grad_dtype=A.GRAD_F32)   # misaligned q
    assert e.value.status == 1
    A.attn_varlen_bwd_static_ws(plan, q, k, v, o, lse, do, *got, grad_dtype=A.GRAD_F32)    # still usable
    torch.cuda.synchronize()
    assert not any(torch.isnan(t).any() for t in got)
