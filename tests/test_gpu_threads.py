"""Two host threads use the library at the same time, each with its own plans, stream and workspace.

The library's shared state (the copy stream that uploads work lists, the error string, the profiling switch) must not
couple them: every thread's results are bit-identical to the ones a single thread gets for the same inputs."""
import threading

import numpy as np
import pytest

from gpu_util import make_case, to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.contiguous().view(torch.int32 if t.element_size() == 4 else torch.int16).cpu().numpy()


def _run(case, stream, rounds):
    """`rounds` times: new plan + forward + backward on `stream`; returns the last round's results as bit patterns."""
    import torch
    import paper_2504_20490_amd as A
    lengths, hq, hkv, d, seed = case
    T = sum(lengths)
    q, k, v, do = (to_dev(x) for x in make_case(lengths, hq, hkv, d, seed=seed))
    o = torch.empty(T, hq, d, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(hq, T, dtype=torch.float32, device="cuda")
    dq = torch.empty(T, hq, d, dtype=torch.float32, device="cuda")
    dk = torch.empty(T, hkv, d, dtype=torch.float32, device="cuda")
    dv = torch.empty(T, hkv, d, dtype=torch.float32, device="cuda")
    cu, _, _ = A.build_cu_seqlens(lengths)
    with torch.cuda.stream(stream):
        for _ in range(rounds):
            plan = A.Plan(cu, hq, hkv, d)                       # uploads its lists through the shared copy stream
            ws = torch.empty(plan.bwd_workspace_bytes(), dtype=torch.uint8, device="cuda")
            for t in (o, lse, dq, dk, dv):
                t.fill_(float("nan"))
            A.attn_varlen_fwd(plan, q, k, v, o, lse, stream=stream)
            A.attn_varlen_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws, grad_dtype=A.GRAD_F32, stream=stream)
            stream.synchronize()                                # the plan and the workspace die with this round
    return {n: _bits(t) for n, t in (("o", o), ("lse", lse), ("dq", dq), ("dk", dk), ("dv", dv))}


def test_two_threads_with_their_own_streams():
    import torch
    cases = [([700, 45, 260, 1, 129, 1500], 4, 2, 128, 41), ([333, 64, 2048, 17], 6, 6, 64, 42)]
    torch.cuda.synchronize()
    alone = [_run(c, torch.cuda.Stream(), 1) for c in cases]
    for a in alone:
        assert not any(np.isnan(w.view(np.float32)).any() for n, w in a.items() if n != "o")

    results, errors = [None, None], []

    def worker(i):
        try:
            torch.cuda.set_device(0)
            results[i] = _run(cases[i], torch.cuda.Stream(), 20)
        except BaseException as e:                              # noqa: BLE001 - reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=240)
    assert not any(t.is_alive() for t in threads), "a worker thread did not finish"
    assert not errors, errors
    for i in range(2):
        for name in alone[i]:
            assert np.array_equal(results[i][name], alone[i][name]), f"thread {i}: {name} differs from the single-thread result"
