"""Forward + backward (and the rotary-embedding calls) recorded into a HIP graph and replayed.

The compute entry points only enqueue kernels on the caller's stream and allocate nothing, so a caller may capture
them.  Every replay is checked bit for bit against eager calls on the same inputs, with the inputs changed and
eager work and synchronisations between the replays."""
import numpy as np
import pytest

from gpu_util import make_case, to_dev

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.contiguous().view(torch.int32 if t.element_size() == 4 else torch.int16).cpu().numpy()


@pytest.mark.parametrize("rope", [False, True])
def test_graph_replays_match_eager_calls(rope):
    import torch
    import paper_2504_20490_amd as A
    lengths, hq, hkv, d = [700, 45, 260, 1, 129], 4, 2, 128
    T = sum(lengths)
    cu, _, _ = A.build_cu_seqlens(lengths)
    plan = A.Plan(cu, hq, hkv, d)                        # plans are made outside the capture: creating one allocates
    positions = max(lengths)
    table = torch.empty(positions, d // 2, 2, dtype=torch.float32, device="cuda")
    A.rope_table(table, positions, d)

    def buffers():
        return dict(qr=torch.empty(T, hq, d, dtype=torch.bfloat16, device="cuda"),
                    kr=torch.empty(T, hkv, d, dtype=torch.bfloat16, device="cuda"),
                    o=torch.empty(T, hq, d, dtype=torch.bfloat16, device="cuda"),
                    lse=torch.empty(hq, T, dtype=torch.float32, device="cuda"),
                    dq=torch.empty(T, hq, d, dtype=torch.float32, device="cuda"),
                    dk=torch.empty(T, hkv, d, dtype=torch.float32, device="cuda"),
                    dv=torch.empty(T, hkv, d, dtype=torch.float32, device="cuda"),
                    ws=torch.empty(plan.bwd_workspace_bytes(), dtype=torch.uint8, device="cuda"))

    q0, k0, v0, do0 = (to_dev(x) for x in make_case(lengths, hq, hkv, d, seed=900))
    q, k, v, do = q0.clone(), k0.clone(), v0.clone(), do0.clone()     # the graph's inputs, refilled between replays

    def calls(b):
        if rope:
            A.rope_qk(plan, q, k, b["qr"], b["kr"], table, positions)
            A.attn_varlen_fwd(plan, b["qr"], b["kr"], v, b["o"], b["lse"])
            A.attn_varlen_bwd_rope(plan, b["qr"], b["kr"], v, b["o"], b["lse"], do, b["dq"], b["dk"], b["dv"], b["ws"],
                                   table, positions, grad_dtype=A.GRAD_F32)
        else:
            A.attn_varlen_fwd(plan, q, k, v, b["o"], b["lse"])
            A.attn_varlen_bwd(plan, q, k, v, b["o"], b["lse"], do, b["dq"], b["dk"], b["dv"], b["ws"],
                              grad_dtype=A.GRAD_F32)

    captured, eager = buffers(), buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls(captured)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls(captured)                                   # stream=None -> torch's current stream = the capturing one
    names = ("o", "lse", "dq", "dk", "dv")
    for replay in range(3):
        if replay:
            new = make_case(lengths, hq, hkv, d, seed=900 + replay)
            for dst, src in zip((q, k, v, do), new):
                dst.copy_(to_dev(src))
        for n in names:
            captured[n].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        calls(eager)                                      # eager work between the replays
        torch.cuda.synchronize()
        for n in names:
            assert np.array_equal(_bits(captured[n]), _bits(eager[n])), f"replay {replay}: {n} differs from the eager result"
            assert not torch.isnan(captured[n].float()).any()
