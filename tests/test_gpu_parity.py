"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded bf16 inputs, element by element.  Tolerances: max-abs 2e-2 and relative Frobenius 1e-2
for O, dQ, dK, dV (bf16 inputs, fp32 accumulation); LSE to 1e-3 absolute."""
import numpy as np
import pytest

import hspmd_workloads as w
import oracle
import gpu_util
from gpu_util import (GpuRun, LSE_ABS, assert_close, default_scale, f64, make_case, to_dev)

pytestmark = pytest.mark.gpu

RAGGED = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 0, 300]


def _full_check(lengths, hq, hkv, d, seed, value_scale=1.0, grad_dtype=None, scale=0.0, magnitude_slack=False,
                slack_roundings=1):
    gpu_util.CONTEXT["case"] = f"small pack {len(lengths)} seqs Hq{hq} Hkv{hkv} d{d} seed{seed}"
    q, k, v, do = make_case(lengths, hq, hkv, d, seed, value_scale)
    run = GpuRun(lengths, q, k, v, do, grad_dtype=grad_dtype, scale=scale).run()
    s = scale if scale > 0 else default_scale(d)
    ro, rlse = oracle.attn_fwd(f64(q), f64(k), f64(v), lengths, s)
    rdq, rdk, rdv = oracle.attn_bwd(f64(q), f64(k), f64(v), f64(do), lengths, s)
    # magnitude_slack: packs outside the benchmark configurations' value range (several query heads per KV head and
    # hundreds of rows push |dK|, |dV| above 10; scaled inputs push |O| above 8, where half a bf16 ulp is 0.03) may add
    # the bf16 rounding of P / dS / O at that magnitude to the max-abs bound -- but only for a tensor whose reference
    # really reaches magnitude 8 (gpu_util.magnitude_bound); every other tensor is held to the nominal bound
    # (slack_roundings: how many such roundings, P, dS and the bf16 operands among them, may line up in one element)
    bound = (lambda ref: gpu_util.magnitude_bound(ref, slack_roundings)) if magnitude_slack else (lambda ref: gpu_util.MAX_ABS)
    assert_close("O", run.host("o"), ro, max_abs=bound(ro))
    lse_peak = float(np.max(np.abs(rlse))) if rlse.size else 0.0
    assert np.max(np.abs(run.host("lse") - rlse)) <= LSE_ABS * (lse_peak / 8.0 if magnitude_slack and lse_peak >= 8.0 else 1.0)
    assert_close("dQ", run.host("dq"), rdq, max_abs=bound(rdq))
    assert_close("dK", run.host("dk"), rdk, max_abs=bound(rdk))
    assert_close("dV", run.host("dv"), rdv, max_abs=bound(rdv))
    gpu_util.CONTEXT["slack"] = None
    return run


def test_random_packs():
    """Thirty small packs with random lengths (including 0 and 1), head counts, group sizes and head dims (seeded)."""
    rng = np.random.default_rng(4242)
    for case in range(30):
        n = int(rng.integers(1, 7))
        lengths = [int(x) for x in rng.choice([0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 400, 640], n)]
        if sum(lengths) == 0:
            lengths[0] = 3
        hkv = int(rng.integers(1, 4))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([64, 128, 104, 80]))
        _full_check(lengths, hq, hkv, d, seed=500 + case, magnitude_slack=True)


def test_c1_tiny_pack():
    cfg = w.config_by_name("C1")
    gpu_util.CONTEXT["case"] = cfg.name
    lengths, q, k, v, do = w.make_inputs(cfg)
    assert lengths == [17, 64, 111]
    run = GpuRun(lengths, q, k, v, do).run()
    s = default_scale(cfg.head_dim)
    ro, rlse = oracle.attn_fwd(f64(q), f64(k), f64(v), lengths, s)
    rdq, rdk, rdv = oracle.attn_bwd(f64(q), f64(k), f64(v), f64(do), lengths, s)
    assert_close("O", run.host("o"), ro)
    assert np.max(np.abs(run.host("lse") - rlse)) <= LSE_ABS
    assert_close("dQ", run.host("dq"), rdq)
    assert_close("dK", run.host("dk"), rdk)
    assert_close("dV", run.host("dv"), rdv)


@pytest.mark.parametrize("hq,hkv,d", [(3, 3, 128), (4, 1, 128), (6, 2, 64), (1, 1, 64), (24, 24, 128)])
def test_ragged_lengths_span_tiles_and_tails(hq, hkv, d):
    lengths = RAGGED if hq < 24 else [1, 129, 0, 77]
    _full_check(lengths, hq, hkv, d, seed=11 + hq)


@pytest.mark.parametrize("hq,hkv,d", [(4, 4, 104), (4, 2, 104), (2, 2, 40), (3, 1, 120), (2, 2, 8), (2, 2, 112), (2, 1, 96),
                                      (2, 2, 88)])
def test_head_dims_between_the_tile_widths(hq, hkv, d):
    """head_dim 104 is the paper's 32B model (hidden 6656 over 64 heads); any multiple of 8 runs on the next tile
    width up.  Outputs are written NaN-filled beforehand, so a column that the kernels leave out would show.
    Up to 112 the kernels of width 128 contract over seven 16-column steps instead of eight (104, 112 and 96, 88: the
    seventh step is then partly or wholly padding); 120 takes all eight."""
    _full_check(RAGGED, hq, hkv, d, seed=30 + d)


def test_head_dim_104_long_sequences_and_strided_views():
    """16 of the 64 heads of the paper's 32B model (a 4-way split of the hidden dimension), one sequence long enough
    for every loop variant, q / k / v as views into one fused QKV buffer."""
    import torch
    lengths, hq, hkv, d = [3000, 333], 16, 16, 104
    q, k, v, do = make_case(lengths, hq, hkv, d, seed=77)
    T = sum(lengths)
    fused = torch.zeros(T, (hq + 2 * hkv) * d, dtype=torch.bfloat16, device="cuda")
    qv = fused[:, : hq * d].view(T, hq, d)
    kv = fused[:, hq * d: (hq + hkv) * d].view(T, hkv, d)
    vv = fused[:, (hq + hkv) * d:].view(T, hkv, d)
    qv.copy_(to_dev(q)); kv.copy_(to_dev(k)); vv.copy_(to_dev(v))
    gpu_util.CONTEXT["case"] = "d104_long"
    run = GpuRun(lengths, q, k, v, do, q_dev=qv, k_dev=kv, v_dev=vv).run()
    s = default_scale(d)
    rows = np.array([0, 1, 127, 128, 2999, 3000, 3332, 1500], dtype=np.int32)
    heads = np.array([0, 15, 7, 3, 15, 0, 9, 8], dtype=np.int32)
    ro, rlse, rdq = oracle.attn_rows(f64(q), f64(k), f64(v), f64(do), lengths, s, rows, heads)
    assert_close("O rows", run.host("o")[rows, heads], ro)
    assert np.max(np.abs(run.host("lse")[heads, rows] - rlse)) <= LSE_ABS
    assert_close("dQ rows", run.host("dq")[rows, heads], rdq)
    keys = np.array([0, 5, 2999, 3000, 3332, 64], dtype=np.int32)
    kvh = np.array([0, 15, 2, 9, 15, 4], dtype=np.int32)
    rdk, rdv = oracle.attn_keys(f64(q), f64(k), f64(v), f64(do), lengths, s, keys, kvh)
    assert_close("dK keys", run.host("dk")[keys, kvh], rdk)
    assert_close("dV keys", run.host("dv")[keys, kvh], rdv)
    assert not np.isnan(run.host("o")).any() and not np.isnan(run.host("dk")).any()


def test_several_tiles_and_uneven_heads():
    # 5 and 11 q tiles, 3 local heads (an uneven share), lengths not multiples of any tile
    _full_check([700, 1300], 3, 3, 128, seed=21)


def test_gqa_group_of_four_multi_tile():
    _full_check([515, 1, 900], 8, 2, 128, seed=22)


@pytest.mark.parametrize("hq,hkv,d", [(16, 2, 128), (8, 1, 64), (16, 1, 104)])
def test_gqa_groups_of_eight_and_sixteen(hq, hkv, d):
    """Eight and sixteen query heads per KV head: the dK/dV workgroup walks the whole group, head after head, over
    several q tiles each, and sums it into one dK / dV tile.  With N(0,1) values the sum over sixteen heads carries
    dV of a sequence's first tokens to |dV| = 17.6 (one KV head) and dK to 8.2: those tensors take the bound for
    references of magnitude >= 8, the others the nominal one."""
    _full_check([300, 777, 64], hq, hkv, d, seed=23 + hq + d, magnitude_slack=True)


def test_explicit_scale_and_small_values():
    _full_check([130, 260], 2, 1, 128, seed=23, value_scale=1.0 / 128 ** 0.5, scale=0.2)


@pytest.mark.parametrize("value_scale,scale", [(3.0, 0.0), (1.0, 1.0), (1e-3, 0.0)])
def test_peaked_and_flat_softmax(value_scale, scale):
    """Scores with a standard deviation of about 9 (q, k scaled by 3) or 11 (softmax scale 1 at head_dim 128): nearly
    one-hot rows, the running maximum moves on most tiles; and scores of about 1e-6: uniform rows."""
    _full_check([200, 333, 64], 2, 2, 128, seed=71, value_scale=value_scale, scale=scale, magnitude_slack=True,
                slack_roundings=4)     # |dQ| reaches 136 here; the relative Frobenius bound stays 1e-2


def test_bf16_gradients():
    # bf16 gradient outputs: same accumulators, rounded once on store.  A bf16 value in [8, 16) has a
    # half-ulp of 0.031, so the absolute bound is widened by that rounding alone.
    lengths = [257, 64, 300]
    q, k, v, do = make_case(lengths, 4, 2, 128, 31)
    import paper_2504_20490_amd as A
    run = GpuRun(lengths, q, k, v, do, grad_dtype=A.GRAD_BF16).run()
    rdq, rdk, rdv = oracle.attn_bwd(f64(q), f64(k), f64(v), f64(do), lengths, default_scale(128))
    for name, ref in (("dq", rdq), ("dk", rdk), ("dv", rdv)):
        assert_close(name, run.host(name), ref, max_abs=gpu_util.magnitude_bound(ref))
    gpu_util.CONTEXT["slack"] = None
    f32 = GpuRun(lengths, q, k, v, do, grad_dtype=A.GRAD_F32).run()
    import torch
    for name in ("dq", "dk", "dv"):
        assert torch.equal(getattr(f32, name).to(torch.bfloat16), getattr(run, name)), name


def test_strided_views_into_a_fused_qkv_buffer():
    import torch
    lengths, hq, hkv, d = [100, 29, 150], 4, 2, 128
    q, k, v, do = make_case(lengths, hq, hkv, d, 41)
    T = sum(lengths)
    fused = torch.zeros(T, (hq + 2 * hkv) * d, dtype=torch.bfloat16, device="cuda")
    fused[:, :hq * d] = to_dev(q).reshape(T, -1)
    fused[:, hq * d:(hq + hkv) * d] = to_dev(k).reshape(T, -1)
    fused[:, (hq + hkv) * d:] = to_dev(v).reshape(T, -1)
    qv = fused[:, :hq * d].view(T, hq, d)
    kv = fused[:, hq * d:(hq + hkv) * d].view(T, hkv, d)
    vv = fused[:, (hq + hkv) * d:].view(T, hkv, d)
    assert qv.stride(0) == (hq + 2 * hkv) * d
    a = GpuRun(lengths, q, k, v, do, q_dev=qv, k_dev=kv, v_dev=vv).run()
    b = GpuRun(lengths, q, k, v, do).run()
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


def _max_abs_ds(lengths, q, k, v, do, s):
    """max |dS| over a pack of short sequences, dense per (sequence, head): the magnitude of the bf16 operand that dQ
    and dK are products of.  It feeds a tolerance, not an expected value."""
    hq, hkv = q.shape[1], k.shape[1]
    G = hq // hkv
    cu = np.concatenate([[0], np.cumsum(lengths)])
    peak = 0.0
    for i, L in enumerate(lengths):
        sl = slice(int(cu[i]), int(cu[i + 1]))
        low = np.tril(np.ones((L, L), dtype=bool))
        for h in range(hq):
            S = np.where(low, s * q[sl, h] @ k[sl, h // G].T, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            dP = do[sl, h] @ v[sl, h // G].T
            dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
            peak = max(peak, float(np.abs(dS).max()))
    return peak


def test_many_tiny_sequences():
    """3000 sequences of 1 .. 12 tokens: one work item per (sequence, head), most of every tile empty.  Every row is
    one of the first rows of its sequence: weights of 1/2 .. 1, so |dS| = |P (dP - D)| reaches 10.4 on this pack (70 of
    its 359K pairs exceed 8) although no gradient element does, and D itself is taken from the bf16-rounded O of rows
    that are close to single V rows.  The bf16 rounding of such a dS (half an ulp of 0.03 times |q| scale, two of them in
    one dK element) is what the widened bound of dQ and dK stands for; O and dV are held to the nominal bound."""
    rng = np.random.default_rng(8)
    lengths = [int(x) for x in rng.integers(1, 13, size=3000)]
    hq, hkv, d, seed = 4, 2, 64, 61
    gpu_util.CONTEXT["case"] = f"small pack {len(lengths)} seqs Hq{hq} Hkv{hkv} d{d} seed{seed}"
    q, k, v, do = make_case(lengths, hq, hkv, d, seed)
    run = GpuRun(lengths, q, k, v, do).run()
    s = default_scale(d)
    ro, rlse = oracle.attn_fwd(f64(q), f64(k), f64(v), lengths, s)
    rdq, rdk, rdv = oracle.attn_bwd(f64(q), f64(k), f64(v), f64(do), lengths, s)
    peak_ds = _max_abs_ds(lengths, f64(q), f64(k), f64(v), f64(do), s)
    assert 8.0 <= peak_ds < 16.0, peak_ds
    assert_close("O", run.host("o"), ro)
    assert np.max(np.abs(run.host("lse") - rlse)) <= LSE_ABS
    assert_close("dQ", run.host("dq"), rdq, max_abs=gpu_util.magnitude_bound(rdq, operand_peak=peak_ds))
    assert_close("dK", run.host("dk"), rdk, max_abs=gpu_util.magnitude_bound(rdk, operand_peak=peak_ds))
    gpu_util.CONTEXT["slack"] = None
    assert_close("dV", run.host("dv"), rdv)


def test_one_very_long_sequence_on_sampled_rows_and_keys():
    """A single 50000-token sequence, one head: 782 key tiles in the longest forward item, 782 q tiles in the
    longest dK/dV item; rows and keys at the ends, at tile edges and in the middle against the oracle."""
    L, d = 50000, 64
    lengths = [L]
    q, k, v, do = make_case(lengths, 1, 1, d, seed=62)
    gpu_util.CONTEXT["case"] = "long50k"
    run = GpuRun(lengths, q, k, v, do).run()
    s = default_scale(d)
    rows = np.array([0, 1, 63, 64, 127, 128, 24999, 25000, 32767, 32768, L - 2, L - 1], dtype=np.int32)
    heads = np.zeros(len(rows), dtype=np.int32)
    ro, rlse, rdq = oracle.attn_rows(f64(q), f64(k), f64(v), f64(do), lengths, s, rows, heads)
    assert_close("O rows", run.host("o")[rows, heads], ro)
    assert np.max(np.abs(run.host("lse")[heads, rows] - rlse)) <= LSE_ABS
    assert_close("dQ rows", run.host("dq")[rows, heads], rdq)
    rdk, rdv = oracle.attn_keys(f64(q), f64(k), f64(v), f64(do), lengths, s, rows, heads)
    # the first keys collect a contribution from every one of the 50000 rows; the nominal bound holds unless an
    # element reaches magnitude 8
    for name, got, ref in (("dK keys", run.host("dk")[rows, heads], rdk), ("dV keys", run.host("dv")[rows, heads], rdv)):
        assert_close(name, got, ref, max_abs=gpu_util.magnitude_bound(ref))
    gpu_util.CONTEXT["slack"] = None
    for name in ("o", "dq", "dk", "dv"):
        assert not np.isnan(run.host(name)).any()


def test_run_to_run_bit_identical_and_plan_reuse():
    import torch
    lengths = [300, 41, 1000, 7]
    q, k, v, do = make_case(lengths, 4, 2, 128, 51)
    run = GpuRun(lengths, q, k, v, do).run()
    first = {n: getattr(run, n).clone() for n in ("o", "lse", "dq", "dk", "dv")}
    for _ in range(3):
        run.run()
        for n, t in first.items():
            assert torch.equal(getattr(run, n), t), n


def test_length_one_and_degenerate_packs():
    import torch
    lengths = [1, 1, 0, 1]
    q, k, v, do = make_case(lengths, 2, 2, 128, 61)
    run = GpuRun(lengths, q, k, v, do).run()
    assert torch.equal(run.o, run.v)                            # O = V row
    assert float((run.dv - run.do.float()).abs().max()) < 1e-5  # dV = dO (P = 1 up to fp32 rounding)
    assert float(run.dq.abs().max()) < 1e-5 and float(run.dk.abs().max()) < 1e-5   # zero up to fp32 rounding
    s = default_scale(128)
    want = s * np.einsum("thc,thc->ht", f64(q), f64(k))
    assert np.max(np.abs(run.host("lse") - want)) <= LSE_ABS
    # empty pack: OK without a launch
    e = np.zeros((0, 2, 128), dtype=np.uint16)
    GpuRun([], e, e, e, e).run()
    GpuRun([0, 0], e, e, e, e).run()


def test_argument_validation_on_device_calls():
    import torch
    import paper_2504_20490_amd as A
    lengths = [40]
    q, k, v, do = make_case(lengths, 2, 2, 128, 71)
    run = GpuRun(lengths, q, k, v, do)
    with pytest.raises(A.HspmdError) as e:
        A.attn_varlen_bwd(run.plan, run.q, run.k, run.v, run.o, run.lse, run.do, run.dq, run.dk, run.dv,
                          torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3
    with pytest.raises(A.HspmdError) as e:
        A.attn_varlen_fwd(run.plan, run.q.view(-1)[1:], run.k, run.v, run.o, run.lse)   # misaligned q
    assert e.value.status == 1
    with pytest.raises(A.HspmdError) as e:
        A.attn_varlen_bwd(run.plan, run.q, run.k, run.v, run.o, run.lse, run.do, run.dq, run.dk, run.dv, run.ws,
                          grad_dtype=5)
    assert e.value.status == 2
    run.run()   # still usable after rejected calls


@pytest.mark.gpu
def test_mfma_rate_probe_is_plausible():
    """The measurement hook returns a rate between a third of and slightly above the nominal 2.5 PFLOP/s."""
    import torch
    import paper_2504_20490_amd as A
    scratch = torch.empty(A.probe_scratch_bytes(), dtype=torch.uint8, device="cuda")
    rate = A.probe_mfma_tflops(scratch, mfma_per_wave=1 << 16)
    assert 800.0 < rate < 2700.0, rate
    # operands that vary like real data: the power-limited clock is lower, never higher
    varied = A.probe_mfma_tflops(scratch, mfma_per_wave=1 << 16, varied_operands=True)
    assert 600.0 < varied < 1.05 * rate, (varied, rate)
    assert torch.isfinite(scratch.view(torch.float32)).all()      # the checksums of the varied run
    with pytest.raises(A.HspmdError):
        A.probe_mfma_tflops(scratch[:16])
    with pytest.raises(A.HspmdError):
        A.probe_mfma_tflops(scratch, mfma_per_wave=0)
    # the variants: every mode runs and lands in a plausible range; idle time lowers the rate, never raises it
    rates = {name: A.probe_mfma_rate(mode, scratch, mfma_per_wave=1 << 16) for name, mode in A.PROBE_MODES.items()}
    assert all(300.0 < r < 2700.0 for r in rates.values()), rates
    idle = [rates[n] for n in A.PROBE_MODES if "one wave per SIMD" in n]
    assert idle[0] > idle[1] > idle[2] > idle[3], idle
    assert rates["32x32x16, A from LDS"] < 1.05 * rates["32x32x16"]
    with pytest.raises(A.HspmdError):
        A.probe_mfma_rate(99, scratch)
