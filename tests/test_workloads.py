"""The seeded input generator: determinism, slice-independence, bf16 rounding and the
length mixes of the five benchmark configurations."""
import math

import numpy as np

import hspmd_workloads as w


def test_stream_is_a_function_of_the_index():
    full = w.make_tensor(7, "k", 100000, threads=1)
    part = w.make_tensor(7, "k", 1000, start=54321, chunk=128, threads=1)
    assert np.array_equal(full[54321:55321], part)
    again = w.make_tensor(7, "k", 100000, chunk=4096, threads=4)
    assert np.array_equal(full, again)
    assert not np.array_equal(full, w.make_tensor(8, "k", 100000))
    assert not np.array_equal(full, w.make_tensor(7, "v", 100000))


def test_values_are_standard_normal_bf16():
    bits = w.make_tensor(3, "q", 1 << 20)
    x = w.bits_to_f32(bits).astype(np.float64)
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1.0) < 5e-3
    assert abs(np.mean(x ** 3)) < 2e-2 and abs(np.mean(x ** 4) - 3.0) < 5e-2
    # rounding: nearest bf16, ties to even
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    r = w.round_to_bf16(f)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625) and r[3] == -2.5
    y = w.normal_f32(1, 1, 0, 4096)
    r = w.round_to_bf16(y)
    assert np.all(np.abs(r - y) <= np.abs(y) * 2.0 ** -8)
    assert np.all((w.bf16_bits(y).astype(np.uint32) << 16).view(np.float32) == r)


def test_length_mixes():
    by_name = {c.name: c for c in w.CONFIGS}
    assert w.lengths_for(by_name["C1_tiny"]) == [17, 64, 111]
    assert w.lengths_for(by_name["C2_uniform"]) == [2048] * 8
    for name, lo, hi in (("C3_mixed16k", 32, 8192), ("C4_asym32k", 64, 16384)):
        c = by_name[name]
        L = w.lengths_for(c)
        assert sum(L) == c.total_tokens and L == w.lengths_for(c)
        assert all(lo <= x <= hi for x in L[:-1]) and 1 <= L[-1] <= hi
    c = by_name["C5_bimodal_gqa"]
    L = w.lengths_for(c)
    assert sum(L) == 65536
    assert all((256 <= x <= 2048) or (16384 <= x <= 32768) for x in L[:-1])
    assert c.q_heads == 32 and c.kv_heads == 8
    c4 = by_name["C4_asym32k"]
    assert c4.q_heads == 24 and c4.q_heads * c4.head_dim * 5 // 3 == 5120   # 24 of 40 heads, hidden 5120


def test_flop_formula():
    assert w.fwd_flops([17, 64, 111], 2, 64) == 2 * (17 * 18 + 64 * 65 + 111 * 112) * 64 * 2 == 4325888
    assert w.fwd_flops([2048] * 8, 32, 128) == 275012124672


def test_make_inputs_shapes():
    c = w.config_by_name("C1")
    L, q, k, v, do = w.make_inputs(c)
    assert q.shape == (192, 2, 64) and k.shape == v.shape == (192, 2, 64) and do.shape == q.shape
    assert q.dtype == np.uint16
    assert not np.array_equal(q, do)
