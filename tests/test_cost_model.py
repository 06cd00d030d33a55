"""Host-side properties of hspmd_attn_estimate_ms (the prediction's accuracy is a GPU test)."""
import numpy as np
import pytest

import paper_2504_20490_amd as A


def _cu(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def test_empty_pack_costs_nothing():
    assert A.estimate_ms([0], 4, 2, 128) == (0.0, 0.0)
    assert A.estimate_ms([0, 0, 0], 4, 2, 64) == (0.0, 0.0)


def test_longer_and_more_sequences_cost_more():
    prev = (0.0, 0.0)
    for L in (256, 1024, 4096, 16384):
        cur = A.estimate_ms(_cu([L] * 4), 16, 16, 128)
        assert cur[0] > prev[0] and cur[1] > prev[1]
        prev = cur
    a = A.estimate_ms(_cu([4096] * 4), 16, 16, 128)
    b = A.estimate_ms(_cu([4096] * 8), 16, 16, 128)
    assert b[0] > a[0] and b[1] > a[1]


def test_quadratic_in_length_and_linear_in_heads_for_large_packs():
    """Large packs are dominated by the step term: one 32k sequence costs about 4x one 16k sequence, and twice the
    heads about twice the time; backward is between 2x and 4x forward."""
    f16, b16 = A.estimate_ms(_cu([16384]), 32, 32, 128)
    f32, b32 = A.estimate_ms(_cu([32768]), 32, 32, 128)
    assert 3.5 < f32 / f16 < 4.2 and 3.5 < b32 / b16 < 4.2
    fh, bh = A.estimate_ms(_cu([16384]), 64, 64, 128)
    assert 1.8 < fh / f16 < 2.1 and 1.8 < bh / b16 < 2.1
    assert 2.0 < b16 / f16 < 4.0


def test_head_dim_64_is_cheaper():
    f128, b128 = A.estimate_ms(_cu([3000, 500, 9000]), 16, 8, 128)
    f64, b64 = A.estimate_ms(_cu([3000, 500, 9000]), 16, 8, 64)
    assert f64 < f128 and b64 < b128


def test_validation():
    with pytest.raises(A.HspmdError):
        A.estimate_ms([0, 10], 3, 2, 128)
    with pytest.raises(A.HspmdError):
        A.estimate_ms([0, 10], 2, 2, 100)
    with pytest.raises(A.HspmdError):
        A.estimate_ms([0, 10, 5], 2, 2, 128)
