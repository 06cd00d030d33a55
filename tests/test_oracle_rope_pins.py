"""Pins of the RoPE oracle against things other than itself: special cases, a hand-worked value, the
complex-number form computed with a library complex multiply, invariants and finite differences."""
import math

import numpy as np
import pytest

from oracle import rope as orope


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_positions_restart_at_every_sequence():
    assert orope.positions_of([3, 0, 2]).tolist() == [0, 1, 2, 0, 1]
    assert orope.positions_of([]).tolist() == []
    with pytest.raises(ValueError):
        orope.positions_of([2, -1])


def test_position_zero_is_the_identity():
    x = _rand((4, 3, 16), 1)
    assert np.array_equal(orope.rope(x, np.zeros(4, dtype=np.int64)), x)


def test_head_dim_two_is_the_plane_rotation():
    """d = 2: one pair, theta_0 = 1, so position p turns the vector by p radians, counter-clockwise."""
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -1.0]]])
    pos = np.array([1, 2, 5])
    y = orope.rope(x, pos)
    for t in range(3):
        c, s = math.cos(pos[t]), math.sin(pos[t])
        want = np.array([[c, -s], [s, c]]) @ x[t, 0]
        assert np.allclose(y[t, 0], want, rtol=0, atol=1e-15)


def test_hand_worked_value():
    """d = 4, base 10000, position 1: theta = (1, 0.01); pairs are (x0, x2) and (x1, x3).
    x = (1, 0, 0, 1): y0 = cos 1, y2 = sin 1, y1 = -sin 0.01, y3 = cos 0.01."""
    y = orope.rope(np.array([[[1.0, 0.0, 0.0, 1.0]]]), np.array([1]))[0, 0]
    want = [0.5403023058681398, -0.009999833334166664, 0.8414709848078965, 0.9999500004166653]
    assert np.allclose(y, want, rtol=0, atol=1e-15)
    # the frequencies fall with the pair index: the second pair of d = 8 turns by base ** (-2/8) = 0.1 per position
    a = orope.angles(np.array([3]), 8, 10000.0)[0]
    assert np.allclose(a, [3.0, 0.3, 0.03, 0.003], rtol=1e-14, atol=0)
    a = orope.angles(np.array([2]), 6, 1000.0)[0]
    assert np.allclose(a, [2.0, 0.2, 0.02], rtol=1e-14, atol=0)


def test_matches_the_complex_form():
    """(x_i + 1j x_{i+d/2}) * exp(1j p theta_i), with the library's complex multiply and exp."""
    T, H, d, base = 9, 2, 12, 500.0
    x = _rand((T, H, d), 2)
    pos = np.array([0, 1, 2, 3, 0, 1, 7, 100, 4095])
    z = x[..., : d // 2] + 1j * x[..., d // 2:]
    theta = np.array([base ** (-2.0 * i / d) for i in range(d // 2)])
    w = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    y = orope.rope(x, pos, base)
    assert np.allclose(y[..., : d // 2], w.real, rtol=0, atol=1e-12)
    assert np.allclose(y[..., d // 2:], w.imag, rtol=0, atol=1e-12)


def test_norms_are_kept_and_scores_depend_on_the_position_difference():
    d = 16
    q, k = _rand((1, 1, d), 3), _rand((1, 1, d), 4)
    for m, n in [(5, 2), (1003, 1000), (40, 37)]:
        qm, kn = orope.rope(q, np.array([m])), orope.rope(k, np.array([n]))
        assert math.isclose(np.linalg.norm(qm), np.linalg.norm(q), rel_tol=1e-14)
        score = float((qm * kn).sum())
        ref = float((orope.rope(q, np.array([3])) * k).sum())      # positions (3, 0): the same difference
        assert math.isclose(score, ref, rel_tol=0, abs_tol=1e-10)
    # and it does depend on the difference
    a = float((orope.rope(q, np.array([3])) * k).sum())
    b = float((orope.rope(q, np.array([4])) * k).sum())
    assert abs(a - b) > 1e-3


def test_transposed_map_is_the_inverse_and_the_gradient():
    T, H, d = 6, 2, 8
    pos = orope.positions_of([4, 2])
    x, g = _rand((T, H, d), 5), _rand((T, H, d), 6)
    assert np.allclose(orope.rope_transposed(orope.rope(x, pos), pos), x, rtol=0, atol=1e-13)
    # <g, rope(x)> as a function of x: its gradient is rope_transposed(g); central differences are exact for a linear map
    grad = orope.rope_transposed(g, pos)
    rng = np.random.default_rng(7)
    for _ in range(20):
        t, h, i = rng.integers(T), rng.integers(H), rng.integers(d)
        e = np.zeros_like(x); e[t, h, i] = 0.5
        fd = float((g * orope.rope(x + e, pos)).sum() - (g * orope.rope(x - e, pos)).sum())
        assert math.isclose(fd, grad[t, h, i], rel_tol=0, abs_tol=1e-12)


def test_bad_arguments():
    with pytest.raises(ValueError):
        orope.rope(np.zeros((2, 1, 4)), np.array([0]))
    with pytest.raises(ValueError):
        orope.angles(np.array([0]), 5, 10000.0)
