"""fp64 CPU oracle for rotary position embedding (RoPE) around packed causal attention (test infrastructure).

THIS IS TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the GPU library never does and shares no code with it.

What it follows.  The paper's models are Llama-style and its table of model configurations lists the position
encoding as RoPE (experimental setup, model configuration table); it gives no formula, so the published
definition of RoPE is written out here (Su et al., RoFormer), in the "rotate-half" pairing that Llama
implementations use: with head dimension d, frequencies theta_i = base ** (-2 i / d) for i = 0 .. d/2-1 and a
token at position p inside its sequence, the pair (x_i, x_{i + d/2}) of every head vector of q and k turns by
the angle p * theta_i:

    y_i        = x_i cos(p theta_i) - x_{i+d/2} sin(p theta_i)
    y_{i+d/2}  = x_{i+d/2} cos(p theta_i) + x_i sin(p theta_i)

The map is linear and orthogonal per token, so the gradient with respect to x of anything that consumes y is
the same rotation by the opposite angle applied to the gradient with respect to y.  Attention on rotated q
and k:  q' = rope(q), k' = rope(k), (O, LSE) = attention(q', k', v);  dq = rope^T(dq'), dk = rope^T(dk').

Positions restart at 0 at every sequence of the pack.  Layout: x [T, H, d] with tokens packed back to back.

Pins (tests/test_oracle_rope_pins.py): position 0 is the identity; d = 2 is the 2x2 rotation matrix; a value
worked out by hand; the complex-number form of the same rotation computed with a library complex multiply;
norms are kept; the score of a rotated pair depends on the position difference only; the transposed map is
the inverse and matches finite differences.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def positions_of(lengths: Sequence[int]) -> np.ndarray:
    """Position of every token of the pack inside its own sequence."""
    if any(L < 0 for L in lengths):
        raise ValueError("negative length")
    if not len(lengths):
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(L, dtype=np.int64) for L in lengths])


def angles(positions: np.ndarray, d: int, base: float) -> np.ndarray:
    """[T, d/2] turning angles p * theta_i."""
    if d % 2:
        raise ValueError("head dimension must be even")
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    return np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]


def _turn(x: np.ndarray, a: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    lo, hi = x[..., :half], x[..., half:]
    c, s = np.cos(a)[:, None, :], np.sin(a)[:, None, :]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def rope(x: np.ndarray, positions: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """y = rope(x) for x [T, H, d] and one position per token."""
    if x.shape[0] != len(positions):
        raise ValueError("one position per token")
    return _turn(x, angles(positions, x.shape[-1], base))


def rope_transposed(dy: np.ndarray, positions: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """Gradient with respect to x of a function of y = rope(x), given its gradient with respect to y."""
    if dy.shape[0] != len(positions):
        raise ValueError("one position per token")
    return _turn(dy, -angles(positions, dy.shape[-1], base))
