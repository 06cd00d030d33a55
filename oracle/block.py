"""fp64 CPU oracle for one block of context-parallel attention (test infrastructure).

THIS IS TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the GPU library never does and shares no code with it.

What it follows.  The paper shards long sequences over devices (context parallelism) and notes that this
needs ring-based send-receive inside attention, which it hides in a fused ``ParallelAttn`` operator
(Section 2.1, "Sharding and Communication in Training", data sharding; system overview, footnote on
``ParallelAttn``).  It gives no formulas.  One ring step on one device is: the device's own chunk of query
rows of every sequence meets one chunk of keys/values (its own or a received one), and the partial results
of the steps are combined.  With causal attention the only new ingredient is that row and key positions
are positions inside the whole sequence:

    query chunk of sequence i: rows at positions q_pos[i] + r, r = 0 .. q_len[i]-1
    key chunk of sequence i  : keys at positions k_pos[i] + j, j = 0 .. k_len[i]-1
    key j is visible to row r  iff  k_pos + j <= q_pos + r

    forward, per block:   S_rj = scale <q_r, k_j> over the visible j
                          LSE_r = ln sum_j exp(S_rj),  O_r = sum_j exp(S_rj - LSE_r) v_j
                          (no visible key: LSE_r = -inf, O_r = 0)
    merge of two blocks:  LSE = ln(exp(LSE_a) + exp(LSE_b)),
                          O = exp(LSE_a - LSE) O_a + exp(LSE_b - LSE) O_b
    backward, per block, given the row statistics of the WHOLE row (LSE_r of all blocks merged,
                          D_r = <dO_r, O_r> of the merged output):
                          P_rj = exp(S_rj - LSE_r), dP_rj = <dO_r, v_j>, dS_rj = P_rj (dP_rj - D_r)
                          dQ_r (this block's share) = scale sum_j dS_rj k_j
                          dK_j = scale sum_{h in group} sum_r dS_rj q_r,  dV_j = sum_{h in group} sum_r P_rj dO_r

These are the definitions written out with dense per-(sequence, head) matrices in numpy fp64: no tiling, no
online softmax.  Layouts as in the packed oracle: q, o, d_o, dq [Tq, Hq, d]; k, v, dk, dv [Tk, Hkv, d];
lse, dsum [Hq, Tq]; grouped KV heads are contiguous groups of query heads.

Pins (tests/test_oracle_block_pins.py): the blocks of any partition of a sequence's keys and rows, merged /
summed, reproduce the packed oracle (a separate C implementation); merge closed forms; blocks that are fully
masked or fully visible; a dense evaluation with a library softmax and reverse-mode autodiff; brute force
over single (row, key) pairs.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def _offsets(lengths: Sequence[int]) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    return cu


def _check(q, k, v, q_lengths, k_lengths, q_pos, k_pos):
    if not (len(q_lengths) == len(k_lengths) == len(q_pos) == len(k_pos)):
        raise ValueError("per-sequence lists differ in length")
    if any(x < 0 for x in list(q_lengths) + list(k_lengths) + list(q_pos) + list(k_pos)):
        raise ValueError("negative length or position")
    Tq, Hq, d = q.shape
    Tk, Hkv, dk = k.shape
    if v.shape != k.shape or dk != d or Hq % Hkv != 0:
        raise ValueError("shape mismatch")
    if sum(q_lengths) != Tq or sum(k_lengths) != Tk:
        raise ValueError("lengths do not sum to the token counts")


def _visible(q_len: int, k_len: int, q_pos: int, k_pos: int) -> np.ndarray:
    """[q_len, k_len] boolean: key j visible to row r."""
    r = np.arange(q_len, dtype=np.int64)[:, None] + q_pos
    j = np.arange(k_len, dtype=np.int64)[None, :] + k_pos
    return j <= r


def block_fwd(q, k, v, q_lengths, k_lengths, q_pos, k_pos, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Partial attention of every sequence's query chunk over its key chunk: (o [Tq,Hq,d], lse [Hq,Tq])."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    _check(q, k, v, q_lengths, k_lengths, q_pos, k_pos)
    Tq, Hq, d = q.shape
    G = Hq // k.shape[1]
    cq, ck = _offsets(q_lengths), _offsets(k_lengths)
    o = np.zeros((Tq, Hq, d)); lse = np.full((Hq, Tq), -np.inf)
    for i in range(len(q_lengths)):
        vis = _visible(q_lengths[i], k_lengths[i], q_pos[i], k_pos[i])
        any_vis = vis.any(axis=1)
        for h in range(Hq):
            qs = q[cq[i]:cq[i + 1], h]; ks = k[ck[i]:ck[i + 1], h // G]; vs = v[ck[i]:ck[i + 1], h // G]
            s = np.where(vis, scale * (qs @ ks.T), -np.inf)
            m = np.where(any_vis, s.max(axis=1, initial=-np.inf), 0.0)
            e = np.exp(s - m[:, None])                     # exp(-inf) = 0 on masked pairs
            z = e.sum(axis=1)
            with np.errstate(divide="ignore", invalid="ignore"):
                p = np.where(any_vis[:, None], e / z[:, None], 0.0)
                lse[h, cq[i]:cq[i + 1]] = np.where(any_vis, m + np.log(z), -np.inf)
            o[cq[i]:cq[i + 1], h] = p @ vs
    return o, lse


def merge(o_a, lse_a, o_b, lse_b) -> Tuple[np.ndarray, np.ndarray]:
    """Combines two partial results of the same rows over disjoint key sets."""
    o_a = np.asarray(o_a, dtype=np.float64); o_b = np.asarray(o_b, dtype=np.float64)
    lse_a = np.asarray(lse_a, dtype=np.float64); lse_b = np.asarray(lse_b, dtype=np.float64)
    m = np.maximum(lse_a, lse_b)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    za, zb = np.exp(lse_a - m_safe), np.exp(lse_b - m_safe)
    with np.errstate(divide="ignore", invalid="ignore"):
        lse = np.where(np.isfinite(m), m_safe + np.log(za + zb), -np.inf)
        wa = np.where(np.isfinite(m), za / (za + zb), 0.0)
        wb = np.where(np.isfinite(m), zb / (za + zb), 0.0)
    o = wa.T[:, :, None] * o_a + wb.T[:, :, None] * o_b
    return o, lse


def block_bwd(q, k, v, d_o, lse, dsum, q_lengths, k_lengths, q_pos, k_pos, scale: float):
    """This block's share of dQ and the gradients of the block's keys/values: (dq [Tq,Hq,d], dk, dv [Tk,Hkv,d]).

    lse, dsum [Hq, Tq] are the statistics of the whole rows (all blocks merged)."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64); dsum = np.asarray(dsum, dtype=np.float64)
    _check(q, k, v, q_lengths, k_lengths, q_pos, k_pos)
    Tq, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    cq, ck = _offsets(q_lengths), _offsets(k_lengths)
    dq = np.zeros((Tq, Hq, d)); dk = np.zeros(k.shape); dv = np.zeros(k.shape)
    for i in range(len(q_lengths)):
        vis = _visible(q_lengths[i], k_lengths[i], q_pos[i], k_pos[i])
        for h in range(Hq):
            g = h // G
            qs = q[cq[i]:cq[i + 1], h]; dos = d_o[cq[i]:cq[i + 1], h]
            ks = k[ck[i]:ck[i + 1], g]; vs = v[ck[i]:ck[i + 1], g]
            s = scale * (qs @ ks.T)
            p = np.where(vis, np.exp(s - lse[h, cq[i]:cq[i + 1]][:, None]), 0.0)
            dp = dos @ vs.T
            ds = p * (dp - dsum[h, cq[i]:cq[i + 1]][:, None])
            dq[cq[i]:cq[i + 1], h] = scale * (ds @ ks)
            dk[ck[i]:ck[i + 1], g] += scale * (ds.T @ qs)
            dv[ck[i]:ck[i + 1], g] += p.T @ dos
    return dq, dk, dv


def row_dot(o, d_o) -> np.ndarray:
    """D[h, t] = <dO[t, h], O[t, h]> as [Hq, Tq]."""
    return np.einsum("thc,thc->ht", np.asarray(o, dtype=np.float64), np.asarray(d_o, dtype=np.float64))
