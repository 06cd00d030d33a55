"""Writes tests/golden/c1_oracle_values.txt: values of the fp64 oracles on the seeded C1 pack.

Calls nothing but the input generator and oracle/ (never the GPU library).  The paper prints no worked
attention example, so these are not the paper's numbers: they pin the oracles as they stood when the
kernels were validated against them, so that a later change to an oracle's arithmetic shows up as a diff
of this file (tests/test_oracle_golden.py compares to 1e-12).  Run from the repository root:

    python tests/golden/make_golden.py
"""
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import hspmd_workloads as w   # noqa: E402
import oracle                 # noqa: E402
from oracle import block as ob, rope as orope   # noqa: E402


def values():
    cfg = w.config_by_name("C1")
    lengths, q, k, v, do = w.make_inputs(cfg)
    f64 = lambda bits: w.bits_to_f32(bits).astype(np.float64)
    q, k, v, do = f64(q), f64(k), f64(v), f64(do)
    s = 1.0 / math.sqrt(cfg.head_dim)
    o, lse = oracle.attn_fwd(q, k, v, lengths, s)
    dq, dk, dv = oracle.attn_bwd(q, k, v, do, lengths, s)
    pos = orope.positions_of(lengths)
    qr = orope.rope(q, pos, 10000.0)
    # one off-diagonal block: rows 40 .. 63 of the second sequence against its keys 0 .. 31
    r0, k0 = 17 + 40, 17
    bo, bl = ob.block_fwd(q[r0:r0 + 24], k[k0:k0 + 32], v[k0:k0 + 32], [24], [32], [40], [0], s)
    out = {}
    picks = [(0, 0, 0), (16, 1, 63), (17, 0, 5), (80, 1, 31), (81, 0, 0), (191, 1, 62)]
    for name, t in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv), ("rope_q", qr)):
        for (tok, h, c) in picks:
            out[f"{name}[{tok},{h},{c}]"] = float(t[tok, h, c])
        out[f"{name}.sum"] = float(t.sum())
        out[f"{name}.abs_sum"] = float(np.abs(t).sum())
    for (h, tok) in [(0, 0), (1, 16), (0, 17), (1, 191)]:
        out[f"lse[{h},{tok}]"] = float(lse[h, tok])
    out["lse.sum"] = float(lse.sum())
    out["block_o[5,1,7]"] = float(bo[5, 1, 7])
    out["block_o.sum"] = float(bo.sum())
    out["block_lse.sum"] = float(bl.sum())
    return out


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_values.txt")
    with open(path, "w") as f:
        f.write("# fp64 oracle values on the seeded C1 pack (3 sequences of 17 / 64 / 111 tokens, 2 heads, head_dim 64);\n")
        f.write("# written by tests/golden/make_golden.py, which calls oracle/ only.  name = value (repr of a double)\n")
        for name, val in values().items():
            f.write(f"{name} = {val!r}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
