"""Refit the coefficients of hspmd_attn_estimate_ms on the GPU at hand.

Runs forward + backward of a set of synthetic packs (uniform and log-normal length mixes, several head
counts) through the library with per-kernel event timing, computes for every pass the two features the
model uses -- inner steps and items of the heaviest XCD queue per resident workgroup -- from the host
scheduler, and fits (launch_us, step_us, item_us) per pass by relative least squares.  Prints the table
that goes into pass_cost_coefficients() (csrc/schedule.cpp).

    python -m paper_2504_20490_amd.fit_cost_model [--head-dim 128]
"""
from __future__ import annotations

import argparse

import numpy as np


def _packs(rng):
    for hq, hkv in [(16, 16), (32, 8), (8, 8), (40, 40)]:
        for length, count in [(512, 32), (1024, 16), (4096, 4), (16384, 1), (256, 64), (8192, 4), (128, 256)]:
            yield [length] * count, hq, hkv
    for _ in range(12):
        n = int(rng.integers(2, 30))
        lens = [int(x) for x in np.clip(np.exp(rng.normal(7.0, 1.2, n)), 16, 20000)]
        yield lens, int(rng.choice([8, 16, 24, 32])), 8


def _measure(A, torch, lengths, hq, hkv, d):
    T = sum(lengths)
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    mk = lambda h: torch.randn(T, h, d, device="cuda", generator=g).to(torch.bfloat16)
    q, k, v, do = mk(hq), mk(hkv), mk(hkv), mk(hq)
    o = torch.empty_like(q)
    lse = torch.empty(hq, T, dtype=torch.float32, device="cuda")
    dq = torch.empty(T, hq, d, dtype=torch.float32, device="cuda")
    dk = torch.empty(T, hkv, d, dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    cu, _, _ = A.build_cu_seqlens(lengths)
    plan = A.Plan(cu, hq, hkv, d)
    ws = torch.empty(plan.bwd_workspace_bytes(), dtype=torch.uint8, device="cuda")

    def step():
        A.attn_varlen_fwd(plan, q, k, v, o, lse)
        A.attn_varlen_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws, grad_dtype=A.GRAD_F32)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    A.profile_enable(True)
    for _ in range(8):
        step()
    torch.cuda.synchronize()
    A.profile_enable(False)
    return {name: ms / n * 1e3 for name, (ms, n) in A.profile_read().items()}   # microseconds


def _features(A, kind, slots, lengths, hq, hkv):
    cu = np.concatenate([[0], np.cumsum(lengths)])
    items = A.schedule(kind, cu, hq, hkv)
    length, tile = items[:, 1].astype(np.int64), items[:, 2].astype(np.int64)
    real = tile >= 0
    rows_q, rows_k = A.tile_rows(A.LIST_FWD), A.tile_rows(A.LIST_DKV)
    if kind == A.LIST_DKV:
        steps = np.where(real, -(-(length - tile * rows_k) // 64) * (hq // hkv), 0)
    else:
        steps = np.where(real, -(-np.minimum(length, (tile + 1) * rows_q) // 64), 0)
    return max(steps[x::8].sum() for x in range(8)) / slots, max(real[x::8].sum() for x in range(8)) / slots


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--head-dim", type=int, default=128, choices=[64, 128])
    args = ap.parse_args()
    import torch
    import paper_2504_20490_amd as A
    A.load_library()
    passes = [(A.LIST_FWD, "fwd_kernel", 64.0), (A.LIST_DQ, "bwd_dq_kernel", 64.0), (A.LIST_DKV, "bwd_dkv_kernel", 32.0)]
    rows = [(lens, hq, hkv, _measure(A, torch, lens, hq, hkv, args.head_dim)) for lens, hq, hkv in _packs(np.random.default_rng(7))]
    print(f"// head_dim {args.head_dim}: {{launch_us, step_us, item_us}} for forward, dQ pass, dK/dV pass ({len(rows)} packs)")
    for kind, name, slots in passes:
        X = np.array([[1.0, *_features(A, kind, slots, lens, hq, hkv)] for lens, hq, hkv, _ in rows])
        y = np.array([ms[name] for *_, ms in rows])
        coef, *_ = np.linalg.lstsq(X / y[:, None], np.ones_like(y), rcond=None)
        err = np.abs(X @ coef / y - 1.0)
        print(f"{{{max(coef[0], 0.0):.1f}, {coef[1]:.3f}, {coef[2]:.2f}}},   // {name}: mean |error| {err.mean():.3f}, max {err.max():.3f}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
