"""Helpers shared by the GPU parity tests: run the C ABI on seeded bf16 inputs, compare with the oracle."""
from __future__ import annotations

import math

import numpy as np

import hspmd_workloads as w

MAX_ABS = 2e-2      # tolerance stated for O, dQ, dK, dV: max-abs error ...
REL_FRO = 1e-2      # ... and relative Frobenius error (bf16 inputs, fp32 accumulation)
LSE_ABS = 1e-3


def f64(bits: np.ndarray) -> np.ndarray:
    return w.bits_to_f32(bits).astype(np.float64)


def to_dev(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def make_case(lengths, hq, hkv, d, seed, value_scale=1.0):
    T = int(sum(lengths))
    q = w.make_tensor(seed, "q", T * hq * d, value_scale).reshape(T, hq, d)
    k = w.make_tensor(seed, "k", T * hkv * d, value_scale).reshape(T, hkv, d)
    v = w.make_tensor(seed, "v", T * hkv * d, value_scale).reshape(T, hkv, d)
    do = w.make_tensor(seed, "do", T * hq * d, value_scale).reshape(T, hq, d)
    return q, k, v, do


class GpuRun:
    """Forward + backward through the C ABI; keeps the device tensors for inspection."""

    def __init__(self, lengths, q_bits, k_bits, v_bits, do_bits, grad_dtype=None, scale=0.0,
                 q_dev=None, k_dev=None, v_dev=None):
        import torch
        import paper_2504_20490_amd as A
        self.A = A
        T, hq, d = q_bits.shape
        hkv = k_bits.shape[1]
        self.shape = (T, hq, hkv, d)
        grad_dtype = A.GRAD_F32 if grad_dtype is None else grad_dtype
        cu, _, total = A.build_cu_seqlens(lengths)
        assert total == T
        self.plan = A.Plan(cu, hq, hkv, d)
        self.q = to_dev(q_bits) if q_dev is None else q_dev
        self.k = to_dev(k_bits) if k_dev is None else k_dev
        self.v = to_dev(v_bits) if v_dev is None else v_dev
        self.do = to_dev(do_bits)
        self.o = torch.full((T, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        self.lse = torch.full((hq, T), float("nan"), dtype=torch.float32, device="cuda")
        gd = torch.float32 if grad_dtype == A.GRAD_F32 else torch.bfloat16
        self.dq = torch.full((T, hq, d), float("nan"), dtype=gd, device="cuda")
        self.dk = torch.full((T, hkv, d), float("nan"), dtype=gd, device="cuda")
        self.dv = torch.full((T, hkv, d), float("nan"), dtype=gd, device="cuda")
        self.ws = torch.empty(max(self.plan.bwd_workspace_bytes(), 16), dtype=torch.uint8, device="cuda")
        self.scale = scale
        self.grad_dtype = grad_dtype

    def forward(self):
        self.A.attn_varlen_fwd(self.plan, self.q, self.k, self.v, self.o, self.lse, self.scale)

    def backward(self):
        self.A.attn_varlen_bwd(self.plan, self.q, self.k, self.v, self.o, self.lse, self.do, self.dq, self.dk,
                               self.dv, self.ws, self.scale, self.grad_dtype)

    def run(self):
        import torch
        self.forward()
        self.backward()
        torch.cuda.synchronize()
        return self

    def host(self, name):
        return getattr(self, name).float().cpu().numpy().astype(np.float64)


def errors(got: np.ndarray, ref: np.ndarray):
    """(max-abs error, relative Frobenius error).  A reference that is identically zero (dQ of a pack of
    length-1 sequences) has no relative error: there the max-abs error alone decides."""
    diff = got - ref
    if not diff.size:
        return 0.0, 0.0
    ref_norm = float(np.linalg.norm(ref))
    return float(np.max(np.abs(diff))), (float(np.linalg.norm(diff)) / ref_norm if ref_norm > 0.0 else 0.0)


CONTEXT = {"case": ""}   # set by a test; written into the optional report


def _report(name, ma, rf, ref):
    """With HSPMD_PARITY_REPORT=<path> every comparison appends one JSON line (the measured errors that the
    results table quotes)."""
    import json
    import os
    path = os.environ.get("HSPMD_PARITY_REPORT")
    if not path:
        return
    with open(path, "a") as f:
        rec = {"case": CONTEXT["case"], "tensor": name, "max_abs": ma, "rel_fro": rf,
               "max_ref": float(np.max(np.abs(ref))) if ref.size else 0.0, "elements": int(ref.size)}
        if CONTEXT.get("where"):
            rec["where"] = CONTEXT["where"]
        if CONTEXT.get("slack"):
            rec["slack"] = CONTEXT["slack"]
        f.write(json.dumps(rec) + "\n")


def assert_close(name, got, ref, max_abs=MAX_ABS, rel_fro=REL_FRO):
    assert not np.isnan(got).any(), f"{name}: NaN in GPU output (unwritten or invalid elements)"
    ma, rf = errors(got, ref)
    _report(name, ma, rf, ref)
    assert ma <= max_abs and rf <= rel_fro, f"{name}: max_abs {ma:.3e} (<= {max_abs}), rel_fro {rf:.3e} (<= {rel_fro})"
    return ma, rf


SLACK_FROM = 8.0    # a bf16 value in [8, 16) has half an ulp of 2^-5 = 0.031 > MAX_ABS


def magnitude_bound(ref: np.ndarray, roundings: int = 1, operand_peak: float = 0.0) -> float:
    """max-abs bound for packs outside the benchmark configurations' value range: the nominal MAX_ABS, widened by
    `roundings` bf16 roundings (2^-9 relative each: P, dS and O are rounded to bf16 on their way into or out of the
    matrix cores) ONLY when the reference tensor really holds an element of magnitude >= 8, where one such
    rounding alone exceeds the nominal bound.  Tensors below that are held to the nominal bound.
    operand_peak: the largest magnitude of the bf16 OPERAND that the tensor is a product of (max |dS| for dQ and dK),
    when the caller has evaluated it: a pack of very short sequences has |dS| >= 8 without |dK| >= 8."""
    peak = max(float(np.max(np.abs(ref))) if ref.size else 0.0, float(operand_peak))
    if peak < SLACK_FROM:
        CONTEXT["slack"] = None
        return MAX_ABS
    CONTEXT["slack"] = {"max_ref": peak, "roundings": roundings}
    SLACK_USED.append((CONTEXT["case"], peak))
    return MAX_ABS + roundings * 2.0 ** -9 * peak


SLACK_USED = []     # (case, max|ref|) of every comparison that took the widened bound, for the record


def default_scale(d):
    return 1.0 / math.sqrt(d)
