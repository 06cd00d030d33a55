#!/usr/bin/env python3
"""Benchmark of libhspmd_attn on one MI355X.

One step = one pass of the whole hot path over one pack: packed-sequence offsets and the
cost-sorted work lists (host, built from the length list), forward, and backward (dQ pass, which
also computes the row statistic D, and dK/dV pass).  Inputs are resident in HBM before the timed region starts.  The workload is the
32768-token log-normal pack on an uneven head share (24 of 40 heads, head_dim 128), the
configuration the headline metric is quoted on.

Prints ONE JSON line.  `value` is useful causal TFLOP/s for forward+backward, with
forward FLOPs = 2 * sum L(L+1) * d * heads and backward counted as 2.5x forward.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (no sparsity)

# GEMMs (2*d flops per visible (query, key) pair and head each) that each kernel's pass needs
GEMMS = {"fwd_kernel": 2, "bwd_dq_kernel": 3, "bwd_dkv_kernel": 4}


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary (a --pmc run cannot share a process with
    the timing run), and where it comes from.  The summary names the digest of the kernel sources it was measured
    with; when the library has changed since, the figure is withheld (None) rather than shown beside fresh timings."""
    from paper_2504_20490_amd.build import sources_digest
    rel = os.path.join("profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    value, digest = None, None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    value = float(line.split(":", 1)[1])
                elif line.startswith("kernel_sources_sha256_16:"):
                    digest = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no committed counter summary for this kernel and workload"
    if value is None:
        return None, f"{rel} holds no figure"
    if digest != sources_digest():
        return None, f"{rel} was measured with other kernel sources ({digest}); withheld"
    return value, f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of these kernel sources, not this run)"


class PowerSampler:
    """Socket power (W) and shader clock (MHz) of GPU 0 while the timed steps run, read with the system management
    tools (`amd-smi metric -p`, `rocm-smi --showclocks`) from a side thread about twice a second.  Needs a timed region
    of several seconds (--steps in the thousands): the tools take a few hundred milliseconds per reading, and the
    readings are averages over about a second.  Evidence for the power limit the kernels run into, not a benchmark
    figure; absent tools give no readings."""

    def __init__(self):
        import threading
        self.power, self.sclk = [], []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        if self._stop.wait(1.5):            # let the clocks settle under the load
            return
        while not self._stop.is_set():
            try:
                out = subprocess.run(["amd-smi", "metric", "-p"], capture_output=True, text=True, timeout=10).stdout
                m = re.search(r"SOCKET_POWER:\s*([0-9.]+)\s*W", out)
                if m:
                    self.power.append(float(m.group(1)))
                out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10).stdout
                m = re.search(r"sclk clock level:[^(]*\(([0-9.]+)Mhz\)", out)
                if m:
                    self.sclk.append(float(m.group(1)))
            except (OSError, subprocess.SubprocessError):
                return
            self._stop.wait(0.3)

    def start(self):
        self._thread.start()

    def stop(self):
        self._stop.set()
        self._thread.join(timeout=30)
        mean = lambda v: round(sum(v) / len(v), 1) if v else None
        return {"socket_power_w": mean(self.power), "sclk_mhz": mean(self.sclk), "readings": len(self.power)}


def cpu_baseline(cfg, lengths, q, k, v, do, rope=False):
    """The fp64 oracle, as it stands, on a bounded sample of the same pack: whole sequences of the
    pack (shortest first, up to a pair budget) and eight KV groups, forward + backward (with `rope`:
    around the rotary-embedding oracle)."""
    import numpy as np
    import hspmd_workloads as w
    import oracle

    cu = np.concatenate([[0], np.cumsum(lengths)])
    budget = 7.0e7          # visible (query, key) pairs per head in the sample: ~10-20 s of CPU work
    order = sorted(range(len(lengths)), key=lambda i: lengths[i])
    chosen, pairs = [], 0
    for i in order:
        p = lengths[i] * (lengths[i] + 1) // 2
        if chosen and pairs + p > budget:
            break
        chosen.append(i)
        pairs += p
    heads = min(cfg.q_heads, 8 * (cfg.q_heads // cfg.kv_heads))
    kvh = heads // (cfg.q_heads // cfg.kv_heads)
    tok = np.concatenate([np.arange(cu[i], cu[i + 1]) for i in chosen])
    f64 = lambda bits: w.bits_to_f32(bits).astype(np.float64)
    qs, ks, vs, dos = f64(q[tok][:, :heads]), f64(k[tok][:, :kvh]), f64(v[tok][:, :kvh]), f64(do[tok][:, :heads])
    sl = [lengths[i] for i in chosen]
    s = 1.0 / math.sqrt(cfg.head_dim)
    t0 = time.perf_counter()
    if rope:
        from oracle import rope as orope
        pos = orope.positions_of(sl)
        qs, ks = orope.rope(qs, pos), orope.rope(ks, pos)
    oracle.attn_fwd(qs, ks, vs, sl, s)
    grads = oracle.attn_bwd(qs, ks, vs, dos, sl, s)
    if rope:
        orope.rope_transposed(grads[0], pos), orope.rope_transposed(grads[1], pos)
    dt = time.perf_counter() - t0
    flops = 3.5 * w.fwd_flops(sl, heads, cfg.head_dim)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"sequences of lengths {sl} of the same pack, {heads} q heads / {kvh} kv heads, "
                      f"fwd+bwd in fp64, {dt:.1f} s"}


def run_probe(args) -> int:
    """The matrix-core probes (hspmd_probe_mfma_rate), each run for a few seconds with the socket power and the shader
    clock read beside it: which MFMA shape delivers more inside the chip's power limit, what streaming an operand
    from LDS costs, and whether idle time of the matrix pipes is returned as clock.  A side measurement: prints one
    JSON line of its own kind."""
    import torch
    import paper_2504_20490_amd as A

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    A.load_library()
    torch.cuda.set_device(0)
    scratch = torch.empty(A.probe_scratch_bytes(), dtype=torch.uint8, device="cuda:0")
    rows = []
    for name, mode in A.PROBE_MODES.items():
        A.probe_mfma_rate(mode, scratch, mfma_per_wave=1 << 16)
        sampler = PowerSampler()
        sampler.start()
        t0, rate = time.perf_counter(), 0.0
        while time.perf_counter() - t0 < args.probe_seconds:
            rate = A.probe_mfma_rate(mode, scratch, mfma_per_wave=1 << 20)
        rows.append({"probe": name, "tflops": round(rate, 1), **sampler.stop()})
    print(json.dumps({"metric": "dense bf16 MFMA rate of register-level probes (side measurement)", "unit": "TFLOP/s",
                      "n_gpus": 1, "peak": PEAK_BF16_TFLOPS, "probes": rows}))
    return 0


def run_ring(args) -> int:
    """One rank of an emulated context-parallel ring: every sequence of the pack is cut into N chunks by position,
    this rank owns chunk `--ring-rank` of every sequence as queries and meets the N key/value chunks one after the
    other (block forward + merge; block backward with dQ accumulation).  A step = N block plans (host) + all of
    that.  The sends and receives of a real ring are not part of it."""
    import numpy as np
    import torch
    import hspmd_workloads as w
    import paper_2504_20490_amd as A

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    A.load_library()
    cfg = w.config_by_name(args.workload)
    lengths, q, k, v, do = w.make_inputs(cfg)
    hq, hkv, d = cfg.q_heads, cfg.kv_heads, cfg.head_dim
    n, rank = args.ring, (args.ring - 1 if args.ring_rank < 0 else args.ring_rank)
    if not 0 <= rank < n:
        print("--ring-rank must be in [0, --ring)", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cu = np.concatenate([[0], np.cumsum(lengths)])
    edges = [[(L * c) // n for c in range(n + 1)] for L in lengths]
    tok = lambda c: np.concatenate([np.arange(cu[i] + edges[i][c], cu[i] + edges[i][c + 1]) for i in range(len(lengths))])
    lens = lambda c: [edges[i][c + 1] - edges[i][c] for i in range(len(lengths))]
    pos = lambda c: [edges[i][c] for i in range(len(lengths))]
    cuof = lambda ls: np.concatenate([[0], np.cumsum(ls)]).astype(np.int32)

    def bf(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    tq_idx = tok(rank)
    Tq = len(tq_idx)
    tq, tdo = bf(q[tq_idx]), bf(do[tq_idx])
    kv = [(bf(k[tok(c)]), bf(v[tok(c)])) for c in range(n)]
    o_acc = torch.empty(Tq, hq, d, dtype=torch.float32, device=dev)
    lse_acc = torch.empty(hq, Tq, dtype=torch.float32, device=dev)
    o_part, lse_part = torch.empty_like(o_acc), torch.empty_like(lse_acc)
    o_bf16 = torch.empty(Tq, hq, d, dtype=torch.bfloat16, device=dev)
    dq = torch.empty(Tq, hq, d, dtype=torch.float32, device=dev)
    dkv = [(torch.empty(kk.shape, dtype=torch.float32, device=dev), torch.empty(kk.shape, dtype=torch.float32, device=dev))
           for kk, _ in kv]
    ws = torch.empty(2 * hq * Tq * 4 + 256, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    # one block plan per ring step, made once and refilled with its chunks every step (no allocation per step)
    plans = [A.BlockPlan(cuof(lens(rank)), cuof(lens(c)), pos(rank), pos(c), hq, hkv, d, stream.cuda_stream)
             for c in range(n)]

    def step():
        for c, plan in enumerate(plans):
            plan.update(cuof(lens(rank)), cuof(lens(c)), pos(rank), pos(c))
        for c, plan in enumerate(plans):
            if c == 0:
                A.attn_block_fwd(plan, tq, kv[c][0], kv[c][1], o_acc, lse_acc, stream=stream)
                if n == 1:
                    A.attn_merge(o_acc, lse_acc, o_acc, lse_acc, o_part, lse_part, o_bf16, stream=stream)
            else:
                A.attn_block_fwd(plan, tq, kv[c][0], kv[c][1], o_part, lse_part, stream=stream)
                A.attn_merge(o_acc, lse_acc, o_part, lse_part, o_acc, lse_acc, o_bf16 if c == n - 1 else None, stream=stream)
        for c, plan in enumerate(plans):
            A.attn_block_bwd(plan, tq, kv[c][0], kv[c][1], o_bf16, lse_acc, tdo, dq, dkv[c][0], dkv[c][1], ws,
                             dq_accumulate=c > 0, reuse_statistics=c > 0, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    A.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    A.profile_enable(False)
    prof = A.profile_read()
    for p in plans:
        p.destroy()
    probe = torch.empty(A.probe_scratch_bytes(), dtype=torch.uint8, device=dev)
    mfma_measured = A.probe_mfma_tflops(probe, stream=stream)

    # visible (row, key) pairs of this rank's rows: row at position p of its sequence sees p + 1 keys
    pairs = sum(sum(range(edges[i][rank] + 1, edges[i][rank + 1] + 1)) for i in range(len(lengths)))
    fwd = 4.0 * d * hq * pairs
    ms_per_step = elapsed / args.steps * 1e3
    tflops = 3.5 * fwd / (ms_per_step * 1e-3) / 1e12
    kern = {name: (ms / max(args.steps, 1)) for name, (ms, cnt) in prof.items() if cnt}     # per step: all blocks of a step
    dominant = max(GEMMS, key=lambda name: kern.get(name, 0.0))
    achieved = GEMMS[dominant] * (fwd / 2.0) / (kern[dominant] * 1e-3) / 1e12 if kern[dominant] > 0 else 0.0
    out = {
        "metric": "context-parallel block step: varlen causal attn fwd+bwd TFLOP/s of one ring rank",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} cut into {n} chunks by position, rank {rank} (queries: chunk {rank} of every "
                               f"sequence; keys: all {n} chunks in turn)", "query_tokens": Tq, "q_heads": hq, "kv_heads": hkv,
                   "head_dim": d, "lengths": lengths, "visible_pairs_per_head": pairs, "fwd_useful_flops": fwd,
                   "step": f"{n} block plan refills + {n} block fwd + merges + {n} block bwd (D once, dQ accumulated)"},
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "kernel_ms_per_step": {name: round(ms, 4) for name, ms in kern.items()},
        "roofline": {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None,
                     "flops_per_launch": GEMMS[dominant] * (fwd / 2.0) / n,
                     "measured_mfma_peak": round(mfma_measured, 1),
                     "note": f"{GEMMS[dominant]} GEMMs over the rank's visible pairs; the {n} launches of a step "
                             "together, timed with HIP events on the launch stream"},
    }
    if not args.no_cpu_baseline:
        from oracle import block as ob
        # bounded sample: the shortest sequences of the pack (up to a pair budget), 2 q heads of one KV group
        f64 = lambda bits: w.bits_to_f32(bits).astype(np.float64)
        order = sorted(range(len(lengths)), key=lambda i: lengths[i])
        chosen, budget = [], 0
        for i in order:
            p_i = sum(range(edges[i][rank] + 1, edges[i][rank + 1] + 1))
            if chosen and budget + p_i > 6.0e6:
                break
            chosen.append(i); budget += p_i
        heads = min(hq, 2)
        s = 1.0 / math.sqrt(d)
        t1 = time.perf_counter()
        for i in chosen:
            rows = np.arange(cu[i] + edges[i][rank], cu[i] + edges[i][rank + 1])
            qs, dos = f64(q[rows][:, :heads]), f64(do[rows][:, :heads])
            o_sum = np.zeros((len(rows), heads, d)); l_sum = np.full((heads, len(rows)), -np.inf)
            blocks = []
            for c in range(n):
                keys = np.arange(cu[i] + edges[i][c], cu[i] + edges[i][c + 1])
                ks, vs = f64(k[keys][:, :1]), f64(v[keys][:, :1])
                geom = ([len(rows)], [len(keys)], [edges[i][rank]], [edges[i][c]], s)
                po, pl = ob.block_fwd(qs, ks, vs, *geom)
                o_sum, l_sum = ob.merge(o_sum, l_sum, po, pl)
                blocks.append((ks, vs, geom))
            dsum = ob.row_dot(o_sum, dos)
            for ks, vs, geom in blocks:
                ob.block_bwd(qs, ks, vs, dos, l_sum, dsum, *geom)
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": 3.5 * 4.0 * d * heads * budget / dt / 1e12, "unit": "TFLOP/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f"block oracle (numpy fp64) on sequences {[lengths[i] for i in chosen]} of the "
                                         f"same pack, {heads} q heads / 1 kv head, all {n} blocks fwd + merge + bwd, {dt:.1f} s"}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C4", help="C1..C5 (default: the 32768-token asymmetric-head pack)")
    ap.add_argument("--grad-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--order", default="xcd_cost", choices=["xcd_cost", "natural", "cost"],
                    help="launch order of the work lists; the default is the library's, the others exist to "
                         "measure what it buys")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the steps, run one plain device copy of 1 GiB (a kernel of known HBM traffic "
                         "that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--ring", type=int, default=0,
                    help="N > 0: measure the block variant instead: one rank of a context-parallel ring of N chunks "
                         "(see run_ring); the default 0 measures the packed path")
    ap.add_argument("--ring-rank", type=int, default=-1, help="which chunk the rank owns (default: the last, heaviest)")
    ap.add_argument("--inputs", default="workload", choices=["workload", "zeros"],
                    help="zeros: all-zero q, k, v, dO (same instruction stream, almost no switching activity): shows how "
                         "much of the kernel time is the power-limited clock.  A side measurement, not a benchmark result")
    ap.add_argument("--sample-power", action="store_true",
                    help="read the socket power and the shader clock with amd-smi / rocm-smi while the timed steps run "
                         "(use several thousand --steps: the readings are one-second averages); reported under 'power'")
    ap.add_argument("--probe", action="store_true",
                    help="run the matrix-core probes instead of the attention step (see run_probe)")
    ap.add_argument("--probe-seconds", type=float, default=4.0, help="how long each probe runs while power is sampled")
    ap.add_argument("--rope", action="store_true",
                    help="add rotary embedding to the step: q, k rotated by the elementwise kernel before the forward, "
                         "dQ and dK turned back inside the backward epilogues (side measurement)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the batch on one GPU; --gpus above 1 is not part of this "
              "build (no collectives, no sharding across GPUs).", file=sys.stderr)
        return 2

    if args.probe:
        return run_probe(args)
    if args.ring > 0:
        return run_ring(args)

    import numpy as np
    import torch
    import hspmd_workloads as w
    import paper_2504_20490_amd as A

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    A.load_library()     # no fallback: raises if the HIP library is missing

    cfg = w.config_by_name(args.workload)
    lengths, q, k, v, do = w.make_inputs(cfg)
    T, hq, hkv, d = cfg.total_tokens, cfg.q_heads, cfg.kv_heads, cfg.head_dim
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def bf(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    tq, tk, tv, tdo = bf(q), bf(k), bf(v), bf(do)
    if args.inputs == "zeros":
        for t in (tq, tk, tv, tdo):
            t.zero_()
    o = torch.empty_like(tq)
    lse = torch.empty(hq, T, dtype=torch.float32, device=dev)
    grad = A.GRAD_F32 if args.grad_dtype == "f32" else A.GRAD_BF16
    gd = torch.float32 if grad == A.GRAD_F32 else torch.bfloat16
    dq = torch.empty(T, hq, d, dtype=gd, device=dev)
    dk = torch.empty(T, hkv, d, dtype=gd, device=dev)
    dv = torch.empty_like(dk)
    ws = torch.empty(2 * hq * T * 4 + 256, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    order = {"xcd_cost": A.ORDER_XCD_COST, "natural": A.ORDER_NATURAL, "cost": A.ORDER_COST}[args.order]

    if args.rope:
        positions = max(lengths)
        table = torch.empty(positions, d // 2, 2, dtype=torch.float32, device=dev)
        A.rope_table(table, positions, d, 10000.0, stream=stream)      # per model, not per step
        tq_rot, tk_rot = torch.empty_like(tq), torch.empty_like(tk)

    # One plan for the whole run, made before the first step as a training loop would; every step refills it with
    # its pack (hspmd_attn_plan_update: the work lists are rebuilt on the host and uploaded into storage the plan
    # owns, while the previous step's kernels run): no device allocation, no free and no device-wide wait per step.
    cu0, _, _ = A.build_cu_seqlens(lengths)
    plan = A.Plan(cu0, hq, hkv, d, stream.cuda_stream, order=order)

    def step():
        cu, _, _ = A.build_cu_seqlens(lengths)                 # packed offsets
        plan.update(cu)                                        # cost-sorted work lists of this step's pack
        if args.rope:
            A.rope_qk(plan, tq, tk, tq_rot, tk_rot, table, positions, stream=stream)
            A.attn_varlen_fwd(plan, tq_rot, tk_rot, tv, o, lse, stream=stream)
            A.attn_varlen_bwd_rope(plan, tq_rot, tk_rot, tv, o, lse, tdo, dq, dk, dv, ws, table, positions,
                                   grad_dtype=grad, stream=stream)
            return
        A.attn_varlen_fwd(plan, tq, tk, tv, o, lse, stream=stream)
        A.attn_varlen_bwd(plan, tq, tk, tv, o, lse, tdo, dq, dk, dv, ws, grad_dtype=grad, stream=stream)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)              # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sampler = PowerSampler() if args.sample_power else None
    A.profile_enable(not args.sample_power)      # a long power run would pile up two events per launch: timing off
    torch.cuda.synchronize()
    if sampler:
        sampler.start()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
        if sampler and i % 64 == 63:
            torch.cuda.synchronize()             # keep the launch queue short; the device stays busy
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    power = sampler.stop() if sampler else None
    A.profile_enable(False)
    if args.sample_power:                        # per-kernel times from a short timed run of the same step
        A.profile_enable(True)
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        A.profile_enable(False)
    stats = A.profile_read_stats()
    prof = {name: (st["mean"] * st["launches"], st["launches"]) for name, st in stats.items()}

    # host-only share of a step (offsets + work lists + upload into the plan), timed separately for the record
    t1 = time.perf_counter()
    for _ in range(5):
        cu, _, _ = A.build_cu_seqlens(lengths)
        plan.update(cu)
    plan_ms = (time.perf_counter() - t1) / 5 * 1e3
    plan.destroy()

    # measured matrix-core rate of this device (register-only MFMA loop): a second denominator beside the nominal peak
    probe = torch.empty(A.probe_scratch_bytes(), dtype=torch.uint8, device=dev)
    mfma_measured = A.probe_mfma_tflops(probe, stream=stream)
    # the same loop on operands that vary like real data: the chip is power-limited, its clock depends on the toggling
    mfma_measured_varied = A.probe_mfma_tflops(probe, stream=stream, varied_operands=True)
    del probe

    ms_per_step = elapsed / args.steps * 1e3
    fwd = w.fwd_flops(lengths, hq, d)
    useful = 3.5 * fwd
    tflops = useful / (ms_per_step * 1e-3) / 1e12
    pair_flops = fwd / 2.0          # one GEMM over the visible pairs: 2*d flops per pair and head

    kern = {name: ms / n for name, (ms, n) in prof.items() if n}
    dominant = max(GEMMS, key=lambda name: kern.get(name, 0.0))
    dom_ms = kern[dominant]
    achieved = GEMMS[dominant] * pair_flops / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0

    from paper_2504_20490_amd.build import sources_digest
    traffic, traffic_source = read_traffic(dominant, cfg.name.split("_")[0])
    out = {
        "metric": "varlen causal attn fwd+bwd TFLOP/s and % bf16 MFMA peak, 32k-token mix",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.note}", "total_tokens": T, "q_heads": hq, "kv_heads": hkv,
                   "head_dim": d, "num_seqs": len(lengths), "lengths": lengths,
                   "sum_L_Lplus1": 2 * w.causal_pairs(lengths), "fwd_useful_flops": fwd,
                   "grad_dtype": args.grad_dtype, "order": args.order,
                   "kernel_sources_sha256_16": sources_digest(),
                   "step": "build_cu_seqlens + work lists (plan refill, no device allocation) + fwd + "
                           "bwd(dQ pass with the row statistic D, dK/dV pass)"},
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "kernel_ms": {name: round(ms, 4) for name, ms in kern.items()},
        "kernel_ms_median": {name: round(st["median"], 4) for name, st in stats.items()},
        "kernel_ms_min": {name: round(st["min"], 4) for name, st in stats.items()},
        "host_plan_ms": round(plan_ms, 4),
        "roofline": {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "flops_per_launch": GEMMS[dominant] * pair_flops,
                     "measured_mfma_peak": round(mfma_measured, 1),
                     "frac_of_measured_peak": round(achieved / mfma_measured, 4) if mfma_measured > 0 else None,
                     "measured_mfma_peak_varied_operands": round(mfma_measured_varied, 1),
                     "frac_of_measured_peak_varied_operands":
                         round(achieved / mfma_measured_varied, 4) if mfma_measured_varied > 0 else None,
                     "note": f"{GEMMS[dominant]} GEMMs over the visible pairs; avg of {prof[dominant][1]} launches "
                             "timed with HIP events on the launch stream"},
    }
    if power is not None:
        out["power"] = power
    if args.inputs == "zeros":
        out["metric"] = "varlen causal attn fwd+bwd on ALL-ZERO inputs (clock-dependence probe, not a benchmark result)"
        out["data"] = "zeros"
    if args.rope:
        # the rotation kernel is an HBM stream: q and k read once and written once
        rope_bytes = 2.0 * 2.0 * T * (hq + hkv) * d
        rope_ms = kern.get("rope_qk_kernel", 0.0)
        gbs = rope_bytes / (rope_ms * 1e-3) / 1e9 if rope_ms > 0 else 0.0
        out["metric"] = "varlen causal attn fwd+bwd with rotary embedding, attention TFLOP/s, 32k-token mix"
        out["config"]["step"] = ("build_cu_seqlens + work lists (plan refill) + rope(q, k) + fwd + "
                                 "bwd(dQ pass with D, dK/dV pass; dQ, dK turned back)")
        out["rope_roofline"] = {"bound": "hbm", "kernel": "rope_qk_kernel", "achieved": round(gbs, 1), "peak": 8000.0,
                                "unit": "GB/s", "frac": round(gbs / 8000.0, 4), "traffic": None,
                                "bytes_per_launch": rope_bytes}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, lengths, q, k, v, do, rope=args.rope)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
