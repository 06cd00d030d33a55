"""ctypes binding of the C ABI declared in include/hspmd_attn.h (same names, no arithmetic)."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libhspmd_attn.so")

LIST_FWD, LIST_DQ, LIST_DKV = 0, 1, 2
GRAD_BF16, GRAD_F32 = 0, 1
ORDER_XCD_COST, ORDER_NATURAL, ORDER_COST = 0, 1, 2

_STATUS = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE_TOO_SMALL", 4: "HIP"}


class HspmdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"hspmd status {_STATUS.get(status, status)}: {message}")
        self.status = status


class WorkItem(ctypes.Structure):
    _fields_ = [("token_start", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("tile", ctypes.c_int32), ("head", ctypes.c_int32)]


class BlockItem(ctypes.Structure):
    _fields_ = [("q_start", ctypes.c_int32), ("q_len", ctypes.c_int32), ("k_start", ctypes.c_int32),
                ("k_len", ctypes.c_int32), ("offset", ctypes.c_int32), ("tile", ctypes.c_int32),
                ("head", ctypes.c_int32), ("q_pos", ctypes.c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_2504_20490_amd.build "
            "or __graft_entry__.build())")
    lib = ctypes.CDLL(_LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    vp = ctypes.c_void_p
    lib.hspmd_last_error.restype = ctypes.c_char_p
    lib.hspmd_last_error.argtypes = []
    lib.hspmd_attn_tile_rows.restype = ctypes.c_int32
    lib.hspmd_attn_tile_rows.argtypes = [ctypes.c_int]
    lib.hspmd_build_cu_seqlens.restype = ctypes.c_int
    lib.hspmd_build_cu_seqlens.argtypes = [i32p, ctypes.c_int32, i32p, i32p, i64p]
    lib.hspmd_attn_schedule.restype = ctypes.c_int
    lib.hspmd_attn_schedule.argtypes = [ctypes.c_int, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.POINTER(WorkItem), ctypes.c_int64, i64p]
    lib.hspmd_attn_schedule_ordered.restype = ctypes.c_int
    lib.hspmd_attn_schedule_ordered.argtypes = [ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int32, ctypes.c_int32,
                                                ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(WorkItem),
                                                ctypes.c_int64, i64p]
    lib.hspmd_attn_plan_create_ordered.restype = ctypes.c_int
    lib.hspmd_attn_plan_create_ordered.argtypes = [i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                   ctypes.c_int, vp, ctypes.POINTER(vp)]
    lib.hspmd_attn_plan_create.restype = ctypes.c_int
    lib.hspmd_attn_plan_create.argtypes = [i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           vp, ctypes.POINTER(vp)]
    lib.hspmd_attn_plan_update.restype = ctypes.c_int
    lib.hspmd_attn_plan_update.argtypes = [vp, i32p, ctypes.c_int32]
    lib.hspmd_attn_block_plan_update.restype = ctypes.c_int
    lib.hspmd_attn_block_plan_update.argtypes = [vp, i32p, i32p, i32p, i32p, ctypes.c_int32]
    lib.hspmd_attn_plan_destroy.restype = ctypes.c_int
    lib.hspmd_attn_plan_destroy.argtypes = [vp]
    lib.hspmd_attn_plan_total_tokens.restype = ctypes.c_int64
    lib.hspmd_attn_plan_total_tokens.argtypes = [vp]
    lib.hspmd_attn_plan_num_items.restype = ctypes.c_int64
    lib.hspmd_attn_plan_num_items.argtypes = [vp, ctypes.c_int]
    lib.hspmd_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.hspmd_attn_bwd_workspace_bytes.argtypes = [vp]
    lib.hspmd_attn_varlen_fwd.restype = ctypes.c_int
    lib.hspmd_attn_varlen_fwd.argtypes = [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                          vp, vp, vp]
    lib.hspmd_attn_varlen_bwd.restype = ctypes.c_int
    lib.hspmd_attn_varlen_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_float, vp, vp, vp, ctypes.c_int, vp, ctypes.c_size_t, vp]
    lib.hspmd_attn_varlen_bwd_static_ws.restype = ctypes.c_int
    lib.hspmd_attn_varlen_bwd_static_ws.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                                    ctypes.c_float, vp, vp, vp, ctypes.c_int, vp]
    lib.hspmd_profile_enable.restype = ctypes.c_int
    lib.hspmd_profile_enable.argtypes = [ctypes.c_int32]
    lib.hspmd_rope_table_bytes.restype = ctypes.c_size_t
    lib.hspmd_rope_table_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.hspmd_rope_table.restype = ctypes.c_int
    lib.hspmd_rope_table.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, vp]
    lib.hspmd_rope_qk.restype = ctypes.c_int
    lib.hspmd_rope_qk.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp, vp, ctypes.c_int64, ctypes.c_int64, vp,
                                  ctypes.c_int32, ctypes.c_int32, vp]
    lib.hspmd_attn_varlen_bwd_rope.restype = ctypes.c_int
    lib.hspmd_attn_varlen_bwd_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                               ctypes.c_float, vp, vp, vp, ctypes.c_int, vp, ctypes.c_int32, vp,
                                               ctypes.c_size_t, vp]
    lib.hspmd_attn_block_bwd_rope.restype = ctypes.c_int
    lib.hspmd_attn_block_bwd_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                              vp, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, ctypes.c_int32, vp,
                                              ctypes.c_size_t, vp]
    lib.hspmd_attn_estimate_ms.restype = ctypes.c_int
    lib.hspmd_attn_estimate_ms.argtypes = [i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.hspmd_attn_block_schedule.restype = ctypes.c_int
    lib.hspmd_attn_block_schedule.argtypes = [ctypes.c_int, i32p, i32p, i32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(BlockItem),
                                              ctypes.c_int64, i64p]
    lib.hspmd_attn_block_plan_create.restype = ctypes.c_int
    lib.hspmd_attn_block_plan_create.argtypes = [i32p, i32p, i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                 ctypes.c_int32, vp, ctypes.POINTER(vp)]
    lib.hspmd_attn_plan_total_kv_tokens.restype = ctypes.c_int64
    lib.hspmd_attn_plan_total_kv_tokens.argtypes = [vp]
    lib.hspmd_attn_block_fwd.restype = ctypes.c_int
    lib.hspmd_attn_block_fwd.argtypes = [vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_float, vp, vp, vp]
    lib.hspmd_attn_merge.restype = ctypes.c_int
    lib.hspmd_attn_merge.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.hspmd_attn_block_bwd.restype = ctypes.c_int
    lib.hspmd_attn_block_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                         vp, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.hspmd_probe_scratch_bytes.restype = ctypes.c_size_t
    lib.hspmd_probe_scratch_bytes.argtypes = []
    lib.hspmd_probe_mfma_tflops.restype = ctypes.c_int
    lib.hspmd_probe_mfma_tflops.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                            ctypes.POINTER(ctypes.c_double)]
    lib.hspmd_probe_mfma_tflops_varied.restype = ctypes.c_int
    lib.hspmd_probe_mfma_tflops_varied.argtypes = lib.hspmd_probe_mfma_tflops.argtypes
    lib.hspmd_probe_mfma_rate.restype = ctypes.c_int
    lib.hspmd_probe_mfma_rate.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                          ctypes.POINTER(ctypes.c_double)]
    lib.hspmd_profile_read.restype = ctypes.c_int
    lib.hspmd_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), i64p]
    lib.hspmd_profile_read_stats.restype = ctypes.c_int
    lib.hspmd_profile_read_stats.argtypes = [ctypes.POINTER(ctypes.c_double), i64p, ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_double)]
    lib.hspmd_kernel_name.restype = ctypes.c_char_p
    lib.hspmd_kernel_name.argtypes = [ctypes.c_int32]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise HspmdError(status, load_library().hspmd_last_error().decode())


def _i32(a: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr32(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def tile_rows(kind: int) -> int:
    return int(load_library().hspmd_attn_tile_rows(kind))


def build_cu_seqlens(lengths: Sequence[int]) -> Tuple[np.ndarray, int, int]:
    """Returns (cu_seqlens int32 [B+1], max_seqlen, total_tokens)."""
    lib = load_library()
    raw = np.asarray(lengths, dtype=np.int64)
    if raw.size and (raw.max() > np.iinfo(np.int32).max or raw.min() < np.iinfo(np.int32).min):
        raise HspmdError(1, "sequence length does not fit int32")
    lens = _i32(lengths)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    mx = ctypes.c_int32(0)
    tot = ctypes.c_int64(0)
    _check(lib.hspmd_build_cu_seqlens(_ptr32(lens), len(lens), _ptr32(cu), ctypes.byref(mx), ctypes.byref(tot)))
    return cu, int(mx.value), int(tot.value)


def schedule(kind: int, cu_seqlens: Sequence[int], q_heads: int, kv_heads: int, num_queues: int = 8,
             order: int = ORDER_XCD_COST) -> np.ndarray:
    """Host-only: the launch-ordered work list as an int32 array [slots, 4]
    (token_start, seq_len, tile, head); padding slots have tile == -1."""
    lib = load_library()
    cu = _i32(cu_seqlens)
    n = ctypes.c_int64(0)
    _check(lib.hspmd_attn_schedule_ordered(kind, order, _ptr32(cu), len(cu) - 1, q_heads, kv_heads, num_queues, None, 0,
                                           ctypes.byref(n)))
    out = np.zeros((n.value, 4), dtype=np.int32)
    if n.value:
        _check(lib.hspmd_attn_schedule_ordered(kind, order, _ptr32(cu), len(cu) - 1, q_heads, kv_heads, num_queues,
                                               out.ctypes.data_as(ctypes.POINTER(WorkItem)), n.value, ctypes.byref(n)))
    return out


class Plan:
    """Device-resident work lists for one pack and one local head configuration."""

    def __init__(self, cu_seqlens: Sequence[int], q_heads: int, kv_heads: int, head_dim: int, stream: int = 0,
                 order: int = ORDER_XCD_COST):
        lib = load_library()
        cu = _i32(cu_seqlens)
        handle = ctypes.c_void_p(None)
        _check(lib.hspmd_attn_plan_create_ordered(_ptr32(cu), len(cu) - 1, q_heads, kv_heads, head_dim, order,
                                                  ctypes.c_void_p(stream), ctypes.byref(handle)))
        self._h = handle
        self.q_heads, self.kv_heads, self.head_dim = q_heads, kv_heads, head_dim
        self.total_tokens = int(lib.hspmd_attn_plan_total_tokens(handle))

    @property
    def handle(self) -> ctypes.c_void_p:
        if self._h is None:
            raise HspmdError(1, "plan already destroyed")
        return self._h

    def update(self, cu_seqlens: Sequence[int]) -> None:
        """Refill with the next pack (same head counts, head_dim and order): no device allocation in the steady state."""
        lib = load_library()
        cu = _i32(cu_seqlens)
        _check(lib.hspmd_attn_plan_update(self.handle, _ptr32(cu), len(cu) - 1))
        self.total_tokens = int(lib.hspmd_attn_plan_total_tokens(self.handle))

    def num_items(self, kind: int) -> int:
        return int(load_library().hspmd_attn_plan_num_items(self.handle, kind))

    def bwd_workspace_bytes(self) -> int:
        return int(load_library().hspmd_attn_bwd_workspace_bytes(self.handle))

    def destroy(self) -> None:
        if self._h is not None:
            h, self._h = self._h, None
            _check(load_library().hspmd_attn_plan_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _dev_ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def attn_varlen_fwd(plan: Plan, q, k, v, o, lse, softmax_scale: float = 0.0, stream=None) -> None:
    """q [T,Hq,d] / k,v [T,Hkv,d] bf16 device tensors (token stride = stride(0), unit inner strides);
    o bf16 [T,Hq,d] contiguous and lse fp32 [Hq,T] are written."""
    lib = load_library()
    _check(lib.hspmd_attn_varlen_fwd(plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v),
                                     _token_stride(q, plan.q_heads, plan.head_dim),
                                     _token_stride(k, plan.kv_heads, plan.head_dim),
                                     float(softmax_scale), _dev_ptr(o), _dev_ptr(lse), _stream_handle(stream)))


def attn_varlen_bwd(plan: Plan, q, k, v, o, lse, d_o, dq, dk, dv, workspace, softmax_scale: float = 0.0,
                    grad_dtype: int = GRAD_BF16, stream=None) -> None:
    """dq/dk/dv (bf16 or fp32 according to grad_dtype) are fully overwritten; workspace is any device
    tensor of at least plan.bwd_workspace_bytes() bytes."""
    lib = load_library()
    _check(lib.hspmd_attn_varlen_bwd(plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(o), _dev_ptr(lse),
                                     _dev_ptr(d_o),
                                     _token_stride(q, plan.q_heads, plan.head_dim),
                                     _token_stride(k, plan.kv_heads, plan.head_dim),
                                     float(softmax_scale), _dev_ptr(dq), _dev_ptr(dk), _dev_ptr(dv), int(grad_dtype),
                                     _dev_ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream_handle(stream)))


STATIC_WORKSPACE_BYTES = 16 * 1024 * 1024 + 256


def attn_varlen_bwd_static_ws(plan: Plan, q, k, v, o, lse, d_o, dq, dk, dv, softmax_scale: float = 0.0,
                              grad_dtype: int = GRAD_BF16, stream=None) -> None:
    """attn_varlen_bwd without a workspace argument: the library's fixed device array is used (no allocation)."""
    lib = load_library()
    _check(lib.hspmd_attn_varlen_bwd_static_ws(plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(o),
                                               _dev_ptr(lse), _dev_ptr(d_o),
                                               _token_stride(q, plan.q_heads, plan.head_dim),
                                               _token_stride(k, plan.kv_heads, plan.head_dim),
                                               float(softmax_scale), _dev_ptr(dq), _dev_ptr(dk), _dev_ptr(dv),
                                               int(grad_dtype), _stream_handle(stream)))


def _token_stride(x, heads: int, head_dim: int) -> int:
    return x.stride(0) if x.dim() == 3 and x.shape[0] > 1 else heads * head_dim


def rope_table_bytes(positions: int, head_dim: int) -> int:
    return int(load_library().hspmd_rope_table_bytes(int(positions), int(head_dim)))


def rope_table(table, positions: int, head_dim: int, base: float = 10000.0, stream=None) -> None:
    """Fills `table` (device fp32 tensor of at least rope_table_bytes(positions, head_dim) bytes) with the
    (cos, sin) pairs [positions, head_dim / 2, 2]."""
    if table.numel() * table.element_size() < rope_table_bytes(positions, head_dim):
        raise ValueError("table tensor is too small")
    _check(load_library().hspmd_rope_table(_dev_ptr(table), int(positions), int(head_dim), float(base),
                                           _stream_handle(stream)))


def rope_qk(plan: Plan, q, k, q_out, k_out, table, table_positions: int, inverse: bool = False, stream=None) -> None:
    """q_out, k_out = rope(q), rope(k) (in place when q_out is q and k_out is k)."""
    _check(load_library().hspmd_rope_qk(plan.handle, _dev_ptr(q), _dev_ptr(k),
                                        _token_stride(q, plan.q_heads, plan.head_dim),
                                        _token_stride(k, plan.kv_heads, plan.head_dim), _dev_ptr(q_out), _dev_ptr(k_out),
                                        _token_stride(q_out, plan.q_heads, plan.head_dim),
                                        _token_stride(k_out, plan.kv_heads, plan.head_dim), _dev_ptr(table),
                                        int(table_positions), 1 if inverse else 0, _stream_handle(stream)))


def attn_varlen_bwd_rope(plan: Plan, q, k, v, o, lse, d_o, dq, dk, dv, workspace, table, table_positions: int,
                         softmax_scale: float = 0.0, grad_dtype: int = GRAD_BF16, stream=None) -> None:
    """attn_varlen_bwd for rotated q, k; dq and dk come back with respect to the unrotated tensors."""
    _check(load_library().hspmd_attn_varlen_bwd_rope(
        plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(o), _dev_ptr(lse), _dev_ptr(d_o),
        _token_stride(q, plan.q_heads, plan.head_dim), _token_stride(k, plan.kv_heads, plan.head_dim),
        float(softmax_scale), _dev_ptr(dq), _dev_ptr(dk), _dev_ptr(dv), int(grad_dtype), _dev_ptr(table),
        int(table_positions), _dev_ptr(workspace), workspace.numel() * workspace.element_size(), _stream_handle(stream)))


NUM_KERNELS = 5


def profile_enable(on: bool) -> None:
    _check(load_library().hspmd_profile_enable(1 if on else 0))


def profile_read():
    """Returns {kernel name: (total ms, launches)} for the kernels launched since the last read."""
    lib = load_library()
    ms = (ctypes.c_double * NUM_KERNELS)()
    n = (ctypes.c_int64 * NUM_KERNELS)()
    _check(lib.hspmd_profile_read(ms, n))
    return {lib.hspmd_kernel_name(i).decode(): (float(ms[i]), int(n[i])) for i in range(NUM_KERNELS) if n[i] > 0}


def profile_read_stats():
    """Returns {kernel name: {"mean", "min", "median" (ms per launch), "launches"}} for the kernels launched since the
    last read."""
    lib = load_library()
    total, mn, med = ((ctypes.c_double * NUM_KERNELS)() for _ in range(3))
    n = (ctypes.c_int64 * NUM_KERNELS)()
    _check(lib.hspmd_profile_read_stats(total, n, mn, med))
    return {lib.hspmd_kernel_name(i).decode(): {"mean": float(total[i]) / int(n[i]), "min": float(mn[i]),
                                                "median": float(med[i]), "launches": int(n[i])}
            for i in range(NUM_KERNELS) if n[i] > 0}


def probe_scratch_bytes() -> int:
    return int(load_library().hspmd_probe_scratch_bytes())


def probe_mfma_tflops(scratch, mfma_per_wave: int = 1 << 18, stream=None, varied_operands: bool = False) -> float:
    """Measured dense bf16 MFMA rate (TFLOP/s) of the current device; scratch is a device tensor of at least
    probe_scratch_bytes() bytes.  varied_operands: pseudo-random operand values instead of constants (the clock
    the chip sustains depends on the switching activity).  Synchronises the stream."""
    out = ctypes.c_double(0.0)
    lib = load_library()
    fn = lib.hspmd_probe_mfma_tflops_varied if varied_operands else lib.hspmd_probe_mfma_tflops
    _check(fn(int(mfma_per_wave), _dev_ptr(scratch), scratch.numel() * scratch.element_size(), _stream_handle(stream),
              ctypes.byref(out)))
    return float(out.value)


PROBE_MODES = {"32x32x16 constant operands": 0, "32x32x16": 1, "16x16x32": 2, "32x32x16, A from LDS": 3,
               "16x16x32, A from LDS": 4, "32x32x16, one wave per SIMD": 5,
               "32x32x16, one wave per SIMD, 256 idle clocks per 512": 6,
               "32x32x16, one wave per SIMD, 512 idle clocks per 512": 7,
               "32x32x16, one wave per SIMD, 1024 idle clocks per 512": 8}


def probe_mfma_rate(mode: int, scratch, mfma_per_wave: int = 1 << 18, stream=None) -> float:
    """Dense bf16 rate (TFLOP/s) of one variant of the matrix-core probe (PROBE_MODES); synchronises the stream."""
    out = ctypes.c_double(0.0)
    _check(load_library().hspmd_probe_mfma_rate(int(mode), int(mfma_per_wave), _dev_ptr(scratch),
                                                scratch.numel() * scratch.element_size(), _stream_handle(stream),
                                                ctypes.byref(out)))
    return float(out.value)


# ---------------------------------------------------------------------------------- block variant
def block_schedule(kind: int, cu_q: Sequence[int], cu_k: Sequence[int], q_pos: Sequence[int], k_pos: Sequence[int],
                   q_heads: int, kv_heads: int, num_queues: int = 8) -> np.ndarray:
    """Host-only: the launch-ordered block work list as an int32 array [slots, 8]
    (q_start, q_len, k_start, k_len, offset, tile, head, q_pos); padding slots have tile == -1."""
    lib = load_library()
    cq, ck, qp, kp = _i32(cu_q), _i32(cu_k), _i32(q_pos), _i32(k_pos)
    if not (len(cq) == len(ck) == len(qp) + 1 == len(kp) + 1):
        raise HspmdError(1, "per-sequence arrays differ in length")
    n = ctypes.c_int64(0)
    args = (kind, _ptr32(cq), _ptr32(ck), _ptr32(qp), _ptr32(kp), len(qp), q_heads, kv_heads, num_queues)
    _check(lib.hspmd_attn_block_schedule(*args, None, 0, ctypes.byref(n)))
    out = np.zeros((n.value, 8), dtype=np.int32)
    if n.value:
        _check(lib.hspmd_attn_block_schedule(*args, out.ctypes.data_as(ctypes.POINTER(BlockItem)), n.value, ctypes.byref(n)))
    return out


class BlockPlan(Plan):
    """Work lists of one step of context-parallel attention: per sequence a query chunk and a key chunk."""

    def __init__(self, cu_q: Sequence[int], cu_k: Sequence[int], q_pos: Sequence[int], k_pos: Sequence[int],
                 q_heads: int, kv_heads: int, head_dim: int, stream: int = 0):
        lib = load_library()
        cq, ck, qp, kp = _i32(cu_q), _i32(cu_k), _i32(q_pos), _i32(k_pos)
        if not (len(cq) == len(ck) == len(qp) + 1 == len(kp) + 1):
            raise HspmdError(1, "per-sequence arrays differ in length")
        handle = ctypes.c_void_p(None)
        _check(lib.hspmd_attn_block_plan_create(_ptr32(cq), _ptr32(ck), _ptr32(qp), _ptr32(kp), len(qp), q_heads,
                                                kv_heads, head_dim, ctypes.c_void_p(stream), ctypes.byref(handle)))
        self._h = handle
        self.q_heads, self.kv_heads, self.head_dim = q_heads, kv_heads, head_dim
        self.total_tokens = int(lib.hspmd_attn_plan_total_tokens(handle))
        self.total_kv_tokens = int(lib.hspmd_attn_plan_total_kv_tokens(handle))

    def update(self, cu_q: Sequence[int], cu_k: Sequence[int], q_pos: Sequence[int], k_pos: Sequence[int]) -> None:
        """Refill with the chunks of the next ring step or pack: no device allocation in the steady state."""
        lib = load_library()
        cq, ck, qp, kp = _i32(cu_q), _i32(cu_k), _i32(q_pos), _i32(k_pos)
        if not (len(cq) == len(ck) == len(qp) + 1 == len(kp) + 1):
            raise HspmdError(1, "per-sequence arrays differ in length")
        _check(lib.hspmd_attn_block_plan_update(self.handle, _ptr32(cq), _ptr32(ck), _ptr32(qp), _ptr32(kp), len(qp)))
        self.total_tokens = int(lib.hspmd_attn_plan_total_tokens(self.handle))
        self.total_kv_tokens = int(lib.hspmd_attn_plan_total_kv_tokens(self.handle))


def _opt_ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(None) if t is None else _dev_ptr(t)


def attn_block_fwd(plan: BlockPlan, q, k, v, o_partial, lse_partial, softmax_scale: float = 0.0, stream=None) -> None:
    """q [Tq,Hq,d], k/v [Tk,Hkv,d] bf16; o_partial fp32 [Tq,Hq,d] and lse_partial fp32 [Hq,Tq] are written."""
    _check(load_library().hspmd_attn_block_fwd(plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v),
                                               _token_stride(q, plan.q_heads, plan.head_dim),
                                               _token_stride(k, plan.kv_heads, plan.head_dim), float(softmax_scale),
                                               _dev_ptr(o_partial), _dev_ptr(lse_partial), _stream_handle(stream)))


def attn_merge(o_a, lse_a, o_b, lse_b, o_out, lse_out, o_out_bf16=None, stream=None) -> None:
    """(o_out, lse_out) = (o_a, lse_a) merged with (o_b, lse_b); the output may be the `a` buffers."""
    T, hq, d = o_a.shape
    _check(load_library().hspmd_attn_merge(T, hq, d, _dev_ptr(o_a), _dev_ptr(lse_a), _dev_ptr(o_b), _dev_ptr(lse_b),
                                           _dev_ptr(o_out), _dev_ptr(lse_out), _opt_ptr(o_out_bf16),
                                           _stream_handle(stream)))


def attn_block_bwd(plan: BlockPlan, q, k, v, o, lse, d_o, dq, dk, dv, workspace, softmax_scale: float = 0.0,
                   dq_accumulate: bool = False, reuse_statistics: bool = False, stream=None) -> None:
    """o (bf16) / lse: merged results of the whole rows; dq fp32 (overwritten or accumulated), dk/dv fp32 written."""
    _check(load_library().hspmd_attn_block_bwd(plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _opt_ptr(o),
                                               _opt_ptr(lse), _dev_ptr(d_o),
                                               _token_stride(q, plan.q_heads, plan.head_dim),
                                               _token_stride(k, plan.kv_heads, plan.head_dim), float(softmax_scale),
                                               _dev_ptr(dq), 1 if dq_accumulate else 0, _dev_ptr(dk), _dev_ptr(dv),
                                               1 if reuse_statistics else 0, _dev_ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def attn_block_bwd_rope(plan: BlockPlan, q, k, v, o, lse, d_o, dq, dk, dv, workspace, table, table_positions: int,
                        softmax_scale: float = 0.0, dq_accumulate: bool = False, reuse_statistics: bool = False,
                        stream=None) -> None:
    """attn_block_bwd for rotated q, k chunks; dq and dk come back with respect to the unrotated tensors."""
    _check(load_library().hspmd_attn_block_bwd_rope(
        plan.handle, _dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _opt_ptr(o), _opt_ptr(lse), _dev_ptr(d_o),
        _token_stride(q, plan.q_heads, plan.head_dim), _token_stride(k, plan.kv_heads, plan.head_dim),
        float(softmax_scale), _dev_ptr(dq), 1 if dq_accumulate else 0, _dev_ptr(dk), _dev_ptr(dv),
        1 if reuse_statistics else 0, _dev_ptr(table), int(table_positions), _dev_ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def estimate_ms(cu_seqlens: Sequence[int], q_heads: int, kv_heads: int, head_dim: int) -> Tuple[float, float]:
    """Host-only: predicted (forward ms, backward ms) of the kernels for this pack on an MI355X."""
    cu = _i32(cu_seqlens)
    f, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(load_library().hspmd_attn_estimate_ms(_ptr32(cu), len(cu) - 1, q_heads, kv_heads, head_dim,
                                                 ctypes.byref(f), ctypes.byref(b)))
    return float(f.value), float(b.value)
