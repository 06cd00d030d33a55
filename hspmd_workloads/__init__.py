"""Seeded synthetic inputs for packed variable-length causal attention.

This module is shared by the tests, the benchmark, the CPU oracle's callers and
the GPU path's callers.  It holds NO attention arithmetic: only a counter-based
random generator, the length mixes of the five benchmark configurations and the
bf16 rounding of the generated values.

The mixed-length evaluation of the paper (Section "Evaluations", scenario (c):
a 32B model trained on packed CommonCrawl / GitHub batches with 16K and 32K
context limits, where 97% of the sequences are shorter than 8K) is not
reproducible without its datasets; the length mixes below stand in for it:
long-tailed lengths with most of the mass below 8K and a tail that reaches the
context limit.

Generator: element ``i`` of stream ``(seed, tensor_id)`` is a pure function of
``(seed, tensor_id, i)`` (splitmix64 finaliser -> two 53-bit uniforms ->
Box-Muller), so any process can regenerate any slice of any tensor without
generating the rest and without depending on a framework RNG stream.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Sequence, Tuple

import numpy as np

__all__ = [
    "Config", "CONFIGS", "config_by_name", "lengths_for", "normal_f32",
    "round_to_bf16", "bf16_bits", "make_tensor", "make_inputs",
    "causal_pairs", "fwd_flops", "TENSOR_IDS",
]

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

TENSOR_IDS = {"q": 1, "k": 2, "v": 3, "do": 4, "lengths": 9}


def _mix64_inplace(z: np.ndarray, tmp: np.ndarray) -> None:
    """splitmix64 output function (Steele, Lea, Flood 2014), in place on uint64."""
    np.right_shift(z, _U64(30), out=tmp); z ^= tmp; z *= _M1
    np.right_shift(z, _U64(27), out=tmp); z ^= tmp; z *= _M2
    np.right_shift(z, _U64(31), out=tmp); z ^= tmp


def _stream_key(seed: int, stream: int) -> np.uint64:
    z = np.asarray([(seed * 0x100000001B3 + stream) & (2**64 - 1)], dtype=_U64)
    with np.errstate(over="ignore"):
        _mix64_inplace(z, np.empty_like(z))
    return z[0]


_BLOCK = 1 << 15   # samples per inner block: keeps the temporaries cache-resident


def _uniform53_block(key: np.uint64, counter: np.ndarray, tmp: np.ndarray) -> np.ndarray:
    """Uniform doubles in (0, 1) for uint64 counters: 53 random bits + half a step."""
    with np.errstate(over="ignore"):
        z = (counter + _U64(1)) * _GOLDEN + key
        _mix64_inplace(z, tmp)
    z >>= _U64(11)
    return (z.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform_f64(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """Uniform(0,1) samples ``start .. start+count-1`` of stream (seed, tensor_id)."""
    key = _stream_key(seed, tensor_id)
    out = np.empty(count, dtype=np.float64)
    for off in range(0, count, _BLOCK):
        n = min(_BLOCK, count - off)
        ctr = np.arange(start + off, start + off + n, dtype=_U64)
        out[off:off + n] = _uniform53_block(key, ctr, np.empty(n, dtype=_U64))
    return out


def normal_f64(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """Standard normal samples ``start .. start+count-1`` of a stream, float64.

    Sample ``i`` uses uniforms ``2i`` and ``2i+1`` of the stream (Box-Muller,
    cosine branch only, so that every sample depends on its own index alone)."""
    key = _stream_key(seed, tensor_id)
    out = np.empty(count, dtype=np.float64)
    for off in range(0, count, _BLOCK):
        n = min(_BLOCK, count - off)
        ctr = np.arange(start + off, start + off + n, dtype=_U64)
        ctr *= _U64(2)
        tmp = np.empty(n, dtype=_U64)
        u1 = _uniform53_block(key, ctr, tmp)
        ctr += _U64(1)
        u2 = _uniform53_block(key, ctr, tmp)
        np.log(u1, out=u1)
        u1 *= -2.0
        np.sqrt(u1, out=u1)
        u2 *= 2.0 * math.pi
        np.cos(u2, out=u2)
        u1 *= u2
        out[off:off + n] = u1
    return out


def normal_f32(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    return normal_f64(seed, tensor_id, start, count).astype(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16 value, returned as float32."""
    return bits_to_f32(bf16_bits(x))


@dataclasses.dataclass(frozen=True)
class Config:
    """One benchmark configuration: a length mix, a local head share, values."""
    name: str
    total_tokens: int
    q_heads: int          # local query heads on this GPU (may be an uneven share)
    kv_heads: int         # local KV heads (q_heads % kv_heads == 0)
    head_dim: int
    value_seed: int
    length_seed: int
    value_scale: float    # multiplies the N(0,1) samples before bf16 rounding
    kind: str             # "fixed" | "lognormal" | "bimodal"
    fixed_lengths: Tuple[int, ...] = ()
    mu: float = 0.0
    sigma: float = 0.0
    lo: int = 0
    hi: int = 0
    note: str = ""


CONFIGS: Tuple[Config, ...] = (
    Config("C1_tiny", 192, 2, 2, 64, 0, 0, 1.0, "fixed", fixed_lengths=(17, 64, 111),
           note="3 sequences, 2 heads, head_dim 64"),
    Config("C2_uniform", 16384, 32, 32, 128, 2, 0, 1.0, "fixed", fixed_lengths=(2048,) * 8,
           note="8 x 2048, dense-batch equivalent"),
    Config("C3_mixed16k", 16384, 32, 32, 128, 3, 1003, 1.0, "lognormal",
           mu=math.log(1024.0), sigma=1.0, lo=32, hi=8192,
           note="log-normal lengths filled to 16384 tokens"),
    Config("C4_asym32k", 32768, 24, 24, 128, 4, 1004, 1.0, "lognormal",
           mu=math.log(2048.0), sigma=1.2, lo=64, hi=16384,
           note="24 of 40 heads (3:2 uneven split of a hidden-5120 model), 32768 tokens"),
    Config("C5_bimodal_gqa", 65536, 32, 8, 128, 5, 1005, 1.0 / math.sqrt(128.0), "bimodal",
           lo=256, hi=2048, note="70% U[256,2048], 30% U[16384,32768]; 32 q heads on 8 kv heads"),
    # the shape of the paper's own 32B model (model configuration table: hidden 6656, 64 heads, head_dim 104) under a
    # 4-way split of the hidden dimension, on its default workload of 4K-token sequences
    Config("P1_paper32b_4k", 32768, 16, 16, 104, 6, 0, 1.0, "fixed", fixed_lengths=(4096,) * 8,
           note="8 x 4096, 16 of 64 heads, head_dim 104"),
)


def config_by_name(name: str) -> Config:
    for c in CONFIGS:
        if c.name == name or c.name.split("_")[0] == name:
            return c
    raise KeyError(name)


def _fill(draw, total: int) -> List[int]:
    """Append drawn lengths until ``total`` tokens; the last one is cut to fit
    (it may fall below the clip floor; it is kept, not merged)."""
    out: List[int] = []
    running = 0
    i = 0
    while running < total:
        length = int(draw(i))
        i += 1
        if running + length > total:
            length = total - running
        out.append(length)
        running += length
    return out


def lengths_for(cfg: Config) -> List[int]:
    """The realised sequence lengths of a configuration (deterministic)."""
    if cfg.kind == "fixed":
        assert sum(cfg.fixed_lengths) == cfg.total_tokens
        return list(cfg.fixed_lengths)
    sid = TENSOR_IDS["lengths"]
    if cfg.kind == "lognormal":
        def draw(i: int) -> int:
            z = float(normal_f64(cfg.length_seed, sid, i, 1)[0])
            length = math.floor(math.exp(cfg.mu + cfg.sigma * z) + 0.5)
            return min(max(length, cfg.lo), cfg.hi)
        return _fill(draw, cfg.total_tokens)
    if cfg.kind == "bimodal":
        def draw(i: int) -> int:
            u = uniform_f64(cfg.length_seed, sid, 2 * i, 2)
            if u[0] < 0.7:
                lo, hi = 256, 2048
            else:
                lo, hi = 16384, 32768
            return lo + min(int(u[1] * (hi - lo + 1)), hi - lo)
        return _fill(draw, cfg.total_tokens)
    raise ValueError(cfg.kind)


def make_tensor(seed: int, name: str, n_elements: int, scale: float = 1.0,
                start: int = 0, chunk: int = 1 << 20, threads: int = 8) -> np.ndarray:
    """bf16 bit patterns (uint16) of ``scale * N(0,1)`` samples ``start..``.

    The float32 value of a sample is ``float32(z) * float32(scale)`` rounded to
    bf16 with round-to-nearest-even; both the oracle's callers and the GPU
    path's callers reinterpret these same bits.  The result does not depend on
    ``chunk`` or ``threads`` (every sample is a function of its own index)."""
    tid = TENSOR_IDS[name]
    out = np.empty(n_elements, dtype=np.uint16)
    s32 = np.float32(scale)

    def fill(off: int) -> None:
        n = min(chunk, n_elements - off)
        z = normal_f32(seed, tid, start + off, n)
        if scale != 1.0:
            z = z * s32
        out[off:off + n] = bf16_bits(z)

    offsets = range(0, n_elements, chunk)
    if len(offsets) > 4 and threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(fill, offsets))
    else:
        for off in offsets:
            fill(off)
    return out


def make_inputs(cfg: Config, lengths: Sequence[int] | None = None):
    """Return ``(lengths, q, k, v, do)``: bf16 bit patterns, token-major
    ``[T, heads, head_dim]`` (uint16 arrays)."""
    if lengths is None:
        lengths = lengths_for(cfg)
    total = int(sum(lengths))
    d = cfg.head_dim
    q = make_tensor(cfg.value_seed, "q", total * cfg.q_heads * d, cfg.value_scale).reshape(total, cfg.q_heads, d)
    k = make_tensor(cfg.value_seed, "k", total * cfg.kv_heads * d, cfg.value_scale).reshape(total, cfg.kv_heads, d)
    v = make_tensor(cfg.value_seed, "v", total * cfg.kv_heads * d, cfg.value_scale).reshape(total, cfg.kv_heads, d)
    do = make_tensor(cfg.value_seed, "do", total * cfg.q_heads * d, cfg.value_scale).reshape(total, cfg.q_heads, d)
    return list(lengths), q, k, v, do


def causal_pairs(lengths: Sequence[int]) -> int:
    """Number of visible (query, key) pairs: sum of L(L+1)/2."""
    return sum(int(l) * (int(l) + 1) // 2 for l in lengths)


def fwd_flops(lengths: Sequence[int], q_heads: int, head_dim: int) -> int:
    """Useful forward FLOPs: two GEMMs of 2*d flops per visible pair and head,
    i.e. 2 * sum L(L+1) * d * heads.  Backward is counted as 2.5x this."""
    return 4 * causal_pairs(lengths) * head_dim * q_heads
