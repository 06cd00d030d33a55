"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times, at the nominal bounds
(max-abs 2e-2 and relative Frobenius 1e-2 for O, dQ, dK, dV; LSE to 1e-3), with no magnitude slack.

C2, C3, C4: EVERY element of O, LSE, dQ, dK and dV of the whole pack against the full fp64 oracle.  The oracle needs
tens of seconds per configuration on the machine's host cores, so a configuration is checked in slices of heads (the heads
are independent; each slice is held to the bounds on its own, which is stricter than one comparison over the pack) and
the GPU runs once per configuration.  The worst element of every comparison is located (sequence, token, head, column)
in the assertion message and in the optional report.

C5 (10 TFLOP of fp64 work in full): every element of the twelve sequences of up to 3311 tokens, and, for the 29082-
and the 18500-token sequences, sampled rows (first rows, tile edges, one row in each half of a q tile, the end) and
sampled keys on the last KV group (whose four query heads are summed inside the dK/dV workgroup): the EARLY keys
0, 1, 63, 64, 127, 128, L/3, L/2, which collect a contribution from almost every row of the sequence and are the
heaviest elements of dK / dV, as well as the last ones.

Plus properties that hold at any size (no NaN anywhere, row 0 of every sequence has dQ ~ 0 and O = V)."""
import numpy as np
import pytest

import hspmd_workloads as w
import oracle
import gpu_util
from gpu_util import GpuRun, LSE_ABS, assert_close, default_scale, f64

pytestmark = pytest.mark.gpu

_CACHE = {}


def _config_run(name):
    """One GPU run per configuration, shared by its head slices (only the latest configuration is kept)."""
    if name not in _CACHE:
        import torch
        _CACHE.clear()
        cfg = w.config_by_name(name)
        lengths, q, k, v, do = w.make_inputs(cfg)
        run = GpuRun(lengths, q, k, v, do).run()
        for t in (run.o, run.lse, run.dq, run.dk, run.dv):
            assert not torch.isnan(t).any()
        G = cfg.q_heads // cfg.kv_heads
        cu = np.concatenate([[0], np.cumsum(lengths)])
        first = torch.from_numpy(cu[:-1][np.asarray(lengths) > 0]).cuda()
        assert float(run.dq[first].abs().max()) < 1e-5      # sum_j dS_0j = 0 up to fp32 rounding of P, dP, D
        for g in range(cfg.kv_heads):
            assert torch.equal(run.o[first][:, g * G:(g + 1) * G], run.v[first][:, g:g + 1].expand(-1, G, -1))
        host = {n: run.host(n) for n in ("o", "lse", "dq", "dk", "dv")}
        _CACHE[name] = (cfg, lengths, q, k, v, do, cu, host)
    return _CACHE[name]


def _where(cu, token):
    i = int(np.searchsorted(cu, token, side="right") - 1)
    return i, int(token - cu[i])


def _close_whole(name, got, ref, cu, head0):
    """assert_close at the nominal bounds, naming the worst element of a [tokens, heads, d] tensor."""
    t, h, c = np.unravel_index(int(np.argmax(np.abs(got - ref))), ref.shape)
    i, r = _where(cu, t)
    where = f"worst element: sequence {i} (L={int(cu[i + 1] - cu[i])}) token {r} head {head0 + int(h)} column {int(c)}, " \
            f"ref {ref[t, h, c]:+.4f} got {got[t, h, c]:+.4f}"
    gpu_util.CONTEXT["where"] = where
    try:
        return assert_close(name, got, ref)
    except AssertionError as e:
        raise AssertionError(f"{e}; {where}") from None
    finally:
        gpu_util.CONTEXT.pop("where", None)


@pytest.mark.parametrize("name,h0,h1", [("C2", 0, 32), ("C3", 0, 16), ("C3", 16, 32),
                                        ("C4", 0, 8), ("C4", 8, 16), ("C4", 16, 24)])
def test_whole_pack_every_element(name, h0, h1):
    cfg, lengths, q, k, v, do, cu, host = _config_run(name)
    assert cfg.q_heads == cfg.kv_heads                       # C2-C4 are MHA: a slice of q heads is the same slice of kv heads
    gpu_util.CONTEXT["case"] = f"{cfg.name} whole pack, heads {h0}..{h1 - 1}"
    s = default_scale(cfg.head_dim)
    hs = slice(h0, h1)
    qs, ks, vs, dos = f64(q[:, hs]), f64(k[:, hs]), f64(v[:, hs]), f64(do[:, hs])
    ro, rlse = oracle.attn_fwd(qs, ks, vs, lengths, s)
    rdq, rdk, rdv = oracle.attn_bwd(qs, ks, vs, dos, lengths, s)
    _close_whole("O", host["o"][:, hs], ro, cu, h0)
    lse_err = np.abs(host["lse"][hs] - rlse)
    assert lse_err.max() <= LSE_ABS, f"LSE max_abs {lse_err.max():.3e}"
    _close_whole("dQ", host["dq"][:, hs], rdq, cu, h0)
    _close_whole("dK", host["dk"][:, hs], rdk, cu, h0)
    _close_whole("dV", host["dv"][:, hs], rdv, cu, h0)


def test_c5_short_sequences_every_element():
    cfg, lengths, q, k, v, do, cu, host = _config_run("C5")
    gpu_util.CONTEXT["case"] = f"{cfg.name} every sequence of up to 3311 tokens, all heads"
    s = default_scale(cfg.head_dim)
    chosen = [i for i, L in enumerate(lengths) if L <= 3311]
    assert len(chosen) == len(lengths) - 2
    tok = np.concatenate([np.arange(cu[i], cu[i + 1]) for i in chosen])
    sl = [lengths[i] for i in chosen]
    sub_cu = np.concatenate([[0], np.cumsum(sl)])
    qs, ks, vs, dos = f64(q[tok]), f64(k[tok]), f64(v[tok]), f64(do[tok])
    ro, rlse = oracle.attn_fwd(qs, ks, vs, sl, s)
    rdq, rdk, rdv = oracle.attn_bwd(qs, ks, vs, dos, sl, s)
    _close_whole("O", host["o"][tok], ro, sub_cu, 0)
    assert np.max(np.abs(host["lse"][:, tok] - rlse)) <= LSE_ABS
    _close_whole("dQ", host["dq"][tok], rdq, sub_cu, 0)
    _close_whole("dK", host["dk"][tok], rdk, sub_cu, 0)
    _close_whole("dV", host["dv"][tok], rdv, sub_cu, 0)


@pytest.mark.parametrize("which", [0, 1])
def test_c5_long_sequences_sampled_rows_and_early_keys(which):
    cfg, lengths, q, k, v, do, cu, host = _config_run("C5")
    hq, hkv, d = cfg.q_heads, cfg.kv_heads, cfg.head_dim
    G = hq // hkv
    s = default_scale(d)
    j = sorted(range(len(lengths)), key=lambda i: -lengths[i])[which]
    L = lengths[j]
    assert L in (29082, 18500)
    gpu_util.CONTEXT["case"] = f"{cfg.name} sequence of {L} tokens, last KV group, sampled rows and keys"
    sl = slice(int(cu[j]), int(cu[j + 1]))
    g = hkv - 1
    hs = slice(g * G, (g + 1) * G)
    qs, ks, vs, dos = f64(q[sl, hs]), f64(k[sl, g:g + 1]), f64(v[sl, g:g + 1]), f64(do[sl, hs])
    last_tile = (L // 128) * 128
    rows = sorted({0, 1, 31, 32, 63, 64, 127, 128, 129, L // 3, L // 3 + 64, L // 2, L // 2 + 64, last_tile - 1,
                   last_tile % L, L - 2, L - 1})
    rows = [r for r in rows if 0 <= r < L]
    tok = np.repeat(rows, G)
    hd = np.tile(np.arange(G), len(rows))
    o_r, lse_r, dq_r = oracle.attn_rows(qs, ks, vs, dos, [L], s, tok, hd)
    assert_close("O rows", host["o"][sl, hs][tok, hd], o_r)
    assert_close("dQ rows", host["dq"][sl, hs][tok, hd], dq_r)
    assert np.max(np.abs(host["lse"][hs, sl][hd, tok] - lse_r)) <= LSE_ABS
    keys = sorted({0, 1, 63, 64, 127, 128, L // 3, L // 2, L - 200, L - 129, L - 64, L - 2, L - 1})
    dk_r, dv_r = oracle.attn_keys(qs, ks, vs, dos, [L], s, keys, [0] * len(keys))
    assert_close("dK keys", host["dk"][sl, g][keys], dk_r)
    assert_close("dV keys", host["dv"][sl, g][keys], dv_r)
    # the early keys alone (the heaviest elements): same bounds
    assert_close("dK early keys", host["dk"][sl, g][keys[:6]], dk_r[:6])
    assert_close("dV early keys", host["dv"][sl, g][keys[:6]], dv_r[:6])


def test_release_cached_run():
    """Frees the cached configuration (device tensors and host copies) before the tests that follow."""
    _CACHE.clear()
