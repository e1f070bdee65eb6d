"""Pins for oracle/forward.py: triple loops, closed forms, library routines, invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import forward as fw
from paper_2604_15750_amd import inputs

RNG = np.random.default_rng(0)


def test_widen_bf16_bits_exact():
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x4049, 0xBF00], dtype=np.uint16)
    # 1.0, -2.0, 1.5, 0, 3.140625 (bf16 nearest below pi), -0.5
    np.testing.assert_array_equal(fw.widen(bits), [1.0, -2.0, 1.5, 0.0, 3.140625, -0.5])
    t = torch.randn(1000, dtype=torch.float32).to(torch.bfloat16)
    np.testing.assert_array_equal(fw.widen(inputs.tensor_to_numpy(t)), t.to(torch.float64).numpy())


def test_matmul_nt_triple_loop():
    x, w = RNG.standard_normal((3, 5)), RNG.standard_normal((4, 5))
    ref = np.zeros((3, 4))
    for r in range(3):
        for o in range(4):
            for i in range(5):
                ref[r, o] += x[r, i] * w[o, i]
    np.testing.assert_allclose(fw.matmul_nt(x, w), ref, rtol=1e-14)
    # a transposed operand would not even have this shape; check a non-symmetric closed case
    assert fw.matmul_nt(np.array([[1.0, 2.0]]), np.array([[3.0, 4.0], [5.0, 6.0], [0.0, 1.0]])).tolist() == [[11.0, 17.0, 2.0]]


def test_rmsnorm_closed_form_and_library():
    out = fw.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)
    rms = math.sqrt(12.5)
    np.testing.assert_allclose(out, [[3 / rms, 8 / rms]], rtol=1e-15)
    x, g = RNG.standard_normal((7, 64)), RNG.standard_normal(64)
    y = fw.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, rtol=1e-14)
    lib = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(fw.rmsnorm(x, g, 1e-5), lib, rtol=1e-13)


def test_swiglu_values_and_library():
    assert fw.swiglu(np.zeros(3), np.array([1.0, -2.0, 5.0])).tolist() == [0.0, 0.0, 0.0]
    np.testing.assert_allclose(fw.swiglu(np.array([1.0]), np.array([2.0])), [2 * 0.7310585786300049], rtol=1e-15)
    np.testing.assert_allclose(fw.swiglu(np.array([40.0]), np.array([3.0])), [120.0], rtol=1e-15)
    g, u = RNG.standard_normal(50), RNG.standard_normal(50)
    lib = (F.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    np.testing.assert_allclose(fw.swiglu(g, u), lib, rtol=1e-13)


def test_rope_rotation_direction_and_pairing():
    # hd = 2: one pair (0, 1), frequency 1: a plain 2-D rotation by `pos` radians, counter-clockwise
    x = np.array([[[1.0, 0.0]]])
    np.testing.assert_allclose(fw.rope(x, [math.pi / 2], 10000.0), [[[0.0, 1.0]]], atol=1e-15)
    # hd = 4: pairs are (0, 2) and (1, 3), the second with frequency theta^(-1/2)
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    out = fw.rope(x, [2.0], 100.0)
    np.testing.assert_allclose(out, [[[math.cos(2.0), math.cos(0.2), math.sin(2.0), math.sin(0.2)]]], atol=1e-15)


def test_rope_identity_isometry_relative():
    q, k = RNG.standard_normal((1, 1, 32)), RNG.standard_normal((1, 1, 32))
    np.testing.assert_array_equal(fw.rope(q, [0], 10000.0), q)
    r = fw.rope(q, [37], 10000.0)
    np.testing.assert_allclose(np.linalg.norm(r), np.linalg.norm(q), rtol=1e-14)
    d1 = np.sum(fw.rope(q, [5], 10000.0) * fw.rope(k, [2], 10000.0))
    d2 = np.sum(fw.rope(q, [105], 10000.0) * fw.rope(k, [102], 10000.0))
    d3 = np.sum(fw.rope(q, [5], 10000.0) * fw.rope(k, [3], 10000.0))
    np.testing.assert_allclose(d1, d2, rtol=1e-10)
    assert abs(d1 - d3) > 1e-3


def _attention_loops(q, k, v):
    A, Hq, hd = q.shape
    T, Hkv, _ = k.shape
    out = np.zeros_like(q)
    for a in range(A):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            s = [sum(q[a, h, e] * k[t, g, e] for e in range(hd)) / math.sqrt(hd) for t in range(T)]
            mx = max(s)
            w = [math.exp(si - mx) for si in s]
            tot = sum(w)
            for e in range(hd):
                out[a, h, e] = sum(w[t] * v[t, g, e] for t in range(T)) / tot
    return out


def test_attention_scalar_loops_and_library():
    q, k, v = RNG.standard_normal((3, 4, 8)), RNG.standard_normal((6, 2, 8)), RNG.standard_normal((6, 2, 8))
    got = fw.attention(q, k, v)
    np.testing.assert_allclose(got, _attention_loops(q, k, v), rtol=1e-12)
    tq = torch.from_numpy(q).permute(1, 0, 2)
    tk = torch.from_numpy(np.repeat(k, 2, axis=1)).permute(1, 0, 2)
    tv = torch.from_numpy(np.repeat(v, 2, axis=1)).permute(1, 0, 2)
    lib = F.scaled_dot_product_attention(tq, tk, tv, is_causal=False).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-11)


def test_attention_special_cases():
    q = RNG.standard_normal((5, 2, 16))
    k1, v1 = RNG.standard_normal((1, 2, 16)), RNG.standard_normal((1, 2, 16))
    np.testing.assert_allclose(fw.attention(q, k1, v1), np.broadcast_to(v1, (5, 2, 16)), rtol=1e-14)
    k = np.repeat(k1, 7, axis=0)
    v = RNG.standard_normal((7, 2, 16))
    np.testing.assert_allclose(fw.attention(q, k, v), np.broadcast_to(v.mean(0), (5, 2, 16)), rtol=1e-13)
    k, perm = RNG.standard_normal((7, 2, 16)), RNG.permutation(7)
    np.testing.assert_allclose(fw.attention(q, k, v), fw.attention(q, k[perm], v[perm]), rtol=1e-12)
    # last query row sees the LAST key as much as the first (no causal mask): plant a huge match
    k[:] = 0
    k[6, :, :] = q[0, :, :] * 50
    np.testing.assert_allclose(fw.attention(q[:1], k, v)[0], v[6], rtol=1e-6)


def _tiny_cfg():
    c = inputs.model_config(2, 32, 4, 2, 8, 48, 64, "f32")
    W = inputs.weights_to_numpy(inputs.make_weights(c, seed=3))
    for key in ("wqkv", "wo", "w_gate_up", "w_down"):  # larger weights so every stage matters
        W[key] = [w * 8 for w in W[key]]
    return c, W


def test_forward_replay_invariant_and_commit():
    cfg, W = _tiny_cfg()
    toks = RNG.integers(0, 63, size=20)
    s = 12
    cache = fw.KVCache(cfg)
    z_full = fw.forward_span(cfg, W, cache, toks, 0, s)
    assert cache.kv_len == s
    z_re = fw.forward_span(cfg, W, cache, toks[s:], s, 0)
    assert cache.kv_len == s
    np.testing.assert_allclose(z_re, z_full[s:], rtol=1e-10, atol=1e-12)
    # changing a span token changes the logits of the other span rows (bidirectional inside the span)
    t2 = toks[s:].copy()
    t2[-1] = (t2[-1] + 1) % 63
    z_ch = fw.forward_span(cfg, W, cache, t2, s, 0)
    assert np.abs(z_ch[0] - z_re[0]).max() > 1e-6


def test_forward_matches_library_composition():
    """The whole stack against torch CPU fp64 library ops on a GQA toy model."""
    cfg, W = _tiny_cfg()
    toks = RNG.integers(0, 63, size=9)
    z = fw.forward_span(cfg, W, fw.KVCache(cfg), toks, 0, 0)
    Hq, Hkv, hd, d = 4, 2, 8, 32
    T = {k: [torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in v] if isinstance(v, list)
         else torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in W.items()}
    h = T["embed"][torch.from_numpy(toks)]
    pos = torch.arange(9, dtype=torch.float64)
    inv = 10000.0 ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    cs = torch.polar(torch.ones(9, hd // 2, dtype=torch.float64), pos[:, None] * inv[None])

    def rot(x):  # complex multiplication on (x_i, x_{i+hd/2}) pairs
        xc = torch.complex(x[..., : hd // 2], x[..., hd // 2 :]) * cs[:, None, :]
        return torch.cat([xc.real, xc.imag], -1)

    for l in range(2):
        x = F.rms_norm(h, (d,), T["norm1"][l], eps=1e-5)
        qkv = F.linear(x, T["wqkv"][l])
        q, k, v = qkv.split([Hq * hd, Hkv * hd, Hkv * hd], dim=-1)
        q, k, v = rot(q.view(9, Hq, hd)), rot(k.view(9, Hkv, hd)), v.view(9, Hkv, hd)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2).repeat_interleave(2, 0),
                                           v.permute(1, 0, 2).repeat_interleave(2, 0))
        h = h + F.linear(o.permute(1, 0, 2).reshape(9, Hq * hd), T["wo"][l])
        x = F.rms_norm(h, (d,), T["norm2"][l], eps=1e-5)
        g, u = F.linear(x, T["w_gate_up"][l]).chunk(2, dim=-1)
        h = h + F.linear(F.silu(g) * u, T["w_down"][l])
    ref = F.linear(F.rms_norm(h, (d,), T["final_norm"], eps=1e-5), T["lm_head"]).numpy()
    np.testing.assert_allclose(z, ref, rtol=1e-9, atol=1e-11)


def test_suffix_entries_replay_invariant():
    """Dual-cache suffix: a pass over [0, s+a+u) that commits [0, s) leaves the keys and values of its other rows as tail
    entries.  Re-running only the rows [s, s+a) with the same tokens, against the cache and the u suffix entries, sees
    exactly the keys the long pass saw, so it reproduces the long pass's logits for those rows; without the suffix it
    does not; and the suffix is not recomputed (changing the block's tokens leaves the tail beyond the block as it was)."""
    cfg = inputs.model_config(2, 64, 4, 2, 32, 96, 50, "f32")
    W = inputs.weights_to_numpy(inputs.make_weights(cfg, seed=3))
    rng = np.random.default_rng(5)
    s, a, u = 7, 5, 6
    toks = rng.integers(0, 49, size=s + a + u)
    cache = fw.KVCache(cfg)
    z_long = fw.forward_span(cfg, W, cache, toks, 0, s)
    tail_before = [t.copy() for t in cache.tail_k]
    z_with = fw.forward_span(cfg, W, cache, toks[s : s + a], s, 0, suffix_len=u)
    assert np.allclose(z_with, z_long[s : s + a], rtol=0, atol=1e-9)
    # same block tokens: the block's entries are recomputed to the same values, the ones beyond it are kept as they were
    assert all(np.allclose(t0, t1, rtol=0, atol=1e-9) and np.array_equal(t0[a:], t1[a:]) for t0, t1 in zip(tail_before, cache.tail_k))
    z_without = fw.forward_span(cfg, W, cache, toks[s : s + a], s, 0)
    assert np.abs(z_without - z_long[s : s + a]).max() > 1e-3
    t2 = toks[s : s + a].copy()
    t2[1] = (t2[1] + 1) % 49
    fw.forward_span(cfg, W, cache, t2, s, 0, suffix_len=u)
    assert all(np.array_equal(t0[a:], t1[a:]) for t0, t1 in zip(tail_before, cache.tail_k))  # entries beyond the block are kept
    with pytest.raises(AssertionError):
        fw.forward_span(cfg, W, cache, toks[s : s + a], s, 0, suffix_len=u + 1)  # no cached keys there
