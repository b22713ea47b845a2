"""Pins of the oracle's cache-level calls and decode attention (Sec. 3.2.1, 3.3, 3.4 item 2)."""
import numpy as np
import pytest
import torch

import kvmix_synth as synth
from oracle.kvmix_ref import RefCache


def u16(a):
    return np.ascontiguousarray(a).view(np.uint16)


def h(a):
    return np.asarray(a, np.uint16).view(np.float16).astype(np.float64)


def build_cache(B, Hq, Hkv, T, W, kb, vb, seed=0, layer=0):
    q, k, v = synth.gen_layer_numpy(seed, layer, B, Hq, Hkv, T)
    n_q = T - W if kb != 16 else 0
    c = RefCache(B, Hq, Hkv, kb, vb, W, max(n_q, 32), ((T - n_q + 63) // 32) * 32)
    if n_q:
        assert c.quantize_pack(u16(k[:, :, :n_q]), u16(v[:, :, :n_q])) == 0
    c.set_window(u16(k[:, :, n_q:]), u16(v[:, :, n_q:]))
    return q, k, v, c


def attn_np(q, K, V, G, scale=None):
    """softmax(q K^T / sqrt(D)) V in binary64; q [B,Hq,D], K/V [B,Hkv,T,D]."""
    B, Hq, D = q.shape
    scale = scale or 1.0 / np.sqrt(D)
    out = np.zeros((B, Hq, D))
    for b in range(B):
        for hh in range(Hq):
            a = K[b, hh // G] @ q[b, hh] * scale
            p = np.exp(a - a.max())
            out[b, hh] = (p / p.sum()) @ V[b, hh // G]
    return out


@pytest.mark.parametrize("kb,vb,G", [(16, 16, 1), (16, 16, 4), (2, 2, 1), (3, 4, 2)])
def test_window_only_equals_library_attention(kb, vb, G):
    """A 16-bit setting, or a window covering the whole context, is exact fp attention: compare
    with torch's scaled_dot_product_attention in fp64."""
    B, Hkv, T = 2, 2, 96
    q, k, v, c = build_cache(B, Hkv * G, Hkv, T, T, kb, vb)
    assert c.n_q == 0
    st, out = c.decode_attn(u16(q))
    assert st == 0
    tq = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    tk = torch.from_numpy(k.astype(np.float64)).repeat_interleave(G, 1)
    tv = torch.from_numpy(v.astype(np.float64)).repeat_interleave(G, 1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0, :].numpy()
    assert np.array_equal(out, want.astype(np.float16).view(np.uint16)) or np.max(np.abs(h(out) - want)) <= 2.0 ** -11 * np.abs(want).max()
    assert np.max(np.abs(h(out) - want)) <= np.maximum(np.abs(want), 2.0 ** -14).max() * 2.0 ** -11


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 3), (4, 4), (2, 4), (3, 2), (1, 1), (1, 3)])
def test_dequant_is_within_half_step_of_inputs(kb, vb):
    """Cache-level round trip: every dequantized Key/Value is within s_i/2 of the fp16 input, with the
    Key step constant along tokens of a channel and the Value step constant along 32 channels of a token."""
    B, Hkv, T, W = 1, 2, 160, 32
    q, k, v, c = build_cache(B, Hkv, Hkv, T, W, kb, vb, seed=3)
    n_q = T - W
    Kd, Vd = c.dequant(0).reshape(B, Hkv, n_q, 128), c.dequant(1).reshape(B, Hkv, n_q, 128)
    ks = h(c.k_scale).reshape(B, Hkv, n_q // 32, 1, 128)          # per (tile, channel)
    vs = h(c.v_scale).reshape(B, Hkv, n_q // 32, 4, 32)            # [tile][g][tau]
    kstep = np.broadcast_to(ks, (B, Hkv, n_q // 32, 32, 128)).reshape(B, Hkv, n_q, 128).copy()
    vstep = np.repeat(vs.transpose(0, 1, 2, 4, 3).reshape(B, Hkv, n_q, 4), 32, axis=-1)
    if kb == 3:
        kstep.reshape(B, Hkv, n_q // 32, 32, 128)[:, :, :, [10, 21], :] *= 7 / 3
    if vb == 3:
        vstep.reshape(B, Hkv, n_q, 4, 32)[..., [10, 21]] *= 7 / 3
    assert np.all(np.abs(Kd - k[:, :, :n_q].astype(np.float64)) <= kstep / 2 * (1 + 1e-6))
    assert np.all(np.abs(Vd - v[:, :, :n_q].astype(np.float64)) <= vstep / 2 * (1 + 1e-6))
    # zero-points are the group minima
    kz = h(c.k_zero).reshape(B, Hkv, n_q // 32, 128)
    assert np.array_equal(kz, k[:, :, :n_q].astype(np.float64).reshape(B, Hkv, n_q // 32, 32, 128).min(3))
    vz = h(c.v_zero).reshape(B, Hkv, n_q // 32, 4, 32)
    want = v[:, :, :n_q].astype(np.float64).reshape(B, Hkv, n_q // 32, 32, 4, 32).min(-1).transpose(0, 1, 2, 4, 3)
    assert np.array_equal(vz, want)


@pytest.mark.parametrize("kb,vb,G", [(2, 2, 1), (3, 4, 1), (4, 3, 4), (2, 4, 8), (1, 2, 2), (4, 1, 1)])
def test_attention_is_plain_attention_over_dequantized_cache(kb, vb, G):
    B, Hkv, T, W = 2, 2, 224, 32
    q, k, v, c = build_cache(B, Hkv * G, Hkv, T, W, kb, vb, seed=5)
    n_q = T - W
    Kf = np.concatenate([c.dequant(0).reshape(B, Hkv, n_q, 128), k[:, :, n_q:].astype(np.float64)], 2)
    Vf = np.concatenate([c.dequant(1).reshape(B, Hkv, n_q, 128), v[:, :, n_q:].astype(np.float64)], 2)
    want = attn_np(q.astype(np.float64), Kf, Vf, G)
    st, out = c.decode_attn(u16(q))
    assert st == 0
    assert np.max(np.abs(h(out) - want)) <= 2.0 ** -11 * np.abs(want).max()
    # softmax_scale argument
    st, out2 = c.decode_attn(u16(q), 0.05)
    assert np.max(np.abs(h(out2) - attn_np(q.astype(np.float64), Kf, Vf, G, 0.05))) <= 2.0 ** -11 * 4


def test_invariances():
    """Softmax attention facts: output inside the convex hull of V~ rows; permuting whole 32-token
    tiles of (K, V) together changes nothing; a single-token context returns that token's V."""
    B, Hkv, G, T, W = 1, 1, 2, 128, 32
    q, k, v, c = build_cache(B, Hkv * G, Hkv, T, W, 2, 2, seed=9)
    st, out = c.decode_attn(u16(q))
    Vf = np.concatenate([c.dequant(1)[0], v[0, 0, T - W:].astype(np.float64)], 0)
    o = h(out)[0]
    assert np.all(o <= Vf.max(0) + 1e-3) and np.all(o >= Vf.min(0) - 1e-3)
    # permute packed tiles
    perm = [2, 0, 1]
    c2 = RefCache(B, Hkv * G, Hkv, 2, 2, W, T - W, 64)
    kk = k[:, :, :T - W].reshape(B, Hkv, 3, 32, 128)[:, :, perm].reshape(B, Hkv, T - W, 128)
    vv = v[:, :, :T - W].reshape(B, Hkv, 3, 32, 128)[:, :, perm].reshape(B, Hkv, T - W, 128)
    c2.quantize_pack(u16(kk), u16(vv))
    c2.set_window(u16(k[:, :, T - W:]), u16(v[:, :, T - W:]))
    st, out2 = c2.decode_attn(u16(q))
    assert np.max(np.abs(h(out2) - h(out))) <= 2.0 ** -10 * np.abs(h(out)).max()
    # single token
    c3 = RefCache(1, 1, 1, 16, 16, 32, 32, 32)
    c3.set_window(u16(k[:, :, :1]), u16(v[:, :, :1]))
    st, out3 = c3.decode_attn(u16(q[:, :1]))
    assert st == 0 and np.array_equal(out3[0, 0], u16(v[0, 0, 0]))


def test_tiny_brute_force():
    """Pure-Python evaluation of the definition on a tiny cache (no numpy linear algebra)."""
    import math
    B, Hkv, G, T, W = 1, 1, 1, 40, 8
    q, k, v, c = build_cache(B, Hkv * G, Hkv, T, W, 4, 2, seed=11)
    Kd, Vd = c.dequant(0)[0], c.dequant(1)[0]
    rows_k = [list(map(float, r)) for r in Kd] + [[float(x) for x in r] for r in k[0, 0, T - W:]]
    rows_v = [list(map(float, r)) for r in Vd] + [[float(x) for x in r] for r in v[0, 0, T - W:]]
    qq = [float(x) for x in q[0, 0]]
    a = [sum(qq[d] * rk[d] for d in range(128)) / math.sqrt(128) for rk in rows_k]
    m = max(a)
    p = [math.exp(x - m) for x in a]
    want = [sum(p[t] * rows_v[t][d] for t in range(T)) / sum(p) for d in range(128)]
    st, out = c.decode_attn(u16(q))
    assert np.max(np.abs(h(out)[0, 0] - np.array(want))) <= 2.0 ** -11 * max(abs(x) for x in want)


def test_per_channel_keys_isolate_outliers():
    """Sec. 3.2.1: per-channel Key groups keep outlier channels from inflating the error of the
    others; grouping the same Keys per token (the Value routine) is far worse."""
    B, Hkv, T = 1, 2, 256
    q, k, v = synth.gen_layer_numpy(21, 0, B, Hkv, Hkv, T)
    ch = synth.outlier_channels(21, 0, Hkv)
    c = RefCache(B, Hkv, Hkv, 2, 2, 32, T, 64)
    c.quantize_pack(u16(k), u16(k))            # Keys through both routines
    e_chan = np.abs(c.dequant(0).reshape(B, Hkv, T, 128) - k.astype(np.float64))
    e_tok = np.abs(c.dequant(1).reshape(B, Hkv, T, 128) - k.astype(np.float64))
    for j in range(Hkv):
        normal = np.setdiff1d(np.arange(128), ch[j])
        assert e_tok[0, j][:, normal].mean() > 1.8 * e_chan[0, j][:, normal].mean()


def test_append_matches_bulk_quantization():
    """Appending token by token through the ring window gives the same packed cache and the same
    attention output as bulk quantization of the aged tokens (Sec. 3.3, Fig. 4)."""
    B, Hkv, G, W, T0, steps = 1, 2, 2, 32, 96, 70
    q, k, v = synth.gen_layer_numpy(31, 0, B, Hkv * G, Hkv, T0 + steps)
    c = RefCache(B, Hkv * G, Hkv, 3, 4, W, 256, 64)
    c.quantize_pack(u16(k[:, :, :T0 - W]), u16(v[:, :, :T0 - W]))
    c.set_window(u16(k[:, :, T0 - W:T0]), u16(v[:, :, T0 - W:T0]))
    for s in range(steps):
        assert c.append(u16(k[:, :, T0 + s]), u16(v[:, :, T0 + s])) == 0
    T = T0 + steps
    assert c.n_q + c.n_w == T and W <= c.n_w < W + 32 and c.n_q % 32 == 0
    c2 = RefCache(B, Hkv * G, Hkv, 3, 4, W, 256, 64)
    c2.quantize_pack(u16(k[:, :, :c.n_q]), u16(v[:, :, :c.n_q]))
    c2.set_window(u16(k[:, :, c.n_q:T]), u16(v[:, :, c.n_q:T]))
    n_t = c.n_q // 32
    assert np.array_equal(c.k_codes[:, :n_t], c2.k_codes[:, :n_t]) and np.array_equal(c.v_codes[:, :n_t], c2.v_codes[:, :n_t])
    assert np.array_equal(c.k_scale[:, :n_t], c2.k_scale[:, :n_t]) and np.array_equal(c.v_zero[:, :n_t], c2.v_zero[:, :n_t])
    st1, o1 = c.decode_attn(u16(q))
    st2, o2 = c2.decode_attn(u16(q))
    assert st1 == 0 and st2 == 0 and np.array_equal(o1, o2)


def test_bit_table_statistics():
    """Sec. 4.2: 20 % of the layers at the high bit-width gives mean Key bits 2.1875 and mean Value
    bits 2.375 for a 32-layer model."""
    k, v = synth.bit_table(32)
    assert set(k) <= {2, 3} and set(v) <= {2, 4}
    assert k.mean() == 2.1875 and v.mean() == 2.375
    k80, v80 = synth.bit_table(80)
    assert k80.mean() == 2.2 and v80.mean() == 2.4
    # effective bits incl. fp16 scale + minimum per 32 elements: compression vs fp16 close to the paper's 4.9x
    assert abs(16 / ((k.mean() + v.mean()) / 2 + 1) - 4.9) < 0.05


def test_error_returns():
    c = RefCache(1, 1, 1, 2, 2, 32, 64, 64)
    bad = np.zeros((1, 1, 48, 128), np.uint16)
    assert c.quantize_pack(bad, bad) == -4              # not a multiple of 32
    big = np.zeros((1, 1, 96, 128), np.uint16)
    assert c.quantize_pack(big, big) == -4              # beyond capacity
    c5 = RefCache(1, 1, 1, 5, 2, 32, 64, 64)
    ok = np.zeros((1, 1, 32, 128), np.uint16)
    assert c5.quantize_pack(ok, ok) == -2
