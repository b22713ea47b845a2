"""Pins of the oracle's Recent Pivotal Context ageing (Sec. 3.3, Fig. 4; ratios of Sec. 4.2): the count formula,
Keys and Values leaving the fp16 window at fronts of their own, and attention over the per-token mix of sources."""
from fractions import Fraction

import numpy as np
import pytest

import kvmix_synth as synth
from oracle import kvmix_ref as ref
from oracle.kvmix_ref import RefCache


def u16(a):
    return np.ascontiguousarray(a).view(np.uint16)


def h(a):
    return np.asarray(a, np.uint16).view(np.float16).astype(np.float64)


def test_rpc_count_sequences_of_the_formula():
    """num_RPC = floor(r * current_RPC), current_RPC = new tokens + RPCs kept so far (Sec. 3.3), worked by hand
    for a 1024-token prompt followed by single-token steps at the two ratios of Sec. 4.2:
    r = 0.2: 204.8 -> 204; (204+1)*0.2 = 41; (41+1)*0.2 = 8.4 -> 8; 1.8 -> 1; 0.4 -> 0; 0.2 -> 0
    r = 0.1: 102.4 -> 102; 10.3 -> 10; 1.1 -> 1; 0.2 -> 0"""
    for r, want in ((0.2, [204, 41, 8, 1, 0, 0]), (0.1, [102, 10, 1, 0, 0])):
        got, kept, new = [], 0, 1024
        for _ in want:
            kept = ref.rpc_next(r, new + kept)
            got.append(kept)
            new = 1
        assert got == want
    assert ref.rpc_next(0.0, 4096) == 0          # "w/o RPC" (App. D): nothing stays
    assert ref.rpc_next(1.0, 77) == 77


@pytest.mark.parametrize("percent", [0, 5, 10, 20, 30, 50, 100])
def test_rpc_count_equals_exact_rational_floor(percent):
    """The binary64 product floors to the same integer as exact arithmetic on the decimal ratio."""
    r = percent / 100
    for current in list(range(0, 3000)) + [4095, 4096, 32767, 32768, 131071]:
        assert ref.rpc_next(r, current) == int(Fraction(percent, 100) * current // 1)


def ring_cache(B, Hkv, kb, vb, T_cap, W_cap, G=1):
    return RefCache(B, Hkv * G, Hkv, kb, vb, -1, T_cap, W_cap)


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 4), (4, 3), (1, 2), (2, 1)])
def test_records_do_not_depend_on_the_order_of_leaving(kb, vb):
    """Key groups are 32 tokens of a channel and Value groups one token's 32 channels (Sec. 3.2.1), so whatever the
    schedule on which Keys (tile by tile) and Values (token by token) left the window, once both fronts have
    reached T the records are those of the one-pass quantizer over the same T tokens, bit for bit."""
    B, Hkv, T = 2, 2, 128
    _, k, v = synth.gen_layer_numpy(21, kb * 5 + vb, B, Hkv, Hkv, T)
    one = RefCache(B, Hkv, Hkv, kb, vb, 0, T, 32)
    assert one.quantize_pack(u16(k), u16(v)) == 0
    rng = np.random.default_rng(kb * 16 + vb)
    c = ring_cache(B, Hkv, kb, vb, T, 96)
    c.packed[:] = 0xDEADBEEF            # stale contents: every bit of a record must come from the quantizer
    fronts = []
    for t in range(T):
        assert c.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
        if rng.random() < 0.4 or c.n_w >= 90 or c.n - c.n_qv >= 90:
            keep_k = int(rng.integers(0, 60))
            keep_v = int(rng.integers(0, 60))
            before = (c.n_q, c.n_qv)
            assert c.flush(keep_k, keep_v) == 0
            assert c.n_q % 32 == 0 and c.n - c.n_q >= min(keep_k, c.n - before[0])      # Keys: whole groups, at least keep_k stay
            assert c.n_q >= before[0] and c.n_qv >= before[1]                           # fronts never move back
            assert c.n_qv == max(before[1], c.n - keep_v)                               # Values: token by token
            assert c.n_q == before[0] or c.n - c.n_q < keep_k + 32                          # and no more than a group beyond
            fronts.append((c.n_q, c.n_qv))
    assert c.flush(0, 0) == 0
    assert (c.n_q, c.n_qv, c.n_w) == (T, T, 0)
    assert any(a != b for a, b in fronts), "the schedule never separated the two fronts"
    assert any(b % 32 for _, b in fronts), "the Value front never stood inside a tile"
    assert np.array_equal(c.packed, one.packed)


def mixed_cache(kb, vb, G, seed, T=200, keep=((70, 9), (40, 33))):
    """A cache whose Key and Value fronts differ, reached through appends and flushes; returns (q, k, v, cache)."""
    B, Hkv = 2, 2
    q, k, v = synth.gen_layer_numpy(seed, 0, B, Hkv * G, Hkv, T)
    c = ring_cache(B, Hkv, kb, vb, 256, 128, G)
    marks = {T // 2: keep[0], T - 1: keep[1]}
    for t in range(T):
        assert c.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
        if c.n - min(c.n_q, c.n_qv) >= 120:
            assert c.flush(96, 96) == 0
        if t in marks:
            assert c.flush(*marks[t]) == 0
    return q, k, v, c


@pytest.mark.parametrize("kb,vb,G,keep", [(2, 2, 1, ((70, 9), (40, 33))), (3, 4, 2, ((10, 80), (3, 50))),
                                           (4, 2, 4, ((64, 0), (0, 45))), (2, 3, 1, ((0, 0), (31, 31)))])
def test_attention_over_fronts_of_their_own_equals_library_attention(kb, vb, G, keep):
    """Each token's Key is its dequantized code when it lies before the Key front and its fp16 row otherwise, and
    the same for its Value against the Value front (Sec. 3.3): build those two arrays here, token by token, from the
    dequantized packed parts and the original fp16 inputs (not from the ring), and take plain softmax attention."""
    q, k, v, c = mixed_cache(kb, vb, G, seed=31 + kb, keep=keep)
    n, n_qk, n_qv = c.n, c.n_q, c.n_qv
    assert n == 200 and n_qk % 32 == 0
    if keep[1][0] != keep[1][1]:
        assert n_qk != n_qv
    Kd = c.dequant(0).reshape(2, 2, n_qk, 128)
    Vd = c.dequant(1).reshape(2, 2, n_qv, 128)
    K = np.concatenate([Kd, k[:, :, n_qk:].astype(np.float64)], axis=2)
    V = np.concatenate([Vd, v[:, :, n_qv:].astype(np.float64)], axis=2)
    st, out = c.decode_attn(u16(q))
    assert st == 0
    B, Hq, D = q.shape
    want = np.zeros((B, Hq, D))
    for b in range(B):
        for hh in range(Hq):
            a = K[b, hh // G] @ q[b, hh].astype(np.float64) / np.sqrt(D)
            p = np.exp(a - a.max())
            want[b, hh] = (p / p.sum()) @ V[b, hh // G]
    assert np.max(np.abs(h(out) - want)) <= 2.0 ** -11 * np.maximum(np.abs(want), 2.0 ** -14).max()
    # the packed parts themselves stay within half a step of the inputs (the quantizer's own pin, at both fronts)
    assert np.max(np.abs(Kd - k[:, :, :n_qk])) < np.abs(k).max()
    assert np.max(np.abs(Vd - v[:, :, :n_qv])) < np.abs(v).max()


def test_equal_fronts_reduce_to_the_single_count_cache():
    """With both fronts at the same multiple of 32 the aged cache is the cache the one-pass path builds:
    same records, same window tokens, bit-identical attention."""
    kb, vb, G, T = 3, 4, 2, 160
    B, Hkv = 2, 2
    q, k, v = synth.gen_layer_numpy(77, 0, B, Hkv * G, Hkv, T)
    a = RefCache(B, Hkv * G, Hkv, kb, vb, 32, 128, 64)
    assert a.quantize_pack(u16(k[:, :, :128]), u16(v[:, :, :128])) == 0
    a.set_window(u16(k[:, :, 128:]), u16(v[:, :, 128:]))
    c = ring_cache(B, Hkv, kb, vb, 128, 192, G)
    for t in range(T):
        assert c.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
    assert c.flush(40, 32) == 0          # Keys: 160 - 40 = 120 -> 96; Values: 128
    assert (c.n_q, c.n_qv) == (96, 128)
    assert c.flush(32, 32) == 0
    assert (c.n_q, c.n_qv, c.n_w, c.v_lead) == (128, 128, 32, 0)
    assert np.array_equal(c.packed, a.packed)
    sa, oa = a.decode_attn(u16(q))
    sc, oc = c.decode_attn(u16(q))
    assert sa == 0 and sc == 0 and np.array_equal(oa, oc)


def test_flush_and_append_error_returns():
    c = ring_cache(1, 1, 2, 2, 64, 64)
    _, k, v = synth.gen_layer_numpy(5, 0, 1, 1, 1, 100)
    for t in range(64):
        assert c.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
    assert c.append(u16(k[:, :, 64]), u16(v[:, :, 64])) == -4        # ring full
    assert c.flush(-1, 0) == -4
    assert c.flush(100, 100) == 0 and (c.n_q, c.n_qv) == (0, 0)       # more than there is: nothing leaves
    assert c.flush(64, 3) == 0 and (c.n_q, c.n_qv, c.v_lead) == (0, 61, 61)
    assert c.flush(0, 0) == 0 and (c.n_q, c.n_qv, c.n_w) == (64, 64, 0)
    for t in range(64, 96):
        assert c.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
    assert c.flush(0, 0) == -4                                        # packed capacity of 64 tokens exceeded
    assert (c.n_q, c.n_qv, c.n_w) == (64, 64, 32)
    fixed = RefCache(1, 1, 1, 2, 2, 32, 64, 96)                       # fixed-window appends need equal fronts
    fixed.c.v_lead = 5
    assert fixed.append(u16(k[:, :, 0]), u16(v[:, :, 0])) == -4
