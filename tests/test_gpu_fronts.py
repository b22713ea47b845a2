"""GPU parity: Keys and Values ageing at fronts of their own (Sec. 3.3): kvmix_flush, kvmix_rpc_next and the
attention / decode-step calls on a cache whose Value front differs from its Key front, against the oracle."""
import numpy as np
import pytest

import kvmix_synth as synth
from gpu_common import assert_attn_close, assert_windows_equal, bits_of, t16, u16
from oracle import kvmix_ref as ref
from oracle.kvmix_ref import RefCache

pytestmark = pytest.mark.gpu

POISON = 0xDEADBEEF      # both record buffers start with the same stale contents and must stay identical bit for bit


def make_ring_pair(B, Hq, Hkv, kb, vb, T_cap, W_cap):
    import torch
    import paper_2506_08018_amd as kv
    rc = RefCache(B, Hq, Hkv, kb, vb, -1, T_cap, W_cap)
    shape, cfg = kv.Shape(B, Hq, Hkv), kv.LayerCfg(kb, vb, -1)
    gc = kv.LayerCache(shape, cfg, T_cap, W_cap)
    rc.packed[:] = POISON
    gc.packed.view(torch.int32)[: rc.packed.size] = int(np.array(POISON, np.uint32).astype(np.int32))
    return rc, gc, shape, cfg


def assert_same_state(rc, gc, what):
    assert (gc.n_q, gc.n_w, gc.w0, gc.v_lead) == (rc.n_q, rc.n_w, rc.w0, rc.v_lead), what
    got = bits_of(gc.packed, np.uint32)[: rc.packed.size].reshape(rc.packed.shape)
    if not np.array_equal(got, rc.packed):
        bad = np.argwhere(got != rc.packed)
        raise AssertionError(f"{what}: {len(bad)} record words differ, first at (unit, tile, word) {tuple(bad[0])}: "
                             f"got {got[tuple(bad[0])]:#x} want {rc.packed[tuple(bad[0])]:#x}")


def attn_both(rc, gc, shape, cfg, q, n_splits=0, static=False, what=""):
    import torch
    import paper_2506_08018_amd as kv
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    if static:
        kv.decode_attn_static(shape, cfg, qt, gc, out, n_splits=n_splits)
    else:
        ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
        kv.decode_attn(shape, cfg, qt, gc, out, ws, n_splits=n_splits)
        torch.cuda.synchronize()
        assert not ws[: 4 * shape.units * max(1, shape.Hq // shape.Hkv // 8)].any(), "arrival counters not reset"
    torch.cuda.synchronize()
    assert_attn_close(t16(out), want, what, tight=True)


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 4), (4, 3), (1, 2), (2, 1), (3, 3), (4, 4), (1, 1)])
def test_flush_records_bit_exact_whatever_the_schedule(kb, vb):
    """Tokens enter one by one or in chunks; Keys leave tile by tile, Values token by token, on a seeded schedule.
    After every flush both sides hold the same counters and the same record buffer, bit for bit, stale words
    included (a flush writes the bits of the tokens that leave and nothing else)."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case flush kb={kb} vb={vb}", flush=True)
    B, Hkv, T = 2, 2, 224
    _, k, v = synth.gen_layer_numpy(700 + kb * 10 + vb, 0, B, Hkv, Hkv, T)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    rc, gc, shape, cfg = make_ring_pair(B, Hkv, Hkv, kb, vb, 256, 128)
    rng = np.random.default_rng(kb * 16 + vb)
    t, n_flush, apart, inside = 0, 0, 0, 0
    while t < T:
        room = 128 - (rc.n - min(rc.n_q, rc.n_qv))
        n = int(min(T - t, room, rng.choice([1, 1, 2, 5, 17, 29])))
        if n > 0:
            for i in range(n):
                assert rc.append(u16(k[:, :, t + i]), u16(v[:, :, t + i])) == 0
            if n == 1:
                kv.append(shape, cfg, kt[:, :, t].contiguous(), vt[:, :, t].contiguous(), gc)
            else:
                kv.append_tokens(shape, cfg, kt[:, :, t:t + n], vt[:, :, t:t + n], gc)
            t += n
        if rng.random() < 0.6 or room - n < 8:
            keep_k, keep_v = (int(x) for x in rng.integers(0, 70, 2))
            assert rc.flush(keep_k, keep_v) == 0
            kv.flush(shape, cfg, gc, keep_k, keep_v)
            torch.cuda.synchronize()
            assert_same_state(rc, gc, f"after flush {n_flush} (keep {keep_k}/{keep_v}, n={rc.n})")
            n_flush += 1
            apart += rc.v_lead != 0
            inside += rc.n_qv % 32 != 0
    assert n_flush >= 4 and apart >= 2 and inside >= 2, (n_flush, apart, inside)
    assert rc.flush(0, 0) == 0
    kv.flush(shape, cfg, gc, 0, 0)
    torch.cuda.synchronize()
    assert_same_state(rc, gc, "final")
    assert (gc.n_q, gc.n_qv, gc.n_w) == (T, T, 0)
    # and the buffer is the one-pass quantizer's
    one = RefCache(B, Hkv, Hkv, kb, vb, 0, 256, 32)
    assert one.quantize_pack(u16(k), u16(v)) == 0
    got = bits_of(gc.packed, np.uint32)[: rc.packed.size].reshape(rc.packed.shape)
    assert np.array_equal(got[:, : T // 32], one.packed[:, : T // 32])


STATES = [      # (tokens, [(keep_k, keep_v) flushes in order]): what the fronts look like afterwards is in the comment
    (200, [(70, 9)]),            # K 128, V 191: Value front ahead, inside a tile; window tokens 192..199
    (200, [(9, 70)]),            # K 160, V 130: Key front ahead, Value front inside a tile
    (200, [(40, 33)]),           # K 160, V 167: both fronts in the same tile
    (200, [(0, 0)]),             # K 192, V 200: every Value packed, no window token for the main launch
    (200, [(200, 0)]),           # K 0, V 200: nothing packed on the Key side
    (200, [(64, 200), (64, 72)]),  # K 128, V 128 after a detour: fronts equal again (plain path)
    (97, [(90, 3)]),             # K 0, V 94: short context, a single partial tile pair
    (230, [(100, 100), (38, 101)]),  # K 192, V 130: Key front two tiles ahead
]


@pytest.mark.parametrize("G", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("state", range(len(STATES)))
def test_attention_with_fronts_apart(G, state):
    import torch
    import paper_2506_08018_amd as kv
    T, flushes = STATES[state]
    kb, vb = [(2, 2), (3, 4), (4, 2), (2, 3), (1, 4)][(state + G) % 5]
    print(f"case fronts attn G={G} state={state} T={T} flushes={flushes} kb={kb} vb={vb}", flush=True)
    B, Hkv = 2, 2 if G < 16 else 1
    q, k, v = synth.gen_layer_numpy(800 + state, G, B, Hkv * G, Hkv, T)
    rc, gc, shape, cfg = make_ring_pair(B, Hkv * G, Hkv, kb, vb, 256, 256)
    for t in range(T):
        assert rc.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
    kv.append_tokens(shape, cfg, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), gc)
    for keep_k, keep_v in flushes:
        assert rc.flush(keep_k, keep_v) == 0
        kv.flush(shape, cfg, gc, keep_k, keep_v)
    torch.cuda.synchronize()
    assert_same_state(rc, gc, "before attention")
    for n_splits, static in ((0, False), (1, False), (3, False), (2, True)):
        attn_both(rc, gc, shape, cfg, q, n_splits, static, f"G={G} state={state} splits={n_splits} static={static}")


@pytest.mark.parametrize("kb,vb,G,r_k,r_v", [(3, 2, 1, 0.2, 0.1), (2, 4, 4, 0.1, 0.2), (2, 2, 2, 0.1, 0.1), (3, 4, 8, 0.2, 0.2)])
def test_decode_loop_under_the_count_formula(kb, vb, G, r_k, r_v):
    """A 200-token prompt, then decode steps. Each step: the new token is appended and attended to (fused step),
    then num_RPC = floor(r * (new + kept)) decides per side how many fp16 entries stay and the rest is flushed
    (Sec. 3.3; ratios of Sec. 4.2). Outputs, counters, records and live window tokens against the oracle."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case rpc loop kb={kb} vb={vb} G={G} r={r_k}/{r_v}", flush=True)
    B, Hkv, T0, steps = 2, 2, 200, 75
    q, k, v = synth.gen_layer_numpy(900 + kb, vb, B, Hkv * G, Hkv, T0 + steps)
    rc, gc, shape, cfg = make_ring_pair(B, Hkv * G, Hkv, kb, vb, 288, 256)
    for t in range(T0):
        assert rc.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    kv.append_tokens(shape, cfg, kt[:, :, :T0], vt[:, :, :T0], gc)
    num_k, num_v = kv.rpc_next(r_k, r_v, T0, T0)
    assert (num_k, num_v) == (ref.rpc_next(r_k, T0), ref.rpc_next(r_v, T0))
    assert rc.flush(num_k, num_v) == 0
    kv.flush(shape, cfg, gc, num_k, num_v)
    torch.cuda.synchronize()
    assert_same_state(rc, gc, "after the prompt")
    ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
    out = torch.zeros(B, Hkv * G, 128, dtype=torch.float16, device="cuda")
    seen_unfused = 0
    for s in range(steps):
        t = T0 + s
        qs = np.ascontiguousarray(np.roll(q, s, axis=1))          # a different query each step
        assert rc.append(u16(k[:, :, t]), u16(v[:, :, t])) == 0
        st, want = rc.decode_attn(u16(qs))
        assert st == 0
        seen_unfused += gc.v_lead != 0 and (max(gc.n_q, gc.n_qv) + 31) // 32 * 32 > gc.n
        kv.decode_step(shape, cfg, kt[:, :, t].contiguous(), vt[:, :, t].contiguous(), torch.from_numpy(qs).cuda(), gc, out, ws,
                       n_splits=(0, 1, 2)[s % 3])
        torch.cuda.synchronize()
        assert_attn_close(t16(out), want, f"step {s} (n_q={rc.n_q} n_qv={rc.n_qv} n={rc.n})", tight=True)
        # ageing: the Keys / Values held in fp16 right now are the new one plus those kept so far
        num_k, num_v = kv.rpc_next(r_k, r_v, gc.n - gc.n_q, gc.n - gc.n_qv)
        assert (num_k, num_v) == (ref.rpc_next(r_k, rc.n - rc.n_q), ref.rpc_next(r_v, rc.n - rc.n_qv))
        assert rc.flush(num_k, num_v) == 0
        kv.flush(shape, cfg, gc, num_k, num_v)
        torch.cuda.synchronize()
        assert_same_state(rc, gc, f"after step {s}")
    assert_windows_equal(rc, gc)
    assert seen_unfused > 0          # steps on which the new token shared its tile with the younger front
    assert not ws[: 4 * shape.units].any()


def test_fronts_error_returns():
    import torch
    import paper_2506_08018_amd as kv
    rc, gc, shape, cfg = make_ring_pair(1, 2, 2, 2, 2, 64, 64)
    _, k, v = synth.gen_layer_numpy(5, 0, 1, 2, 2, 64)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    kv.append_tokens(shape, cfg, kt, vt, gc)
    with pytest.raises(kv.KVMixError) as e:                      # ring full
        kv.append(shape, cfg, kt[:, :, 0].contiguous(), vt[:, :, 0].contiguous(), gc)
    assert e.value.status == -4
    with pytest.raises(kv.KVMixError) as e:
        kv.flush(shape, cfg, gc, -1, 0)
    assert e.value.status == -4
    kv.flush(shape, cfg, gc, 64, 3)
    assert (gc.n_q, gc.n_qv, gc.v_lead) == (0, 61, 61)
    q = torch.zeros(1, 2, 128, dtype=torch.float16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(kv.KVMixError) as e:                      # fronts apart: the extra partial needs the workspace
        kv.decode_attn(shape, cfg, q, gc, out, None, n_splits=1)
    assert e.value.status == -1
    fixed = kv.LayerCfg(2, 2, 32)                                # fixed-window ageing needs one front
    with pytest.raises(kv.KVMixError) as e:
        kv.append(shape, fixed, kt[:, :, 0].contiguous(), vt[:, :, 0].contiguous(), gc)
    assert e.value.status == -4
    with pytest.raises(kv.KVMixError) as e:
        kv.rpc_next(1.5, 0.1, 10, 10)
    assert e.value.status == -4
    torch.cuda.synchronize()
