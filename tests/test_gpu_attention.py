"""GPU parity: kvmix_decode_attn / kvmix_append vs the oracle (max-abs 2e-3, per-row rel-L2 1e-2)."""
import numpy as np
import pytest

import kvmix_synth as synth
from gpu_common import assert_attn_close, assert_cache_equal, assert_windows_equal, bits_of, make_pair, run_attn, t16, u16

pytestmark = pytest.mark.gpu

COMBOS = [(kb, vb) for kb in (1, 2, 3, 4) for vb in (1, 2, 3, 4)]      # every pair the launch tables instantiate


@pytest.mark.parametrize("kb,vb", COMBOS)
@pytest.mark.parametrize("G", [1, 4])
def test_all_bit_combos(kb, vb, G):
    print(f"case attn kb={kb} vb={vb} G={G}", flush=True)
    B, Hkv, T, W = 2, 2, 32 * 9 + 17, 32            # ragged window: n_w = 49
    q, k, v, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T, W, kb, vb, seed=200 + kb * 10 + vb)
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    got = run_attn(gc, shape, cfg, q)
    assert_attn_close(got, want, f"kb={kb} vb={vb} G={G}", tight=True)


@pytest.mark.parametrize("kb,vb", [(1, 1), (1, 3), (4, 1), (2, 1)])
@pytest.mark.parametrize("G,n_splits", [(8, 1), (8, 3), (2, 3), (4, 1)])
def test_one_bit_settings_across_groups_and_splits(kb, vb, G, n_splits):
    print(f"case one-bit kb={kb} vb={vb} G={G} splits={n_splits}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2 * G, 2, 32 * 26 + 11, 32, kb, vb, seed=250 + kb * 10 + vb + G)
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    got = run_attn(gc, shape, cfg, q, n_splits=n_splits)
    assert_attn_close(got, want, f"kb={kb} vb={vb} G={G} splits={n_splits}", tight=True)


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_gqa_groups_and_scale(G):
    print(f"case gqa G={G}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2 * G, 2, 32 * 20 + 40, 32, 2, 4, seed=300 + G)
    for scale in (0.0, 0.05):
        st, want = rc.decode_attn(u16(q), scale)
        got = run_attn(gc, shape, cfg, q, softmax_scale=scale)
        assert_attn_close(got, want, f"G={G} scale={scale}", tight=True)


@pytest.mark.parametrize("n_splits", [1, 2, 3, 5, 8])
def test_result_independent_of_split_count(n_splits):
    print(f"case splits={n_splits}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(2, 8, 2, 32 * 33 + 5, 64, 3, 4, seed=400)
    st, want = rc.decode_attn(u16(q))
    got = run_attn(gc, shape, cfg, q, n_splits=n_splits)
    assert_attn_close(got, want, f"splits={n_splits}", tight=True)
    again = run_attn(gc, shape, cfg, q, n_splits=n_splits)   # counters were reset: second call still right
    assert_attn_close(again, want, f"splits={n_splits} (second call)", tight=True)


@pytest.mark.parametrize("kb,vb,G", [(16, 16, 1), (16, 16, 4), (2, 2, 2)])
def test_window_only_is_exact_fp_attention(kb, vb, G):
    """16-bit setting / window covering the context: no packed tokens at all."""
    print(f"case window-only kb={kb} G={G}", flush=True)
    T = 200
    q, k, v, rc, gc, shape, cfg = make_pair(2, 2 * G, 2, T, 256, kb, vb, seed=500)
    assert gc.n_q == 0 and gc.n_w == T
    st, want = rc.decode_attn(u16(q))
    got = run_attn(gc, shape, cfg, q)
    err, _ = assert_attn_close(got, want, "window-only")
    assert err <= 2.0 ** -10 * np.abs(q).max() * 4   # fp32 accumulation: at most an fp16 ulp or two off


def test_edge_contexts():
    """Single-token context; packed tokens only (empty window); exactly one packed tile."""
    import torch
    print("case single token", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2, 2, 1, 32, 16, 16, seed=600)
    st, want = rc.decode_attn(u16(q))
    got = run_attn(gc, shape, cfg, q)
    assert np.array_equal(got, want) and np.array_equal(got[0], u16(v[0, :, 0]))
    print("case empty window", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 4, 2, 96, 0, 2, 3, seed=601)
    assert gc.n_w == 0 and gc.n_q == 96
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    assert_attn_close(run_attn(gc, shape, cfg, q), want, "empty window")
    print("case one tile", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2, 2, 33, 0, 4, 4, seed=602)
    assert gc.n_q == 32 and gc.n_w == 1
    st, want = rc.decode_attn(u16(q))
    assert_attn_close(run_attn(gc, shape, cfg, q), want, "one tile")


def test_sharp_softmax_and_large_values():
    """(a) queries aligned with one packed / one window key (softmax close to one-hot);
    (b) Values of magnitude ~10, where the fp16 output spacing exceeds the absolute bound."""
    from gpu_common import h2f64
    B, Hkv, G, T, W = 1, 2, 2, 32 * 12 + 32, 32
    print("case sharp softmax", flush=True)
    q, k, v = synth.gen_layer_numpy(700, 0, B, Hkv * G, Hkv, T)
    q[0, 0] = (k[0, 0, 77].astype(np.float32) * 0.4).astype(np.float16)
    q[0, 3] = (k[0, 1, T - 5].astype(np.float32) * 0.4).astype(np.float16)
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T, W, 2, 2, q_k_v=(q, k, v))
    st, want = rc.decode_attn(u16(q))
    assert_attn_close(run_attn(gc, shape, cfg, q), want, "sharp softmax")
    print("case large values", flush=True)
    q, k, v = synth.gen_layer_numpy(701, 0, B, Hkv * G, Hkv, T)
    v = (v.astype(np.float32) * 4.0).astype(np.float16)
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T, W, 2, 2, q_k_v=(q, k, v))
    st, want = rc.decode_attn(u16(q))
    got = run_attn(gc, shape, cfg, q)
    err = np.abs(h2f64(got) - h2f64(want))
    big = np.maximum(np.abs(h2f64(want)), np.abs(h2f64(got)))
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(big, 2.0 ** -14))) - 10)
    # outputs above 2 have an fp16 spacing wider than the absolute bound: allow one spacing there
    bad = np.argwhere(err > np.maximum(2e-3, 1.01 * ulp))
    assert len(bad) == 0, [(tuple(i), h2f64(want)[tuple(i)], h2f64(got)[tuple(i)]) for i in bad[:5]]


@pytest.mark.parametrize("G,kb,vb", [(1, 2, 2), (4, 3, 4), (8, 2, 3)])
def test_stale_ring_slots_and_key_outliers(G, kb, vb):
    """(a) Ring slots outside the live window hold leftovers: NaN patterns in the Key ring, infinities and large
    values in the Value ring. Dead slots are never read, the result does not change, also through fused steps whose
    new token lands on such a slot. (b) Key channel outliers of x100 (group scales in the hundreds, folded into
    fp16 operands)."""
    import torch
    print(f"case stale slots / outliers G={G} kb={kb} vb={vb}", flush=True)
    B, Hkv, T, W = 1, 2, 32 * 14 + 9, 32
    q, k, v = synth.gen_layer_numpy(720 + G, 0, B, Hkv * G, Hkv, T)
    k[:, :, :, 5] *= 10.0          # on top of the generator's x10 channels: up to x100
    k[:, 1, :, 77] *= 100.0
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T, W, kb, vb, W_cap=128, q_k_v=(q, k, v))
    assert gc.n_w == 41 and gc.W_cap == 128
    junk_k = torch.full((shape.units, 128 - 41, 128), float("nan"), dtype=torch.float16, device="cuda")
    junk_v = torch.full((shape.units, 128 - 41, 128), -6.0e4, dtype=torch.float16, device="cuda")
    junk_v[:, ::3] = float("inf")
    gc.k_win.view(torch.float16).view(shape.units, 128, 128)[:, 41:] = junk_k
    gc.v_win.view(torch.float16).view(shape.units, 128, 128)[:, 41:] = junk_v
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    for ns in (1, 2):
        assert_attn_close(run_attn(gc, shape, cfg, q, n_splits=ns), want, f"stale slots G={G} splits={ns}")
    import paper_2506_08018_amd as kv
    kn, vn = synth.gen_layer_numpy(721, 1, B, Hkv, Hkv, 3)[1:]
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
    for s_ in range(3):
        assert rc.append(u16(kn[:, :, s_]), u16(vn[:, :, s_])) == 0
        st, want = rc.decode_attn(u16(q))
        kv.decode_step(shape, cfg, torch.from_numpy(kn[:, :, s_].copy()).cuda(), torch.from_numpy(vn[:, :, s_].copy()).cuda(), qt, gc, out, ws)
        torch.cuda.synchronize()
        assert_attn_close(t16(out), want, f"stale slots G={G} fused step {s_}")


@pytest.mark.parametrize("kb,vb,G", [(2, 2, 1), (3, 4, 4)])
def test_append_and_flush_match_oracle(kb, vb, G):
    """Token-by-token appends through the ring window, flushing 32 aged tokens at a time, on both sides."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case append kb={kb} vb={vb} G={G}", flush=True)
    B, Hkv, W, T0, steps = 2, 2, 32, 96, 75
    q, k, v = synth.gen_layer_numpy(800, 0, B, Hkv * G, Hkv, T0 + steps)
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T0, W, kb, vb, T_cap=256, W_cap=64, q_k_v=(q, k[:, :, :T0], v[:, :, :T0]))
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    for s in range(steps):
        assert rc.append(u16(k[:, :, T0 + s]), u16(v[:, :, T0 + s])) == 0
        kv.append(shape, cfg, kt[:, :, T0 + s].contiguous(), vt[:, :, T0 + s].contiguous(), gc)
        assert (gc.n_q, gc.n_w, gc.w0) == (rc.n_q, rc.n_w, rc.w0)
        if s in (0, 31, 32, 33, 74):
            st, want = rc.decode_attn(u16(q))
            assert_attn_close(run_attn(gc, shape, cfg, q), want, f"after append {s}")
    torch.cuda.synchronize()
    assert_cache_equal(rc, gc)
    assert_windows_equal(rc, gc)


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 4), (16, 16)])
def test_append_tokens_equals_single_appends(kb, vb):
    """Chunks of new tokens (1, 7, 32, 45, 100 at a time, from a strided source) against the oracle's
    token-by-token appends: counters, tile records and both windows bit for bit, attention at the end."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case append_tokens kb={kb} vb={vb}", flush=True)
    B, Hkv, G, W, T0 = 2, 2, 2, 32, 64 + 5
    chunks = [1, 7, 32, 45, 100, 3, 31, 64, 33]
    total = sum(chunks)
    q, k, v = synth.gen_layer_numpy(830, 0, B, Hkv * G, Hkv, T0 + total)
    W_cap = 64 if kb != 16 else 448
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T0, W, kb, vb, T_cap=448, W_cap=W_cap, q_k_v=(q, k[:, :, :T0], v[:, :, :T0]))
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    t = T0
    for n in chunks:
        for i in range(n):
            assert rc.append(u16(k[:, :, t + i]), u16(v[:, :, t + i])) == 0
        kv.append_tokens(shape, cfg, kt[:, :, t:t + n], vt[:, :, t:t + n], gc)      # a view: token stride 128, head stride T*128
        t += n
        assert (gc.n_q, gc.n_w, gc.w0) == (rc.n_q, rc.n_w, rc.w0)
    torch.cuda.synchronize()
    if kb != 16:
        assert_cache_equal(rc, gc)
    assert_windows_equal(rc, gc)
    st, want = rc.decode_attn(u16(q))
    assert_attn_close(run_attn(gc, shape, cfg, q), want, "after chunked appends", tight=True)


@pytest.mark.parametrize("kb,vb,G,n_splits", [(2, 2, 1, 0), (2, 3, 2, 3), (3, 4, 4, 1), (4, 2, 8, 2), (16, 16, 2, 0)])
def test_decode_step_equals_append_then_attention(kb, vb, G, n_splits):
    """The fused step (append inside the attention launch, two launches + attention when the window overflows)
    against the oracle's append followed by its attention, at every step across two flushes; the window
    arrays and the tile records end up identical too."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case decode_step kb={kb} vb={vb} G={G} splits={n_splits}", flush=True)
    B, Hkv, W, T0, steps = 2, 2, 32, 96 + 7, 70
    q, k, v = synth.gen_layer_numpy(810 + G, 0, B, Hkv * G, Hkv, T0 + steps)
    W_cap = 64 if kb != 16 else 192
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T0, W, kb, vb, T_cap=256, W_cap=W_cap, q_k_v=(q, k[:, :, :T0], v[:, :, :T0]))
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    ws = torch.zeros(kv.workspace_bytes(shape, 512), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(5)
    for s in range(steps):
        qs = (q.astype(np.float32) * rng.uniform(0.5, 1.5)).astype(np.float16)      # a fresh query every step
        qt = torch.from_numpy(qs).cuda()
        out = torch.zeros_like(qt)
        assert rc.append(u16(k[:, :, T0 + s]), u16(v[:, :, T0 + s])) == 0
        st, want = rc.decode_attn(u16(qs))
        assert st == 0
        kv.decode_step(shape, cfg, kt[:, :, T0 + s].contiguous(), vt[:, :, T0 + s].contiguous(), qt, gc, out, ws, n_splits=n_splits)
        torch.cuda.synchronize()
        assert (gc.n_q, gc.n_w, gc.w0) == (rc.n_q, rc.n_w, rc.w0)
        assert_attn_close(t16(out), want, f"decode_step {s} (n_q {gc.n_q}, n_w {gc.n_w})", tight=True)
    assert not ws[: 4 * shape.units].any()
    if kb != 16:
        assert_cache_equal(rc, gc)
    assert_windows_equal(rc, gc)


@pytest.mark.parametrize("Hq,Hkv,kb,vb,n_splits", [(72, 1, 2, 2, 0), (16, 1, 3, 4, 2), (64, 2, 2, 4, 1), (24, 1, 4, 3, 3)])
def test_multi_query_and_large_groups(Hq, Hkv, kb, vb, n_splits):
    """Multi-query attention and groups of more than 8 query heads per kv head (a 71-head model with one kv head,
    padded to 72 = 9 blocks of 8): every head block of a unit reads the same packed tiles and window."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case mqa Hq={Hq} Hkv={Hkv} kb={kb} vb={vb} splits={n_splits}", flush=True)
    B, T, W = 2, 32 * 22 + 13, 32
    q, k, v, rc, gc, shape, cfg = make_pair(B, Hq, Hkv, T, W, kb, vb, seed=640 + Hq)
    if Hq == 72:
        q[:, 71] = 0          # the padding head: its output is ignored by a caller, here it is simply a zero query
    st, want = rc.decode_attn(u16(q))
    assert st == 0
    got = run_attn(gc, shape, cfg, q, n_splits=n_splits)
    assert_attn_close(got, want, f"Hq={Hq} Hkv={Hkv}", tight=True)
    # fused step with the append inside, twice
    kn, vn = synth.gen_layer_numpy(641, 1, B, Hkv, Hkv, 2)[1:]
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
    for s in range(2):
        assert rc.append(u16(kn[:, :, s]), u16(vn[:, :, s])) == 0
        st, want = rc.decode_attn(u16(q))
        kv.decode_step(shape, cfg, torch.from_numpy(kn[:, :, s].copy()).cuda(), torch.from_numpy(vn[:, :, s].copy()).cuda(), qt, gc, out, ws, n_splits=n_splits)
        torch.cuda.synchronize()
        assert_attn_close(t16(out), want, f"Hq={Hq} Hkv={Hkv} step {s}", tight=True)
    assert not ws[: 4 * shape.units * max(1, Hq // Hkv // 8)].any()


def test_decode_steps_with_window_length_zero():
    """Window length 0: every 32nd step the appended token is itself among the 32 that are quantized (it never
    passes through the ring); in between the window holds 1..31 tokens."""
    import torch
    import paper_2506_08018_amd as kv
    print("case decode_step window 0", flush=True)
    B, Hkv, G, W, T0, steps, kb, vb = 1, 2, 2, 0, 64 + 30, 40, 2, 3
    q, k, v = synth.gen_layer_numpy(815, 0, B, Hkv * G, Hkv, T0 + steps)
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T0, W, kb, vb, T_cap=160, W_cap=32, q_k_v=(q, k[:, :, :T0], v[:, :, :T0]))
    assert (gc.n_q, gc.n_w) == (64, 30)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    for s in range(steps):
        assert rc.append(u16(k[:, :, T0 + s]), u16(v[:, :, T0 + s])) == 0
        st, want = rc.decode_attn(u16(q))
        assert st == 0
        kv.decode_step(shape, cfg, kt[:, :, T0 + s].contiguous(), vt[:, :, T0 + s].contiguous(), qt, gc, out)
        torch.cuda.synchronize()
        assert (gc.n_q, gc.n_w, gc.w0) == (rc.n_q, rc.n_w, rc.w0)
        assert_attn_close(t16(out), want, f"window 0, step {s} (n_q {gc.n_q}, n_w {gc.n_w})", tight=True)
    assert_cache_equal(rc, gc)
    assert_windows_equal(rc, gc)


@pytest.mark.parametrize("kb,vb,G", [(2, 2, 1), (3, 4, 4), (4, 2, 8)])
def test_many_tiles_per_wave(kb, vb, G):
    """Long context in few workgroups: every wave runs many iterations of its prefetch loop."""
    print(f"case many tiles kb={kb} vb={vb} G={G}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2 * G, 2, 32 * 150 + 77, 128, kb, vb, seed=900 + G)
    st, want = rc.decode_attn(u16(q))
    for ns in (1, 2):
        for rep in range(2):
            assert_attn_close(run_attn(gc, shape, cfg, q, n_splits=ns), want, f"many tiles splits={ns} rep={rep}", tight=True)


def test_config1_full_parity():
    """Benchmark configuration 1 in full: 1 layer, B1, 32 heads, T1024, window 32, K2/V2."""
    print("case config1", flush=True)
    c = synth.CONFIGS["cfg1_single_layer"]
    q, k, v, rc, gc, shape, cfg = make_pair(c["B"], c["Hq"], c["Hkv"], c["T"], c["W"], 2, 2, seed=synth.BASE_SEED)
    assert gc.n_q == 992 and gc.n_w == 32
    assert_cache_equal(rc, gc)
    st, want = rc.decode_attn(u16(q))
    for ns in (0, 1, 4):
        assert_attn_close(run_attn(gc, shape, cfg, q, n_splits=ns), want, f"config1 splits={ns}", tight=True)


def test_attn_error_returns():
    import torch
    import paper_2506_08018_amd as kv
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2, 2, 96, 32, 2, 2, seed=1)
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    with pytest.raises(kv.KVMixError) as e:      # splits > 1 without workspace
        kv.decode_attn(shape, cfg, qt, gc, out, None, n_splits=2)
    assert e.value.status == -1
    small = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(kv.KVMixError) as e:
        kv.decode_attn(shape, cfg, qt, gc, out, small, n_splits=2)
    assert e.value.status == -6
    with pytest.raises(kv.KVMixError) as e:      # G = 3 unsupported
        kv.decode_attn(kv.Shape(1, 6, 2), cfg, qt, gc, out, None)
    assert e.value.status == -4
    with pytest.raises(kv.KVMixError) as e:      # G = 12: above 8 only multiples of 8
        kv.decode_attn(kv.Shape(1, 24, 2), cfg, qt, gc, out, None)
    assert e.value.status == -4
    assert not out.any()


@pytest.mark.parametrize("n_splits", [1, 4])
def test_graph_replays_match_eager(n_splits):
    """kvmix_decode_attn recorded into a HIP graph (it allocates nothing and clears its arrival counters in the
    kernel): every replay, with eager work and synchronizations in between and a new query each time, gives the
    eager result (to the last-bit freedom of the dynamic tile order) and matches the oracle."""
    import torch
    import paper_2506_08018_amd as kv
    print(f"case graph replay splits={n_splits}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(2, 8, 2, 32 * 21 + 9, 64, 3, 2, seed=950)
    ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
    qt = torch.from_numpy(q).cuda()
    out_g = torch.zeros_like(qt)
    out_e = torch.zeros_like(qt)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        kv.decode_attn(shape, cfg, qt, gc, out_g, ws, n_splits=n_splits)      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        kv.decode_attn(shape, cfg, qt, gc, out_g, ws, n_splits=n_splits)
    rng = np.random.default_rng(3)
    for rep in range(4):
        qn = (q.astype(np.float32) * rng.uniform(0.6, 1.4)).astype(np.float16)
        qt.copy_(torch.from_numpy(qn).cuda())                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        kv.decode_attn(shape, cfg, qt, gc, out_e, ws, n_splits=n_splits)
        torch.cuda.synchronize()
        # waves claim tiles dynamically, so the summation order (and the last fp16 bit) may differ between launches
        assert_attn_close(t16(out_g), t16(out_e), f"graph replay {rep} vs eager", tight=True)
        st, want = rc.decode_attn(u16(qn))
        assert_attn_close(t16(out_g), want, f"graph replay {rep}", tight=True)
        assert not ws[: 4 * shape.units].any()
