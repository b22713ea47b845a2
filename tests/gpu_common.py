"""Helpers for the GPU parity tests: build the same cache on both sides from the same seeded inputs."""
import numpy as np

import kvmix_synth as synth
from oracle.kvmix_ref import RefCache

ATOL = 2e-3   # max-abs bound on fp16 attention outputs (spec tolerance)
RTOL_L2 = 1e-2  # per-row relative L2 bound


def u16(a):
    return np.ascontiguousarray(a).view(np.uint16)


def h2f64(a):
    return np.asarray(a, np.uint16).view(np.float16).astype(np.float64)


def t16(t):
    """torch fp16 tensor -> numpy uint16 bits on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_of(t, dtype):
    """raw uint8 device buffer -> numpy array of `dtype` on the host."""
    return t.cpu().numpy().view(dtype)


def make_pair(B, Hq, Hkv, T, W, kb, vb, seed=0, layer=0, T_cap=None, W_cap=None, q_k_v=None):
    """Seeded inputs; the oldest T - W' tokens packed (W' = W rounded so that n_q % 32 == 0), the rest
    in the window. Returns (q, k, v numpy fp16, RefCache, gpu LayerCache, Shape, LayerCfg)."""
    import torch
    import paper_2506_08018_amd as kv
    q, k, v = q_k_v if q_k_v is not None else synth.gen_layer_numpy(seed, layer, B, Hq, Hkv, T)
    n_q = 0 if kb == 16 else max(0, (T - W) // 32 * 32)
    n_w = T - n_q
    T_cap = T_cap or max(n_q, 32)
    W_cap = W_cap or ((n_w + 63) // 32) * 32
    rc = RefCache(B, Hq, Hkv, kb, vb, W, T_cap, W_cap)
    shape, cfg = kv.Shape(B, Hq, Hkv), kv.LayerCfg(kb, vb, W)
    gc = kv.LayerCache(shape, cfg, T_cap, W_cap)
    kt = torch.from_numpy(k).cuda()
    vt = torch.from_numpy(v).cuda()
    if n_q:
        assert rc.quantize_pack(u16(k[:, :, :n_q]), u16(v[:, :, :n_q])) == 0
        kv.quantize_pack(shape, cfg, kt[:, :, :n_q], vt[:, :, :n_q], gc)
    rc.set_window(u16(k[:, :, n_q:]), u16(v[:, :, n_q:]))
    gc.set_window(kt[:, :, n_q:], vt[:, :, n_q:])
    return q, k, v, rc, gc, shape, cfg


def gpu_fields(gc, rc):
    """The GPU cache's record buffer cut into fields with the layout statement's decoder (on the host)."""
    from oracle.kvmix_ref import split_records
    want = rc.packed
    got = bits_of(gc.packed, np.uint32)[: want.size].reshape(want.shape)
    return got, split_records(got, rc.kb, rc.vb)


def assert_cache_equal(rc, gc, n_tiles=None):
    """Bit-exact comparison of the tile records (codes, scales and minima) of the packed tiles."""
    nt = rc.n_q // 32 if n_tiles is None else n_tiles
    got_packed, got = gpu_fields(gc, rc)
    want = rc.fields()
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero"):   # field by field first: better messages
        g, w = got[name][:, :nt], want[name][:, :nt]
        if not np.array_equal(g, w):
            bad = np.argwhere(g != w)
            raise AssertionError(f"{name}: {len(bad)} mismatching entries, first at {bad[0]}: got {g[tuple(bad[0])]:#x} want {w[tuple(bad[0])]:#x}")
    assert np.array_equal(got_packed[:, :nt], rc.packed[:, :nt]), "tile records differ outside the decoded fields"


def assert_windows_equal(rc, gc):
    """The live tokens of both fp16 ring windows, bit for bit (slots outside the n_w live ones are unspecified: a
    token that is quantized within the call that brought it never has to pass through the ring)."""
    kw, vw = bits_of(gc.k_win, np.uint16).reshape(rc.k_win.shape), bits_of(gc.v_win, np.uint16).reshape(rc.v_win.shape)
    W = rc.k_win.shape[1]
    slots = [(rc.w0 + r) % W for r in range(rc.n_w)]
    assert np.array_equal(kw[:, slots], rc.k_win[:, slots]), "Key window"
    assert np.array_equal(vw[:, slots], rc.v_win[:, slots]), "Value window"


TIGHT_ABS = 1e-4  # accumulation noise floor (fp32 sums, matrix-core product truncation) on top of one fp16 spacing


def assert_attn_close(got_bits, want_bits, what="", tight=False, tight_abs=None):
    """Spec bound (max-abs 2e-3, per-row rel-L2 1e-2). tight=True additionally requires every output
    to be within one fp16 spacing (+ TIGHT_ABS) of the oracle: what fp32 accumulation of well-scaled
    inputs delivers, and what catches a mis-scaled partial sum that the loose bound would let through."""
    got, want = h2f64(got_bits), h2f64(want_bits)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - want)
    if tight:
        big = np.maximum(np.abs(want), np.abs(got))
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(big, 2.0 ** -14))) - 10)
        bad = np.argwhere(err > 1.01 * ulp + (TIGHT_ABS if tight_abs is None else tight_abs))
        assert len(bad) == 0, f"{what}: {len(bad)} outputs off by more than one fp16 spacing, e.g. " + \
            str([(tuple(int(x) for x in i), want[tuple(i)], got[tuple(i)]) for i in bad[:4]])
    rows = want.reshape(-1, want.shape[-1])
    rel = np.linalg.norm((got - want).reshape(rows.shape), axis=1) / np.maximum(np.linalg.norm(rows, axis=1), 1e-30)
    assert err.max() <= ATOL, f"{what}: max abs err {err.max():.3e} > {ATOL}"
    assert rel.max() <= RTOL_L2, f"{what}: max rel-L2 err {rel.max():.3e} > {RTOL_L2}"
    return err.max(), rel.max()


def run_attn(gc, shape, cfg, q, n_splits=0, softmax_scale=0.0):
    import torch
    import paper_2506_08018_amd as kv
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    ws = torch.zeros(kv.workspace_bytes(shape, gc.T_cap), dtype=torch.uint8, device="cuda")
    kv.decode_attn(shape, cfg, qt, gc, out, ws, softmax_scale=softmax_scale, n_splits=n_splits)
    torch.cuda.synchronize()
    assert not ws[: 4 * shape.units * max(1, shape.Hq // shape.Hkv // 8)].any(), "arrival counters not reset"
    return t16(out)
