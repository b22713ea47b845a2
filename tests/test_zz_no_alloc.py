"""GPU check of kvmix_decode_attn_static (the entry point that allocates nothing: split partials in the library's
fixed device array) against kvmix_decode_attn with a caller workspace, on two calls in a row, the second smaller."""
import numpy as np
import pytest

from gpu_common import assert_attn_close, make_pair, run_attn, t16, u16

pytestmark = pytest.mark.gpu


def run_static(gc, shape, cfg, q, n_splits):
    import torch
    import paper_2506_08018_amd as kv
    qt = torch.from_numpy(q).cuda()
    out = torch.zeros_like(qt)
    kv.decode_attn_static(shape, cfg, qt, gc, out, n_splits=n_splits)
    torch.cuda.synchronize()
    return t16(out)


def test_static_scratch_matches_workspace_entry_point():
    import torch
    import paper_2506_08018_amd as kv
    # first call: 4 units x 8 splits x 4 heads; second call right after it: fewer units, fewer splits, shorter context
    for (B, Hkv, G, T, W, kb, vb, ns) in [(2, 2, 4, 32 * 40 + 21, 64, 3, 4, 8), (1, 2, 2, 32 * 9 + 5, 32, 2, 2, 3), (1, 1, 1, 100, 32, 2, 4, 1)]:
        print(f"case static scratch B={B} Hkv={Hkv} G={G} T={T} splits={ns}", flush=True)
        q, k, v, rc, gc, shape, cfg = make_pair(B, Hkv * G, Hkv, T, W, kb, vb, seed=970 + ns)
        want_ws = run_attn(gc, shape, cfg, q, n_splits=ns)          # the existing entry point, caller workspace
        got = run_static(gc, shape, cfg, q, ns)
        assert_attn_close(got, want_ws, f"static vs workspace entry, splits={ns}", tight=True)
        st, want = rc.decode_attn(u16(q))
        assert st == 0
        assert_attn_close(got, want, f"static vs oracle, splits={ns}", tight=True)
        again = run_static(gc, shape, cfg, q, ns)                   # the array's counters were left zero
        assert_attn_close(again, want, f"static second call, splits={ns}", tight=True)


def test_static_scratch_rejects_oversized_requests():
    import torch
    import paper_2506_08018_amd as kv
    # 512 units x 8 splits x 8 heads x 520 B = 17 MB of partials: beyond the fixed array
    shape, cfg = kv.Shape(64, 64, 8), kv.LayerCfg(2, 2, 32)
    gc = kv.LayerCache(shape, cfg, 32 * 64, 64)
    gc.c.n_q = 32 * 64
    q = torch.zeros((64, 64, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(kv.KVMixError) as e:
        kv.decode_attn_static(shape, cfg, q, gc, out, n_splits=8)
    assert e.value.status == -6
    assert not out.any()
