"""GPU parity: kvmix_quantize_pack / kvmix_dequant vs the oracle, bit-exact on codes, scales and zero-points."""
import numpy as np
import pytest

import kvmix_synth as synth
from gpu_common import assert_cache_equal, bits_of, make_pair, u16

pytestmark = pytest.mark.gpu

COMBOS = [(kb, vb) for kb in (1, 2, 3, 4) for vb in (1, 2, 3, 4)]      # every pair the launch tables instantiate


@pytest.mark.parametrize("kb,vb", COMBOS)
def test_quantize_pack_bit_exact(kb, vb):
    print(f"case quantize_pack kb={kb} vb={vb}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(2, 4, 2, 32 * 7 + 32, 32, kb, vb, seed=100 + kb * 10 + vb)
    assert gc.n_q == rc.n_q == 32 * 7
    assert_cache_equal(rc, gc)


def adversarial_kv(seed, B, Hkv, T):
    """Groups the quantizer has to get exactly right: constant, two-valued, full fp16 range, subnormal,
    signed zeros, exact ties."""
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((B, Hkv, T, 128)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, T, 128)).astype(np.float32)
    for a in (k, v):
        a[:, :, 0:32, 0:32] = 1.25                                   # constant (both axes)
        a[:, :, 32:64, :] = np.where(rng.random((B, Hkv, 32, 128)) < 0.5, -3.0, 5.0)
        a[:, :, 64:96, 0:64] = rng.choice([-65504.0, 65504.0, 0.0, 1.0], (B, Hkv, 32, 64))
        a[:, :, 64:96, 64:128] = rng.uniform(-6e-5, 6e-5, (B, Hkv, 32, 64))   # fp16 subnormals
        a[:, :, 96:128, :] = rng.integers(0, 16, (B, Hkv, 32, 128)) * 0.5      # many exact ties
        a[:, :, 128:160, :] = np.where(rng.random((B, Hkv, 32, 128)) < 0.5, -0.0, 0.0)
        a[:, :, 128:160, ::7] = 2.0 ** -20
        a[:, :, 160:192, :] *= 1000.0
    return k.astype(np.float16), v.astype(np.float16)


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 3), (4, 4), (1, 1), (1, 4), (3, 1)])   # 1 bit: ranges beyond fp16 store the largest fp16 step
def test_quantize_pack_adversarial_groups(kb, vb):
    print(f"case adversarial kb={kb} vb={vb}", flush=True)
    B, Hkv, T = 1, 2, 256
    k, v = adversarial_kv(7, B, Hkv, T)
    q = np.zeros((B, Hkv, 128), np.float16)
    _, _, _, rc, gc, shape, cfg = make_pair(B, Hkv, Hkv, T + 32, 32, kb, vb, q_k_v=(q, np.concatenate([k, k[:, :, :32]], 2), np.concatenate([v, v[:, :, :32]], 2)))
    assert_cache_equal(rc, gc)


def test_quantize_pack_offsets_and_strides():
    """Writing at a token offset into a larger cache, from a strided (sliced) source."""
    import torch
    import paper_2506_08018_amd as kv
    from oracle.kvmix_ref import RefCache
    B, Hkv, T = 2, 2, 192
    q, k, v = synth.gen_layer_numpy(5, 0, B, Hkv, Hkv, T)
    rc = RefCache(B, Hkv, Hkv, 3, 4, 32, 256, 64)
    shape, cfg = kv.Shape(B, Hkv, Hkv), kv.LayerCfg(3, 4, 32)
    gc = kv.LayerCache(shape, cfg, 256, 64)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    for (a, b_) in ((0, 64), (64, 160), (160, 192)):
        print(f"case offsets chunk {a}:{b_}", flush=True)
        assert rc.quantize_pack(u16(k[:, :, a:b_]), u16(v[:, :, a:b_])) == 0
        kv.quantize_pack(shape, cfg, kt[:, :, a:b_], vt[:, :, a:b_], gc)   # non-contiguous views: strides passed through
    torch.cuda.synchronize()
    assert gc.n_q == rc.n_q == 192
    assert_cache_equal(rc, gc)


@pytest.mark.parametrize("kb,vb", [(2, 4), (3, 2), (4, 3)])
def test_dequant_matches_oracle(kb, vb):
    import torch
    import paper_2506_08018_amd as kv
    print(f"case dequant kb={kb} vb={vb}", flush=True)
    q, k, v, rc, gc, shape, cfg = make_pair(1, 2, 2, 160, 32, kb, vb, seed=9)
    for which in (0, 1):
        out = torch.zeros((shape.units, gc.n_q, 128), dtype=torch.float32, device="cuda")
        kv.dequant(shape, cfg, gc, which, out)
        got = out.cpu().numpy().astype(np.float64)
        want = rc.dequant(which)
        assert np.all(np.abs(got - want) <= 2.0 ** -22 * (np.abs(want) + np.abs(got) + 1e-30) + 2.0 ** -22 * 70.0)


def test_error_returns_launch_nothing():
    import torch
    import paper_2506_08018_amd as kv
    shape, cfg = kv.Shape(1, 2, 2), kv.LayerCfg(2, 2, 32)
    gc = kv.LayerCache(shape, cfg, 64, 64)
    k = torch.zeros((1, 2, 48, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(kv.KVMixError) as e:
        kv.quantize_pack(shape, cfg, k, k, gc)
    assert e.value.status == -4
    k = torch.zeros((1, 2, 96, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(kv.KVMixError) as e:
        kv.quantize_pack(shape, cfg, k, k, gc)
    assert e.value.status == -4
    with pytest.raises(kv.KVMixError) as e:
        kv.quantize_pack(shape, kv.LayerCfg(5, 2, 32), k[:, :, :32], k[:, :, :32], gc)
    assert e.value.status == -2
    with pytest.raises(kv.KVMixError) as e:
        kv.quantize_pack(kv.Shape(1, 2, 2, 64, 32), cfg, k[:, :, :32], k[:, :, :32], gc)
    assert e.value.status == -4
    with pytest.raises(kv.KVMixError) as e:
        kv.quantize_pack(kv.Shape(1, 2, 2, 128, 64), cfg, k[:, :, :32], k[:, :, :32], gc)
    assert e.value.status == -3
    assert gc.n_q == 0 and not bits_of(gc.packed, np.uint32).any()
