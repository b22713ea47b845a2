"""Seeded synthetic inputs shared by the oracle-side and the HIP-side callers.

Holds none of the method's arithmetic: only random tensors with the structure of the paper's
workloads (Sec. 3.2.1: Key caches carry a few large-magnitude channels; Sec. 4.1/4.2: Llama-2-7B,
Llama-3-8B, Mistral-7B head geometries, group 32, 20 % of the layers at the high bit-width) and
the benchmark configurations. They stand in for caches of the paper's models on LongBench-length
prompts; no model weights or benchmark text are involved.
"""
import numpy as np

BASE_SEED = 2506
# Packed-cache capacity of the benchmark caches beyond the context length T: room for this many generated tokens
# (a multiple of 32). The tile count per unit sets the address stride between units, which the memory system is
# sensitive to (one stride measured 25 % slower than its neighbours); capacity is the caller's choice.
GEN_ROOM = 320
OUTLIER_CHANNELS = 4
OUTLIER_GAIN = 10.0

# The five benchmark workloads (T = context including the token being decoded).
CONFIGS = {
    "cfg1_single_layer": dict(L=1, B=1, Hq=32, Hkv=32, T=1024, W=32, bits="2/2"),
    "cfg2_llama2_7b": dict(L=32, B=8, Hq=32, Hkv=32, T=4096, W=128, bits="table"),
    "cfg3_mistral_7b_gqa": dict(L=32, B=16, Hq=32, Hkv=8, T=8192, W=128, bits="table"),
    "cfg4_llama3_8b_long": dict(L=32, B=1, Hq=32, Hkv=8, T=32768, W=256, bits="table"),
    "cfg5_70b_stress": dict(L=80, B=64, Hq=64, Hkv=8, T=4096, W=128, bits="table"),
}


def bit_table(L, seed=BASE_SEED, k_high=3, v_high=4, low=2, frac=0.2):
    """Per-layer (k_bits, v_bits): a seeded choice of round(frac*L) layers at the high Key
    bit-width and, independently, as many at the high Value bit-width (Sec. 4.2: 3/2-bit Keys,
    4/2-bit Values, 20 % high: means 2.1875 / 2.375 at 32 layers)."""
    rng = np.random.default_rng([seed, 0xB175])
    n_high = int(round(frac * L))
    k = np.full(L, low, np.int32)
    v = np.full(L, low, np.int32)
    k[rng.choice(L, n_high, replace=False)] = k_high
    v[rng.choice(L, n_high, replace=False)] = v_high
    if L == 1:
        k[:] = low
        v[:] = low
    return k, v


def outlier_channels(seed, layer, n_units_heads, D=128):
    """[Hkv][OUTLIER_CHANNELS] distinct channel indices per kv head."""
    rng = np.random.default_rng([seed, layer, 0xC4A7])
    return np.stack([rng.choice(D, OUTLIER_CHANNELS, replace=False) for _ in range(n_units_heads)])


def gen_layer_numpy(seed, layer, B, Hq, Hkv, T, D=128):
    """q [B,Hq,D], K [B,Hkv,T,D], V [B,Hkv,T,D] as fp16 (numpy float16), N(0,1) with the
    seeded outlier Key channels multiplied by OUTLIER_GAIN."""
    rng = np.random.default_rng([seed, layer, 0xDA7A])
    q = rng.standard_normal((B, Hq, D), dtype=np.float32)
    k = rng.standard_normal((B, Hkv, T, D), dtype=np.float32)
    v = rng.standard_normal((B, Hkv, T, D), dtype=np.float32)
    ch = outlier_channels(seed, layer, Hkv, D)
    for j in range(Hkv):
        k[:, j, :, ch[j]] *= OUTLIER_GAIN
    return q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)


def gen_layer_torch(device, seed, layer, B, Hq, Hkv, T, D=128):
    """Same recipe drawn by torch's generator on `device` (a different random stream than the
    numpy one; callers that need the oracle's view copy the tensors to the host)."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + int(layer))
    q = torch.randn((B, Hq, D), generator=g, device=device, dtype=torch.float32).to(torch.float16)
    k = torch.randn((B, Hkv, T, D), generator=g, device=device, dtype=torch.float32)
    v = torch.randn((B, Hkv, T, D), generator=g, device=device, dtype=torch.float32).to(torch.float16)
    ch = torch.as_tensor(outlier_channels(seed, layer, Hkv, D), device=device)
    for j in range(Hkv):
        k[:, j, :, ch[j]] *= OUTLIER_GAIN
    return q, k.to(torch.float16), v


def as_bits(a16):
    """numpy float16 array -> uint16 bit patterns (a view)."""
    return np.ascontiguousarray(a16).view(np.uint16)
