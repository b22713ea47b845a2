"""Pins of the packed-tile encoding: density from the paper (Sec. 3.2.2 step 4 and the 3-bit
block of 11), bijectivity, and the pack/unpack identity."""
import numpy as np
import pytest

BITS = [1, 2, 3, 4]


@pytest.mark.parametrize("bits", BITS)
def test_density(ref, bits):
    # 32/bit elements per 32-bit word for 2 and 4 bit; 3 words per group of 32 for 3 bit
    # (blocks of 11 = 10 x 3 bit + 1 x 2 bit = 32 bits; 11 + 11 + 10 elements)
    words = ref.words_per_tile(bits)
    n_groups = 128  # 32 x 128 codes / 32
    assert words == n_groups * {1: 1, 2: 2, 3: 3, 4: 4}[bits]   # 1, 2, 4 bit: 32 / bit codes per word
    if bits in (2, 4):
        assert 32 * 128 // words == 32 // bits
    assert 10 * 3 + 2 == 32 and 11 + 11 + 10 == 32


@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("bits", BITS)
def test_bijection(ref, which, bits):
    """Every code owns its own bits: one-hot tiles light pairwise-disjoint bit sets whose union is
    the whole tile (minus the unused bits of 3-bit groups)."""
    qm = 2 ** bits - 1
    seen = np.zeros(ref.words_per_tile(bits), np.uint32)
    rng = np.random.default_rng(5)
    picks = set((int(t), int(d)) for t, d in zip(rng.integers(0, 32, 400), rng.integers(0, 128, 400)))
    picks |= {(0, 0), (31, 127), (10, 5), (21, 77), (5, 10), (7, 21), (9, 42)}
    for (t, d) in picks:
        c = np.zeros((32, 128), np.uint8)
        c[t, d] = qm
        tile = ref.pack_tile(which, bits, c)
        assert bin(int.from_bytes(tile.tobytes(), "little")).count("1") == bits
        assert not np.any(seen & tile)
        seen |= tile
    full = ref.pack_tile(which, bits, np.full((32, 128), qm, np.uint8))
    nbits = bin(int.from_bytes(full.tobytes(), "little")).count("1")
    assert nbits == 32 * 128 * bits
    assert not np.any(seen & ~full)


@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("bits", BITS)
def test_pack_unpack_identity(ref, which, bits):
    rng = np.random.default_rng(bits * 2 + which)
    for _ in range(5):
        c = rng.integers(0, 2 ** bits, (32, 128)).astype(np.uint8)
        tile = ref.pack_tile(which, bits, c)
        assert np.array_equal(ref.unpack_tile(which, bits, tile), c)


def test_three_bit_unused_bits_zero_after_quantize(ref):
    """After the quantizer, the two 2-bit elements of each 3-bit group leave their third bit
    unused: exactly 2 of 96 bits per group stay zero even for saturated inputs."""
    from oracle.kvmix_ref import RefCache
    rng = np.random.default_rng(0)
    k = rng.standard_normal((1, 1, 32, 128)).astype(np.float16)
    v = rng.standard_normal((1, 1, 32, 128)).astype(np.float16)
    c = RefCache(1, 1, 1, 3, 3, 32, 32, 64)
    assert c.quantize_pack(k.view(np.uint16), v.view(np.uint16)) == 0
    kc = ref.unpack_tile(0, 3, c.k_codes[0, 0])
    vc = ref.unpack_tile(1, 3, c.v_codes[0, 0])
    assert kc[[10, 21], :].max() <= 3 and kc.max() == 7     # Key groups run along tokens
    assert vc[:, [10, 21, 42, 53, 74, 85, 106, 117]].max() <= 3 and vc.max() == 7  # Value groups along channels


@pytest.mark.parametrize("kb,vb", [(2, 2), (3, 4), (4, 3)])
def test_tile_record_places_every_group(ref, kb, vb):
    """The tile record written by the cache-level quantize-pack holds, at the places the layout statement
    names (metadata word 4l+f, code sections after the 256 metadata words), exactly what the group
    quantizer returns for each Key group (one channel, 32 tokens) and Value group (one token, 32 channels)."""
    from oracle.kvmix_ref import RefCache, record_words
    rng = np.random.default_rng(kb * 10 + vb)
    k = (rng.standard_normal((1, 2, 64, 128)) * rng.uniform(0.2, 5.0, (1, 2, 1, 128))).astype(np.float16)
    v = (rng.standard_normal((1, 2, 64, 128)) * rng.uniform(0.2, 5.0, (1, 2, 64, 1))).astype(np.float16)
    c = RefCache(1, 2, 2, kb, vb, 32, 96, 64)
    assert c.quantize_pack(k.view(np.uint16), v.view(np.uint16)) == 0
    assert record_words(kb, vb) == 256 + 128 * kb + 128 * vb and c.packed.shape == (2, 3, record_words(kb, vb))
    assert not c.packed[:, 2].any()                       # the unused third tile stays zero
    for u in range(2):
        for t in range(2):
            rec = c.packed[u, t]
            meta16 = rec[:256].view(np.uint16)            # little-endian: low half first
            kcodes = ref.unpack_tile(0, kb, rec[256:256 + 128 * kb])
            vcodes = ref.unpack_tile(1, vb, rec[256 + 128 * kb:])
            for d in range(128):
                codes, s, z = ref.quantize_group(k[0, u, 32 * t:32 * t + 32, d].view(np.uint16), kb)
                l = d // 2
                assert meta16[2 * (4 * l + 0) + d % 2] == s and meta16[2 * (4 * l + 1) + d % 2] == z
                assert np.array_equal(kcodes[:, d], codes)
            for tau in range(32):
                for g in range(4):
                    codes, s, z = ref.quantize_group(v[0, u, 32 * t + tau, 32 * g:32 * g + 32].view(np.uint16), vb)
                    l = 16 * g + tau // 2
                    assert meta16[2 * (4 * l + 2) + tau % 2] == s and meta16[2 * (4 * l + 3) + tau % 2] == z
                    assert np.array_equal(vcodes[tau, 32 * g:32 * g + 32], codes)
    f = c.fields()                                         # the test helper agrees with the same statement
    assert f["k_scale"][1, 0, 77] == c.packed[1, 0, 4 * 38].item() >> 16
    assert f["v_zero"][0, 1, 2, 9] == c.packed[0, 1, 4 * (32 + 4) + 3].item() >> 16
