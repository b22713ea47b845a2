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


def header_decode_tile(is_value, bits, words):
    """Decoder written from the layout statement of include/kvmix.h alone (Key / Value code position lines, then the
    1-, 2-, 4- and 3-bit word and bit formulas), independent of the oracle's own unpacking: codes [32][128]."""
    words = [int(w) for w in words]
    codes = np.zeros((32, 128), np.uint8)
    for tau in range(32):
        for d in range(128):
            if not is_value:
                ks, kq, j, hh = d // 32, (d % 32) // 8, (d % 8) // 2, d % 2
                m, i = (tau % 8) // 4, 4 * (tau // 8) + tau % 4
                slot = ks + 4 * m
            else:
                kq, j, hh, i, slot = tau // 8, (tau % 8) // 2, tau % 2, d % 16, d // 16
            l = 16 * kq + i
            plane_bit = 16 * hh + 8 * (j % 2) + 2 * (slot % 4) + slot // 4
            if bits == 1:
                c = (words[2 * l + j // 2] >> plane_bit) & 1
            elif bits == 2:
                c = (words[4 * l + j] >> (16 * hh + 2 * slot)) & 3
            elif bits == 4:
                c = (words[256 * (slot // 4) + 4 * l + j] >> (16 * hh + 4 * (slot % 4))) & 15
            else:
                c = ((words[4 * l + j] >> (16 * hh + 2 * slot)) & 3) + 4 * ((words[256 + 2 * l + j // 2] >> plane_bit) & 1)
            codes[tau, d] = c
    return codes


@pytest.mark.parametrize("kb,vb", [(1, 4), (2, 3), (3, 2), (4, 1)])
def test_records_decode_with_an_independent_reader_of_the_layout_statement(ref, kb, vb):
    """The codes found in a quantized tile record by a decoder that knows only the header's position formulas are
    the group quantizer's codes, for 1 / 2 / 3 / 4 bit and both Key and Value sections: a slot or word swap in the
    oracle's packing that stays bijective would pass the oracle's own pack / unpack identity but not this."""
    from oracle.kvmix_ref import RefCache
    rng = np.random.default_rng(40 + kb * 5 + vb)
    k = (rng.standard_normal((1, 1, 32, 128)) * rng.uniform(0.2, 5.0, (1, 1, 1, 128))).astype(np.float16)
    v = (rng.standard_normal((1, 1, 32, 128)) * rng.uniform(0.2, 5.0, (1, 1, 32, 1))).astype(np.float16)
    c = RefCache(1, 1, 1, kb, vb, 32, 32, 64)
    assert c.quantize_pack(k.view(np.uint16), v.view(np.uint16)) == 0
    rec = c.packed[0, 0]
    kcodes = header_decode_tile(False, kb, rec[256:256 + 128 * kb])
    vcodes = header_decode_tile(True, vb, rec[256 + 128 * kb:])
    for d in range(128):
        codes, _, _ = ref.quantize_group(k[0, 0, :, d].view(np.uint16), kb)
        assert np.array_equal(kcodes[:, d], codes), f"Key channel {d}"
    for tau in range(32):
        for g in range(4):
            codes, _, _ = ref.quantize_group(v[0, 0, tau, 32 * g:32 * g + 32].view(np.uint16), vb)
            assert np.array_equal(vcodes[tau, 32 * g:32 * g + 32], codes), f"Value token {tau} block {g}"
    # and the oracle's own reader agrees with the independent one
    assert np.array_equal(ref.unpack_tile(0, kb, rec[256:256 + 128 * kb]), kcodes)
    assert np.array_equal(ref.unpack_tile(1, vb, rec[256 + 128 * kb:]), vcodes)


def test_three_bit_word_as_the_paper_words_it(ref):
    """Sec. 3.2.2: blocks of 11 per 32-bit integer, ten 3-bit fields and one 2-bit field. The literal form of a
    group (three words) and the bit-plane form in the tile record hold the same 32 codes in the same number of
    bits; the literal word's field places are checked by hand."""
    from oracle.kvmix_ref import RefCache
    # field places: element j of a block at bits [3j, 3j+3), the 11th at bits [30, 32)
    for i in range(32):
        codes = np.zeros(32, np.uint8)
        top = 3 if i in (10, 21) else 7
        codes[i] = top
        w = ref.pack_literal3(codes)
        blk, j = divmod(i, 11)
        want = np.zeros(3, np.uint32)
        want[blk] = top << (3 * j if j < 10 else 30)
        assert np.array_equal(w, want)
    full = ref.pack_literal3(np.array([3 if i in (10, 21) else 7 for i in range(32)], np.uint8))
    assert full[0] == 0xFFFFFFFF and full[1] == 0xFFFFFFFF and full[2] == 0x3FFFFFFF      # 11 + 11 + 10 elements
    # a quantized 3-bit tile: every group's codes survive both forms, and both take 3 words per group
    rng = np.random.default_rng(3)
    k = rng.standard_normal((1, 1, 32, 128)).astype(np.float16)
    v = rng.standard_normal((1, 1, 32, 128)).astype(np.float16)
    c = RefCache(1, 1, 1, 3, 3, 32, 32, 64)
    assert c.quantize_pack(k.view(np.uint16), v.view(np.uint16)) == 0
    kc = ref.unpack_tile(0, 3, c.k_codes[0, 0])
    vc = ref.unpack_tile(1, 3, c.v_codes[0, 0])
    n_words = 0
    for d in range(128):
        codes, _, _ = ref.quantize_group(k[0, 0, :, d].view(np.uint16), 3)
        lit = ref.pack_literal3(codes)
        n_words += lit.size
        assert np.array_equal(ref.unpack_literal3(lit), codes) and np.array_equal(kc[:, d], codes)
    assert n_words == c.k_codes[0, 0].size == 128 * 3
    for tau in range(32):
        for g in range(4):
            codes, _, _ = ref.quantize_group(v[0, 0, tau, 32 * g:32 * g + 32].view(np.uint16), 3)
            assert np.array_equal(ref.unpack_literal3(ref.pack_literal3(codes)), codes)
            assert np.array_equal(vc[tau, 32 * g:32 * g + 32], codes)
