"""Pins against the numbers the paper prints (tests/golden/paper_values.txt, each with its place in the paper)."""
import os

import numpy as np

import kvmix_synth as synth

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_values.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_bit_table_means_round_to_the_paper_s():
    g = golden()
    kb, vb = synth.bit_table(32, synth.BASE_SEED)
    assert round(float(np.mean(kb)), 2) == g["mean_key_bits"] and round(float(np.mean(vb)), 2) == g["mean_value_bits"]
    assert set(np.unique(kb)) <= {2, 3} and set(np.unique(vb)) <= {2, 4}


def test_packed_cache_reaches_the_paper_s_compression(ref):
    """Bytes of the tile records (codes + fp16 scale and minimum per group of 32) against the fp16 cache, at the
    benchmark's bit table: the paper's 4.9x within 2 %."""
    from oracle.kvmix_ref import record_words
    g = golden()
    kb, vb = synth.bit_table(32, synth.BASE_SEED)
    packed = sum(record_words(int(a), int(b)) * 4 for a, b in zip(kb, vb))        # bytes per (unit, 32-token tile), all layers
    fp16 = 32 * 2 * 32 * 128 * 2                                                    # layers x (K, V) x tokens x channels x 2 B
    assert abs(fp16 / packed / g["memory_compression"] - 1.0) < 0.02
    assert int(g["group_size"]) == 32


def test_codes_per_word(ref):
    g = golden()
    for bits, name in ((1, "codes_per_word_1bit"), (2, "codes_per_word_2bit"), (4, "codes_per_word_4bit")):
        assert 32 * 128 // ref.words_per_tile(bits) == int(g[name])
    # 3 bit: the literal word of the oracle holds the paper's 11 codes (a 12th would not fit: 10 x 3 + 2 = 32 bits),
    # and a group of 32 is two such blocks and one of 10, three words in all, also in the tile record's form
    n = int(g["codes_per_word_3bit"])
    codes = np.zeros(32, np.uint8)
    codes[:n] = [7] * (n - 1) + [3]
    w = ref.pack_literal3(codes)
    assert w[0] == 0xFFFFFFFF and w[1] == 0 and w[2] == 0
    assert ref.words_per_tile(3) * 32 // (32 * 128) == 3
