"""ctypes view of the CPU oracle (oracle/kvmix_ref.c) on numpy arrays.

Test infrastructure only: imported by tests/, the smoke check and bench.py's cpu_baseline leg.
It never imports the HIP package.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "group")]


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k_bits", "v_bits", "window")]


class _Cache(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("k_win", C.c_void_p), ("v_win", C.c_void_p)] + \
               [(n, C.c_int32) for n in ("T_cap", "W_cap", "n_q", "n_w", "w0", "v_lead")]


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.kvmix_ref_h2d.restype = C.c_double
        L.kvmix_ref_h2d.argtypes = [C.c_uint16]
        L.kvmix_ref_d2h.restype = C.c_uint16
        L.kvmix_ref_d2h.argtypes = [C.c_double]
        L.kvmix_ref_dequant_elem.restype = C.c_double
        L.kvmix_ref_dequant_elem.argtypes = [C.c_int, C.c_int, C.c_int, C.c_uint16, C.c_uint16]
        L.kvmix_ref_quantize_group.restype = None
        L.kvmix_ref_quantize_group.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvmix_ref_pack_tile.restype = None
        L.kvmix_ref_pack_tile.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.kvmix_ref_unpack_tile.restype = None
        L.kvmix_ref_unpack_tile.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.kvmix_ref_pack_literal3.restype = None
        L.kvmix_ref_pack_literal3.argtypes = [C.c_void_p, C.c_void_p]
        L.kvmix_ref_unpack_literal3.restype = None
        L.kvmix_ref_unpack_literal3.argtypes = [C.c_void_p, C.c_void_p]
        L.kvmix_ref_num_threads.restype = C.c_int
        L.kvmix_ref_set_num_threads.restype = None
        L.kvmix_ref_set_num_threads.argtypes = [C.c_int]
        L.kvmix_ref_record_words.restype = C.c_int
        L.kvmix_ref_record_words.argtypes = [C.c_int, C.c_int]
        L.kvmix_ref_quantize_pack.restype = C.c_int
        L.kvmix_ref_quantize_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                              C.c_int64, C.c_int, C.c_int, C.c_void_p]
        L.kvmix_ref_append.restype = C.c_int
        L.kvmix_ref_append.argtypes = [C.c_void_p] * 5
        L.kvmix_ref_dequant.restype = C.c_int
        L.kvmix_ref_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.kvmix_ref_rpc_next.restype = C.c_int
        L.kvmix_ref_rpc_next.argtypes = [C.c_double, C.c_int]
        L.kvmix_ref_flush.restype = C.c_int
        L.kvmix_ref_flush.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        L.kvmix_ref_decode_attn.restype = C.c_int
        L.kvmix_ref_decode_attn.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().kvmix_ref_num_threads()


def set_num_threads(n: int) -> None:
    lib().kvmix_ref_set_num_threads(int(n))


def h2d(h: int) -> float:
    return lib().kvmix_ref_h2d(int(h))


def d2h(x: float) -> int:
    return lib().kvmix_ref_d2h(float(x))


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def quantize_group(x16, bits):
    """x16: uint16[32] fp16 bit patterns -> (codes uint8[32], scale bits, zero bits)."""
    x16 = np.ascontiguousarray(x16, dtype=np.uint16)
    assert x16.shape == (32,)
    codes = np.zeros(32, np.uint8)
    s = np.zeros(1, np.uint16)
    z = np.zeros(1, np.uint16)
    lib().kvmix_ref_quantize_group(_ptr(x16), int(bits), _ptr(codes), _ptr(s), _ptr(z))
    return codes, int(s[0]), int(z[0])


def dequant_group(codes, bits, scale, zero):
    L = lib()
    return np.array([L.kvmix_ref_dequant_elem(int(c), i, int(bits), int(scale), int(zero)) for i, c in enumerate(codes)])


def words_per_tile(bits: int) -> int:
    return 128 * bits


def pack_tile(which, bits, codes):
    """codes: uint8[32 tokens][128 channels] -> uint32[128*bits] tile words (which: 0 Key, 1 Value)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    assert codes.shape == (32, 128)
    tile = np.zeros(words_per_tile(bits), np.uint32)
    lib().kvmix_ref_pack_tile(int(which), int(bits), _ptr(codes), _ptr(tile))
    return tile


def unpack_tile(which, bits, tile):
    tile = np.ascontiguousarray(tile, dtype=np.uint32)
    assert tile.shape == (words_per_tile(bits),)
    codes = np.zeros((32, 128), np.uint8)
    lib().kvmix_ref_unpack_tile(int(which), int(bits), _ptr(tile), _ptr(codes))
    return codes


def pack_literal3(codes):
    """32 codes of a 3-bit group -> the three 32-bit words of the paper's own wording (blocks of 11)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    assert codes.shape == (32,)
    words = np.zeros(3, np.uint32)
    lib().kvmix_ref_pack_literal3(_ptr(codes), _ptr(words))
    return words


def unpack_literal3(words):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    assert words.shape == (3,)
    codes = np.zeros(32, np.uint8)
    lib().kvmix_ref_unpack_literal3(_ptr(words), _ptr(codes))
    return codes


def rpc_next(r: float, current: int) -> int:
    """num_RPC = floor(r * current_RPC) (Sec. 3.3)."""
    return lib().kvmix_ref_rpc_next(float(r), int(current))


def record_words(k_bits: int, v_bits: int) -> int:
    return lib().kvmix_ref_record_words(int(k_bits), int(v_bits))


def split_records(packed, k_bits, v_bits):
    """Test helper: cut a buffer of tile records, uint32 [units][tiles][record words], into its fields by the
    layout statement (metadata word 4l+f, first value in the low half): returns a dict with k_codes, v_codes
    (uint32 [units][tiles][128*bits]), k_scale, k_zero (uint16 [units][tiles][128], by channel) and v_scale,
    v_zero (uint16 [units][tiles][4][32], by [channel block][token]). Little-endian host."""
    packed = np.ascontiguousarray(packed, dtype=np.uint32)
    units, tiles, rw = packed.shape
    assert rw == 256 + 128 * k_bits + 128 * v_bits
    meta = np.ascontiguousarray(packed[:, :, :256])
    lo = (meta & 0xFFFF).astype(np.uint16).reshape(units, tiles, 64, 4)     # first value of word 4l+f
    hi = (meta >> 16).astype(np.uint16).reshape(units, tiles, 64, 4)        # second value
    pair = np.stack([lo, hi], axis=-1)                                      # [u][t][l][f][first/second]
    out = {"k_codes": packed[:, :, 256:256 + 128 * k_bits], "v_codes": packed[:, :, 256 + 128 * k_bits:]}
    for f, name in enumerate(("k_scale", "k_zero")):
        out[name] = pair[:, :, :, f, :].reshape(units, tiles, 128)          # channel 2l + second
    for f, name in enumerate(("v_scale", "v_zero")):
        out[name] = pair[:, :, :, 2 + f, :].reshape(units, tiles, 4, 32)    # l = 16g + tau/2, tau = 2(l%16) + second
    return out


class RefCache:
    """One layer's cache in host memory, driven through the oracle's cache-level calls."""

    def __init__(self, B, Hq, Hkv, k_bits, v_bits, window, T_cap, W_cap, D=128, group=32):
        self.shape = _Shape(B, Hq, Hkv, D, group)
        self.cfg = _Cfg(k_bits, v_bits, window)
        self.units = B * Hkv
        tiles = T_cap // 32
        kb = k_bits if k_bits != 16 else 2
        vb = v_bits if v_bits != 16 else 2
        self.kb, self.vb = kb, vb
        self.packed = np.zeros((self.units, tiles, record_words(kb, vb)), np.uint32)
        self.k_win = np.zeros((self.units, W_cap, 128), np.uint16)
        self.v_win = np.zeros((self.units, W_cap, 128), np.uint16)
        self.c = _Cache(_ptr(self.packed).value, _ptr(self.k_win).value, _ptr(self.v_win).value, T_cap, W_cap, 0, 0, 0, 0)

    def fields(self):
        """The record buffer cut into codes / scales / minima (copies), see split_records."""
        return split_records(self.packed, self.kb, self.vb)

    k_codes = property(lambda self: self.fields()["k_codes"])
    v_codes = property(lambda self: self.fields()["v_codes"])
    k_scale = property(lambda self: self.fields()["k_scale"])
    k_zero = property(lambda self: self.fields()["k_zero"])
    v_scale = property(lambda self: self.fields()["v_scale"])
    v_zero = property(lambda self: self.fields()["v_zero"])

    # counters live in the C struct
    n_q = property(lambda self: self.c.n_q)
    n_w = property(lambda self: self.c.n_w)
    w0 = property(lambda self: self.c.w0)
    v_lead = property(lambda self: self.c.v_lead)
    n_qv = property(lambda self: self.c.n_q + self.c.v_lead)       # packed Value tokens
    n = property(lambda self: self.c.n_q + self.c.n_w)             # tokens of the sequence

    def flush(self, keep_k, keep_v):
        """Age the cache: at most the keep_k / keep_v most recent Keys / Values stay fp16 (Keys in steps of 32)."""
        return lib().kvmix_ref_flush(C.byref(self.shape), C.byref(self.cfg), C.byref(self.c), int(keep_k), int(keep_v))

    def quantize_pack(self, k, v, t0=None):
        """k, v: uint16 [B][Hkv][n_tokens][128] contiguous. Appends at t0 (default n_q) and advances n_q."""
        k = np.ascontiguousarray(k, dtype=np.uint16)
        v = np.ascontiguousarray(v, dtype=np.uint16)
        B, Hkv, n, D = k.shape
        assert v.shape == k.shape and B * Hkv == self.units and D == 128
        if t0 is None:
            t0 = self.c.n_q
        st = lib().kvmix_ref_quantize_pack(C.byref(self.shape), C.byref(self.cfg), _ptr(k), _ptr(v), D, n * D,
                                           Hkv * n * D, n, t0, C.byref(self.c))
        if st == 0:
            self.c.n_q = max(self.c.n_q, t0 + n)
        return st

    def set_window(self, k, v):
        """k, v: uint16 [B][Hkv][n_w][128]: the window tokens, oldest first (ring start reset to 0)."""
        n = k.shape[2]
        k = np.asarray(k, dtype=np.uint16).reshape(self.units, n, 128)
        v = np.asarray(v, dtype=np.uint16).reshape(self.units, n, 128)
        assert n <= self.c.W_cap
        self.k_win[:, :n, :] = k
        self.v_win[:, :n, :] = v
        self.c.n_w = n
        self.c.w0 = 0

    def append(self, k_new, v_new):
        k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
        v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
        assert k_new.size == self.units * 128 and v_new.size == self.units * 128
        return lib().kvmix_ref_append(C.byref(self.shape), C.byref(self.cfg), _ptr(k_new), _ptr(v_new), C.byref(self.c))

    def dequant(self, which):
        out = np.zeros((self.units, self.c.n_q + (self.c.v_lead if which else 0), 128), np.float64)
        st = lib().kvmix_ref_dequant(C.byref(self.shape), C.byref(self.cfg), C.byref(self.c), int(which), _ptr(out))
        assert st == 0, st
        return out

    def decode_attn(self, q, softmax_scale=0.0):
        """q: uint16 [B][Hq][128] -> (status, out uint16 [B][Hq][128])."""
        q = np.ascontiguousarray(q, dtype=np.uint16)
        out = np.zeros((self.shape.B, self.shape.Hq, 128), np.uint16)
        st = lib().kvmix_ref_decode_attn(C.byref(self.shape), C.byref(self.cfg), _ptr(q), C.byref(self.c),
                                         C.c_float(softmax_scale), _ptr(out))
        return st, out
