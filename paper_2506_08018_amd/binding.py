"""ctypes marshalling for include/kvmix.h. No arithmetic of the method lives here."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvmix.so")
_lib = None


class KVMixError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "group")]

    def __init__(self, B, Hq, Hkv, D=128, group=32):
        super().__init__(B, Hq, Hkv, D, group)

    @property
    def units(self):
        return self.B * self.Hkv


class LayerCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k_bits", "v_bits", "window")]


class _CacheStruct(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("packed", "k_win", "v_win")] + \
               [(n, C.c_int32) for n in ("T_cap", "W_cap", "n_q", "n_w", "w0", "v_lead")]


def lib():
    """Load libkvmix.so (built in-tree by paper_2506_08018_amd/build.py). Fails loudly when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2506_08018_amd.build` "
                              "(there is no CPU fallback)")
        # PyTorch first: it brings its own copy of the HIP runtime, and the buffers handed to this library are torch's.
        # Loaded the other way round, the library binds to another copy of the runtime, to which torch's pointers
        # mean nothing (every launch then fails with a HIP error).
        import torch  # noqa: F401
        L = C.CDLL(_LIB_PATH)
        P, I, I64, SZ = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
        L.kvmix_version.restype = I
        L.kvmix_strerror.restype = C.c_char_p
        L.kvmix_strerror.argtypes = [I]
        L.kvmix_last_hip_error.restype = I
        L.kvmix_cache_bytes.restype = I
        L.kvmix_cache_bytes.argtypes = [P, P, I, I, P, P]
        L.kvmix_workspace_bytes.restype = I
        L.kvmix_workspace_bytes.argtypes = [P, I, P]
        L.kvmix_quantize_pack.restype = I
        L.kvmix_quantize_pack.argtypes = [P, P, P, P, I64, I64, I64, I, I, P, P]
        L.kvmix_append.restype = I
        L.kvmix_append.argtypes = [P, P, P, P, P, P]
        L.kvmix_append_tokens.restype = I
        L.kvmix_append_tokens.argtypes = [P, P, P, P, I64, I64, I64, I, P, P]
        L.kvmix_decode_attn.restype = I
        L.kvmix_decode_attn.argtypes = [P, P, P, P, C.c_float, P, P, SZ, I, P]
        L.kvmix_decode_attn_static.restype = I
        L.kvmix_decode_attn_static.argtypes = [P, P, P, P, C.c_float, P, I, P]
        L.kvmix_decode_step.restype = I
        L.kvmix_decode_step.argtypes = [P, P, P, P, P, P, C.c_float, P, P, SZ, I, P]
        L.kvmix_stream_read.restype = I
        L.kvmix_stream_read.argtypes = [P, SZ, I, I, P, P]
        L.kvmix_rpc_next.restype = I
        L.kvmix_rpc_next.argtypes = [C.c_double, C.c_double, I, I, P, P]
        L.kvmix_flush.restype = I
        L.kvmix_flush.argtypes = [P, P, P, I, I, P]
        L.kvmix_dequant.restype = I
        L.kvmix_dequant.argtypes = [P, P, P, I, P, P]
        _lib = L
    return _lib


def version():
    return lib().kvmix_version()


def strerror(status):
    return lib().kvmix_strerror(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise KVMixError(status, where)


def _stream(stream=None):
    """hipStream_t of torch's current stream, or of the given torch stream / raw handle."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def cache_bytes(shape, cfg, T_cap, W_cap):
    """-> dict of byte sizes: packed (the tile records), win (each of the two window arrays)."""
    out = [C.c_size_t(0) for _ in range(2)]
    _check(lib().kvmix_cache_bytes(C.byref(shape), C.byref(cfg), T_cap, W_cap, *[C.byref(o) for o in out]), "kvmix_cache_bytes")
    return dict(zip(("packed", "win"), (o.value for o in out)))


def workspace_bytes(shape, T_max):
    n = C.c_size_t(0)
    _check(lib().kvmix_workspace_bytes(C.byref(shape), T_max, C.byref(n)), "kvmix_workspace_bytes")
    return n.value


class LayerCache:
    """One layer's cache: device buffers (torch uint8/int16 tensors) plus the host-side struct."""

    def __init__(self, shape, cfg, T_cap, W_cap, device="cuda"):
        import torch
        self.shape, self.cfg = shape, cfg
        sz = cache_bytes(shape, cfg, T_cap, W_cap)
        z = lambda n: torch.zeros(max(n, 16), dtype=torch.uint8, device=device)
        self.packed = z(sz["packed"])
        self.k_win, self.v_win = z(sz["win"]), z(sz["win"])
        self.c = _CacheStruct(self.packed.data_ptr(), self.k_win.data_ptr(), self.v_win.data_ptr(), T_cap, W_cap, 0, 0, 0, 0)

    v_lead = property(lambda self: self.c.v_lead)
    n_qv = property(lambda self: self.c.n_q + self.c.v_lead)
    n = property(lambda self: self.c.n_q + self.c.n_w)
    n_q = property(lambda self: self.c.n_q)
    n_w = property(lambda self: self.c.n_w)
    w0 = property(lambda self: self.c.w0)
    T_cap = property(lambda self: self.c.T_cap)
    W_cap = property(lambda self: self.c.W_cap)

    def nbytes(self):
        return sum(t.numel() for t in (self.packed, self.k_win, self.v_win))

    def set_window(self, k, v):
        """k, v: fp16 tensors [B][Hkv][n_w][128] (oldest first); plain copies into the ring, start slot 0."""
        import torch
        units, W = self.shape.units, self.c.W_cap
        n = k.shape[2]
        assert n <= W
        kw = self.k_win.view(torch.float16).view(units, W, 128)
        vw = self.v_win.view(torch.float16).view(units, W, 128)
        kw[:, :n, :] = k.reshape(units, n, 128)
        vw[:, :n, :] = v.reshape(units, n, 128)
        self.c.n_w = n
        self.c.w0 = 0


def quantize_pack(shape, cfg, k, v, cache, t0=None):
    """k, v: fp16 CUDA tensors [B][Hkv][n_tokens][128] (last dim contiguous). Writes at token offset t0
    (default n_q) and advances cache.n_q."""
    assert k.dtype == v.dtype and k.element_size() == 2 and k.stride(3) == 1 and v.stride() == k.stride()
    n = k.shape[2]
    if t0 is None:
        t0 = cache.c.n_q
    st = lib().kvmix_quantize_pack(C.byref(shape), C.byref(cfg), k.data_ptr(), v.data_ptr(), k.stride(2), k.stride(1),
                                   k.stride(0), n, t0, C.byref(cache.c), _stream())
    _check(st, "kvmix_quantize_pack")
    cache.c.n_q = max(cache.c.n_q, t0 + n)


def append(shape, cfg, k_new, v_new, cache):
    """k_new, v_new: fp16 CUDA tensors [B][Hkv][128], contiguous."""
    assert k_new.is_contiguous() and v_new.is_contiguous()
    _check(lib().kvmix_append(C.byref(shape), C.byref(cfg), k_new.data_ptr(), v_new.data_ptr(), C.byref(cache.c), _stream()),
           "kvmix_append")


def append_tokens(shape, cfg, k_new, v_new, cache):
    """k_new, v_new: fp16 CUDA tensors [B][Hkv][n][128] (last dim contiguous, any strides otherwise)."""
    assert k_new.element_size() == 2 and k_new.stride(3) == 1 and v_new.stride() == k_new.stride() and v_new.shape == k_new.shape
    st = lib().kvmix_append_tokens(C.byref(shape), C.byref(cfg), k_new.data_ptr(), v_new.data_ptr(), k_new.stride(2),
                                   k_new.stride(1), k_new.stride(0), k_new.shape[2], C.byref(cache.c), _stream())
    _check(st, "kvmix_append_tokens")


def decode_attn(shape, cfg, q, cache, out, workspace=None, softmax_scale=0.0, n_splits=0, stream=None):
    """q, out: fp16 CUDA tensors [B][Hq][128], contiguous. workspace: uint8 CUDA tensor (zeroed once) or None.
    stream: torch stream or raw hipStream_t handle (default: torch's current stream)."""
    assert q.is_contiguous() and out.is_contiguous()
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    st = lib().kvmix_decode_attn(C.byref(shape), C.byref(cfg), q.data_ptr(), C.byref(cache.c), C.c_float(softmax_scale),
                                 out.data_ptr(), wp, wn, n_splits, _stream(stream))
    _check(st, "kvmix_decode_attn")
    return out


def decode_attn_static(shape, cfg, q, cache, out, softmax_scale=0.0, n_splits=0, stream=None):
    """decode_attn without a workspace argument: the split partials live in the library's own fixed device array."""
    assert q.is_contiguous() and out.is_contiguous()
    st = lib().kvmix_decode_attn_static(C.byref(shape), C.byref(cfg), q.data_ptr(), C.byref(cache.c), C.c_float(softmax_scale),
                                        out.data_ptr(), n_splits, _stream(stream))
    _check(st, "kvmix_decode_attn_static")
    return out


def decode_step(shape, cfg, k_new, v_new, q, cache, out, workspace=None, softmax_scale=0.0, n_splits=0, stream=None):
    """append(k_new, v_new) followed by decode_attn(q), in one launch unless the window overflows."""
    assert k_new.is_contiguous() and v_new.is_contiguous() and q.is_contiguous() and out.is_contiguous()
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    st = lib().kvmix_decode_step(C.byref(shape), C.byref(cfg), k_new.data_ptr(), v_new.data_ptr(), q.data_ptr(),
                                 C.byref(cache.c), C.c_float(softmax_scale), out.data_ptr(), wp, wn, n_splits, _stream(stream))
    _check(st, "kvmix_decode_step")
    return out


def rpc_next(r_k, r_v, current_k, current_v):
    """(num_k, num_v) = floor(r * current) for a layer's Keys and Values."""
    nk, nv = C.c_int(0), C.c_int(0)
    _check(lib().kvmix_rpc_next(float(r_k), float(r_v), int(current_k), int(current_v), C.byref(nk), C.byref(nv)), "kvmix_rpc_next")
    return nk.value, nv.value


def flush(shape, cfg, cache, keep_k, keep_v, stream=None):
    """Quantize the Keys / Values that are no longer among the keep_k / keep_v most recent ones."""
    _check(lib().kvmix_flush(C.byref(shape), C.byref(cfg), C.byref(cache.c), int(keep_k), int(keep_v), _stream(stream)), "kvmix_flush")


def stream_read(buf, workgroups, threads=768, nbytes=None, sink=None, stream=None):
    """Load-only pass over the first nbytes (default: all) of the CUDA tensor `buf` in the attention kernel's launch shape."""
    n = buf.numel() * buf.element_size() if nbytes is None else int(nbytes)
    st = lib().kvmix_stream_read(buf.data_ptr(), n, workgroups, threads, sink.data_ptr() if sink is not None else None, _stream(stream))
    _check(st, "kvmix_stream_read")


def dequant(shape, cfg, cache, which, out):
    """out: fp32 CUDA tensor [units][n_q (Keys) or n_q + v_lead (Values)][128]."""
    _check(lib().kvmix_dequant(C.byref(shape), C.byref(cfg), C.byref(cache.c), which, out.data_ptr(), _stream()), "kvmix_dequant")
    return out
