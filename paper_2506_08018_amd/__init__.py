"""KVmix hot path on MI355X: thin Python binding over the C-ABI library libkvmix.so.

Every step of the path runs in the HIP kernels of csrc/; this package only marshals arguments.
PyTorch is used for device memory and streams.
"""
from .binding import (KVMixError, LayerCache, LayerCfg, Shape, append, append_tokens, cache_bytes, decode_attn, decode_attn_static, decode_step, dequant, flush, lib,
                      quantize_pack, rpc_next, stream_read, strerror, version, workspace_bytes)

__all__ = ["KVMixError", "LayerCache", "LayerCfg", "Shape", "append", "append_tokens", "cache_bytes", "decode_attn", "decode_attn_static", "decode_step", "dequant", "flush", "lib",
           "quantize_pack", "rpc_next", "stream_read", "strerror", "version", "workspace_bytes"]
