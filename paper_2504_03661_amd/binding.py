"""ctypes binding of libpq_attn.so: argument marshalling only.

Function names and argument order are those of include/pq_attn.h.  Tensor
arguments may be torch tensors (their data_ptr() is passed), raw integer device
addresses, or None for NULL.  Nothing here computes: if the shared library has
not been built the import of this module still works, but the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

PQ_F16, PQ_F32 = 0, 1
PQ_CODES_K, PQ_CODES_V = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpq_attn.so")
_lib = None


class PQAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {pq_status_string(status)} (status {status})")


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "n_subspaces", "n_centroids", "max_context", "max_recent",
        "dtype", "device", "n_splits", "reserved")]


@dataclass
class PQAttnConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    n_subspaces: int = 64
    n_centroids: int = 256
    max_context: int = 0
    max_recent: int = 0
    dtype: int = PQ_F16
    device: int = 0
    n_splits: int = 0
    reserved: int = 0

    def c_struct(self) -> _Config:
        return _Config(*(int(getattr(self, n)) for n, _ in _Config._fields_))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the in-tree library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2504_03661_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    cfgp = ctypes.POINTER(_Config)
    L.pq_attn_validate_config.restype = ctypes.c_int
    L.pq_attn_validate_config.argtypes = [cfgp]
    L.pq_attn_codes_bytes.restype = i64
    L.pq_attn_codes_bytes.argtypes = [cfgp]
    L.pq_attn_create.restype = ctypes.c_int
    L.pq_attn_create.argtypes = [cfgp, ctypes.POINTER(vp)]
    L.pq_attn_destroy.restype = ctypes.c_int
    L.pq_attn_destroy.argtypes = [vp]
    L.pq_attn_n_splits.restype = ctypes.c_int
    L.pq_attn_n_splits.argtypes = [vp]
    L.pq_attn_n_passes.restype = ctypes.c_int
    L.pq_attn_n_passes.argtypes = [vp]
    L.pq_attn_heads_per_workgroup.restype = ctypes.c_int
    L.pq_attn_heads_per_workgroup.argtypes = [vp]
    L.pq_attn_set_codebooks.restype = ctypes.c_int
    L.pq_attn_set_codebooks.argtypes = [vp, vp, vp, vp]
    L.pq_attn_decode.restype = ctypes.c_int
    L.pq_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp]
    L.pq_attn_decode_noalloc.restype = ctypes.c_int
    L.pq_attn_decode_noalloc.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp]
    L.pq_encode_append.restype = ctypes.c_int
    L.pq_encode_append.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    L.pq_pack_codes.restype = ctypes.c_int
    L.pq_pack_codes.argtypes = [vp, i32, vp, i32, vp, vp]
    L.pq_unpack_codes.restype = ctypes.c_int
    L.pq_unpack_codes.argtypes = [vp, i32, vp, i32, vp, vp]
    L.pq_kmeans_workspace_bytes.restype = ctypes.c_int64
    L.pq_kmeans_workspace_bytes.argtypes = [vp]
    L.pq_kmeans_fit.restype = ctypes.c_int
    L.pq_kmeans_fit.argtypes = [vp, vp, i32, vp, i32, vp, ctypes.c_int64, vp]
    L.pq_stream_read_probe.restype = ctypes.c_int
    L.pq_stream_read_probe.argtypes = [vp, vp, ctypes.c_int64, vp]
    L.pq_attn_device_error.restype = ctypes.c_int
    L.pq_attn_device_error.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32)]
    L.pq_status_string.restype = ctypes.c_char_p
    L.pq_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())  # torch tensor


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(status: int, where: str) -> None:
    if status != 0:
        raise PQAttnError(status, where)


def pq_status_string(status: int) -> str:
    return load_library().pq_status_string(int(status)).decode()


def pq_attn_validate_config(cfg: PQAttnConfig) -> int:
    return int(load_library().pq_attn_validate_config(ctypes.byref(cfg.c_struct())))


def pq_attn_codes_bytes(cfg: PQAttnConfig) -> int:
    n = int(load_library().pq_attn_codes_bytes(ctypes.byref(cfg.c_struct())))
    if n < 0:
        raise PQAttnError(n, "pq_attn_codes_bytes")
    return n


def pq_attn_create(cfg: PQAttnConfig) -> int:
    out = ctypes.c_void_p()
    _check(load_library().pq_attn_create(ctypes.byref(cfg.c_struct()), ctypes.byref(out)), "pq_attn_create")
    return out.value


def pq_attn_destroy(ctx: int) -> None:
    _check(load_library().pq_attn_destroy(ctx), "pq_attn_destroy")


def pq_attn_n_splits(ctx: int) -> int:
    return int(load_library().pq_attn_n_splits(ctx))


def pq_attn_n_passes(ctx: int) -> int:
    return int(load_library().pq_attn_n_passes(ctx))


def pq_attn_heads_per_workgroup(ctx: int) -> int:
    return int(load_library().pq_attn_heads_per_workgroup(ctx))


def pq_attn_set_codebooks(ctx, k_codebook, v_codebook, stream=None) -> None:
    _check(load_library().pq_attn_set_codebooks(ctx, _addr(k_codebook), _addr(v_codebook), _stream(stream)),
           "pq_attn_set_codebooks")


def pq_attn_decode(ctx, q, k_codes, v_codes, ctx_len, k_codebook, v_codebook, recent_k, recent_v, recent_len,
                   scale, out, stream=None) -> None:
    _check(load_library().pq_attn_decode(ctx, _addr(q), _addr(k_codes), _addr(v_codes), _addr(ctx_len),
                                         _addr(k_codebook), _addr(v_codebook), _addr(recent_k), _addr(recent_v),
                                         _addr(recent_len), float(scale), _addr(out), _stream(stream)),
           "pq_attn_decode")


def pq_attn_decode_noalloc(cfg: PQAttnConfig, q, k_codes, v_codes, ctx_len, k_codebook, v_codebook, recent_k, recent_v,
                           recent_len, scale, out, stream=None) -> None:
    _check(load_library().pq_attn_decode_noalloc(ctypes.byref(cfg.c_struct()), _addr(q), _addr(k_codes), _addr(v_codes),
                                                 _addr(ctx_len), _addr(k_codebook), _addr(v_codebook), _addr(recent_k),
                                                 _addr(recent_v), _addr(recent_len), float(scale), _addr(out),
                                                 _stream(stream)), "pq_attn_decode_noalloc")


def pq_encode_append(ctx, new_k, new_v, n_new, k_codebook, v_codebook, k_codes, v_codes, ctx_len,
                     stream=None) -> None:
    _check(load_library().pq_encode_append(ctx, _addr(new_k), _addr(new_v), int(n_new), _addr(k_codebook),
                                           _addr(v_codebook), _addr(k_codes), _addr(v_codes), _addr(ctx_len),
                                           _stream(stream)), "pq_encode_append")


def pq_pack_codes(ctx, kind, token_major, n_tokens, packed, stream=None) -> None:
    _check(load_library().pq_pack_codes(ctx, int(kind), _addr(token_major), int(n_tokens), _addr(packed),
                                        _stream(stream)), "pq_pack_codes")


def pq_unpack_codes(ctx, kind, packed, n_tokens, token_major, stream=None) -> None:
    _check(load_library().pq_unpack_codes(ctx, int(kind), _addr(packed), int(n_tokens), _addr(token_major),
                                          _stream(stream)), "pq_unpack_codes")


def pq_kmeans_workspace_bytes(ctx) -> int:
    n = int(load_library().pq_kmeans_workspace_bytes(ctx))
    if n < 0:
        raise PQAttnError(n, "pq_kmeans_workspace_bytes")
    return n


def pq_kmeans_fit(ctx, samples, n_samples, codebook, n_iters, workspace, workspace_bytes, stream=None) -> None:
    _check(load_library().pq_kmeans_fit(ctx, _addr(samples), int(n_samples), _addr(codebook), int(n_iters),
                                        _addr(workspace), int(workspace_bytes), _stream(stream)), "pq_kmeans_fit")


def pq_stream_read_probe(ctx, src, n_bytes, stream=None) -> None:
    _check(load_library().pq_stream_read_probe(ctx, _addr(src), int(n_bytes), _stream(stream)), "pq_stream_read_probe")


def pq_attn_device_error(ctx) -> int:
    flags = ctypes.c_uint32(0)
    _check(load_library().pq_attn_device_error(ctx, ctypes.byref(flags)), "pq_attn_device_error")
    return int(flags.value)
