"""ctypes front end of the CPU oracle (oracle/pq_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the GPU library never does.

Inputs are the logical numpy tensors of the problem statement (Eq. 5-6): the
query, token-major uint8 codes, per-head codebooks, the recent full-precision
window, the scale.  Floating inputs of any width are widened (exactly) to
float64 before the C code sees them; the scale is the fp32 number the GPU gets,
widened.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        i32, i64, dbl, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        L.oracle_pq_decode.restype = ctypes.c_int
        L.oracle_pq_decode.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, i64, vp,
                                       dbl, vp, i64, vp, vp]
        L.oracle_pq_encode.restype = ctypes.c_int
        L.oracle_pq_encode.argtypes = [i32, i32, i32, i32, i32, i64, vp, vp, vp]
        L.oracle_pq_dequantize.restype = None
        L.oracle_pq_dequantize.argtypes = [vp, vp, i64, i32, i32, i32, vp]
        L.oracle_dense_attention.restype = None
        L.oracle_dense_attention.argtypes = [vp, vp, vp, i64, i32, dbl, vp, vp]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.restype = None
        L.oracle_set_num_threads.argtypes = [i32]
        # the same routines for 16-bit centroid indices (more than 256 centroids per subspace)
        for name in ("oracle_pq_decode", "oracle_pq_encode", "oracle_pq_dequantize"):
            wide = getattr(L, name + "_u16")
            wide.restype = getattr(L, name).restype
            wide.argtypes = getattr(L, name).argtypes
        _lib = L
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _code_width(n_centroids: int):
    """(numpy dtype of a centroid index, suffix of the C routine) for a codebook of this size."""
    assert 1 <= n_centroids <= 65536
    return (np.uint8, "") if n_centroids <= 256 else (np.uint16, "_u16")


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for later calls (timing the oracle on one core); n <= 0 restores one thread per processor."""
    lib().oracle_set_num_threads(int(n))


def dequantize(codes: np.ndarray, codebook: np.ndarray) -> np.ndarray:
    """Eq. 5 for one head: codes [n, M] (uint8, or uint16 for more than 256 centroids), codebook [M, C, ds]
    -> [n, M*ds] float64."""
    cb = _f64(codebook)
    _, C, ds = cb.shape
    code_t, suffix = _code_width(C)
    assert int(np.max(codes, initial=0)) < C
    codes = np.ascontiguousarray(codes, dtype=code_t)
    n, M = codes.shape
    out = np.empty((n, M * ds), dtype=np.float64)
    getattr(lib(), "oracle_pq_dequantize" + suffix)(_ptr(codes), _ptr(cb), n, M, C, ds, _ptr(out))
    return out


def dense_attention(q, keys, values, scale) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 for one query row.  Returns (out [d], softmax weights [n])."""
    q, keys, values = _f64(q), _f64(keys), _f64(values)
    n, d = keys.shape
    out = np.empty((d,), dtype=np.float64)
    w = np.empty((n,), dtype=np.float64)
    lib().oracle_dense_attention(_ptr(q), _ptr(keys), _ptr(values), n, d, float(np.float32(scale)), _ptr(out),
                                 _ptr(w))
    return out, w


def decode(q, k_codes, v_codes, ctx_len, k_codebook, v_codebook, recent_k=None, recent_v=None, recent_len=None,
           scale=None, pairs: Optional[Sequence[Tuple[int, int]]] = None, return_weight_sum: bool = False):
    """Eq. 6 for every (sequence, query head), or only for `pairs` [(b, hq), ...].

    Returns out [B, Hq, d] float64 (rows outside `pairs` are NaN), and with
    return_weight_sum also the [B, Hq] sums of the softmax weights.
    """
    qd = _f64(q)
    B, Hq, d = qd.shape
    kcb, vcb = _f64(k_codebook), _f64(v_codebook)
    C, ds = kcb.shape[2], kcb.shape[3]
    code_t, suffix = _code_width(C)
    if C < np.iinfo(code_t).max + 1:
        assert int(np.max(k_codes, initial=0)) < C and int(np.max(v_codes, initial=0)) < C
    k_codes = np.ascontiguousarray(k_codes, dtype=code_t)
    v_codes = np.ascontiguousarray(v_codes, dtype=code_t)
    _, Hkv, ctx_cap, M = k_codes.shape
    assert v_codes.shape == k_codes.shape
    assert kcb.shape == vcb.shape and kcb.shape[0] == Hkv and kcb.shape[1] == M
    assert M * ds == d
    cl = np.ascontiguousarray(ctx_len, dtype=np.int32)
    assert cl.shape == (B,) and (cl >= 0).all() and (cl <= ctx_cap).all()
    rk = rv = rl = None
    rec_cap = 0
    if recent_k is not None:
        rl = np.ascontiguousarray(recent_len, dtype=np.int32)
        rec_cap = recent_k.shape[2]
        assert (rl >= 0).all() and (rl <= rec_cap).all()
        # rows beyond recent_len are not part of the window; they may hold NaN
        rk, rv = _f64(recent_k), _f64(recent_v)
        assert rk.shape == (B, Hkv, rec_cap, d) and rv.shape == rk.shape
    if scale is None:
        scale = np.float32(1.0 / np.sqrt(np.float64(d)))
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    wsum = np.full((B, Hq), np.nan, dtype=np.float64)
    pr = None
    n_pairs = 0
    if pairs is not None:
        # each listed row is computed by one thread: a pair listed twice would be written by two
        pr = np.ascontiguousarray(np.unique(np.asarray(pairs, dtype=np.int32).reshape(-1, 2), axis=0))
        n_pairs = pr.shape[0]
        assert (pr[:, 0] >= 0).all() and (pr[:, 0] < B).all() and (pr[:, 1] >= 0).all() and (pr[:, 1] < Hq).all()
    rc = getattr(lib(), "oracle_pq_decode" + suffix)(B, Hq, Hkv, d, M, C, _ptr(qd), _ptr(k_codes), _ptr(v_codes), ctx_cap, _ptr(cl),
                                _ptr(kcb), _ptr(vcb), _ptr(rk), _ptr(rv), rec_cap, _ptr(rl),
                                float(np.float32(scale)), _ptr(pr), n_pairs, _ptr(out), _ptr(wsum))
    if rc != 0:
        raise RuntimeError("oracle_pq_decode failed (shape error or out of memory)")
    return (out, wsum) if return_weight_sum else out


def encode(x, codebook) -> np.ndarray:
    """Eq. 4: x [B, Hkv, n, d], codebook [Hkv, M, C, ds] -> codes [B, Hkv, n, M] (uint8; uint16 when C > 256)."""
    xd, cb = _f64(x), _f64(codebook)
    B, Hkv, n, d = xd.shape
    _, M, C, ds = cb.shape
    assert cb.shape[0] == Hkv and M * ds == d
    code_t, suffix = _code_width(C)
    codes = np.empty((B, Hkv, n, M), dtype=code_t)
    rc = getattr(lib(), "oracle_pq_encode" + suffix)(B, Hkv, d, M, C, n, _ptr(xd), _ptr(cb), _ptr(codes))
    if rc != 0:
        raise RuntimeError("oracle_pq_encode failed (shape error)")
    return codes
