"""Seeded synthetic inputs for PQ decode attention and PQ encode.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no distances, no tables, no softmax, no packing).  Both the
CPU oracle's tests and the GPU library's tests / benchmark draw their inputs
here so that the two sides see identical bits.

All tensors are numpy arrays in the *logical* layouts of the problem statement:

    q            [B, Hq, d]                 dtype
    k_codebook   [Hkv, M, C, ds]            dtype   (ds = d / M; C = 256, or 4096 for the 12-bit setting)
    v_codebook   [Hkv, M, C, ds]            dtype
    k_codes      [B, Hkv, ctx_cap, M]       uint8   (token-major; uint16 when C = 4096)
    v_codes      [B, Hkv, ctx_cap, M]       uint8
    ctx_len      [B]                        int32
    recent_k/v   [B, Hkv, rec_cap, d]       dtype   (rows >= recent_len[b] are NaN)
    recent_len   [B]                        int32
    new_k/new_v  [B, Hkv, n_new, d]         dtype   (only when n_new > 0)

The inputs stand in for the KV activations of the paper's models (32 heads of
128 dims, 1K-128K contexts, Table I / Table IV); those need trained weights and
datasets which are not available, so only their shapes are reproduced.

Draw order is fixed (q, K codebook, V codebook, K codes, V codes, recent_len,
recent K, recent V, new K, new V) on one counter-based Philox stream, so a
(spec, seed) pair names the data exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 250403661
N_CENTROIDS = 256


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_subspaces: int
    context: int                 # quantized tokens per sequence after any append
    dtype: str                   # "f16" | "f32"
    recent_cap: int = 0          # rows allocated for the recent window
    recent_fixed: Optional[int] = None   # every sequence has this many rows ...
    recent_uniform: bool = False         # ... or uniform in [0, recent_cap)
    outlier_frac: float = 0.0    # fraction of centroid coordinates scaled up
    outlier_scale: float = 1.0
    n_new: int = 0               # tokens appended per step through encode
    seed: int = BASE_SEED
    ctx_lens: Optional[tuple] = None     # explicit per-sequence lengths (tests)
    n_centroids: int = N_CENTROIDS       # 256 (8-bit codes) or 4096 (12-bit codes, held in uint16)

    @property
    def sub_dim(self) -> int:
        return self.head_dim // self.n_subspaces

    @property
    def np_dtype(self):
        return np.float16 if self.dtype == "f16" else np.float32


def config(index: int) -> Workload:
    """The five named workloads (index 0..4)."""
    s = BASE_SEED + index
    if index == 0:
        return Workload("cfg0_tiny", 1, 1, 1, 128, 64, 1024, "f32", seed=s)
    if index == 1:
        return Workload("cfg1_llama2_7b_32k", 1, 32, 32, 128, 64, 32768, "f16",
                        recent_cap=128, recent_fixed=128, seed=s)
    if index == 2:
        return Workload("cfg2_batched_8x32k", 8, 32, 32, 128, 64, 32768, "f16",
                        recent_cap=256, recent_uniform=True, seed=s)
    if index == 3:
        return Workload("cfg3_gqa_128k", 1, 32, 8, 128, 64, 131072, "f16",
                        recent_cap=128, recent_fixed=128,
                        outlier_frac=0.02, outlier_scale=20.0, seed=s)
    if index == 4:
        return Workload("cfg4_2bit_encode_16x64k", 16, 32, 32, 128, 32, 65536, "f16",
                        n_new=64, seed=s)
    raise ValueError("config index must be 0..4")


def scaled(w: Workload, **changes) -> Workload:
    """A copy of `w` with some fields changed (smaller context, batch, ...)."""
    return replace(w, **changes)


def _normal(rng, shape, np_dtype):
    # drawn in fp32, rounded to nearest into the storage type
    return rng.standard_normal(shape, dtype=np.float32).astype(np_dtype)


def generate(w: Workload, ctx_cap: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw every tensor of workload `w`.

    With n_new > 0 the cache holds `context - n_new` tokens per sequence before
    the step; the step appends n_new tokens and then attends over `context`.
    `ctx_cap` (>= context) is the allocated token capacity of the code tensors.
    """
    rng = np.random.Generator(np.random.Philox(w.seed))
    B, Hq, Hkv, d, M = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_subspaces
    ds = w.sub_dim
    dt = w.np_dtype
    cap = int(ctx_cap) if ctx_cap is not None else w.context
    assert cap >= w.context

    out: Dict[str, np.ndarray] = {}
    out["q"] = _normal(rng, (B, Hq, d), dt)

    def codebook():
        cb = rng.standard_normal((Hkv, M, w.n_centroids, ds), dtype=np.float32)
        if w.outlier_frac > 0.0:
            mask = rng.random((Hkv, M, w.n_centroids, ds)) < w.outlier_frac
            cb = np.where(mask, cb * np.float32(w.outlier_scale), cb)
        return cb.astype(dt)

    out["k_codebook"] = codebook()
    out["v_codebook"] = codebook()

    def codes():
        return rng.integers(0, w.n_centroids, size=(B, Hkv, cap, M),
                            dtype=np.uint8 if w.n_centroids <= 256 else np.uint16)

    out["k_codes"] = codes()
    out["v_codes"] = codes()

    if w.ctx_lens is not None:
        lens = np.asarray(w.ctx_lens, dtype=np.int32)
        assert lens.shape == (B,) and lens.max(initial=0) <= cap
    else:
        lens = np.full((B,), w.context - w.n_new, dtype=np.int32)
    out["ctx_len"] = lens

    if w.recent_cap > 0:
        if w.recent_uniform:
            rl = rng.integers(0, w.recent_cap, size=(B,), dtype=np.int32)
        else:
            rl = np.full((B,), w.recent_fixed if w.recent_fixed is not None else w.recent_cap,
                         dtype=np.int32)
        rk = _normal(rng, (B, Hkv, w.recent_cap, d), dt)
        rv = _normal(rng, (B, Hkv, w.recent_cap, d), dt)
        # rows that are not part of the window are poisoned: reading one is a bug
        for b in range(B):
            rk[b, :, rl[b]:, :] = np.nan
            rv[b, :, rl[b]:, :] = np.nan
        out["recent_len"], out["recent_k"], out["recent_v"] = rl, rk, rv
    else:
        out["recent_len"] = np.zeros((B,), dtype=np.int32)
        out["recent_k"] = None
        out["recent_v"] = None

    if w.n_new > 0:
        out["new_k"] = _normal(rng, (B, Hkv, w.n_new, d), dt)
        out["new_v"] = _normal(rng, (B, Hkv, w.n_new, d), dt)
    return out


def attention_scale(w: Workload) -> np.float32:
    """1/sqrt(d_k) as the fp32 number both sides receive."""
    return np.float32(1.0 / np.sqrt(np.float64(w.head_dim)))


def training_samples(n_kv_heads: int, n_samples: int, head_dim: int = 128, n_subspaces: int = 64, seed: int = 0,
                     duplicate_init: int = 0, n_centroids: int = N_CENTROIDS) -> Dict[str, np.ndarray]:
    """Stand-in for the sampled K (or V) activations that the offline codebook training clusters
    (Section III-A, "Offline PQ Codebook Training"): per head, `n_samples` fp16 vectors ~ N(0, 1) times a
    per-channel factor drawn log-uniformly in [0.5, 4] (a few channels much larger than the rest, the
    shape the paper's Fig. 2-3 describe).  The initial codebook is the sub-vectors of the head's first
    C = n_centroids samples (centroid c of subspace i = sample c's i-th sub-vector); with `duplicate_init`
    = k the last k initial centroids of every subspace repeat the first k, so that some clusters stay
    empty.

        samples   [Hkv, n_samples, d]      float16
        init      [Hkv, M, C, ds]          float16
    """
    assert n_samples >= n_centroids
    rng = np.random.Generator(np.random.Philox(key=BASE_SEED + 7919 * (seed + 1)))
    ds = head_dim // n_subspaces
    chan = np.exp(rng.uniform(np.log(0.5), np.log(4.0), size=(n_kv_heads, 1, head_dim)))
    x = (rng.standard_normal((n_kv_heads, n_samples, head_dim)) * chan).astype(np.float32).astype(np.float16)
    init = np.ascontiguousarray(
        x[:, :n_centroids].reshape(n_kv_heads, n_centroids, n_subspaces, ds).transpose(0, 2, 1, 3))
    if duplicate_init > 0:
        init[:, :, n_centroids - duplicate_init:] = init[:, :, :duplicate_init]
    return {"samples": x, "init": init}
