"""Device-side plumbing shared by the GPU tests, the smoke check and the benchmark.

Uploads a workload (numpy tensors in the logical layouts of the problem statement)
with torch, owns the device buffers, and calls the C ABI through the binding.
torch is used for device memory and streams only; every step of the path runs in
the library's kernels.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as B


def _dev(a: Optional[np.ndarray], device) -> Optional[torch.Tensor]:
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:          # 12-bit codes: the same bits as int16, a dtype every torch build moves
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


class PQSession:
    """One context plus the device tensors of one workload."""

    def __init__(self, data: Dict[str, np.ndarray], n_q_heads: int, dtype: str, max_context: Optional[int] = None,
                 n_splits: int = 0, device: int = 0, code_copies: int = 1, register_codebooks: bool = True):
        if not torch.cuda.is_available():
            raise RuntimeError("PQSession needs a GPU: the library has no CPU path")
        self.device = torch.device("cuda", device)
        k_codes = data["k_codes"]
        Bn, Hkv, n_tok, M = k_codes.shape
        d = data["q"].shape[-1]
        self.B, self.Hq, self.Hkv, self.d, self.M = Bn, n_q_heads, Hkv, d, M
        self.dtype = dtype
        rk = data.get("recent_k")
        self.cfg = B.PQAttnConfig(
            batch=Bn, n_q_heads=n_q_heads, n_kv_heads=Hkv, head_dim=d, n_subspaces=M,
            n_centroids=int(data["k_codebook"].shape[2]),
            max_context=int(max_context if max_context is not None else n_tok),
            max_recent=0 if rk is None else int(rk.shape[2]),
            dtype=B.PQ_F16 if dtype == "f16" else B.PQ_F32, device=device, n_splits=n_splits)
        self.ctx = B.pq_attn_create(self.cfg)
        self.n_splits = B.pq_attn_n_splits(self.ctx)
        self.n_passes = B.pq_attn_n_passes(self.ctx)
        self.heads_per_workgroup = B.pq_attn_heads_per_workgroup(self.ctx)
        self.codes_bytes = B.pq_attn_codes_bytes(self.cfg)

        self.q = _dev(data["q"], self.device)
        self.k_codebook = _dev(data["k_codebook"], self.device)
        self.v_codebook = _dev(data["v_codebook"], self.device)
        self.recent_k = _dev(rk, self.device)
        self.recent_v = _dev(data.get("recent_v"), self.device)
        self.recent_len = _dev(data["recent_len"].astype(np.int32), self.device) if rk is not None else None
        self.ctx_len = _dev(data["ctx_len"].astype(np.int32), self.device)
        self.out = torch.empty((Bn, n_q_heads, d), dtype=torch.float32, device=self.device)

        # `code_copies` distinct packed copies of the code tensors (the benchmark rotates
        # through them so that reads come from HBM, not from the memory-side cache)
        self.k_codes, self.v_codes = [], []
        tm_k = _dev(k_codes, self.device)
        tm_v = _dev(data["v_codes"], self.device)
        for _ in range(code_copies):
            pk = torch.zeros(self.codes_bytes, dtype=torch.uint8, device=self.device)
            pv = torch.zeros(self.codes_bytes, dtype=torch.uint8, device=self.device)
            B.pq_pack_codes(self.ctx, B.PQ_CODES_K, tm_k, n_tok, pk)
            B.pq_pack_codes(self.ctx, B.PQ_CODES_V, tm_v, n_tok, pv)
            self.k_codes.append(pk)
            self.v_codes.append(pv)
        torch.cuda.synchronize(self.device)
        del tm_k, tm_v
        if register_codebooks:
            B.pq_attn_set_codebooks(self.ctx, self.k_codebook, self.v_codebook)

    def decode(self, scale: float, copy: int = 0, pass_codebooks: bool = False, out: Optional[torch.Tensor] = None):
        o = self.out if out is None else out
        B.pq_attn_decode(self.ctx, self.q, self.k_codes[copy], self.v_codes[copy], self.ctx_len,
                         self.k_codebook if pass_codebooks else None, self.v_codebook if pass_codebooks else None,
                         self.recent_k, self.recent_v, self.recent_len, float(scale), o)
        return o

    def prepared_decode(self, scale: float, copy: int = 0):
        """A zero-argument callable that launches decode on the CURRENT stream with the argument
        marshalling done once (the benchmark's inner loop must not be bound by Python)."""
        lib = B.load_library()
        import ctypes
        vp = ctypes.c_void_p
        stream = int(torch.cuda.current_stream().cuda_stream) or None
        args = (vp(self.ctx), vp(self.q.data_ptr()), vp(self.k_codes[copy].data_ptr()),
                vp(self.v_codes[copy].data_ptr()), vp(self.ctx_len.data_ptr()), None, None,
                vp(self.recent_k.data_ptr()) if self.recent_k is not None else None,
                vp(self.recent_v.data_ptr()) if self.recent_v is not None else None,
                vp(self.recent_len.data_ptr()) if self.recent_len is not None else None,
                ctypes.c_float(float(scale)), vp(self.out.data_ptr()), vp(stream) if stream else None)
        fn = lib.pq_attn_decode

        def call():
            rc = fn(*args)
            if rc != 0:
                raise B.PQAttnError(rc, "pq_attn_decode")
        return call

    def prepared_append(self, new_k: torch.Tensor, new_v: torch.Tensor, copy: int = 0):
        lib = B.load_library()
        import ctypes
        vp = ctypes.c_void_p
        stream = int(torch.cuda.current_stream().cuda_stream) or None
        args = (vp(self.ctx), vp(new_k.data_ptr()), vp(new_v.data_ptr()), ctypes.c_int32(new_k.shape[2]), None, None,
                vp(self.k_codes[copy].data_ptr()), vp(self.v_codes[copy].data_ptr()), vp(self.ctx_len.data_ptr()),
                vp(stream) if stream else None)
        fn = lib.pq_encode_append

        def call():
            rc = fn(*args)
            if rc != 0:
                raise B.PQAttnError(rc, "pq_encode_append")
        return call

    def append(self, new_k: torch.Tensor, new_v: torch.Tensor, copy: int = 0, pass_codebooks: bool = False):
        n_new = new_k.shape[2]
        B.pq_encode_append(self.ctx, new_k, new_v, n_new,
                           self.k_codebook if pass_codebooks else None, self.v_codebook if pass_codebooks else None,
                           self.k_codes[copy], self.v_codes[copy], self.ctx_len)

    def unpack(self, kind: int, n_tokens: int, copy: int = 0) -> np.ndarray:
        wide = self.cfg.n_centroids > 256                     # 12-bit codes travel token-major as 16-bit words
        tm = torch.empty((self.B, self.Hkv, n_tokens, self.M), dtype=torch.int16 if wide else torch.uint8,
                         device=self.device)
        src = self.k_codes[copy] if kind == B.PQ_CODES_K else self.v_codes[copy]
        B.pq_unpack_codes(self.ctx, kind, src, n_tokens, tm)
        torch.cuda.synchronize(self.device)
        out = tm.cpu().numpy()
        return out.view(np.uint16) if wide else out

    def device_error(self) -> int:
        return B.pq_attn_device_error(self.ctx)

    def close(self):
        if self.ctx:
            B.pq_attn_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
