"""pq_attn_decode_noalloc — decode with every piece of scratch in an array that is part of the library's device
code, for callers that cannot allocate — against pq_attn_decode on the same inputs: two calls in a row on the one
array, the second with a smaller input (fewer heads, shorter context, the other kernel)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import pq_oracle as O
from paper_2504_03661_amd import PQAttnConfig, binding as B
from paper_2504_03661_amd.harness import PQSession
from synth import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-3, 1e-3


def close(got, ref, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref).max()
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    assert err <= MAX_ABS and rel <= REL_L2, f"{what}: max_abs={err:.3e} rel_l2={rel:.3e}"


def run_both(name, B_, Hq, Hkv, M, ctx, rcap, dtype, seed):
    print(f"no-alloc case {name}: B={B_} Hq={Hq} Hkv={Hkv} M={M} ctx={ctx} recent<{rcap} {dtype}", flush=True)
    w = W.Workload(name, B_, Hq, Hkv, 128, M, ctx, dtype, recent_cap=rcap, recent_uniform=rcap > 0, seed=seed)
    data = W.generate(w)
    scale = W.attention_scale(w)
    with PQSession(data, Hq, dtype) as s:
        want = s.decode(scale).clone()
        torch.cuda.synchronize()
        got = torch.full_like(want, float("nan"))
        B.pq_attn_decode_noalloc(s.cfg, s.q, s.k_codes[0], s.v_codes[0], s.ctx_len, s.k_codebook, s.v_codebook,
                                 s.recent_k, s.recent_v, s.recent_len, scale, got)
        torch.cuda.synchronize()
        got, want = got.cpu().numpy(), want.cpu().numpy()
    close(got, want, f"{name}: no-alloc entry point against pq_attn_decode")
    ref = O.decode(data["q"], data["k_codes"], data["v_codes"], data["ctx_len"], data["k_codebook"], data["v_codebook"],
                   data["recent_k"], data["recent_v"], data["recent_len"], scale=scale)
    close(got, ref, f"{name}: no-alloc entry point against the oracle")


def test_two_calls_in_a_row_the_second_smaller():
    run_both("na_big", 2, 8, 8, 64, 9000, 40, "f16", 8101)       # per-head kernel, 16 rows x several splits
    run_both("na_small", 1, 4, 2, 64, 1300, 7, "f16", 8102)      # grouped-query kernel, fewer rows, shorter context
    run_both("na_big_again", 2, 8, 8, 32, 9000, 0, "f16", 8103)  # and back up: M = 32, no window
    run_both("na_f32", 1, 2, 2, 64, 700, 5, "f32", 8104)


def test_replays_from_a_graph():
    """The call launches kernels only (codebook re-pack, ticket fill, decode), so a caller can record it into a HIP
    graph: replays with eager work and synchronisations between them give what the eager call gives."""
    w = W.Workload("na_graph", 1, 8, 2, 128, 64, 6000, "f16", recent_cap=12, recent_uniform=True, seed=8105)
    data = W.generate(w)
    scale = W.attention_scale(w)
    rng = np.random.default_rng(6)
    queries = [torch.from_numpy(rng.standard_normal(data["q"].shape).astype(np.float16)).cuda() for _ in range(3)]
    with PQSession(data, 8, "f16") as s:
        def call(out):
            B.pq_attn_decode_noalloc(s.cfg, s.q, s.k_codes[0], s.v_codes[0], s.ctx_len, s.k_codebook, s.v_codebook,
                                     s.recent_k, s.recent_v, s.recent_len, scale, out)
        eager = []
        for q in queries:
            s.q.copy_(q)
            o = torch.empty_like(s.out)
            call(o)
            eager.append(o)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()                           # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            call(s.out)                                      # warm-up on the capturing stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            call(s.out)
        for rep in range(6):
            i = rep % 3
            s.q.copy_(queries[i])
            s.out.fill_(float("nan"))                        # eager work between the replays
            g.replay()
            torch.cuda.synchronize()
            dev = (s.out - eager[i]).abs().max().item()
            assert dev <= 4e-6, f"replay {rep} differs from the eager call by {dev:.3e}"


def test_limits_are_rejected_before_anything_is_launched():
    lib = B.load_library()
    q = torch.zeros(16, device="cuda")

    def call(cfg):
        p = ctypes.c_void_p(q.data_ptr())
        return lib.pq_attn_decode_noalloc(ctypes.byref(cfg.c_struct()), p, p, p, p, p, p, None, None, None, 1.0, p, None)

    ok = dict(batch=1, n_q_heads=4, n_kv_heads=4, max_context=256)
    assert call(PQAttnConfig(**{**ok, "n_q_heads": 64, "n_kv_heads": 64})) == -4          # 4 MiB of fp16 codebooks
    assert call(PQAttnConfig(**{**ok, "n_q_heads": 32, "n_kv_heads": 32, "dtype": B.PQ_F32})) == -4
    assert call(PQAttnConfig(**{**ok, "batch": 300})) == -4                               # 1200 rows
    assert call(PQAttnConfig(**{**ok, "batch": 64, "n_splits": 8})) == -4                 # 2048 partial rows
    assert call(PQAttnConfig(**{**ok, "n_subspaces": 32, "n_centroids": 4096})) == -3     # 12-bit codes
    assert call(PQAttnConfig(**{**ok, "batch": 0})) == -2
    assert lib.pq_attn_decode_noalloc(None, None, None, None, None, None, None, None, None, None, 1.0, None, None) == -1
