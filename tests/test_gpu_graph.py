"""pq_attn_decode and pq_encode_append launch kernels and nothing else, so a caller can capture them in a HIP graph:
every replay must give what the eager call gives (replays interleaved with eager work and synchronisations)."""
import numpy as np
import pytest
import torch

from oracle import pq_oracle as O
from paper_2504_03661_amd import PQ_CODES_K
from paper_2504_03661_amd.harness import PQSession
from synth import workloads as W

pytestmark = pytest.mark.gpu

CASES = [
    # name, B, Hq, Hkv, M, context, recent rows, centroids, n_splits
    ("per_head", 2, 4, 4, 64, 9000, 40, 256, 3),
    ("grouped", 1, 8, 2, 64, 20000, 16, 256, 4),
    ("two_bit", 2, 2, 2, 32, 5000, 0, 256, 2),
    ("two_bit_grouped", 1, 8, 2, 32, 12000, 9, 256, 3),
    ("pq12_fused", 1, 2, 2, 32, 9000, 8, 4096, 2),
    ("pq12_two_pass", 1, 2, 2, 32, 9000, 8, 4096, -2),
    ("pq12_grouped", 1, 8, 2, 32, 9000, 8, 4096, 2),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_decode_replays_from_a_graph(case):
    name, B_, Hq, Hkv, M, ctx, rcap, C, splits = case
    w = W.Workload("graph_" + name, B_, Hq, Hkv, 128, M, ctx, "f16", recent_cap=rcap, recent_uniform=rcap > 0, seed=77,
                   n_centroids=C)
    data = W.generate(w)
    scale = W.attention_scale(w)
    rng = np.random.default_rng(5)
    queries = [torch.from_numpy(rng.standard_normal(data["q"].shape).astype(np.float16)).cuda() for _ in range(3)]
    with PQSession(data, Hq, "f16", n_splits=splits) as s:
        eager = []
        for q in queries:
            s.q.copy_(q)
            eager.append(s.decode(scale).clone())
        torch.cuda.synchronize()
        ref = O.decode(queries[0].cpu().numpy(), data["k_codes"], data["v_codes"], data["ctx_len"], data["k_codebook"],
                       data["v_codebook"], data["recent_k"], data["recent_v"], data["recent_len"], scale=scale)
        assert np.abs(eager[0].cpu().numpy() - ref).max() <= 2e-3
        side = torch.cuda.Stream()                           # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            s.decode(scale)                                  # warm-up on the capturing stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            s.decode(scale)
        for rep in range(6):
            i = rep % 3
            s.q.copy_(queries[i])
            s.out.fill_(float("nan"))                        # eager work between the replays
            g.replay()
            torch.cuda.synchronize()
            dev = (s.out - eager[i]).abs().max().item()
            assert dev <= 4e-6, f"{name}: replay {rep} differs from the eager call by {dev:.3e}"


@pytest.mark.parametrize("M,C", [(64, 256), (32, 4096)], ids=["8bit", "12bit"])
def test_append_and_decode_in_one_graph(M, C):
    """One decoding step as a caller would capture it: append 3 tokens per head, then attend.  (12-bit codes: the
    append stages its codes in memory the context allocated at creation, so the very first append is capturable.)"""
    w = W.Workload("graph_step", 2, 4, 4, 128, M, 700, "f16", n_new=3, seed=78, n_centroids=C)
    data = W.generate(w, ctx_cap=800)
    scale = W.attention_scale(w)
    nk, nv = torch.from_numpy(data["new_k"]).cuda(), torch.from_numpy(data["new_v"]).cuda()
    with PQSession(data, 4, "f16", max_context=800) as s:
        base = s.ctx_len.clone()
        s.append(nk, nv)
        want = s.decode(scale).clone()
        want_codes = s.unpack(PQ_CODES_K, 700)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        s.ctx_len.copy_(base)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            s.append(nk, nv)
            s.decode(scale)
        for rep in range(3):
            s.ctx_len.copy_(base)
            s.out.zero_()
            g.replay()
            torch.cuda.synchronize()
            assert s.ctx_len.cpu().tolist() == (base + 3).cpu().tolist()
            assert (s.out - want).abs().max().item() <= 4e-6
            np.testing.assert_array_equal(s.unpack(PQ_CODES_K, 700), want_codes)
