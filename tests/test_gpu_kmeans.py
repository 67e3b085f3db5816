"""GPU parity of the offline codebook training (pq_kmeans_fit) against the k-means oracle: the trained
fp16 codebooks must be bit-identical (assignment is decided in IEEE double on both sides, member sums
are exact, the mean is rounded the same way)."""
import numpy as np
import pytest
import torch

from oracle import pq_kmeans_oracle as K
from paper_2504_03661_amd import PQAttnConfig, PQAttnError, binding as B
from synth import workloads as W

pytestmark = pytest.mark.gpu


def make_ctx(Hkv, M, dtype=B.PQ_F16, n_centroids=256):
    cfg = PQAttnConfig(batch=1, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, n_subspaces=M, n_centroids=n_centroids,
                       max_context=64, max_recent=0, dtype=dtype, device=0, n_splits=0)
    return B.pq_attn_create(cfg)


def gpu_fit(ctx, samples, init, iters):
    x = torch.from_numpy(samples).cuda()
    cb = torch.from_numpy(init.copy()).cuda()
    nbytes = B.pq_kmeans_workspace_bytes(ctx)
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")     # workspace contents are arbitrary
    B.pq_kmeans_fit(ctx, x, samples.shape[1], cb, iters, ws, nbytes)
    torch.cuda.synchronize()
    return cb.cpu().numpy()


@pytest.mark.parametrize("Hkv,M,n,iters,dup", [(2, 64, 3000, 1, 0), (2, 64, 3000, 3, 6), (3, 32, 1025, 2, 3),
                                               (1, 32, 256, 4, 0), (1, 64, 5000, 5, 0)])
def test_trained_codebook_is_bit_identical_to_the_oracle(Hkv, M, n, iters, dup):
    d = W.training_samples(Hkv, n, 128, M, seed=Hkv * 100 + M + n, duplicate_init=dup)
    want, _ = K.kmeans_lloyd(d["samples"], d["init"], iters)
    ctx = make_ctx(Hkv, M)
    try:
        got = gpu_fit(ctx, d["samples"], d["init"], iters)
    finally:
        B.pq_attn_destroy(ctx)
    assert got.dtype == np.float16 and got.shape == want.shape
    diff = got.view(np.uint16) != want.view(np.uint16)
    assert not diff.any(), f"{int(diff.sum())} of {diff.size} centroid coordinates differ"
    if dup and iters == 1:
        assert (got[:, :, 256 - dup:].view(np.uint16) == d["init"][:, :, 256 - dup:].view(np.uint16)).all()


@pytest.mark.parametrize("n,iters,dup", [(5000, 2, 0), (8192 + 77, 1, 9)])
def test_trained_12bit_codebook_is_bit_identical_to_the_oracle(n, iters, dup):
    """4096 centroids per subspace (M = 32): assignment in chunks of 8192 samples, sums added straight to memory."""
    d = W.training_samples(2, n, 128, 32, seed=n, duplicate_init=dup, n_centroids=4096)
    want, _ = K.kmeans_lloyd(d["samples"], d["init"], iters)
    ctx = make_ctx(2, 32, n_centroids=4096)
    try:
        got = gpu_fit(ctx, d["samples"], d["init"], iters)
    finally:
        B.pq_attn_destroy(ctx)
    diff = got.view(np.uint16) != want.view(np.uint16)
    assert not diff.any(), f"{int(diff.sum())} of {diff.size} centroid coordinates differ"


def test_training_lowers_the_quantization_error_and_the_codebook_serves_encode():
    d = W.training_samples(2, 4096, 128, 64, seed=77)
    ctx = make_ctx(2, 64)
    try:
        got = gpu_fit(ctx, d["samples"], d["init"], 8)
    finally:
        B.pq_attn_destroy(ctx)
    before, after = K.inertia(d["samples"], d["init"]), K.inertia(d["samples"], got)
    assert after < 0.6 * before


def test_fit_argument_errors():
    ctx = make_ctx(1, 64)
    ctx32 = make_ctx(1, 64, B.PQ_F32)
    try:
        x = torch.zeros((1, 300, 128), dtype=torch.float16, device="cuda")
        cb = torch.zeros((1, 64, 256, 2), dtype=torch.float16, device="cuda")
        n = B.pq_kmeans_workspace_bytes(ctx)
        ws = torch.zeros(n, dtype=torch.uint8, device="cuda")
        for args, status in [((x, 0, cb, 1, ws, n), -2), ((x, 300, cb, 0, ws, n), -2), ((x, 300, cb, 1, ws, n - 1), -4),
                             ((x, (1 << 20) + 1, cb, 1, ws, n), -4), ((None, 300, cb, 1, ws, n), -1),
                             ((x, 300, None, 1, ws, n), -1), ((x, 300, cb, 1, None, n), -1)]:
            with pytest.raises(PQAttnError) as e:
                B.pq_kmeans_fit(ctx, *args)
            assert e.value.status == status
        with pytest.raises(PQAttnError) as e:
            B.pq_kmeans_workspace_bytes(ctx32)
        assert e.value.status == -3
        with pytest.raises(PQAttnError) as e:
            B.pq_kmeans_fit(ctx32, x, 300, cb, 1, ws, n)
        assert e.value.status == -3
    finally:
        B.pq_attn_destroy(ctx)
        B.pq_attn_destroy(ctx32)
