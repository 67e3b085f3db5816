"""Pins of the k-means oracle (oracle/pq_kmeans_oracle.py) against things other than itself: a
library k-means, a pure-Python Lloyd iteration with exact rational means, and the invariants of
the algorithm (Section II-C training phase; Section III-A, "Offline PQ Codebook Training")."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.cluster.vq import kmeans2

from oracle import pq_kmeans_oracle as K
from synth import workloads as W


def blobs(rng, n):
    """256 clusters on a 16 x 16 grid of spacing 1, 0.02 wide: every point is nearest to its own centre."""
    gx, gy = np.meshgrid(np.arange(16.0), np.arange(16.0))
    centres = np.stack([gx.ravel(), gy.ravel()], axis=1)
    which = np.concatenate([np.arange(256), rng.integers(0, 256, size=n - 256)])
    return centres, which, centres[which] + 0.02 * rng.standard_normal((n, 2))


@pytest.mark.parametrize("ds,iters", [(2, 1), (2, 4), (4, 3)])
def test_float64_mode_equals_scipy_kmeans2(ds, iters):
    # one head, one subspace, float64 throughout; scipy's kmeans2 with an explicit initial matrix runs the
    # same Lloyd iteration (assign, mean, empty clusters keep their centroid)
    rng = np.random.default_rng(3 + ds)
    x = rng.standard_normal((3000, ds))
    init = x[:256].copy()
    ref, ref_labels = kmeans2(x, init, iter=iters, minit="matrix", missing="warn")
    cb, labels = K.kmeans_lloyd(x[None], init[None, None], iters, store_dtype=None)
    np.testing.assert_allclose(cb[0, 0], ref, rtol=1e-12, atol=1e-12)
    # kmeans2 returns the labels of its last assignment step (the one the final means were taken over)
    assert (labels[0, :, 0] == ref_labels).all()


def python_lloyd_fp16(x, cent, iters):
    """Lloyd iteration in pure Python: exact rational distances and means, rounded float32 then float16."""
    x = [[Fraction(float(v)) for v in row] for row in x]
    cent = [[Fraction(float(v)) for v in row] for row in cent]
    for _ in range(iters):
        members = [[] for _ in cent]
        for row in x:
            dist = [sum((a - b) ** 2 for a, b in zip(row, c)) for c in cent]
            members[dist.index(min(dist))].append(row)          # index(): lowest index among equal minima
        for c, rows in enumerate(members):
            if rows:
                mean = [sum(col) / len(rows) for col in zip(*rows)]
                cent[c] = [Fraction(float(np.float16(np.float32(float(m))))) for m in mean]
    return np.array([[float(v) for v in row] for row in cent], dtype=np.float16)


def test_fp16_mode_equals_exact_rational_lloyd_on_a_tiny_case():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((90, 2)).astype(np.float16)
    init = x[:6].copy()
    init[5] = init[1]                                             # a duplicate: cluster 5 can never win a tie
    want = python_lloyd_fp16(x, init, 3)
    # the oracle's encode needs 256 centroids only by convention of the GPU side; any count works on the CPU
    got, _ = K.kmeans_lloyd(x[None], init[None, None], 3)
    assert got.dtype == np.float16
    assert (got[0, 0].view(np.uint16) == want.view(np.uint16)).all()
    one, _ = K.kmeans_lloyd(x[None], init[None, None], 1)
    assert (one[0, 0, 5].view(np.uint16) == init[5].view(np.uint16)).all()   # empty in iteration 1: kept its centroid


def test_update_is_the_correctly_rounded_mean_whatever_the_member_order():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((5000, 4)) * 30).astype(np.float16)
    labels = rng.integers(0, 7, size=5000)
    cent = np.zeros((8, 4), dtype=np.float16)                      # cluster 7 has no members
    cent[7] = [1, 2, 3, 4]
    a = K.lloyd_update(x, labels, cent, np.float16)
    perm = rng.permutation(5000)
    b = K.lloyd_update(x[perm], labels[perm], cent, np.float16)
    assert (a.view(np.uint16) == b.view(np.uint16)).all()
    for c in range(7):
        rows = [[Fraction(float(v)) for v in r] for r in x[labels == c]]
        mean = [sum(col) / len(rows) for col in zip(*rows)]
        want = np.array([float(m) for m in mean]).astype(np.float32).astype(np.float16)   # float(Fraction): correctly rounded
        assert (a[c].view(np.uint16) == want.view(np.uint16)).all()
    assert (a[7] == cent[7]).all()


def test_inertia_never_increases_in_float64_mode():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((2, 4000, 8))
    cb = np.ascontiguousarray(x[:, :256].reshape(2, 256, 2, 4).transpose(0, 2, 1, 3))
    last = K.inertia(x, cb)
    for _ in range(5):
        cb, _ = K.kmeans_lloyd(x, cb, 1, store_dtype=None)
        now = K.inertia(x, cb)
        assert now <= last * (1 + 1e-12)
        last = now


def test_separated_blobs_are_recovered_and_are_a_fixed_point():
    rng = np.random.default_rng(21)
    centres, which, x = blobs(rng, 6000)
    init = rng.permutation(centres + 0.1)                          # displaced centres, in another order
    cb, labels = K.kmeans_lloyd(x[None], init[None, None], 2, store_dtype=None)
    means = np.stack([x[which == c].mean(0) for c in range(256)])
    order = np.lexsort((cb[0, 0][:, 0].round(), cb[0, 0][:, 1].round()))      # back to grid order
    np.testing.assert_allclose(cb[0, 0][order], means, rtol=0, atol=1e-12)
    again, _ = K.kmeans_lloyd(x[None], cb, 1, store_dtype=None)
    np.testing.assert_allclose(again, cb, rtol=0, atol=1e-12)


def test_generator_shapes_and_duplicates():
    d = W.training_samples(3, 700, 128, 32, seed=4, duplicate_init=5)
    assert d["samples"].shape == (3, 700, 128) and d["samples"].dtype == np.float16
    assert d["init"].shape == (3, 32, 256, 4)
    assert (d["init"][:, :, 251:] == d["init"][:, :, :5]).all()
    assert (d["init"][1, 2, 7] == d["samples"][1, 7, 8:12]).all()
    cb, labels = K.kmeans_lloyd(d["samples"], d["init"], 1)
    # in the first iteration the duplicates receive no member (ties go to the lowest index) and stay put
    assert (labels < 251).all()
    assert (cb[:, :, 251:].view(np.uint16) == d["init"][:, :, 251:].view(np.uint16)).all()
