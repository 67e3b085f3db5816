"""CPU oracle of the offline codebook training: k-means per subspace by Lloyd's iteration.

TEST INFRASTRUCTURE ONLY: tests and the benchmark's cpu_baseline leg may import this; the GPU
library never does.

The paper trains one codebook per (KV head, subspace) with k-means on sampled key / value
vectors (Section II-C, "training phase"; Section III-A, "Offline PQ Codebook Training") and says
nothing about initialisation, iteration count, empty clusters or the arithmetic.  What is computed
here, in the textbook's order:

  repeat n_iters times
    1. assignment: every sample sub-vector goes to its nearest centroid, squared Euclidean
       distance, equal distances to the lowest index — the same rule, and the same oracle routine,
       as the encode of Eq. 4;
    2. update: every centroid with at least one member becomes the arithmetic mean of its
       members; a centroid without members stays where it is.

The initial centroids are an input.  Centroids are stored in the codebook's dtype between
iterations, as the trained codebook is (fp16 in the paper's models):

  * store_dtype = float16: the member sum is exact (fp16 values are integers times 2^-24, summed as
    integers), mean = double(sum) * 2^-24 / count in IEEE double, then rounded to float32 and from
    there to float16.  Every step is a single correctly rounded operation, so the result is one
    definite fp16 number whatever the order of the members.
  * store_dtype = None: plain float64 throughout (sums accumulated in sample order); used to pin
    this routine against a library k-means.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from . import pq_oracle


def lloyd_update(x: np.ndarray, labels: np.ndarray, centroids: np.ndarray, store_dtype) -> np.ndarray:
    """One update step for one (head, subspace): x [n, ds], labels [n], centroids [C, ds]."""
    C, ds = centroids.shape
    counts = np.bincount(labels, minlength=C)
    if store_dtype is None:
        sums = np.zeros((C, ds), dtype=np.float64)
        np.add.at(sums, labels, x.astype(np.float64))
        new = np.array(centroids, dtype=np.float64)
        has = counts > 0
        new[has] = sums[has] / counts[has, None]
        return new
    assert store_dtype == np.float16 and x.dtype == np.float16
    fixed = (x.astype(np.float64) * 2.0 ** 24).astype(np.int64)       # exact: |x| * 2^24 < 2^41
    sums = np.zeros((C, ds), dtype=np.int64)
    np.add.at(sums, labels, fixed)                                      # exact integer sums
    new = np.array(centroids, dtype=np.float16)
    has = counts > 0
    mean = sums[has].astype(np.float64) * 2.0 ** -24 / counts[has, None].astype(np.float64)
    new[has] = mean.astype(np.float32).astype(np.float16)
    return new


def kmeans_lloyd(samples: np.ndarray, codebook: np.ndarray, n_iters: int,
                 store_dtype: Optional[type] = np.float16) -> Tuple[np.ndarray, np.ndarray]:
    """samples [Hkv, n, d], codebook [Hkv, M, C, ds] (initial centroids) -> (trained codebook, labels
    [Hkv, n, M] of the last assignment step)."""
    x = np.asarray(samples)
    cb = np.array(codebook, dtype=np.float64 if store_dtype is None else store_dtype)
    Hkv, n, d = x.shape
    _, M, C, ds = cb.shape
    assert cb.shape[0] == Hkv and M * ds == d
    labels = np.zeros((Hkv, n, M), dtype=np.int64)
    for _ in range(n_iters):
        labels = pq_oracle.encode(x[None], cb)[0].astype(np.int64)     # step 1
        for h in range(Hkv):
            for i in range(M):                                         # step 2
                cb[h, i] = lloyd_update(x[h, :, i * ds:(i + 1) * ds], labels[h, :, i], cb[h, i], store_dtype)
    return cb, labels


def inertia(samples: np.ndarray, codebook: np.ndarray) -> float:
    """Sum over all sample sub-vectors of the squared distance to the nearest centroid (float64)."""
    x = np.asarray(samples, dtype=np.float64)
    cb = np.asarray(codebook, dtype=np.float64)
    Hkv, n, d = x.shape
    _, M, C, ds = cb.shape
    total = 0.0
    for h in range(Hkv):
        for i in range(M):
            diff = x[h, :, None, i * ds:(i + 1) * ds] - cb[h, i][None]
            total += float((diff * diff).sum(-1).min(-1).sum())
    return total
