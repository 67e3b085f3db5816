"""The fp16 encode decides codes in fp64 but first filters centroids with fp32 matrix-core sums; the filter is safe
if its threshold tau is at least twice the largest deviation of a computed value from the true one.  This test
re-computes the kernel's tau (with the constants of csrc/pq_filter_constants.h, which both encode kernels include) and checks it against an
emulation of the sums under the WORST rounding the bound allows for — every fp32 addition truncated toward zero,
terms added one after the other — on random inputs of very different magnitudes."""
import os
import re

import numpy as np
import pytest

_HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2504_03661_amd", "csrc",
                       "pq_filter_constants.h")


def _constant(name):
    """The value the kernels are compiled with: parsed from the header both encode kernels include."""
    m = re.search(r"^#define\s+" + name + r"\s+([0-9.eE+-]+)f\s*$", open(_HEADER).read(), re.M)
    assert m, name
    return np.float32(m.group(1))


K_REL, K_ABS, X2F = _constant("PQ_FILTER_TAU_REL"), _constant("PQ_FILTER_TAU_ABS"), _constant("PQ_FILTER_X2_FACTOR")


def trunc32(v):
    """float64 -> the float32 obtained by truncating toward zero."""
    f = np.asarray(v, dtype=np.float64).astype(np.float32)
    over = np.abs(f.astype(np.float64)) > np.abs(v)
    return np.where(over, np.nextafter(f, np.float32(0)), f).astype(np.float32)


def kernel_tau_and_off(x, n_max, c_max):
    """As the kernels compute them, in float32: x [n, ds] (float32 views of fp16 values)."""
    x1 = np.zeros(len(x), np.float32)
    x2 = np.zeros(len(x), np.float32)
    for j in range(x.shape[1]):
        x1 = x1 + np.abs(x[:, j])
        x2 = x2 + x[:, j] * x[:, j]
    t0 = n_max + x1 * c_max + X2F * x2
    off = X2F * x2 + np.float32(2.0) * (K_REL * (np.float32(2.0) * t0) + K_ABS)
    tau = K_REL * (t0 + off) + K_ABS
    return tau, off + tau


@pytest.mark.parametrize("ds", [2, 4])
@pytest.mark.parametrize("c_scale,x_scale", [(1.0, 1.0), (1e-3, 1e-3), (30.0, 1.0), (1.0, 200.0), (30.0, 100.0), (1e-5, 3.0)])
def test_tau_covers_twice_the_worst_case_error(ds, c_scale, x_scale):
    rng = np.random.default_rng(int(1000 * ds + 7 * c_scale + x_scale) % 2**31)
    c = (rng.standard_normal((256, ds)) * c_scale).astype(np.float16).astype(np.float32)
    x = (rng.standard_normal((512, ds)) * x_scale).astype(np.float16).astype(np.float32)
    # centroid rows as the kernel builds them
    n = np.zeros(256, np.float32)
    for j in range(ds):
        n = n + c[:, j] * c[:, j]                             # exact squares, rounded sums
    h = np.float32(0.5) * n
    hh = h.astype(np.float16)
    hl = (h - hh.astype(np.float32)).astype(np.float16)
    assert np.isfinite(hh.astype(np.float32)).all() and (h < 60000).all()
    n_max, c_max = h.max(), np.abs(c).max()
    tau, off = kernel_tau_and_off(x, n_max, c_max)
    # computed value: C operand first, then the products, then h and l, every add truncated
    acc = np.repeat(off[:, None], 256, axis=1).astype(np.float32)
    for j in range(ds):
        prod = -(x[:, j].astype(np.float64)[:, None] * c[:, j].astype(np.float64)[None, :])      # exact in fp32
        acc = trunc32(acc.astype(np.float64) + prod)
    acc = trunc32(acc.astype(np.float64) + hh.astype(np.float64)[None, :])
    acc = trunc32(acc.astype(np.float64) + hl.astype(np.float64)[None, :])
    # true value: off + |c|^2 / 2 - x . c in float64 (exact to 1e-16 relative of the magnitudes)
    true = off.astype(np.float64)[:, None] + 0.5 * (c.astype(np.float64) ** 2).sum(1)[None, :] \
        - x.astype(np.float64) @ c.astype(np.float64).T
    err = np.abs(acc.astype(np.float64) - true).max(axis=1)
    assert (2.0 * err <= tau.astype(np.float64)).all(), (2.0 * err / tau).max()
    assert (2.0 * err <= 0.85 * tau.astype(np.float64)).all()          # and with room to spare
    assert (acc > 0).all()                                  # the offset keeps every value positive: integer order = float order
    # pass 2: the C operand becomes off - (best + tau) and a NEGATIVE computed value marks a candidate.  Under the same
    # worst-case rounding (truncation toward zero makes negative values less negative) every centroid that is not
    # marked must have a strictly larger true value than the true minimiser, which itself must be marked.
    best = acc.min(axis=1)
    d = (off - (best + tau)).astype(np.float32)
    for rounding in (trunc32, lambda v: np.asarray(v, np.float64).astype(np.float32)):
        acc2 = np.repeat(d[:, None], 256, axis=1).astype(np.float32)
        for j in range(ds):
            prod = -(x[:, j].astype(np.float64)[:, None] * c[:, j].astype(np.float64)[None, :])
            acc2 = rounding(acc2.astype(np.float64) + prod)
        acc2 = rounding(acc2.astype(np.float64) + hh.astype(np.float64)[None, :])
        acc2 = rounding(acc2.astype(np.float64) + hl.astype(np.float64)[None, :])
        marked = np.signbit(acc2)
        rows = np.arange(len(x))
        assert marked[rows, true.argmin(axis=1)].all()
        unmarked_min = np.where(marked, np.inf, true).min(axis=1)
        assert (unmarked_min > true.min(axis=1)).all()
        if c_scale >= 1e-3:                                 # (tiny centroids all sit within the absolute floor of tau)
            assert marked.sum(axis=1).max() <= 64           # a filter, not a pass-through


def test_truncation_helper():
    v = np.array([1.0 + 2.0 ** -24, -(1.0 + 2.0 ** -24), 1.0 + 3 * 2.0 ** -24, 0.1])
    t = trunc32(v)
    assert t[0] == np.float32(1.0) and t[1] == np.float32(-1.0) and t[2] == np.float32(1.0 + 2.0 ** -23)
    assert abs(float(t[3])) <= 0.1
