"""Pins for the CPU oracle: each test holds oracle/ to something other than itself.

What fixes the expected value in each test is named in its docstring: a library
routine (scipy softmax, torch scaled_dot_product_attention, scipy.cluster.vq.vq),
a closed form, an invariant, or brute force written with different machinery
(vectorised numpy gathers instead of loops).  None of them needs a GPU.
"""
import os

import numpy as np
import pytest
import scipy.cluster.vq
import scipy.special
import torch

from oracle import pq_oracle as O
from synth import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small(seed=0, B=2, Hq=4, Hkv=4, d=16, M=8, N=37, R=5, dtype="f32", lens=None):
    w = W.Workload("t", B, Hq, Hkv, d, M, N, dtype, recent_cap=max(R, 0), recent_fixed=R if R > 0 else None,
                   seed=1000 + seed, ctx_lens=lens)
    return w, W.generate(w)


def brute_force(data, scale, b, hq, G=1):
    """Dense attention over explicitly decoded K/V with library softmax (scipy)."""
    hkv = hq // G
    N = int(data["ctx_len"][b])
    kc = data["k_codes"][b, hkv, :N].astype(np.int64)          # [N, M]
    vc = data["v_codes"][b, hkv, :N].astype(np.int64)
    kcb = data["k_codebook"][hkv].astype(np.float64)           # [M, C, ds]
    vcb = data["v_codebook"][hkv].astype(np.float64)
    M = kc.shape[1]
    sub = np.arange(M)[None, :]
    d = kcb.shape[0] * kcb.shape[2]
    K = kcb[sub, kc].reshape(N, d)                              # gather + concatenate (Eq. 5)
    V = vcb[sub, vc].reshape(N, d)
    R = int(data["recent_len"][b])
    if R:
        K = np.concatenate([K, data["recent_k"][b, hkv, :R].astype(np.float64)])
        V = np.concatenate([V, data["recent_v"][b, hkv, :R].astype(np.float64)])
    s = (K @ data["q"][b, hq].astype(np.float64)) * float(np.float32(scale))
    return scipy.special.softmax(s) @ V


def run_oracle(w, data, **kw):
    return O.decode(data["q"], data["k_codes"], data["v_codes"], data["ctx_len"], data["k_codebook"],
                    data["v_codebook"], data["recent_k"], data["recent_v"], data["recent_len"],
                    scale=W.attention_scale(w), **kw)


@pytest.mark.parametrize("seed,dtype,M,R", [(0, "f32", 8, 5), (1, "f16", 4, 0), (2, "f16", 16, 9), (3, "f32", 2, 1)])
def test_decode_matches_brute_force_library_softmax(seed, dtype, M, R):
    """Brute force on tiny inputs: numpy gather + scipy.special.softmax."""
    w, data = small(seed, d=16, M=M, R=R, dtype=dtype, lens=(37, 11))
    out = run_oracle(w, data)
    for b in range(w.batch):
        for h in range(w.n_q_heads):
            np.testing.assert_allclose(out[b, h], brute_force(data, W.attention_scale(w), b, h), rtol=1e-12,
                                       atol=1e-14)


def test_decode_reduces_to_dense_attention_when_codebook_holds_the_vectors():
    """Special case that is textbook attention: centroid t of every subspace is the
    t-th source sub-vector and code[t, i] = t, so K^ = K and V^ = V exactly; the
    expected value comes from torch's scaled_dot_product_attention in float64."""
    rng = np.random.default_rng(5)
    B, H, d, M, N = 1, 3, 32, 8, 200
    ds = d // M
    K = rng.standard_normal((H, N, d))
    V = rng.standard_normal((H, N, d))
    q = rng.standard_normal((B, H, d))
    kcb = np.zeros((H, M, 256, ds))
    vcb = np.zeros((H, M, 256, ds))
    kcb[:, :, :N, :] = K.reshape(H, N, M, ds).transpose(0, 2, 1, 3)
    vcb[:, :, :N, :] = V.reshape(H, N, M, ds).transpose(0, 2, 1, 3)
    codes = np.broadcast_to(np.arange(N, dtype=np.uint8)[None, None, :, None], (B, H, N, M)).copy()
    scale = np.float32(1 / np.sqrt(d))
    out = O.decode(q, codes, codes, np.array([N], np.int32), kcb, vcb, scale=scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).reshape(1, H, 1, d), torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        scale=float(scale)).reshape(H, d).numpy()
    np.testing.assert_allclose(out[0], ref, rtol=1e-11, atol=1e-13)


def test_hand_worked_example_from_golden_file():
    """Closed form: softmax([0, ln 3]) = [1/4, 3/4]; derivation in the fixture."""
    vals = {}
    for line in open(os.path.join(GOLDEN, "hand_worked_attention.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array([float(x) for x in v])
    kcb = np.zeros((1, 2, 2, 1)); kcb[0, 0, :, 0] = [0, 1]; kcb[0, 1, :, 0] = [0, 2]
    vcb = np.zeros((1, 2, 2, 1)); vcb[0, 0, :, 0] = [1, 5]; vcb[0, 1, :, 0] = [-2, 2]
    kc = np.array([[[[0, 1], [1, 0]]]], np.uint8)
    vc = np.array([[[[0, 1], [1, 0]]]], np.uint8)
    scale = np.float32(1 / np.sqrt(2.0))
    # q chosen so that float(scale) * q[0] * 1 == ln 3 to the last bit that matters
    q = np.array([[[np.log(3.0) / float(scale), 0.0]]])
    out = O.decode(q, kc, vc, np.array([2], np.int32), kcb, vcb, scale=scale)
    np.testing.assert_allclose(out[0, 0], vals["out_no_recent"], rtol=1e-14)
    _, wts = O.dense_attention(q[0, 0], O.dequantize(kc[0, 0], kcb[0]), O.dequantize(vc[0, 0], vcb[0]), scale)
    np.testing.assert_allclose(wts, vals["weights_no_recent"], rtol=1e-14)
    rk = np.array([[[[2.0, 7.0]]]]); rv = np.array([[[[-8.0, 11.0]]]])
    out = O.decode(q, kc, vc, np.array([2], np.int32), kcb, vcb, rk, rv, np.array([1], np.int32), scale=scale)
    np.testing.assert_allclose(out[0, 0], vals["out_with_recent"], rtol=1e-14)


def test_softmax_weights_sum_to_one_and_output_in_convex_hull():
    """Invariants of softmax attention: weights sum to 1; each output coordinate lies
    between the minimum and maximum of that coordinate over the value rows."""
    w, data = small(7, B=3, Hq=4, Hkv=4, d=32, M=16, N=300, R=12, lens=(300, 1, 77))
    out, wsum = run_oracle(w, data, return_weight_sum=True)
    np.testing.assert_allclose(wsum, 1.0, rtol=0, atol=1e-14)
    for b in range(w.batch):
        for h in range(w.n_q_heads):
            N, R = data["ctx_len"][b], data["recent_len"][b]
            V = np.concatenate([O.dequantize(data["v_codes"][b, h, :N], data["v_codebook"][h]),
                                data["recent_v"][b, h, :R].astype(np.float64)])
            assert (out[b, h] <= V.max(0) + 1e-12).all() and (out[b, h] >= V.min(0) - 1e-12).all()


def test_adding_a_constant_to_all_scores_changes_nothing():
    """Softmax shift invariance, exercised through the keys: adding a vector u to every
    key adds the same q.u to every score.  Built with the codebook-holds-the-vectors case."""
    rng = np.random.default_rng(11)
    H, d, M, N = 1, 8, 4, 50
    ds = d // M
    K = rng.standard_normal((N, d)); V = rng.standard_normal((N, d)); q = rng.standard_normal((1, 1, d))
    u = rng.standard_normal(d)
    codes = np.broadcast_to(np.arange(N, dtype=np.uint8)[None, None, :, None], (1, 1, N, M)).copy()

    def cb(X):
        c = np.zeros((1, M, 256, ds)); c[0, :, :N, :] = X.reshape(N, M, ds).transpose(1, 0, 2); return c
    a = O.decode(q, codes, codes, np.array([N], np.int32), cb(K), cb(V))
    b = O.decode(q, codes, codes, np.array([N], np.int32), cb(K + u), cb(V))
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)


def test_zero_query_gives_mean_of_value_rows():
    """Closed form: q = 0 makes every weight 1/n."""
    w, data = small(3, B=1, Hq=2, Hkv=2, d=16, M=8, N=64, R=7)
    data["q"][:] = 0
    out = run_oracle(w, data)
    for h in range(2):
        V = np.concatenate([O.dequantize(data["v_codes"][0, h, :64], data["v_codebook"][h]),
                            data["recent_v"][0, h, :7].astype(np.float64)])
        np.testing.assert_allclose(out[0, h], V.mean(0), rtol=1e-13, atol=1e-15)


def test_all_codes_equal_returns_that_decoded_value_row():
    """Closed form: identical rows -> output is that row whatever the weights."""
    w, data = small(4, B=1, Hq=1, Hkv=1, d=16, M=8, N=90, R=0)
    data["v_codes"][:] = data["v_codes"][0, 0, 0]
    out = run_oracle(w, data)
    row = data["v_codebook"][0][np.arange(8), data["v_codes"][0, 0, 0].astype(int)].reshape(-1).astype(np.float64)
    np.testing.assert_allclose(out[0, 0], row, rtol=1e-14)


def test_single_token_returns_its_value_and_empty_sequence_returns_zeros():
    """N = 1, R = 0 -> the decoded value row exactly; N + R = 0 -> zeros (documented reading)."""
    w, data = small(5, B=2, Hq=1, Hkv=1, d=16, M=8, N=4, R=0, lens=(1, 0))
    out, wsum = run_oracle(w, data, return_weight_sum=True)
    row = data["v_codebook"][0][np.arange(8), data["v_codes"][0, 0, 0].astype(int)].reshape(-1).astype(np.float64)
    assert (out[0, 0] == row).all()
    assert (out[1, 0] == 0).all() and wsum[1, 0] == 0


def test_dominant_key_selects_its_value_row():
    """Limit: one score far above the rest -> the output tends to that value row."""
    w, data = small(6, B=1, Hq=1, Hkv=1, d=16, M=8, N=40, R=3)
    q = data["q"][0, 0].astype(np.float64)
    data["recent_k"][0, 0, 1] = (q / np.linalg.norm(q) * 1e3).astype(np.float32)
    out = run_oracle(w, data)
    np.testing.assert_allclose(out[0, 0], data["recent_v"][0, 0, 1].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_token_permutation_invariance():
    w, data = small(8, B=1, Hq=2, Hkv=2, d=16, M=8, N=120, R=0)
    a = run_oracle(w, data)
    perm = np.random.default_rng(0).permutation(120)
    data["k_codes"] = data["k_codes"][:, :, perm]
    data["v_codes"] = data["v_codes"][:, :, perm]
    b = run_oracle(w, data)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_moving_a_token_from_codes_to_recent_window_changes_nothing():
    """One softmax over the concatenation (reading of Eq. 7's two terms): a token may sit
    in the quantized part or, with its decoded rows, in the full-precision part."""
    w, data = small(9, B=1, Hq=2, Hkv=2, d=16, M=8, N=50, R=4, dtype="f32")
    a = run_oracle(w, data)
    moved = dict(data)
    R0 = 4
    rk = np.full((1, 2, 6, 16), np.nan, np.float64); rv = rk.copy()
    rk[:, :, :R0] = data["recent_k"][:, :, :R0]; rv[:, :, :R0] = data["recent_v"][:, :, :R0]
    for h in range(2):
        rk[0, h, R0] = O.dequantize(data["k_codes"][0, h, 49:50], data["k_codebook"][h])[0]
        rv[0, h, R0] = O.dequantize(data["v_codes"][0, h, 49:50], data["v_codebook"][h])[0]
    moved.update(recent_k=rk, recent_v=rv, recent_len=np.array([R0 + 1], np.int32), ctx_len=np.array([49], np.int32))
    b = run_oracle(w, moved)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_with_replicated_kv_heads():
    """Query head h reads KV head h // G (contiguous groups)."""
    G = 4
    w = W.Workload("g", 2, 8, 2, 16, 8, 60, "f16", recent_cap=6, recent_fixed=6, seed=77)
    data = W.generate(w)
    a = run_oracle(w, data)
    rep = dict(data)
    for k in ("k_codes", "v_codes", "recent_k", "recent_v"):
        rep[k] = np.repeat(data[k], G, axis=1)
    for k in ("k_codebook", "v_codebook"):
        rep[k] = np.repeat(data[k], G, axis=0)
    b = run_oracle(w, rep)
    np.testing.assert_array_equal(a, b)


def test_batch_rows_are_independent_and_pairs_subset_matches():
    w, data = small(10, B=3, Hq=2, Hkv=2, d=16, M=8, N=33, R=2, lens=(33, 5, 20))
    full = run_oracle(w, data)
    part = run_oracle(w, data, pairs=[(1, 1), (2, 0), (1, 1)])      # a repeated pair is computed once
    assert (part[1, 1] == full[1, 1]).all() and (part[2, 0] == full[2, 0]).all()
    assert np.isnan(part[0, 0]).all()
    alone = {k: (v[1:2] if (v is not None and k not in ("k_codebook", "v_codebook")) else v) for k, v in data.items()}
    w1 = W.scaled(w, batch=1)
    np.testing.assert_array_equal(run_oracle(w1, alone)[0], full[1])


def test_table_sum_form_equals_dequantized_form():
    """Eq. 7's identity: q.K^_t equals the sum over subspaces of table entries
    LUT[i][code] with LUT[i] = q^i . (C_K^i)^T, here evaluated in double with einsum."""
    w, data = small(12, B=1, Hq=1, Hkv=1, d=32, M=16, N=500, R=0)
    q = data["q"][0, 0].astype(np.float64)
    kcb = data["k_codebook"][0].astype(np.float64)
    lut = np.einsum("ij,icj->ic", q.reshape(16, 2), kcb)
    codes = data["k_codes"][0, 0].astype(int)
    s_table = lut[np.arange(16)[None, :], codes].sum(1) * float(W.attention_scale(w))
    p = scipy.special.softmax(s_table)
    _, wts = O.dense_attention(q, O.dequantize(data["k_codes"][0, 0], kcb),
                               O.dequantize(data["v_codes"][0, 0], data["v_codebook"][0]), W.attention_scale(w))
    np.testing.assert_allclose(wts, p, rtol=1e-11)


# --------------------------------------------------------------------------- encode


def test_encode_matches_library_vector_quantizer():
    """scipy.cluster.vq.vq is a library nearest-centroid routine (random data: no ties)."""
    w = W.Workload("e", 2, 3, 3, 16, 4, 8, "f32", n_new=8, seed=21)
    data = W.generate(w)
    codes = O.encode(data["new_k"], data["k_codebook"])
    ds = 4
    for b in range(2):
        for h in range(3):
            for i in range(4):
                obs = data["new_k"][b, h, :, i * ds:(i + 1) * ds].astype(np.float64)
                ref, _ = scipy.cluster.vq.vq(obs, data["k_codebook"][h, i].astype(np.float64))
                np.testing.assert_array_equal(codes[b, h, :, i], ref)


def test_encode_matches_vectorised_argmin_fp16():
    """Brute force with numpy broadcasting; np.argmin returns the first (lowest) index."""
    w = W.Workload("e", 1, 2, 2, 32, 8, 20, "f16", n_new=20, seed=22)
    data = W.generate(w)
    codes = O.encode(data["new_v"], data["v_codebook"])
    x = data["new_v"].astype(np.float64).reshape(1, 2, 20, 8, 1, 4)
    cb = data["v_codebook"].astype(np.float64)[None, :, None]          # [1,H,1,M,C,ds]
    diff = x - cb
    dist = diff[..., 0] ** 2
    for j in range(1, 4):
        dist = dist + diff[..., j] ** 2
    np.testing.assert_array_equal(codes, dist.argmin(-1).astype(np.uint8))


def test_encode_exact_hit_duplicates_and_roundtrip():
    """Distance 0 wins; a duplicated centroid row resolves to the lowest index;
    encode(decode(codes)) == codes when centroids are pairwise distinct."""
    rng = np.random.default_rng(3)
    H, M, ds = 2, 4, 2
    cb = rng.standard_normal((H, M, 256, ds)).astype(np.float16)
    codes = rng.integers(0, 256, size=(1, H, 50, M), dtype=np.uint8)
    # make centroids pairwise distinct per (head, subspace) for the round trip
    for h in range(H):
        for i in range(M):
            assert len({tuple(r) for r in cb[h, i].tolist()}) == 256
    x = np.stack([O.dequantize(codes[0, h], cb[h]) for h in range(H)])[None]
    np.testing.assert_array_equal(O.encode(x, cb), codes)
    # duplicate: centroid 200 becomes a copy of centroid 17, and 3 a copy of 250
    cb2 = cb.copy()
    cb2[:, :, 200] = cb2[:, :, 17]
    cb2[:, :, 3] = cb2[:, :, 250]
    c17 = np.full((1, H, 1, M), 200, np.uint8)
    x17 = np.stack([O.dequantize(c17[0, h], cb2[h]) for h in range(H)])[None]
    assert (O.encode(x17, cb2) == 17).all()
    c250 = np.full((1, H, 1, M), 250, np.uint8)
    x250 = np.stack([O.dequantize(c250[0, h], cb2[h]) for h in range(H)])[None]
    assert (O.encode(x250, cb2) == 3).all()


def test_encode_equidistant_tie_goes_to_lowest_index():
    """Two different centroids at exactly the same distance: x = 0 between +a and -a."""
    cb = np.full((1, 1, 256, 2), 100.0)
    cb[0, 0, 9] = [0.5, -0.25]
    cb[0, 0, 4] = [-0.5, 0.25]
    cb[0, 0, 77] = [0.25, 0.5]     # same norm, third tie
    x = np.zeros((1, 1, 1, 2))
    assert O.encode(x, cb)[0, 0, 0, 0] == 4


# ------------------------------------------------------------------ 12-bit codes (4096 centroids, 16-bit indices)


def test_wide_code_routines_agree_with_the_byte_routines_on_byte_sized_codebooks():
    """The 16-bit-index build of the oracle is the same source: on a 256-centroid problem it must return
    exactly what the byte build returns (checked against brute force above)."""
    w, data = small(7, d=16, M=4, R=3, dtype="f16", lens=(29, 8))
    ref = run_oracle(w, data)
    L = O.lib()
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    k16 = np.ascontiguousarray(data["k_codes"], dtype=np.uint16)
    v16 = np.ascontiguousarray(data["v_codes"], dtype=np.uint16)
    out = np.full(ref.shape, np.nan)
    wsum = np.full(ref.shape[:2], np.nan)
    q, kcb, vcb, rk, rv = f64(data["q"]), f64(data["k_codebook"]), f64(data["v_codebook"]), f64(data["recent_k"]), f64(data["recent_v"])
    cl = np.ascontiguousarray(data["ctx_len"], dtype=np.int32)
    rl = np.ascontiguousarray(data["recent_len"], dtype=np.int32)
    p = lambda a: a.ctypes.data
    rc = L.oracle_pq_decode_u16(w.batch, w.n_q_heads, w.n_kv_heads, 16, 4, 256, p(q), p(k16), p(v16), k16.shape[2], p(cl),
                                p(kcb), p(vcb), p(rk), p(rv), rk.shape[2], p(rl), float(W.attention_scale(w)), None, 0,
                                p(out), p(wsum))
    assert rc == 0
    assert (out == ref).all()


@pytest.mark.parametrize("seed,R", [(0, 4), (1, 0)])
def test_decode_with_4096_centroids_matches_brute_force_library_softmax(seed, R):
    """Brute force (numpy gather + scipy softmax) on a tiny 12-bit problem: M = 4 subspaces of 4 dims, 4096
    centroids each, codes up to 4095 held in uint16."""
    w = W.Workload("t12", 2, 2, 2, 16, 4, 45, "f16", recent_cap=R, recent_fixed=R if R else None, seed=2000 + seed,
                   ctx_lens=(45, 13), n_centroids=4096)
    data = W.generate(w)
    assert data["k_codes"].dtype == np.uint16 and data["k_codes"].max() > 255
    out = run_oracle(w, data)
    for b in range(2):
        for h in range(2):
            np.testing.assert_allclose(out[b, h], brute_force(data, W.attention_scale(w), b, h), rtol=1e-12, atol=1e-13)


def test_encode_with_4096_centroids_matches_library_vector_quantizer():
    """scipy.cluster.vq.vq on each subspace (float64 Euclidean nearest neighbour); random data, no ties."""
    rng = np.random.default_rng(12)
    cb = rng.standard_normal((1, 2, 4096, 4)).astype(np.float16)
    x = rng.standard_normal((1, 1, 300, 8)).astype(np.float16)
    codes = O.encode(x, cb)
    assert codes.dtype == np.uint16 and codes.max() > 255
    for i in range(2):
        want, _ = scipy.cluster.vq.vq(x[0, 0, :, 4 * i:4 * i + 4].astype(np.float64), cb[0, i].astype(np.float64))
        assert (codes[0, 0, :, i] == want).all()
    # exact hits and duplicated centroids: the lowest index wins
    cb[0, 0, 4000] = cb[0, 0, 17]
    x[0, 0, 0, :4] = cb[0, 0, 4000]
    assert O.encode(x, cb)[0, 0, 0, 0] == 17


def _exact_nearest(x16, cb16):
    """Nearest centroid in EXACT arithmetic: every fp16 value is an integer multiple of 2^-24, so squared distances
    are integers (Python ints, no rounding anywhere); ties go to the lowest index.  x16 [n, ds], cb16 [C, ds]."""
    xi = [[int(v) for v in row] for row in (x16.astype(np.float64) * 2.0 ** 24)]
    ci = [[int(v) for v in row] for row in (cb16.astype(np.float64) * 2.0 ** 24)]
    out = np.empty(len(xi), dtype=np.int64)
    for t, xr in enumerate(xi):
        best, best_d = 0, None
        for c, cr in enumerate(ci):
            d = sum((a - b) * (a - b) for a, b in zip(xr, cr))
            if best_d is None or d < best_d:
                best, best_d = c, d
        out[t] = best
    return out


@pytest.mark.parametrize("ds", [2, 4])
@pytest.mark.parametrize("case", ["unit", "outliers_x20", "codebook_x150", "tokens_x300", "subnormal", "midpoints", "ties",
                                  "wide_differences"])
def test_encode_equals_exact_integer_argmin_at_any_magnitude(case, ds):
    """Eq. 4 / Section II-C ask for the nearest centroid; the oracle evaluates the squared distance in IEEE double.
    Where double rounding could matter (values far above 1: two roundings per distance; tokens a few fp16 steps off
    the midpoint of close centroid pairs; subnormals; exact ties) its codes are pinned to exact integer arithmetic."""
    rng = np.random.default_rng(zlib_seed(case) + ds)
    C, n = 256, 160
    cb = rng.standard_normal((C, ds)).astype(np.float32)
    x = rng.standard_normal((n, ds)).astype(np.float32)
    if case == "outliers_x20":                    # 2 % of centroid coordinates scaled by 20, as in the GQA workload
        cb = np.where(rng.random(cb.shape) < 0.02, cb * 20.0, cb)
    elif case == "codebook_x150":
        cb = cb * 150.0
        x = x * 100.0
    elif case == "tokens_x300":
        x[::3] *= 300.0
    elif case == "subnormal":
        cb, x = cb * 1e-6, x * 1e-6
        cb[::2] = 0.0
        x[:8] = 0.0
    cb = cb.astype(np.float16)
    x = x.astype(np.float16)
    if case == "midpoints":                       # tokens within +-2 fp16 steps of the midpoint of a close pair
        cbf = cb.astype(np.float32)
        cbf[128:] = cbf[:128] + (rng.standard_normal((128, ds)) * 0.05).astype(np.float32)
        cb = cbf.astype(np.float16)
        pair = rng.integers(0, 128, size=n)
        mid = 0.5 * (cb[pair].astype(np.float32) + cb[pair + 128].astype(np.float32))
        jit = rng.integers(-2, 3, size=mid.shape) * np.abs(np.spacing(mid.astype(np.float16))).astype(np.float32)
        x = (mid + jit).astype(np.float16)
    elif case == "ties":                          # duplicated centroids and tokens exactly between two centroids
        cb[200] = cb[17]
        cb[255] = cb[3]
        cb[40] = 0
        cb[41] = 0
        cb[41, 0] = np.float16(0.5)
        x[:4] = 0
        x[:4, 0] = np.float16(0.25)
        x[4:20] = cb[rng.integers(0, 256, size=16)]
    elif case == "wide_differences":
        # Tokens at (X, 0, ..) with X one of 512, 1024, 2048, one centroid at the origin and one at (2^-15, y, 0, ..) with y^2
        # a little below X 2^-14: the second is nearer by about 1e-4, but only if the difference X - 2^-15 (25 and
        # more significant bits) is kept exactly; every other centroid lies on the far side of the origin.
        cb = cb.astype(np.float32)
        cb[:, 0] = -np.abs(cb[:, 0]) - 0.01
        cb = cb.astype(np.float16)
        cb[10] = 0
        cb[11] = 0
        cb[11, 0] = np.float16(2.0 ** -15)
        big = float(rng.choice([512.0, 1024.0, 2048.0]))
        x[:] = 0
        x[:, 0] = np.float16(big)
        cb[11, 1] = np.float16(np.sqrt(big * 2.0 ** -14) * 0.999)
        assert float(cb[11, 1]) ** 2 < big * 2.0 ** -14 - 2.0 ** -30
    assert np.isfinite(cb.astype(np.float32)).all() and np.isfinite(x.astype(np.float32)).all()
    codes = O.encode(x.reshape(1, 1, n, ds), cb.reshape(1, 1, C, ds))[0, 0, :, 0]
    want = _exact_nearest(x, cb)
    np.testing.assert_array_equal(codes, want)
    if case == "ties":
        assert (codes != 200).all() and (codes != 255).all()
    if case == "wide_differences":
        assert (codes == 11).all()


def zlib_seed(name):
    import zlib
    return zlib.crc32(name.encode()) % 100000


# ------------------------------------------------------------------ property-based: random tiny shapes

from hypothesis import given, settings, strategies as st  # noqa: E402


@settings(max_examples=30, deadline=None)
@given(seed=st.integers(0, 10_000), B=st.integers(1, 3), Hkv=st.integers(1, 2), G=st.integers(1, 3),
       M=st.sampled_from([1, 2, 4, 8]), ds=st.sampled_from([1, 2, 4]), C=st.sampled_from([2, 7, 256, 300, 4096]),
       N=st.integers(0, 40), R=st.integers(0, 6), f16=st.booleans())
def test_decode_equals_brute_force_on_random_tiny_shapes(seed, B, Hkv, G, M, ds, C, N, R, f16):
    """Brute force (numpy gather + scipy softmax) over drawn shapes: any subspace count and width, any
    codebook size (byte and 16-bit indices), grouped heads, ragged and empty sequences, with and without window."""
    rng = np.random.default_rng(seed)
    lens = tuple(int(x) for x in rng.integers(0, N + 1, size=B))
    w = W.Workload("h", B, Hkv * G, Hkv, M * ds, M, max(N, 1), "f16" if f16 else "f32", recent_cap=R,
                   recent_uniform=R > 0, seed=seed, ctx_lens=lens, n_centroids=C)
    data = W.generate(w)
    out = run_oracle(w, data)
    for b in range(B):
        for h in range(Hkv * G):
            if lens[b] + int(data["recent_len"][b]) == 0:
                assert (out[b, h] == 0).all()
            else:
                np.testing.assert_allclose(out[b, h], brute_force(data, W.attention_scale(w), b, h, G), rtol=1e-11,
                                           atol=1e-12)


@settings(max_examples=25, deadline=None)
@given(seed=st.integers(0, 10_000), M=st.sampled_from([1, 3, 8]), ds=st.sampled_from([1, 2, 4]),
       C=st.sampled_from([1, 5, 256, 1000]), n=st.integers(0, 30), f16=st.booleans())
def test_encode_equals_vectorised_argmin_on_random_tiny_shapes(seed, M, ds, C, n, f16):
    """numpy argmin over explicitly computed squared distances (first minimum = lowest index); the drawn values
    are multiples of 1/8 in [-4, 4], so every distance is exact in double and equal distances do occur."""
    rng = np.random.default_rng(seed)
    dt = np.float16 if f16 else np.float32
    cb = (rng.integers(-32, 33, size=(2, M, C, ds)) / 8.0).astype(dt)
    x = (rng.integers(-32, 33, size=(1, 2, n, M * ds)) / 8.0).astype(dt)
    codes = O.encode(x, cb)
    xs = x.astype(np.float64).reshape(1, 2, n, M, 1, ds)
    d2 = ((xs - cb.astype(np.float64)[None, :, None]) ** 2).sum(-1)         # [1, 2, n, M, C]
    assert (codes == d2.argmin(-1)).all()
