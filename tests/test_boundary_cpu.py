"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad configurations before touching HIP."""
import ctypes
import os
import re

import pytest

import paper_2504_03661_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pq_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = declared_functions()
    assert {"pq_attn_create", "pq_attn_decode", "pq_encode_append"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n


def test_binding_has_the_same_names():
    for n in declared_functions():
        assert hasattr(P, n), n


def good(**kw):
    c = P.PQAttnConfig(batch=1, n_q_heads=32, n_kv_heads=32, max_context=32768, max_recent=128)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("changes,status", [
    ({}, 0),
    ({"n_subspaces": 32}, 0),
    ({"n_q_heads": 32, "n_kv_heads": 8}, 0),
    ({"dtype": P.PQ_F32}, 0),
    ({"batch": 0}, -2),
    ({"n_q_heads": 30, "n_kv_heads": 8}, -2),          # Hq % Hkv
    ({"head_dim": 128, "n_subspaces": 48}, -2),        # d % M
    ({"max_context": 0}, -2),
    ({"max_recent": -1}, -2),
    ({"dtype": 7}, -2),
    ({"reserved": 1}, -2),
    ({"n_centroids": 4096, "n_subspaces": 32}, 0),     # the 12-bit setting
    ({"n_centroids": 4096}, -3),                       # 12-bit codes need M = 32 ...
    ({"n_centroids": 4096, "n_subspaces": 32, "dtype": P.PQ_F32}, -3),   # ... and fp16
    ({"n_centroids": 1024, "n_subspaces": 32}, -3),
    ({"n_subspaces": 16}, -3),
    ({"head_dim": 64, "n_subspaces": 32}, -3),
    ({"n_splits": 1000}, -3),
    ({"n_splits": -1}, -2),                            # a negative split count is the 12-bit contexts' alone:
    ({"n_centroids": 4096, "n_subspaces": 32, "n_splits": -3}, 0),      # two-pass decode with 3 token ranges
    ({"n_centroids": 4096, "n_subspaces": 32, "n_splits": -65}, -3),
])
def test_validate_config(changes, status):
    assert P.pq_attn_validate_config(good(**changes)) == status


def test_codes_bytes_rounds_capacity_to_64_token_blocks():
    assert P.pq_attn_codes_bytes(good()) == 32 * 32768 * 64
    assert P.pq_attn_codes_bytes(good(max_context=1000)) == 32 * 1024 * 64
    assert P.pq_attn_codes_bytes(good(max_context=65, n_subspaces=32, batch=3)) == 3 * 32 * 128 * 32
    # 12-bit codes: 48 bytes per token, capacity in 128-token blocks
    assert P.pq_attn_codes_bytes(good(max_context=130, n_subspaces=32, n_centroids=4096, batch=2)) == 2 * 32 * 256 * 48
    with pytest.raises(P.PQAttnError):
        P.pq_attn_codes_bytes(good(batch=-1))


def test_null_arguments_are_rejected_without_a_gpu():
    lib = P.load_library()
    assert lib.pq_attn_create(None, None) == -1
    assert lib.pq_attn_destroy(None) == -1
    assert lib.pq_attn_decode(None, None, None, None, None, None, None, None, None, None, 1.0, None, None) == -1
    assert lib.pq_encode_append(None, None, None, 1, None, None, None, None, None, None) == -1
    assert lib.pq_attn_decode_noalloc(None, None, None, None, None, None, None, None, None, None, 1.0, None, None) == -1
    assert lib.pq_attn_validate_config(None) == -1
    assert lib.pq_pack_codes(None, 0, None, 1, None, None) == -1
    assert lib.pq_unpack_codes(None, 0, None, 1, None, None) == -1
    assert lib.pq_attn_set_codebooks(None, None, None, None) == -1
    assert lib.pq_kmeans_workspace_bytes(None) == -1
    assert lib.pq_kmeans_fit(None, None, 1, None, 1, None, 0, None) == -1
    assert lib.pq_stream_read_probe(None, None, 16, None) == -1
    assert lib.pq_attn_device_error(None, None) == -1
    assert lib.pq_attn_n_splits(None) == -1
    assert lib.pq_attn_n_passes(None) == -1
    assert lib.pq_attn_heads_per_workgroup(None) == -1
    out = ctypes.c_void_p()
    # bad config is reported before any HIP call
    assert lib.pq_attn_create(ctypes.byref(good(batch=0).c_struct()), ctypes.byref(out)) == -2
    assert out.value is None


def test_noalloc_entry_point_checks_its_limits_on_the_host():
    """pq_attn_decode_noalloc validates the configuration and the limits of its static scratch before any HIP call
    (the pointers only have to be non-NULL for that)."""
    lib = P.load_library()
    buf = ctypes.create_string_buffer(64)
    p = ctypes.cast(buf, ctypes.c_void_p)

    def call(cfg):
        return lib.pq_attn_decode_noalloc(ctypes.byref(cfg.c_struct()), p, p, p, p, p, p, None, None, None, 1.0, p, None)

    assert call(good(batch=0)) == -2
    assert call(good(n_q_heads=64, n_kv_heads=64)) == -4                      # 4 MiB of fp16 codebooks
    assert call(good(dtype=P.PQ_F32)) == -4                                   # 32 heads in fp32: 4 MiB
    assert call(good(batch=64)) == -4                                         # 2048 (sequence, head) rows
    assert call(good(batch=16, n_splits=4)) == -4                             # 2048 partial rows
    assert call(good(n_subspaces=32, n_centroids=4096)) == -3                 # 12-bit codes
    assert lib.pq_attn_decode_noalloc(ctypes.byref(good().c_struct()), p, p, p, p, p, p, p, None, None, 1.0, p, None) == -1
    assert lib.pq_attn_decode_noalloc(ctypes.byref(good().c_struct()), p, p, p, p, p, p, None, None, None,
                                      float("nan"), p, None) == -2


def test_status_strings():
    assert P.pq_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -6, -7, -99):
        assert P.pq_status_string(s)
