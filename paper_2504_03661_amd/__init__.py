"""MI355X-native PQ decode attention (MILLION's hot path): thin binding over libpq_attn.so."""
from .binding import (  # noqa: F401
    PQ_CODES_K, PQ_CODES_V, PQ_F16, PQ_F32, PQAttnConfig, PQAttnError, library_path, load_library,
    pq_attn_codes_bytes, pq_attn_create, pq_attn_decode, pq_attn_decode_noalloc, pq_attn_destroy, pq_attn_device_error, pq_attn_heads_per_workgroup, pq_attn_n_passes, pq_attn_n_splits,
    pq_attn_set_codebooks, pq_attn_validate_config, pq_encode_append, pq_kmeans_fit, pq_kmeans_workspace_bytes, pq_pack_codes, pq_status_string,
    pq_stream_read_probe, pq_unpack_codes,
)
