/*
 * pq_attn — single-query decode attention over a product-quantized (PQ) KV cache,
 * and the nearest-centroid encode that appends tokens to it, for AMD MI355X (gfx950).
 *
 * Plain C ABI: every pointer argument says whether it is host or device memory,
 * every size is in elements unless it says bytes.  No call takes ownership of
 * caller memory; the context owns only its own scratch (re-packed codebooks,
 * split partials, tickets).  Calls are asynchronous on the HIP stream passed in
 * (a hipStream_t cast to void*, NULL = the default stream) and never synchronise
 * the host, except pq_attn_create / pq_attn_destroy / pq_attn_device_error.
 *
 * Notation (Section III-A, Eq. 4-6): B sequences, Hq query heads, Hkv KV heads
 * (query head h reads KV head h / (Hq/Hkv)), d = head_dim, M subspaces of width
 * ds = d / M, C = 256 centroids per subspace (8-bit codes), N_b quantized tokens
 * and R_b recent full-precision tokens of sequence b.
 *
 * Code tensors.  Logically Delta_K, Delta_V are [B][Hkv][N][M] uint8 (Eq. 4).  On the
 * device each is an opaque buffer of pq_attn_codes_bytes() bytes in a layout chosen
 * for the scan kernels (K and V use different layouts).  pq_encode_append writes
 * that layout directly; pq_pack_codes / pq_unpack_codes convert from / to the
 * logical token-major form.
 *
 * Every function returns a pq_status (0 = PQ_OK, negative = error) unless noted.
 * On an argument error nothing is launched.
 */
#ifndef PQ_ATTN_H
#define PQ_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pq_attn_ctx pq_attn_ctx;

typedef enum {
    PQ_OK = 0,
    PQ_ERR_NULL = -1,        /* a required pointer is NULL                               */
    PQ_ERR_SHAPE = -2,       /* sizes are inconsistent (Hq % Hkv, d % M, negative, ...)    */
    PQ_ERR_UNSUPPORTED = -3, /* a consistent shape this build has no kernel for          */
    PQ_ERR_CAPACITY = -4,    /* n_new / n_tokens exceeds the configured capacity         */
    PQ_ERR_HIP = -6,         /* a HIP runtime call failed                                */
    PQ_ERR_ALLOC = -7        /* device or host allocation failed                         */
} pq_status;

typedef enum { PQ_F16 = 0, PQ_F32 = 1 } pq_dtype;
typedef enum { PQ_CODES_K = 0, PQ_CODES_V = 1 } pq_code_kind;

typedef struct {
    int32_t batch;        /* B >= 1                                                         */
    int32_t n_q_heads;    /* Hq                                                             */
    int32_t n_kv_heads;   /* Hkv, Hq % Hkv == 0                                             */
    int32_t head_dim;     /* d; supported: 128                                              */
    int32_t n_subspaces;  /* M; supported: 64 (ds = 2, 4 bits/dim) and 32 (ds = 4, 2 bits/dim) */
    int32_t n_centroids;  /* C; supported: 256 (nbits = 8), and 4096 (nbits = 12) with M = 32, fp16 */
    int32_t max_context;  /* token capacity of the code tensors per (sequence, KV head),    */
                          /* 1 .. 2^24                                                      */
    int32_t max_recent;   /* row capacity of the recent window tensors (0: no window), <= 2^24 */
    int32_t dtype;        /* pq_dtype of q, codebooks, recent K/V and new K/V               */
    int32_t device;       /* HIP device ordinal                                             */
    int32_t n_splits;     /* context splits per (sequence, query head); 0 = choose.         */
                          /* 4096-centroid contexts only: -k asks for the two-pass decode   */
                          /* (split by subspace group) with k token ranges; "0 = choose"    */
                          /* takes it by itself when (sequence, head) pairs are few         */
    int32_t reserved;     /* must be 0                                                      */
} pq_attn_config;

/* Checks the configuration on the host (no GPU needed): PQ_OK or the error
 * pq_attn_create would return for it. */
int pq_attn_validate_config(const pq_attn_config *cfg /* host */);

/* Bytes of ONE device code tensor (K or V) for this configuration: the token
 * capacity is rounded up to whole 64-token blocks.  Returns a negative pq_status
 * for an invalid configuration.  Host-only. */
int64_t pq_attn_codes_bytes(const pq_attn_config *cfg /* host */);

/* Creates a context on cfg->device: allocates the context-owned scratch and
 * synchronises.  *out is set only on PQ_OK.  The caller frees it with
 * pq_attn_destroy (which synchronises the device first). */
int pq_attn_create(const pq_attn_config *cfg /* host */, pq_attn_ctx **out /* host */);
int pq_attn_destroy(pq_attn_ctx *ctx);

/* Number of context splits the decode kernel uses (after "0 = choose"). */
int pq_attn_n_splits(const pq_attn_ctx *ctx);

/* Kernels one pq_attn_decode call launches: 1 (fused), or 2 for a 4096-centroid
 * context that decodes in two passes (partial scores per subspace group, then
 * softmax and values). */
int pq_attn_n_passes(const pq_attn_ctx *ctx);

/* Query heads one decode workgroup serves: 1 for the kernels that build per-query
 * tables, 2..4 for the grouped-query kernels (one pass over a KV head's codes for
 * that many query heads: a KV head's Hq / Hkv >= 2 query heads are cut into
 * ceil(Hq / Hkv / 4) sub-groups of 2..4 heads, sizes as equal as possible, and the
 * largest is returned; chosen when the context is fp16 — for 4096-centroid contexts only where the shape is large
 * enough to pay for it: fewer than 5 compute units per (sequence, query head), or
 * a capacity of 1.5 M (query head, token) pairs, and n_splits >= 0). */
int pq_attn_heads_per_workgroup(const pq_attn_ctx *ctx);

/* Registers the codebooks trained offline (Section III-A, "Offline PQ Codebook
 * Training"): C_K, C_V as [Hkv][M][C][ds] in the context dtype, device memory.
 * The kernels launched by this call copy them into context-owned memory (a plain
 * copy for the encode kernels, a centroid-major image for the decode kernels); the
 * caller's tensors are read by those kernels only and may be freed, overwritten
 * or reused once they have run (i.e. after later work on the same stream, or a
 * stream synchronisation).  The library keeps no pointer to them.
 *
 * pq_attn_decode and pq_encode_append take codebook pointers too: non-NULL
 * pointers are registered by that call, on its stream, before its kernels (the
 * copy costs a few microseconds per call — register once and pass NULL in a
 * decoding loop).  A codebook changed in place has to be registered again.
 * Registration must be stream-ordered with every other call on the context that
 * uses the codebooks: with two streams (asynchronous quantization), register
 * first, synchronise, then pass NULL on both. */
int pq_attn_set_codebooks(pq_attn_ctx *ctx, const void *k_codebook /* device */,
                          const void *v_codebook /* device */, void *hip_stream);

/* Decode attention for one new token per sequence over the quantized cache plus
 * the recent window (Eq. 6, evaluated as Eq. 7: per-head tables q^i.(C_K^i)^T are
 * sampled by the K codes, one softmax shared with the full-precision rows, values
 * aggregated through C_V by the V codes; Section III-B "Efficient Attention
 * Implementation" and steps 1-4 of Section III-C).
 *
 *   q           device [B][Hq][d]                 dtype
 *   k_codes     device, pq_attn_codes_bytes()     device layout (PQ_CODES_K)
 *   v_codes     device, pq_attn_codes_bytes()     device layout (PQ_CODES_V)
 *   ctx_len     device [B] int32                  N_b, clamped to [0, max_context]
 *   k_codebook  device [Hkv][M][C][ds] dtype      or NULL = the registered ones
 *   v_codebook  likewise
 *   recent_k/v  device [B][Hkv][max_recent][d]    dtype; both NULL = no window
 *   recent_len  device [B] int32                  R_b, clamped to [0, max_recent]; NULL = all 0
 *   scale       1/sqrt(d) of Eq. 1; must be finite (PQ_ERR_SHAPE otherwise)
 *   out         device [B][Hq][d] float32
 *
 * Rows >= R_b of the recent tensors and tokens >= N_b of the code tensors are never
 * used in the result.  A sequence with N_b + R_b == 0 gets a row of zeros.
 * Codebooks, q and the recent rows must be finite.  Calls on one context must be
 * stream-ordered with each other (they share the context's scratch). */
int pq_attn_decode(pq_attn_ctx *ctx, const void *q, const uint8_t *k_codes, const uint8_t *v_codes,
                   const int32_t *ctx_len, const void *k_codebook, const void *v_codebook, const void *recent_k,
                   const void *recent_v, const int32_t *recent_len, float scale, float *out, void *hip_stream);

/* pq_attn_decode for callers that cannot allocate device memory — code recorded into a HIP graph, tight
 * serving loops, harnesses that forbid hipMalloc — and therefore cannot hold a context: the same kernels, the
 * same result, with every piece of scratch (codebook images, split partials, tickets) in one array that is
 * part of the library's device code (4.5 MiB per GPU the library runs on, held until the process ends).  The call allocates and
 * frees nothing and does not synchronise.
 *
 *   cfg         host; as for pq_attn_create (cfg->device names the GPU).  The code tensors use the layout
 *               of a context created from the same configuration (pq_pack_codes / pq_encode_append of such a
 *               context produce them).
 *   k_codebook, v_codebook   device [Hkv][M][256][ds] dtype, required: re-packed into the scratch by every call
 *   all other arguments as in pq_attn_decode
 *
 * Limits (PQ_ERR_CAPACITY beyond them): 8-bit codes only (4096 centroids: PQ_ERR_UNSUPPORTED); one codebook
 * tensor at most 2 MiB (32 KV heads in fp16, 16 in fp32); batch * n_q_heads <= 1024; with an explicit
 * n_splits, batch * n_q_heads * n_splits <= 1024 ("0 = choose" never exceeds it).
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * threads, or with a call still in flight) race; stream-order them.  The first call on a device looks the array's
 * address up (no allocation, but a runtime query): make that call before any stream capture starts. */
int pq_attn_decode_noalloc(const pq_attn_config *cfg /* host */, const void *q, const uint8_t *k_codes,
                           const uint8_t *v_codes, const int32_t *ctx_len, const void *k_codebook,
                           const void *v_codebook, const void *recent_k, const void *recent_v,
                           const int32_t *recent_len, float scale, float *out, void *hip_stream);

/* Quantizes n_new full-precision tokens per (sequence, KV head) and appends their
 * codes (Eq. 4 with Section II-C's nearest-centroid assignment; step 5 of Section
 * III-C): for every sub-vector the index of the centroid at the smallest squared
 * Euclidean distance; equal distances go to the lowest index.  The distance is decided
 * in IEEE double as dist = fma(x_j - c_j, x_j - c_j, dist), j = 0 .. ds-1 in order.
 *
 *   new_k/new_v device [B][Hkv][n_new][d] dtype (finite values)
 *   k_codebook / v_codebook as in pq_attn_decode
 *   k_codes / v_codes       written at token positions ctx_len[b] .. ctx_len[b]+n_new-1
 *   ctx_len     device [B] int32, incremented by n_new on the stream
 *
 * The call may run on another stream concurrently with pq_attn_decode on the same context if the
 * two are given different length arrays and the decode does not attend over the positions being
 * written (asynchronous quantization, Section III-B); the caller publishes the new lengths afterwards.
 *
 * With 12-bit codes the call stages the codes in context-owned memory sized at pq_attn_create (except for
 * 8 or fewer new tokens per KV head over all sequences, which go straight into the code tensors); a long
 * append runs as several chunks through it (more launches, no allocation, no synchronisation).  Two appends
 * on one context must not overlap.
 *
 * 0 < n_new <= max_context, else PQ_ERR_CAPACITY.  Tokens that would land beyond
 * max_context for some sequence are dropped, that sequence's length saturates, and
 * bit 0 of the device error word is set (see pq_attn_device_error). */
int pq_encode_append(pq_attn_ctx *ctx, const void *new_k, const void *new_v, int32_t n_new, const void *k_codebook,
                     const void *v_codebook, uint8_t *k_codes, uint8_t *v_codes, int32_t *ctx_len, void *hip_stream);

/* Layout conversion of code tensors (device to device, asynchronous).
 *   token_major device [B][Hkv][n_tokens][M] uint8 (uint16 for 12-bit codes), n_tokens <= max_context
 *   packed      device, pq_attn_codes_bytes()
 * pack writes tokens 0..n_tokens-1 of every head; unpack reads them. */
int pq_pack_codes(pq_attn_ctx *ctx, int32_t kind /* pq_code_kind */, const void *token_major, int32_t n_tokens,
                  uint8_t *packed, void *hip_stream);
int pq_unpack_codes(pq_attn_ctx *ctx, int32_t kind, const uint8_t *packed, int32_t n_tokens, void *token_major,
                    void *hip_stream);

/* Offline codebook training (Section II-C, training phase; Section III-A, "Offline PQ Codebook Training"):
 * k-means per (KV head, subspace) on sampled key or value vectors, n_iters iterations of Lloyd's algorithm
 * from the caller's initial centroids.  Assignment: nearest centroid by the rule and arithmetic of
 * pq_encode_append (IEEE double, ties to the lowest index).  Update: a centroid with members becomes their
 * mean — exact member sum, divided in double, rounded to float and then to fp16 — and one without keeps its
 * value.  The result does not depend on the order in which samples are processed.
 *
 *   samples    device [Hkv][n_samples][d] fp16 (finite), 1 <= n_samples <= 2^20 (else PQ_ERR_CAPACITY)
 *   codebook   device [Hkv][M][C][ds] fp16: initial centroids in, trained centroids out (in place)
 *   workspace  device, 8-byte aligned, at least pq_kmeans_workspace_bytes(ctx) bytes (else PQ_ERR_CAPACITY);
 *              contents need not be initialised and are garbage afterwards
 *
 * fp16 contexts only (PQ_ERR_UNSUPPORTED otherwise); with 12-bit codes the codebook is [Hkv][32][4096][4].  Asynchronous on the stream.  Training a codebook that
 * is registered with the context in place requires pq_attn_set_codebooks afterwards. */
int64_t pq_kmeans_workspace_bytes(const pq_attn_ctx *ctx);
int pq_kmeans_fit(pq_attn_ctx *ctx, const void *samples /* device */, int32_t n_samples, void *codebook /* device */,
                  int32_t n_iters, void *workspace /* device */, int64_t workspace_bytes, void *hip_stream);

/* Measurement aid, not part of the method: one kernel that only reads `bytes` bytes (a multiple of
 * 16, 16-byte aligned, device memory) with the load instruction the decode kernels use for codes.
 * The benchmark times it to report what HBM delivers to a pure read on the box it runs on, beside
 * the nominal peak.  Asynchronous on the stream. */
int pq_stream_read_probe(pq_attn_ctx *ctx, const void *src /* device */, int64_t bytes, void *hip_stream);

/* Synchronises the device, returns the sticky device error word in *flags and
 * clears it.  Bit 0: an append overflowed max_context. */
int pq_attn_device_error(pq_attn_ctx *ctx, uint32_t *flags /* host */);

/* Static, never NULL. */
const char *pq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PQ_ATTN_H */
