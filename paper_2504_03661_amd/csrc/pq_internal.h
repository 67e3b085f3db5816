// Internal declarations shared by the translation units of libpq_attn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pq_attn.h"

// ---------------------------------------------------------------------------------
// Device layouts of the code tensors.  Both are functions of (token t, subspace i)
// only, so an append is a set of byte stores and needs no read-modify-write.
//
// K codes ("lane-skewed 64-token blocks"): the score pass gives every lane of a
// wavefront one token and walks the subspaces in a per-lane rotated order, so that
// in any one LDS gather the 64 lanes touch 64 different table columns (= banks)
// whatever the code values are.  A block holds 64 tokens, M bytes each, as M/16
// chunks of 1 KiB; chunk k holds, for lane l = t % 64, the 16 bytes that lane
// consumes at steps s = 16k .. 16k+15, and the byte at step s is the code of
// subspace (s + rot) % M.  One wavefront load of a chunk is 1 KiB contiguous.
// rot = l for the per-head table kernel (every lane on its own column); rot = l rounded down to
// a multiple of 4 for the grouped-query kernel, whose 4x4x4 matrix instruction makes the four
// tokens of a lane quad walk the same dimensions together (PQ_K_SKEW_LANE / PQ_K_SKEW_QUAD).
//
// V codes ("16-token tiles, subspace-major"): the value pass gives every lane one
// subspace (lane = output dims) and walks tokens; a tile is 16 tokens x M
// subspaces with the 16 tokens of one subspace contiguous, so a lane's 16-byte
// load is its subspace's next 16 tokens and a wavefront load is 1 KiB contiguous.
// ---------------------------------------------------------------------------------
#define PQ_K_SKEW_LANE 0
#define PQ_K_SKEW_QUAD 1

__host__ __device__ inline int64_t pq_k_code_offset(int64_t t, int i, int M, int skew)
{
    const int l = (int)(t & 63);
    const int rot = skew == PQ_K_SKEW_QUAD ? (l & ~3) : l;
    const int s = (i - rot) & (M - 1);  // M is a power of two
    return (t >> 6) * (64 * (int64_t)M) + (int64_t)(s >> 4) * 1024 + l * 16 + (s & 15);
}

__host__ __device__ inline int64_t pq_v_code_offset(int64_t t, int i, int M)
{
    return (t >> 4) * (16 * (int64_t)M) + (int64_t)i * 16 + (t & 15);
}

// Floats per split partial: [0] running maximum (log2 domain), [1] sum of weights,
// [2..3] unused, [4..4+d) unnormalised output.
#define PQ_PART_STRIDE 132
#define PQ_MAX_SPLITS 64
#define PQ_MAX_TOKENS (1 << 24)  // capacity limit that keeps the kernels' index arithmetic in 32 bits
#define PQ_HEAD_DIM 128
#define PQ_ERRFLAG_APPEND_OVERFLOW 1u

struct pq_attn_ctx {
    pq_attn_config cfg;
    int ds;               // sub-vector width
    int group;            // Hq / Hkv
    int n_splits;
    int k_skew;           // PQ_K_SKEW_*: which decode kernel this context runs, hence its K code layout
    int64_t cap_padded;   // max_context rounded up to 64 tokens
    size_t elem_bytes;    // 2 or 4
    void *kcb_packed;     // [Hkv][256][M][ds] dtype   (centroid-major)
    void *vcb_packed;     // [Hkv][256][M][ds] dtype
    const void *reg_k;    // caller pointers the packed copies were made from
    const void *reg_v;
    float *partials;      // [B*Hq][n_splits][PQ_PART_STRIDE]
    unsigned int *tickets;  // [B*Hq], zero between calls
    unsigned int *dev_err;  // sticky error word
};

struct pq_decode_args {
    const void *q;
    const uint8_t *k_codes, *v_codes;
    const int32_t *ctx_len;
    const void *kcb_packed, *vcb_packed;
    const void *recent_k, *recent_v;
    const int32_t *recent_len;
    float *out;
    float *partials;
    unsigned int *tickets;
    float scale_log2e;
    int B, Hq, Hkv, G, S;  // G = Hq / Hkv
    int max_context, max_recent;
    int64_t head_stride;  // bytes of one (sequence, KV head) in a code tensor
};

struct pq_encode_args {
    const void *x[2];        // new_k, new_v   [B][Hkv][n_new][d]
    const void *codebook[2];  // natural layout [Hkv][M][256][ds]
    uint8_t *codes[2];
    const int32_t *ctx_len;
    int B, Hkv, n_new, max_context;
    int k_skew;
    int64_t head_stride;
};

// launchers (each returns hipGetLastError() after its launches)
hipError_t pq_launch_decode(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s);
hipError_t pq_launch_decode_grouped(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s);
// true when the grouped-query kernel serves this configuration (fp16, M = 64, 2..4 query heads per KV head)
bool pq_config_uses_grouped_kernel(const pq_attn_config *cfg);
hipError_t pq_launch_encode(const pq_attn_ctx *ctx, const pq_encode_args &a, int32_t *ctx_len, unsigned int *dev_err,
                            hipStream_t s);
hipError_t pq_launch_pack_codebook(const pq_attn_ctx *ctx, const void *src, void *dst, hipStream_t s);
hipError_t pq_launch_pack_codes(const pq_attn_ctx *ctx, int kind, const uint8_t *token_major, int n_tokens,
                                uint8_t *packed, bool unpack, hipStream_t s);
hipError_t pq_launch_stream_read(const void *src, int64_t bytes, uint32_t *sink, hipStream_t s);
// offline codebook training (fp16 contexts): accumulator bytes the caller's workspace must hold, and n_iters Lloyd
// iterations over samples [Hkv][n_samples][d], codebook [Hkv][M][256][ds] updated in place
int64_t pq_kmeans_accumulator_bytes(const pq_attn_ctx *ctx);
hipError_t pq_launch_kmeans(const pq_attn_ctx *ctx, const void *samples, int n_samples, void *codebook, int n_iters,
                            void *workspace, hipStream_t s);
