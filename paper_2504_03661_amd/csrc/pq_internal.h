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
    const int rot = skew == PQ_K_SKEW_QUAD ? (l >> 2) * (M >> 4) : l;  // by quad: 4 (M = 64) or 2 (M = 32) subspaces per score step
    const int s = (i - rot) & (M - 1);  // M is a power of two
    return (t >> 6) * (64 * (int64_t)M) + (int64_t)(s >> 4) * 1024 + l * 16 + (s & 15);
}

__host__ __device__ inline int64_t pq_v_code_offset(int64_t t, int i, int M)
{
    return (t >> 4) * (16 * (int64_t)M) + (int64_t)i * 16 + (t & 15);
}

// ---------------------------------------------------------------------------------
// 12-bit codes (M = 32 subspaces of 4 dims, 4096 centroids): 48 bytes per token and tensor.
// Every unit below is 12 bytes = eight 12-bit codes, code s of a unit in bits 12 s .. 12 s + 11
// (little-endian), and a wavefront loads 64 consecutive units (768 bytes) with one 12-byte load
// per lane.  The decode kernel walks the subspaces in groups (its tables for all 32 do not fit
// in LDS), so both layouts are group-major inside a block of tokens.
//
// K codes: blocks of 64 tokens x 4 groups of 8 subspaces; unit (block, group, lane = token % 64)
// holds that token's codes of subspaces 8 g .. 8 g + 7 in order.
//
// V codes: blocks of 128 tokens x 8 groups of 4 subspaces; unit (block, group, lane) with
// lane = 4 * (token % 16) + (subspace % 4) holds the codes of that subspace for the 8 tokens
// token % 16 + 16 k of the block, k = 0 .. 7 (the value pass gives a lane one subspace and every
// 16th token).
// The token capacity of a tensor is rounded up to 128 tokens.
// ---------------------------------------------------------------------------------
#define PQ12_M 32
#define PQ12_CENTROIDS 4096
#define PQ12_TOKEN_BYTES 48

// byte offset of the 12-byte unit and index (0..7) of the code inside it
__host__ __device__ inline int64_t pq12_k_unit(int64_t t, int i, int *slot)
{
    *slot = i & 7;
    return (((t >> 6) * 4 + (i >> 3)) * 64 + (t & 63)) * 12;
}

__host__ __device__ inline int64_t pq12_v_unit(int64_t t, int i, int *slot)
{
    const int r = (int)(t & 127);
    *slot = r >> 4;
    return (((t >> 7) * 8 + (i >> 2)) * 64 + (r & 15) * 4 + (i & 3)) * 12;
}

// Floats per split partial: [0] running maximum (log2 domain), [1] sum of weights,
// [2..3] unused, [4..4+d) unnormalised output.
#define PQ_PART_STRIDE 132
#define PQ_MAX_SPLITS 64
#define PQ_MAX_TOKENS (1 << 24)  // capacity limit that keeps the kernels' index arithmetic in 32 bits
#define PQ_HEAD_DIM 128
#define PQ_ERRFLAG_APPEND_OVERFLOW 1u
// limits of pq_attn_decode_noalloc's static scratch: bytes of one centroid-major codebook image set (K or V, all KV
// heads) and (sequence, query head, split) rows of partials / (sequence, query head) tickets
#define PQ_NOALLOC_CODEBOOK_BYTES (2 << 20)
#define PQ_NOALLOC_MAX_ROWS 1024

struct pq_attn_ctx {
    pq_attn_config cfg;
    int ds;               // sub-vector width
    int group;            // Hq / Hkv
    int n_splits;
    int k_skew;           // PQ_K_SKEW_*: which decode kernel this context runs, hence its K code layout
    int64_t cap_padded;   // max_context rounded up to 64 tokens
    size_t elem_bytes;    // 2 or 4
    void *kcb_packed;     // [Hkv][256][M][ds] dtype   (centroid-major); 12-bit contexts: the natural layout
    void *vcb_packed;     // [Hkv][256][M][ds] dtype
    void *kcb_natural;    // the context's own copy of the registered codebooks in the caller's layout
    void *vcb_natural;    // [Hkv][M][C][ds] (what the encode kernels read); 12-bit contexts: = *_packed
    bool registered;      // codebooks have been registered (the copies above hold them)
    float *partials;      // [B*Hq][n_splits][PQ_PART_STRIDE]
    unsigned int *tickets;  // [B*Hq], zero between calls
    unsigned int *dev_err;  // sticky error word
    // 12-bit contexts: token-major uint16 staging of an append's codes, sized once at creation; a longer
    // append runs as several chunks of at most stage_tokens tokens per (sequence, KV head)
    uint16_t *stage[2];
    int32_t stage_tokens;
    // 12-bit contexts that decode in two passes: partial scores [B*Hq][4][cap_padded]; n_splits then counts the
    // token ranges of the second pass
    float *scores12;
    bool grouped12;       // 12-bit context that runs the grouped-query kernel
    int n_cu;             // compute units of the device
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
    int Gs;                // grouped-query kernels: the largest number of query heads a workgroup takes (2..4)
    int n_sub;             // ... and the sub-groups a KV head's G query heads are cut into: ceil(G / 4) groups whose
                           // sizes differ by at most one (7 = 4 + 3, 5 = 3 + 2, 10 = 4 + 3 + 3)
    int max_context, max_recent;
    int n_cu;              // compute units of the device (the live split count of a batch's sequences follows it)
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
// true when the grouped-query kernel serves this configuration (fp16, M = 64 or 32, 8-bit codes, Hq / Hkv >= 2).  A KV
// head's g query heads are cut into pq_grouped_sub_groups(g) = ceil(g / 4) sub-groups of 2..4 heads whose sizes differ by
// at most one, one workgroup each; pq_grouped_heads_per_workgroup(g) is the largest of them (0 for g < 2)
bool pq_config_uses_grouped_kernel(const pq_attn_config *cfg);
int pq_grouped_sub_groups(int g);
int pq_grouped_heads_per_workgroup(int g);
hipError_t pq_launch_encode(const pq_attn_ctx *ctx, const pq_encode_args &a, int32_t *ctx_len, unsigned int *dev_err,
                            hipStream_t s);
// lengths += n_new, saturating at max_context (sets the overflow flag)
hipError_t pq_launch_bump_len(int32_t *ctx_len, int B, int n_new, int max_context, unsigned int *dev_err, hipStream_t s);
// src [Hkv][M][256][ds] (caller memory) -> packed [Hkv][256][M][ds] and a plain copy in the source layout
hipError_t pq_launch_pack_codebook(const pq_attn_ctx *ctx, const void *src, void *packed, void *natural, hipStream_t s);
hipError_t pq_launch_pack_codes(const pq_attn_ctx *ctx, int kind, const uint8_t *token_major, int n_tokens,
                                uint8_t *packed, bool unpack, hipStream_t s);
hipError_t pq_launch_stream_read(const void *src, int64_t bytes, uint32_t *sink, hipStream_t s);
// offline codebook training (fp16 contexts): accumulator bytes the caller's workspace must hold, and n_iters Lloyd
// iterations over samples [Hkv][n_samples][d], codebook [Hkv][M][256][ds] updated in place
int64_t pq_kmeans_accumulator_bytes(const pq_attn_ctx *ctx);
hipError_t pq_launch_kmeans(const pq_attn_ctx *ctx, const void *samples, int n_samples, void *codebook, int n_iters,
                            void *workspace, hipStream_t s);

// 12-bit contexts (n_centroids = 4096): decode, encode into the token-major staging buffers followed by the
// packing of the staged codes behind the current lengths, and the layout conversions of whole tensors
bool pq_config_is_12bit(const pq_attn_config *cfg);
hipError_t pq12_launch_decode(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s);
// 12-bit contexts with 2, 3 or 4 query heads per workgroup reading one KV head (pq12_decode_grouped.hip)
bool pq12_config_uses_grouped_kernel(const pq_attn_config *cfg, int n_cu);
hipError_t pq12_launch_decode_grouped(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s);
// a.x holds rows [B][Hkv][x_rows][d]; rows 0 .. a.n_new - 1 of every head are encoded and appended
// (a.n_new <= ctx->stage_tokens)
hipError_t pq12_launch_encode_append(const pq_attn_ctx *ctx, const pq_encode_args &a, int64_t x_rows, int32_t *ctx_len,
                                     unsigned int *dev_err, hipStream_t s);
// plain device-to-device copy of `bytes` bytes (a multiple of 16, 16-byte aligned) by a kernel
hipError_t pq_launch_copy16(const void *src, void *dst, int64_t bytes, hipStream_t s);
hipError_t pq12_launch_pack_codes(const pq_attn_ctx *ctx, int kind, const uint16_t *token_major, int n_tokens,
                                  uint8_t *packed, bool unpack, hipStream_t s);
// pieces of the training shared by the 8-bit and the 12-bit path
hipError_t pq_launch_clear_words(void *p, int64_t words, hipStream_t s);
hipError_t pq_launch_kmeans_update(void *codebook, unsigned long long *sums, unsigned int *counts, int64_t n, int ds,
                                   hipStream_t s);
int64_t pq12_kmeans_workspace_bytes(const pq_attn_ctx *ctx);
hipError_t pq12_launch_kmeans(const pq_attn_ctx *ctx, const void *samples, int n_samples, void *codebook, int n_iters,
                              void *workspace, hipStream_t s);
