// Layout conversions: codebooks to the centroid-major image the decode kernel
// streams into LDS, and code tensors between the logical token-major form
// [B][Hkv][n][M] (Delta_K, Delta_V of Eq. 4) and the device layouts.
#include <hip/hip_runtime.h>

#include "pq_device_utils.h"
#include "pq_internal.h"

namespace {

// [Hkv][M][256][ds] -> [Hkv][256][M][ds]; one thread per (head, centroid, subspace)
// (also writes `nat`, unless NULL: a plain copy of src, the context's own codebooks for the encode kernels)
template <typename E>
__global__ void pq_pack_codebook_kernel(const E *src, E *dst, E *nat, int Hkv, int M, int ds)
{
    const int64_t n = (int64_t)Hkv * 256 * M;
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= n)
        return;
    const int i = (int)(x % M);
    const int c = (int)((x / M) % 256);
    const int h = (int)(x / ((int64_t)M * 256));
    const int64_t so = (((int64_t)h * M + i) * 256 + c) * ds;
    E *d = dst + x * ds;
    for (int j = 0; j < ds; ++j) {
        const E v = src[so + j];
        d[j] = v;
        if (nat != nullptr)
            nat[so + j] = v;
    }
}

__global__ void pq_copy16_kernel(const u32x4 *src, u32x4 *dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = src[i];
}

// one thread per code byte of the token-major tensor
__global__ void pq_pack_codes_kernel(const uint8_t *token_major, uint8_t *packed, int64_t n_heads, int n_tokens,
                                     int M, int64_t head_stride, int kind, int unpack, int k_skew)
{
    const int64_t total = n_heads * n_tokens * M;
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= total)
        return;
    const int i = (int)(x % M);
    const int64_t t = (x / M) % n_tokens;
    const int64_t h = x / ((int64_t)M * n_tokens);
    const int64_t off = h * head_stride + (kind == PQ_CODES_K ? pq_k_code_offset(t, i, M, k_skew) : pq_v_code_offset(t, i, M));
    if (unpack)
        const_cast<uint8_t *>(token_major)[x] = packed[off];
    else
        packed[off] = token_major[x];
}

// Reads n 16-byte vectors with the code-stream load and folds them into one word per lane; the
// store (into a scratch word nobody reads) happens for one value in 2^32 and keeps the loads alive.
__global__ __launch_bounds__(1024) void pq_stream_read_kernel(const u32x4 *p, int64_t n, uint32_t *sink)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i < n; i += stride) {
        const uint4 v = load_codes<true>(p + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u)
        *sink = acc;
}

}  // namespace

hipError_t pq_launch_pack_codebook(const pq_attn_ctx *ctx, const void *src, void *dst, void *natural, hipStream_t s)
{
    const int Hkv = ctx->cfg.n_kv_heads, M = ctx->cfg.n_subspaces, ds = ctx->ds;
    const int64_t n = (int64_t)Hkv * 256 * M;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (ctx->cfg.dtype == PQ_F16)
        hipLaunchKernelGGL(pq_pack_codebook_kernel<uint16_t>, grid, block, 0, s, (const uint16_t *)src,
                           (uint16_t *)dst, (uint16_t *)natural, Hkv, M, ds);
    else
        hipLaunchKernelGGL(pq_pack_codebook_kernel<uint32_t>, grid, block, 0, s, (const uint32_t *)src,
                           (uint32_t *)dst, (uint32_t *)natural, Hkv, M, ds);
    return hipGetLastError();
}

hipError_t pq_launch_pack_codes(const pq_attn_ctx *ctx, int kind, const uint8_t *token_major, int n_tokens,
                                uint8_t *packed, bool unpack, hipStream_t s)
{
    const int64_t n_heads = (int64_t)ctx->cfg.batch * ctx->cfg.n_kv_heads;
    const int M = ctx->cfg.n_subspaces;
    const int64_t total = n_heads * n_tokens * M;
    if (total == 0)
        return hipSuccess;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    hipLaunchKernelGGL(pq_pack_codes_kernel, grid, block, 0, s, token_major, packed, n_heads, n_tokens, M,
                       ctx->cap_padded * M, kind, unpack ? 1 : 0, ctx->k_skew);
    return hipGetLastError();
}

hipError_t pq_launch_copy16(const void *src, void *dst, int64_t bytes, hipStream_t s)
{
    const int64_t n = bytes / 16;
    if (n == 0)
        return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(pq_copy16_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s, (const u32x4 *)src,
                       (u32x4 *)dst, n);
    return hipGetLastError();
}

hipError_t pq_launch_stream_read(const void *src, int64_t bytes, uint32_t *sink, hipStream_t s)
{
    hipLaunchKernelGGL(pq_stream_read_kernel, dim3(2048), dim3(1024), 0, s, (const u32x4 *)src, bytes / 16, sink);
    return hipGetLastError();
}
