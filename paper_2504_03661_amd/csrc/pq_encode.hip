// Nearest-centroid encode of new tokens, appended to the code tensors in place.
//
// Eq. 4 read with Section II-C ("assigned to the nearest centroid in its subspace"):
//   code[t][i] = argmin_c sum_j (x[t][i*ds + j] - C^i[c][j])^2,   ties -> lowest c.
// The comparison is decided in IEEE double: inputs widened exactly, and for
// j = 0 .. ds-1 in order dist = fma(x_j - c_j, x_j - c_j, dist): each difference and
// each fused multiply-add rounded once, nothing else contracted (this file is compiled
// with -ffp-contract=off and the loop below also pins it with a pragma).  fp64 vector
// arithmetic runs at the same rate as unpacked fp32 on gfx950, so exactness costs
// nothing here; the scan costs 2 ds + 3 vector operations per (sub-vector, centroid).
//
// Mapping.  One wavefront = one (K or V, sequence, KV head, subspace, 64-token
// chunk).  Lane = token: all 64 lanes walk the 256 centroids in lock step, the
// centroid (widened to double) comes out of LDS as a broadcast read, the running
// best is a compare + two selects, and no cross-lane reduction is needed.  The
// strict "<" on an ascending scan keeps the lowest index among equal distances.
// The code byte is stored straight into the device layout of its tensor.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"

namespace {

// One wavefront per workgroup: its LDS footprint (the widened codebook of one subspace, 4-8 KiB)
// fits beside a resident decode workgroup, so an encode issued on another stream can share the
// compute units with a running decode (asynchronous quantization, Section III-B).
constexpr int ENC_WAVES = 1;

template <typename T> __device__ inline double widen(const void *p, int64_t i);
template <> __device__ inline double widen<__half>(const void *p, int64_t i)
{
    return (double)__half2float(((const __half *)p)[i]);  // fp16 -> fp32 -> fp64, both exact
}
template <> __device__ inline double widen<float>(const void *p, int64_t i)
{
    return (double)((const float *)p)[i];
}

template <int M, int DS, typename T>
__global__ __launch_bounds__(ENC_WAVES * 64) void pq_encode_kernel(const pq_encode_args a)
{
#pragma clang fp contract(off)
    __shared__ double cb[ENC_WAVES][256 * DS];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int which = blockIdx.z;                     // 0: keys, 1: values
    const int i = blockIdx.y * ENC_WAVES + wave;      // subspace
    const int n_chunks = (a.n_new + 63) >> 6;
    const int chunk = blockIdx.x % n_chunks;
    const int head = blockIdx.x / n_chunks;           // b * Hkv + hkv
    const int b = head / a.Hkv;
    const int hkv = head - b * a.Hkv;

    // this wavefront's codebook C^i, widened
    const int64_t cb_base = ((int64_t)hkv * M + i) * 256 * DS;
    for (int e = lane; e < 256 * DS; e += 64)
        cb[wave][e] = widen<T>(a.codebook[which], cb_base + e);
    __builtin_amdgcn_wave_barrier();

    const int tok = chunk * 64 + lane;
    const bool live = tok < a.n_new;
    double x[DS];
#pragma unroll
    for (int j = 0; j < DS; ++j)
        x[j] = live ? widen<T>(a.x[which], ((int64_t)head * a.n_new + tok) * PQ_HEAD_DIM + i * DS + j) : 0.0;

    int best = 0;
    double best_dist = __builtin_huge_val();  // finite inputs: centroid 0 always beats it
    for (int c = 0; c < 256; ++c) {
        double dist = 0.0;
#pragma unroll
        for (int j = 0; j < DS; ++j) {
            const double diff = x[j] - cb[wave][c * DS + j];
            dist = __builtin_fma(diff, diff, dist);
        }
        // strict "<" on an ascending scan: the lowest index among equal distances stays
        best = dist < best_dist ? c : best;
        best_dist = __builtin_fmin(best_dist, dist);
    }

    int n_old = a.ctx_len[b];
    n_old = n_old < 0 ? 0 : n_old;
    const int64_t pos = (int64_t)n_old + tok;
    if (live && pos < a.max_context) {
        uint8_t *dst = a.codes[which] + (int64_t)head * a.head_stride;
        const int64_t off = which == 0 ? pq_k_code_offset(pos, i, M, a.k_skew) : pq_v_code_offset(pos, i, M);
        dst[off] = (uint8_t)best;
    }
}

__global__ void pq_bump_len_kernel(int32_t *ctx_len, int B, int n_new, int max_context, unsigned int *dev_err)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B)
        return;
    int n = ctx_len[b];
    n = n < 0 ? 0 : n;
    int64_t m = (int64_t)n + n_new;
    if (m > max_context) {
        m = max_context;
        atomicOr(dev_err, PQ_ERRFLAG_APPEND_OVERFLOW);
    }
    ctx_len[b] = (int32_t)m;
}

template <int M, int DS, typename T>
void launch(const pq_encode_args &a, hipStream_t s)
{
    const int n_chunks = (a.n_new + 63) >> 6;
    dim3 grid(a.B * a.Hkv * n_chunks, M / ENC_WAVES, 2);
    hipLaunchKernelGGL((pq_encode_kernel<M, DS, T>), grid, dim3(ENC_WAVES * 64), 0, s, a);
}

}  // namespace

hipError_t pq_launch_bump_len(int32_t *ctx_len, int B, int n_new, int max_context, unsigned int *dev_err, hipStream_t s)
{
    hipLaunchKernelGGL(pq_bump_len_kernel, dim3((B + 255) / 256), dim3(256), 0, s, ctx_len, B, n_new, max_context, dev_err);
    return hipGetLastError();
}

hipError_t pq_launch_encode(const pq_attn_ctx *ctx, const pq_encode_args &a, int32_t *ctx_len, unsigned int *dev_err,
                            hipStream_t s)
{
    const bool f16 = ctx->cfg.dtype == PQ_F16;
    if (ctx->cfg.n_subspaces == 64) {
        if (f16) launch<64, 2, __half>(a, s); else launch<64, 2, float>(a, s);
    } else {
        if (f16) launch<32, 4, __half>(a, s); else launch<32, 4, float>(a, s);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    // lengths move only after every encode workgroup has read the old ones (stream order)
    return pq_launch_bump_len(ctx_len, a.B, a.n_new, a.max_context, dev_err, s);
}
