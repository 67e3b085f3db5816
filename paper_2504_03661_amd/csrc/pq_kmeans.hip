// Offline codebook training: k-means per (KV head, subspace) by Lloyd's iteration on sampled
// key / value vectors (Section II-C, training phase; Section III-A, "Offline PQ Codebook Training").
//
// One iteration = two kernels.
//   assign   every sample sub-vector goes to its nearest centroid — the rule and the arithmetic of
//            the encode kernel: squared Euclidean distance decided in IEEE double as
//            dist = fma(x_j - c_j, x_j - c_j, dist), equal distances to the lowest index — and is
//            added to that centroid's member sum and count.  fp16 values are integers times
//            2^-24, so the sums are kept as 64-bit integers: exact, and independent of the order in
//            which the atomics land (n_samples <= 2^20 keeps them below 2^61).
//   update   centroid = double(sum) * 2^-24 / count in IEEE double, rounded to float and from there
//            to fp16; a centroid without members keeps its value.  The kernel also clears the
//            accumulators for the next iteration.
// The paper does not say how it initialises, iterates or treats empty clusters; the initial
// centroids are the caller's, the iteration count too.
//
// Mapping of `assign`: one workgroup = (head, subspace, slice of samples), 4 wavefronts sharing the
// widened codebook (LDS, broadcast reads) and the slice's partial sums (LDS atomics); lane =
// sample; the partial sums reach memory with one 64-bit atomic per touched entry.  Bound by the
// fp64 vector ALU like the encode: (2 ds + 3) operations per (sub-vector, centroid).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_nearest_filter.h"

namespace {

constexpr int KM_WAVES = 4;
constexpr int KM_CHUNKS = 4;                           // 64-sample chunks per wavefront
constexpr int KM_SLICE = KM_WAVES * KM_CHUNKS * 64;    // samples per workgroup

template <int M, int DS>
__global__ __launch_bounds__(KM_WAVES * 64) void pq_kmeans_assign_kernel(const __half *samples, const __half *codebook,
                                                                        unsigned long long *sums, unsigned int *counts,
                                                                        int n_samples, int n_slices)
{
    constexpr int ROW = pq_filter_row_bytes<DS>();
    static_assert(KM_WAVES * 64 == 256, "one thread per centroid below");
    __shared__ double cb[256 * DS];
    __shared__ __attribute__((aligned(16))) unsigned char arow[256 * ROW];
    __shared__ unsigned long long part_sum[256 * DS];
    __shared__ unsigned int part_cnt[256];
    __shared__ float red[2 * KM_WAVES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int head = blockIdx.x / n_slices;
    const int slice = blockIdx.x - head * n_slices;
    const int i = blockIdx.y;  // subspace

    // codebook of this (head, subspace): fp64 copy and matrix-instruction rows for the nearest-centroid filter of
    // the encode (pq_nearest_filter.h), one centroid per thread; accumulators cleared
    const int64_t cb_base = ((int64_t)head * M + i) * 256 * DS;
    float n_max = 0.f, c_max = 0.f;
    bool cb_bad = false;
    pq_filter_build_row<DS>(codebook + cb_base + tid * DS, arow + tid * ROW, cb + tid * DS, n_max, c_max, cb_bad);
    for (int e = tid; e < 256 * DS; e += KM_WAVES * 64)
        part_sum[e] = 0ull;
    part_cnt[tid] = 0u;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        n_max = fmaxf(n_max, __shfl_xor(n_max, o));
        c_max = fmaxf(c_max, __shfl_xor(c_max, o));
    }
    if (lane == 0) {
        red[wave] = n_max;
        red[KM_WAVES + wave] = __builtin_amdgcn_ballot_w64(cb_bad) != 0 ? -1.f : c_max;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < KM_WAVES; ++w) {
        n_max = fmaxf(n_max, red[w]);
        const float cw = red[KM_WAVES + w];
        cb_bad |= cw < 0.f;
        c_max = fmaxf(c_max, cw);
    }
    cb_bad = __builtin_amdgcn_ballot_w64(cb_bad) != 0;

    // this wavefront's KM_CHUNKS 64-sample chunks, assigned together (the same rule and arithmetic as the encode)
    bool live[KM_CHUNKS];
    _Float16 xv[KM_CHUNKS][DS];
#pragma unroll
    for (int ch = 0; ch < KM_CHUNKS; ++ch) {
        const int s = slice * KM_SLICE + (ch * KM_WAVES + wave) * 64 + lane;
        live[ch] = s < n_samples;
        const int ss = live[ch] ? s : 0;
#pragma unroll
        for (int j = 0; j < DS; ++j)
            xv[ch][j] = __builtin_bit_cast(_Float16, samples[((int64_t)head * n_samples + ss) * PQ_HEAD_DIM + i * DS + j]);
    }
    int codes[KM_CHUNKS];
    pq_filter_codes<DS, KM_CHUNKS>(arow, cb, n_max, c_max, cb_bad, xv, live, codes);
#pragma unroll
    for (int ch = 0; ch < KM_CHUNKS; ++ch) {
        if (!live[ch])
            continue;
#pragma unroll
        for (int j = 0; j < DS; ++j) {
            // exact: an fp16 value times 2^24 is an integer below 2^41 in magnitude
            const long long fixed = (long long)((float)xv[ch][j] * 16777216.0f);
            atomicAdd(&part_sum[codes[ch] * DS + j], (unsigned long long)fixed);
        }
        atomicAdd(&part_cnt[codes[ch]], 1u);
    }
    __syncthreads();

    const int64_t acc_base = ((int64_t)head * M + i) * 256;
    for (int e = tid; e < 256 * DS; e += KM_WAVES * 64)
        if (part_sum[e] != 0ull)
            atomicAdd(&sums[acc_base * DS + e], part_sum[e]);
    for (int e = tid; e < 256; e += KM_WAVES * 64)
        if (part_cnt[e] != 0u)
            atomicAdd(&counts[acc_base + e], part_cnt[e]);
}

// one thread per (head, subspace, centroid)
template <int DS>
__global__ void pq_kmeans_update_kernel(__half *codebook, unsigned long long *sums, unsigned int *counts, int64_t n)
{
#pragma clang fp contract(off)
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n)
        return;
    const unsigned int count = counts[e];
    if (count != 0u) {
#pragma unroll
        for (int j = 0; j < DS; ++j) {
            const double sum = (double)(long long)sums[e * DS + j];
            const double mean = sum * 5.9604644775390625e-08 / (double)count;  // 2^-24, then one division
            codebook[e * DS + j] = __float2half_rn((float)mean);
            sums[e * DS + j] = 0ull;
        }
        counts[e] = 0u;
    }
}

__global__ void pq_clear_words_kernel(uint32_t *p, int64_t n)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n)
        p[e] = 0u;
}

}  // namespace

hipError_t pq_launch_clear_words(void *p, int64_t words, hipStream_t s)
{
    hipLaunchKernelGGL(pq_clear_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, (uint32_t *)p, words);
    return hipGetLastError();
}

hipError_t pq_launch_kmeans_update(void *codebook, unsigned long long *sums, unsigned int *counts, int64_t n, int ds,
                                   hipStream_t s)
{
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (ds == 2)
        hipLaunchKernelGGL(pq_kmeans_update_kernel<2>, grid, block, 0, s, (__half *)codebook, sums, counts, n);
    else
        hipLaunchKernelGGL(pq_kmeans_update_kernel<4>, grid, block, 0, s, (__half *)codebook, sums, counts, n);
    return hipGetLastError();
}

int64_t pq_kmeans_accumulator_bytes(const pq_attn_ctx *ctx)
{
    if (pq_config_is_12bit(&ctx->cfg))
        return pq12_kmeans_workspace_bytes(ctx);
    const int64_t n = (int64_t)ctx->cfg.n_kv_heads * ctx->cfg.n_subspaces * 256;
    return n * ctx->ds * 8 + n * 4;
}

hipError_t pq_launch_kmeans(const pq_attn_ctx *ctx, const void *samples, int n_samples, void *codebook, int n_iters,
                            void *workspace, hipStream_t s)
{
    if (pq_config_is_12bit(&ctx->cfg))
        return pq12_launch_kmeans(ctx, samples, n_samples, codebook, n_iters, workspace, s);
    const int Hkv = ctx->cfg.n_kv_heads, M = ctx->cfg.n_subspaces, DS = ctx->ds;
    const int64_t n = (int64_t)Hkv * M * 256;
    unsigned long long *sums = (unsigned long long *)workspace;
    unsigned int *counts = (unsigned int *)(sums + n * DS);
    const int64_t words = pq_kmeans_accumulator_bytes(ctx) / 4;
    hipLaunchKernelGGL(pq_clear_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s,
                       (uint32_t *)workspace, words);
    const int n_slices = (n_samples + KM_SLICE - 1) / KM_SLICE;
    const dim3 grid((unsigned)(Hkv * n_slices), (unsigned)M), block(KM_WAVES * 64);
    for (int it = 0; it < n_iters; ++it) {
        if (M == 64) {
            hipLaunchKernelGGL((pq_kmeans_assign_kernel<64, 2>), grid, block, 0, s, (const __half *)samples,
                               (const __half *)codebook, sums, counts, n_samples, n_slices);
            hipLaunchKernelGGL(pq_kmeans_update_kernel<2>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                               (__half *)codebook, sums, counts, n);
        } else {
            hipLaunchKernelGGL((pq_kmeans_assign_kernel<32, 4>), grid, block, 0, s, (const __half *)samples,
                               (const __half *)codebook, sums, counts, n_samples, n_slices);
            hipLaunchKernelGGL(pq_kmeans_update_kernel<4>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                               (__half *)codebook, sums, counts, n);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    return hipGetLastError();
}
