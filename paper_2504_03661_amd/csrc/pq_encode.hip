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
// This scan (pq_encode_kernel) serves fp32 contexts; fp16 contexts reach the same codes through
// pq_encode_fast_kernel further down, where the matrix cores find the few centroids that can be
// the nearest and the expression above decides among them.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_device_utils.h"
#include "pq_nearest_filter.h"

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

// ---------------------------------------------------------------------------------
// fp16 inputs: the same codes, found with the matrix cores as a filter.
//
// With q(c) = n(c)/2 - x . c (n = |c|^2) the distance is |x|^2 + 2 q, so the nearest centroid minimises q.
// For fp16 inputs every product x_j c_j is exact in fp32, and v_mfma_f32_4x4x4_16B_f16 evaluates
// v(c) = q(c) + off for 4 centroids (rows of A, from LDS) x 64 tokens (columns of B, one per lane) per
// instruction, to within a bound e that follows from the magnitudes (below); off >= |x|^2/2 + e is a
// per-token constant in the C operand that makes every computed value positive, so that values compare
// as integers (v_min3_i32: half a vector operation per value, no NaN quieting).  That is a filter, not the
// decision:
//   pass 1  best = min over all 256 centroids of the computed v;
//   pass 2  the same products again with off - (best + tau) in the C operand: a computed value is negative
//           where it lies within tau of the best one, so a group of 4 centroids is a candidate when the OR of
//           its 4 results has the sign bit set (one v_alignbit shifts that bit into the group mask); count the
//           candidate groups, remember the first and the last;
//   refine  one or two candidate groups (nearly always): the true minimiser is among their centroids — the
//           distances of those 4 (8 if some token of the wavefront has two groups) are evaluated in the
//           defining fp64 arithmetic (see the top of this file),
//           ascending, and the smallest, lowest index first, is the code.  Three or more groups within tau
//           (duplicated centroids, near-ties): the lane walks all of its marked groups the same way.  A
//           codebook or token outside the range the bound covers (no marked group, non-finite values): the
//           64-token chunk runs the full fp64 scan.
// Either way the code is decided by the fp64 expression, so it is bit-exact by construction; the filter only
// has to be SAFE: every centroid outside the candidate groups must have a strictly larger true distance.  With
// |computed - true| <= e for every centroid and c^ the minimiser of the computed values, a centroid c outside
// the candidate groups has true v(c) > best + tau - e and true v(c^) <= best + e: tau >= 2 e suffices (plus the
// two roundings of off - (best + tau), <= 2^-23 T, and strictly: tau exceeds 2 e by 2^-20.4 T).
// Bound on e: A row = (c_0 .. c_{ds-1}, h, l) with h + l = n/2 split into two fp16 (n summed in fp32 from
// exact squares: <= 2^-21.2 n/2 in all), B column = (-x_0 .. -x_{ds-1}, 1, 1); fp32 accumulation of at most 7
// terms, even if every one of the 6 adds truncates, <= 6 x 2^-23 T with T = N + X C + off >= the sum of the
// terms' magnitudes (N = max n/2, C = max |c_j|, X = sum_j |x_j|).  So e <= 2^-19.7 T, and
// tau = 2^-18.3 T + 2^-22 leaves a factor 1.3 beyond the worst case (2.6 if the adds round to nearest), which
// is many orders above the rounding of the fp64 distances themselves.
// The matrix instruction takes fp16 subnormals as they are (no flush: measured, and the default mode of a HIP
// kernel); n/2 beyond the fp16 range does not split into h + l: such a codebook takes the full scan.
// Cost per (sub-vector, centroid): about 2 vector operations instead of 2 ds + 3 in fp64.
__device__ inline float wave_max_f(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

template <int M, int DS, int NQ>
__global__ __launch_bounds__(64) void pq_encode_fast_kernel(const pq_encode_args a, const int rounds)
{
    constexpr int ROW = pq_filter_row_bytes<DS>();
    __shared__ __attribute__((aligned(16))) unsigned char arow[256 * ROW];
    __shared__ double cb[256 * DS];

    const int lane = threadIdx.x;
    const int which = blockIdx.z;  // 0: keys, 1: values
    const int i = blockIdx.y;      // subspace
    const int n_tok = a.B * a.n_new;  // tokens of one KV head over all sequences: they share its codebook
    const int n_chunks = (n_tok + 64 * NQ - 1) / (64 * NQ);
    const int n_jobs = (n_chunks + rounds - 1) / rounds;  // a wavefront takes `rounds` chunks in a row: one codebook set-up
    const int hkv = blockIdx.x / n_jobs;
    const int chunk0 = (blockIdx.x - hkv * n_jobs) * rounds;

    // ---- codebook of this subspace: fp64 copy for the exact evaluations, A rows for the filter
    const __half *src = (const __half *)a.codebook[which] + ((int64_t)hkv * M + i) * 256 * DS;
    float n_max = 0.f, c_max = 0.f;
    bool cb_bad = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int c = lane + 64 * r;
        pq_filter_build_row<DS>(src + c * DS, arow + c * ROW, cb + c * DS, n_max, c_max, cb_bad);
    }
    n_max = wave_max_f(n_max);
    c_max = wave_max_f(c_max);
    cb_bad = __builtin_amdgcn_ballot_w64(cb_bad) != 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

#pragma unroll 1
    for (int chunk = chunk0; chunk < chunk0 + rounds && chunk < n_chunks; ++chunk) {
    // ---- this lane's tokens: one per 64-token sub-chunk
    bool live[NQ];
    int bq[NQ], tq[NQ];
    _Float16 xv[NQ][DS];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int u = (chunk * NQ + q) * 64 + lane;
        live[q] = u < n_tok;
        const int uu = live[q] ? u : 0;
        bq[q] = uu / a.n_new;
        tq[q] = uu - bq[q] * a.n_new;
        const __half *xp =
            (const __half *)a.x[which] + (((int64_t)bq[q] * a.Hkv + hkv) * a.n_new + tq[q]) * PQ_HEAD_DIM + i * DS;
#pragma unroll
        for (int j = 0; j < DS; ++j)
            xv[q][j] = __builtin_bit_cast(_Float16, xp[j]);
    }
    int codes[NQ];
    pq_filter_codes<DS, NQ>(arow, cb, n_max, c_max, cb_bad, xv, live, codes);

#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        int n_old = a.ctx_len[bq[q]];
        n_old = n_old < 0 ? 0 : n_old;
        const int64_t pos = (int64_t)n_old + tq[q];
        if (live[q] && pos < a.max_context) {
            uint8_t *dst = a.codes[which] + ((int64_t)bq[q] * a.Hkv + hkv) * a.head_stride;
            const int64_t off = which == 0 ? pq_k_code_offset(pos, i, M, a.k_skew) : pq_v_code_offset(pos, i, M);
            dst[off] = (uint8_t)codes[q];
        }
    }
    }
}

// ---------------------------------------------------------------------------------
// A handful of tokens per KV head (one decoding step of a small batch): lane = CENTROID.  With one token per
// lane a wavefront would walk 256 centroids for a few live lanes; here every lane holds 4 centroids in
// registers, evaluates the defining fp64 distances of the token at hand to its 4 (ascending, strict "<") and
// the wavefront takes the lexicographic minimum of (distance, index) — the lowest index among equal distances,
// as in the scan.  One wavefront per (K or V, KV head, subspace) loops over the head's tokens of all sequences.
constexpr int FEW_TOKENS = 16;

template <int M, int DS, typename T>
__global__ __launch_bounds__(64) void pq_encode_few_kernel(const pq_encode_args a)
{
#pragma clang fp contract(off)
    const int lane = threadIdx.x;
    const int which = blockIdx.z;
    const int i = blockIdx.y;
    const int hkv = blockIdx.x;
    const int n_tok = a.B * a.n_new;  // <= FEW_TOKENS

    const int64_t cb_base = ((int64_t)hkv * M + i) * 256 * DS;
    double c[4][DS];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < DS; ++j)
            c[r][j] = widen<T>(a.codebook[which], cb_base + (int64_t)(lane + 64 * r) * DS + j);

    // lane u < n_tok fetches token u: its sub-vector, sequence and position
    const int u_mine = lane < n_tok ? lane : 0;
    const int b_mine = u_mine / a.n_new;
    const int t_mine = u_mine - b_mine * a.n_new;
    double x_mine[DS];
#pragma unroll
    for (int j = 0; j < DS; ++j)
        x_mine[j] = widen<T>(a.x[which], (((int64_t)b_mine * a.Hkv + hkv) * a.n_new + t_mine) * PQ_HEAD_DIM + i * DS + j);
    int n_old = a.ctx_len[b_mine];
    n_old = n_old < 0 ? 0 : n_old;

    int code_mine = 0;
    for (int u = 0; u < n_tok; ++u) {
        double x[DS];
#pragma unroll
        for (int j = 0; j < DS; ++j)
            x[j] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x_mine[j]), u),
                                    __builtin_amdgcn_readlane(__double2loint(x_mine[j]), u));
        double bd = __builtin_huge_val();
        int bc = lane;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double dist = 0.0;
#pragma unroll
            for (int j = 0; j < DS; ++j) {
                const double diff = x[j] - c[r][j];
                dist = __builtin_fma(diff, diff, dist);
            }
            bc = dist < bd ? lane + 64 * r : bc;  // ascending index inside the lane, strict "<"
            bd = __builtin_fmin(bd, dist);
        }
        wave_argmin(bd, bc);
        code_mine = lane == u ? bc : code_mine;
    }
    const int64_t pos = (int64_t)n_old + t_mine;
    if (lane < n_tok && pos < a.max_context) {
        uint8_t *dst = a.codes[which] + ((int64_t)b_mine * a.Hkv + hkv) * a.head_stride;
        const int64_t off = which == 0 ? pq_k_code_offset(pos, i, M, a.k_skew) : pq_v_code_offset(pos, i, M);
        dst[off] = (uint8_t)code_mine;
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

template <int M, int DS>
void launch_fast(const pq_encode_args &a, hipStream_t s)
{
    const int n_tok = a.B * a.n_new;
    if (n_tok > 128) {
        // prompt-sized inputs: up to 8 chunks of 256 tokens per wavefront while at least 8192 wavefronts remain
        const int n_chunks = (n_tok + 255) / 256;
        const int64_t waves = (int64_t)a.Hkv * n_chunks * M * 2;
        const int rounds = (int)(waves / 8192 < 1 ? 1 : waves / 8192 > 8 ? 8 : waves / 8192);
        dim3 grid(a.Hkv * ((n_chunks + rounds - 1) / rounds), M, 2);
        hipLaunchKernelGGL((pq_encode_fast_kernel<M, DS, 4>), grid, dim3(64), 0, s, a, rounds);
    } else if (n_tok > 64) {
        dim3 grid(a.Hkv, M, 2);
        hipLaunchKernelGGL((pq_encode_fast_kernel<M, DS, 2>), grid, dim3(64), 0, s, a, 1);
    } else {
        dim3 grid(a.Hkv, M, 2);
        hipLaunchKernelGGL((pq_encode_fast_kernel<M, DS, 1>), grid, dim3(64), 0, s, a, 1);
    }
}

hipError_t pq_launch_encode(const pq_attn_ctx *ctx, const pq_encode_args &a, int32_t *ctx_len, unsigned int *dev_err,
                            hipStream_t s)
{
    const bool f16 = ctx->cfg.dtype == PQ_F16;
    // fp16: from 7 tokens per head the filter kernel is the faster one (32 heads, one new token per sequence: 4
    // sequences 7.4 us, 8 sequences 10.7 us, 16 sequences 17.9 us here against 10.1 us there)
    if ((int64_t)a.B * a.n_new <= (f16 ? 6 : FEW_TOKENS)) {
        const dim3 grid(a.Hkv, ctx->cfg.n_subspaces, 2);
        if (ctx->cfg.n_subspaces == 64) {
            if (f16) hipLaunchKernelGGL((pq_encode_few_kernel<64, 2, __half>), grid, dim3(64), 0, s, a);
            else hipLaunchKernelGGL((pq_encode_few_kernel<64, 2, float>), grid, dim3(64), 0, s, a);
        } else {
            if (f16) hipLaunchKernelGGL((pq_encode_few_kernel<32, 4, __half>), grid, dim3(64), 0, s, a);
            else hipLaunchKernelGGL((pq_encode_few_kernel<32, 4, float>), grid, dim3(64), 0, s, a);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        return pq_launch_bump_len(ctx_len, a.B, a.n_new, a.max_context, dev_err, s);
    }
    // the filter kernel indexes the tokens of a head over all sequences with 32 bits
    const bool fast = f16 && (int64_t)a.B * a.n_new < ((int64_t)1 << 30);
    if (ctx->cfg.n_subspaces == 64) {
        if (fast) launch_fast<64, 2>(a, s); else if (f16) launch<64, 2, __half>(a, s); else launch<64, 2, float>(a, s);
    } else {
        if (fast) launch_fast<32, 4>(a, s); else if (f16) launch<32, 4, __half>(a, s); else launch<32, 4, float>(a, s);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    // lengths move only after every encode workgroup has read the old ones (stream order)
    return pq_launch_bump_len(ctx_len, a.B, a.n_new, a.max_context, dev_err, s);
}
