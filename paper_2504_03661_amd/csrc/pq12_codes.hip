// 12-bit codes (M = 32 subspaces of 4 dims, 4096 centroids per subspace — the paper's 3-bit-per-
// dimension setting, Section IV-A): nearest-centroid encode and the conversions between the logical
// token-major form [B][Hkv][n][32] uint16 and the device layouts of pq_internal.h.
//
// Encode (Eq. 4 with Section II-C's nearest-centroid assignment) follows the 8-bit encode kernel: lane =
// token, squared Euclidean distance decided in IEEE double as dist = fma(x_j - c_j, x_j - c_j, dist),
// strict "<" on an ascending scan so that equal distances go to the lowest index.  A subspace's 4096
// centroids, widened to double, take 128 KiB: they pass through LDS in four tiles of 1024.
// Two 12-bit codes share bytes, so the kernel does not write the device layout itself: codes go to a
// token-major staging buffer and a second kernel packs them behind the current lengths, one thread per
// 12-byte unit (a V unit holds 8 tokens of one subspace: the thread keeps the codes of tokens it does
// not append).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_device_utils.h"
#include "pq_filter_constants.h"

namespace {

constexpr int E12_WAVES = 4;
constexpr int E12_TILE = 1024;  // centroids per LDS tile

__device__ inline void pack8(const uint32_t (&c)[8], uint32_t (&w)[3])
{
    w[0] = c[0] | (c[1] << 12) | (c[2] << 24);
    w[1] = (c[2] >> 8) | (c[3] << 4) | (c[4] << 16) | (c[5] << 28);
    w[2] = (c[5] >> 4) | (c[6] << 8) | (c[7] << 20);
}

__device__ inline void unpack8(const uint32_t (&w)[3], uint32_t (&c)[8])
{
    c[0] = w[0] & 0xfffu;
    c[1] = (w[0] >> 12) & 0xfffu;
    c[2] = ((w[0] >> 24) | (w[1] << 8)) & 0xfffu;
    c[3] = (w[1] >> 4) & 0xfffu;
    c[4] = (w[1] >> 16) & 0xfffu;
    c[5] = ((w[1] >> 28) | (w[2] << 4)) & 0xfffu;
    c[6] = (w[2] >> 8) & 0xfffu;
    c[7] = w[2] >> 20;
}

// One workgroup = (K or V, KV head, subspace) x 4 work items, one per wavefront; a work item is a 64-token
// chunk of one sequence (the sequences of a batch share the head's codebook, so short appends of many
// sequences still fill the workgroup).  x is [B][Hkv][x_head_stride >= n_new][d]; the codes of its first
// n_new rows go to out [B][Hkv][n_new][32].
__global__ __launch_bounds__(E12_WAVES * 64) void pq12_encode_kernel(const __half *x0, const __half *x1,
                                                                    const __half *cb0, const __half *cb1,
                                                                    uint16_t *out0, uint16_t *out1, int B, int Hkv,
                                                                    int n_new, int groups_per_head, int64_t x_head_stride)
{
#pragma clang fp contract(off)
    __shared__ double tile[E12_TILE * 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int which = blockIdx.z;  // 0: keys, 1: values
    const int i = blockIdx.y;      // subspace
    const int n_chunks = (n_new + 63) >> 6;
    const int hkv = blockIdx.x / groups_per_head;
    const int item = (blockIdx.x - hkv * groups_per_head) * E12_WAVES + wave;  // (sequence, chunk) of this wavefront
    const int b = item / n_chunks;
    const int chunk = item - b * n_chunks;
    const int64_t head = (int64_t)b * Hkv + hkv;
    const __half *x = which ? x1 : x0;
    const __half *cb = (which ? cb1 : cb0) + ((int64_t)hkv * PQ12_M + i) * PQ12_CENTROIDS * 4;
    uint16_t *out = which ? out1 : out0;

    const int tok = chunk * 64 + lane;
    const bool live = b < B && tok < n_new;
    double xv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        xv[j] = live ? (double)__half2float(x[(head * x_head_stride + tok) * PQ_HEAD_DIM + i * 4 + j]) : 0.0;

    int best = 0;
    double best_dist = __builtin_huge_val();
    for (int t0 = 0; t0 < PQ12_CENTROIDS; t0 += E12_TILE) {
        __syncthreads();  // the previous tile has been scanned by every wavefront
        for (int e = tid; e < E12_TILE * 4; e += E12_WAVES * 64)
            tile[e] = (double)__half2float(cb[t0 * 4 + e]);
        __syncthreads();
        for (int c = 0; c < E12_TILE; ++c) {
            double dist = 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double diff = xv[j] - tile[c * 4 + j];
                dist = __builtin_fma(diff, diff, dist);
            }
            best = dist < best_dist ? t0 + c : best;  // ascending scan, strict "<": lowest index among equals
            best_dist = __builtin_fmin(best_dist, dist);
        }
    }
    if (live)
        out[(head * n_new + tok) * PQ12_M + i] = (uint16_t)best;
}

// ---------------------------------------------------------------------------------------------------
// The same codes with the matrix cores as a filter (see the 8-bit encode for the argument and the error bound;
// here ds = 4, so an A row is (c_0 .. c_3) and (h, l, 0, 0), two matrix instructions per value quad, 6 fp32
// adds).  A workgroup keeps the 4096 A rows of its (K or V, KV head, subspace) in LDS (64 KiB) and each of its 8
// wavefronts takes up to NQ 64-token sub-chunks of the head's tokens over all sequences.  Pass 1: the minimum
// of the 4096 computed values per token.  Pass 2: one bit per block of 16 centroids that holds a value
// within tau of it (256 bits per token; the sign of the value once best + tau is folded into the C operand).
// One or two marked blocks: their 16 or 32 centroids are evaluated in
// the defining fp64 arithmetic, ascending, lowest index first; more: the lane walks all of its marked blocks the
// same way.  A codebook whose |c|^2 / 2 leaves the fp16 range, or no marked block at all (non-finite values): the
// sub-chunk runs the full fp64 scan.  About 1.1 vector instructions per (sub-vector, centroid)
// instead of 11.
// SPLIT (a head has at most 64 NQ tokens in the call — a decoding step of a batch): with one sub-chunk per
// workgroup seven of its eight wavefronts would idle while one walks all 4096 centroids alone, each step waiting
// out the latency of two dependent matrix instructions (17 tokens per head: 454 us).  Here all eight take the SAME
// tokens and an eighth of the centroids each — 128 of the 1024 groups in pass 1, one of the eight 32-block mask
// words in pass 2 — and exchange the per-token minimum and the mask words through LDS; the words are the ones the
// unsplit walk computes, so the refinement (wavefront 0) and the codes are the same.
// ---------------------------------------------------------------------------------------------------
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4e __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2e __attribute__((ext_vector_type(2)));

constexpr int F12_WAVES = 8;  // wavefronts that share one set of A rows

template <int NQ, bool SPLIT>
__global__ __launch_bounds__(F12_WAVES * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void pq12_encode_fast_kernel(const __half *x0, const __half *x1,
                                                                         const __half *cb0, const __half *cb1,
                                                                         uint16_t *out0, uint16_t *out1, int B, int Hkv,
                                                                         int n_new, int groups_per_head, int64_t x_head_stride)
{
#pragma clang fp contract(off)
    __shared__ __attribute__((aligned(16))) unsigned char arow[PQ12_CENTROIDS * 16];
    __shared__ float red[2 * F12_WAVES + 1];
    __shared__ uint32_t xchg[SPLIT ? F12_WAVES * NQ * 64 : 1];  // SPLIT: per wavefront, sub-chunk and token

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int which = blockIdx.z;  // 0: keys, 1: values
    const int i = blockIdx.y;      // subspace
    const int n_tok = B * n_new;   // tokens of one KV head over all sequences
    const int hkv = blockIdx.x / groups_per_head;
    // of 64 NQ tokens; SPLIT: the workgroup's eight wavefronts share one
    const int chunk = SPLIT ? blockIdx.x - hkv * groups_per_head : (blockIdx.x - hkv * groups_per_head) * F12_WAVES + wave;
    const __half *x = which ? x1 : x0;
    const __half *cb = (which ? cb1 : cb0) + ((int64_t)hkv * PQ12_M + i) * PQ12_CENTROIDS * 4;
    uint16_t *out = which ? out1 : out0;

    // ---- A rows of the 4096 centroids, their largest |c|^2 / 2 and coordinate
    float n_max = 0.f, c_max = 0.f;
    bool cb_bad = false;
    for (int c = tid; c < PQ12_CENTROIDS; c += F12_WAVES * 64) {
        const u32x2e raw = *(const u32x2e *)(cb + c * 4);
        const f16x4 v = __builtin_bit_cast(f16x4, raw);
        float n = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float f = (float)v[j];
            n += f * f;  // exact squares; the sum is rounded (covered by the bound)
            c_max = fmaxf(c_max, fabsf(f));
        }
        const float h = 0.5f * n;
        const _Float16 hh = (_Float16)h;
        const _Float16 hl = (_Float16)(h - (float)hh);
        cb_bad |= !(h < 60000.f);
        n_max = fmaxf(n_max, h);
        const f16x4 tail = {hh, hl, (_Float16)0.f, (_Float16)0.f};
        *(f16x4 *)(arow + c * 16) = v;
        *(f16x4 *)(arow + c * 16 + 8) = tail;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        n_max = fmaxf(n_max, __shfl_xor(n_max, o));
        c_max = fmaxf(c_max, __shfl_xor(c_max, o));
    }
    if (lane == 0) {
        red[wave] = n_max;
        red[F12_WAVES + wave] = __builtin_amdgcn_ballot_w64(cb_bad) != 0 ? -1.f : c_max;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < F12_WAVES; ++w) {
        n_max = fmaxf(n_max, red[w]);
        const float cw = red[F12_WAVES + w];
        cb_bad |= cw < 0.f;
        c_max = fmaxf(c_max, cw);
    }
    cb_bad = __builtin_amdgcn_ballot_w64(cb_bad) != 0;
    if (cb_bad)
        c_max = 0.f;  // unused: every sub-chunk takes the full scan

    // ---- this lane's tokens
    bool live[NQ], bad[NQ];
    f16x4 bop[NQ];
    f32x4e off4[NQ];
    float tau[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int u = (chunk * NQ + q) * 64 + lane;
        live[q] = u < n_tok;
        const int uu = live[q] ? u : 0;
        const int b = uu / n_new;
        const int t = uu - b * n_new;
        // x is [B][Hkv][x_head_stride >= n_new][d]
        const u32x2e raw = *(const u32x2e *)(x + ((((int64_t)b * Hkv + hkv) * x_head_stride + t) * PQ_HEAD_DIM + i * 4));
        const f16x4 v = __builtin_bit_cast(f16x4, raw);
        float x1s = 0.f, x2s = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float f = (float)v[j];
            x1s += fabsf(f);
            x2s += f * f;
        }
        u32x2e neg = raw ^ 0x80008000u;
        asm volatile("" : "+v"(neg));  // keep the negated operand in its registers
        bop[q] = __builtin_bit_cast(f16x4, neg);
        const float t0 = n_max + x1s * c_max + PQ_FILTER_X2_FACTOR * x2s;
        float off = PQ_FILTER_X2_FACTOR * x2s + 2.0f * (PQ_FILTER_TAU_REL * (2.0f * t0) + PQ_FILTER_TAU_ABS);
        tau[q] = PQ_FILTER_TAU_REL * (t0 + off) + PQ_FILTER_TAU_ABS;
        off += tau[q];
        off4[q] = f32x4e{off, off, off, off};
        bad[q] = cb_bad || !(off < 1.0e30f);
    }
    const f16x4 ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)0.f, (_Float16)0.f};
    const unsigned char *my_row = arow + (lane & 3) * 16;
    auto values = [&](int m, int q) -> f32x4e {
        const f16x4 A1 = *(const f16x4 *)(my_row + m * 64);
        const f16x4 A2 = *(const f16x4 *)(my_row + m * 64 + 8);
        return __builtin_amdgcn_mfma_f32_4x4x4f16(A2, ones, __builtin_amdgcn_mfma_f32_4x4x4f16(A1, bop[q], off4[q], 0, 0, 0), 0, 0, 0);
    };

    // ---- pass 1: smallest computed value per token (positive floats order like their bit patterns)
    int best[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
        best[q] = 0x7f800000;
    constexpr int M_PER_WAVE = SPLIT ? PQ12_CENTROIDS / 4 / F12_WAVES : PQ12_CENTROIDS / 4;
    const int m0 = SPLIT ? wave * M_PER_WAVE : 0;
#pragma unroll 2
    for (int m = m0; m < m0 + M_PER_WAVE; ++m) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const f32x4e d = values(m, q);
            best[q] = min(min(best[q], __float_as_int(d[0])), __float_as_int(d[1]));
            best[q] = min(min(best[q], __float_as_int(d[2])), __float_as_int(d[3]));
        }
    }
    if (SPLIT) {  // the minimum over the eight wavefronts' shares
#pragma unroll
        for (int q = 0; q < NQ; ++q)
            xchg[(wave * NQ + q) * 64 + lane] = (uint32_t)best[q];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int w = 0; w < F12_WAVES; ++w)
                best[q] = min(best[q], (int)xchg[(w * NQ + q) * 64 + lane]);
        __syncthreads();  // the words are written again below
    }
    // ---- pass 2: one bit per block of 16 centroids within tau of the minimum.  With off - (best + tau) in the C
    // operand a computed value is negative exactly where it is a candidate: the OR of a block's 16 results carries
    // that in its sign bit, which one v_alignbit shifts into the mask (block 32 wd + k lands in bit 31 - k).
    uint32_t cand[NQ][8];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const float b = __int_as_float(best[q]);
        bad[q] |= !(b > 0.f && b < 1.0e30f);
        const float d = off4[q][0] - (b + tau[q]);
        off4[q] = f32x4e{d, d, d, d};
    }
#pragma unroll
    for (int wd = 0; wd < 8; ++wd) {
        if (SPLIT && wd != wave)  // wave-uniform: this wavefront's word only
            continue;
        uint32_t bits[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q)
            bits[q] = 0u;
#pragma unroll 1
        for (int k = 0; k < 32; ++k) {  // block 32 wd + k: groups 4 (32 wd + k) .. + 3
            uint32_t any[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                any[q] = 0u;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const f32x4e d = values(4 * (32 * wd + k) + g4, q);
                    any[q] |= (__float_as_uint(d[0]) | __float_as_uint(d[1])) | (__float_as_uint(d[2]) | __float_as_uint(d[3]));
                }
            }
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                bits[q] = __builtin_amdgcn_alignbit(bits[q], any[q], 31);
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q)
            cand[q][wd] = bits[q];
        if (SPLIT) {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                xchg[(wave * NQ + q) * 64 + lane] = bits[q];
        }
    }
    if (SPLIT) {
        __syncthreads();
        if (wave != 0)
            return;  // wavefront 0 refines and stores for the workgroup
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int wd = 0; wd < 8; ++wd)
                cand[q][wd] = xchg[(wd * NQ + q) * 64 + lane];
    }

    // ---- refine / full scan, store
    double xd[4];
    auto exact = [&](int c, int &code, double &bd) {
        const f16x4 v = *(const f16x4 *)(arow + c * 16);
        double dist = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double diff = xd[j] - (double)(float)v[j];
            dist = __builtin_fma(diff, diff, dist);
        }
        code = dist < bd ? c : code;  // ascending callers, strict "<": the lowest index among equal distances stays
        bd = __builtin_fmin(bd, dist);
    };
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        // the token again (its registers were given up during the passes)
        const int u = (chunk * NQ + q) * 64 + lane;
        const int uu = live[q] ? u : 0;
        const int b = uu / n_new;
        const int t = uu - b * n_new;
        {
            const u32x2e raw = *(const u32x2e *)(x + ((((int64_t)b * Hkv + hkv) * x_head_stride + t) * PQ_HEAD_DIM + i * 4));
            const f16x4 v = __builtin_bit_cast(f16x4, raw);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xd[j] = (double)(float)v[j];
        }
        int cnt = 0, first = 0, last = 0;
#pragma unroll
        for (int wd = 7; wd >= 0; --wd) {
            const uint32_t wbits = cand[q][wd];
            cnt += __builtin_popcount(wbits);
            first = wbits ? 32 * wd + __builtin_clz(wbits) : first;
        }
#pragma unroll
        for (int wd = 0; wd < 8; ++wd) {
            const uint32_t wbits = cand[q][wd];
            last = wbits ? 32 * wd + 31 - __builtin_ctz(wbits) : last;
        }
        int code = 0;
        double bd = __builtin_huge_val();
        for (int k = 0; k < 16; ++k)
            exact(16 * first + k, code, bd);
        if (__builtin_amdgcn_ballot_w64(live[q] && cnt == 2) != 0) {  // wave-uniform; lanes with one block repeat it
            for (int k = 0; k < 16; ++k)
                exact(16 * last + k, code, bd);
        }
        // more than two marked blocks (a cluster of near-ties, a token far outside the codebook's range): this
        // lane walks all of its marked blocks, ascending — the nearest centroid and every tie lie in them
        const bool many = live[q] && !bad[q] && cnt > 2;
        if (__builtin_amdgcn_ballot_w64(many) != 0) {  // wave-uniform
            int code_m = 0;
            double bd_m = __builtin_huge_val();
#pragma unroll
            for (int wd = 0; wd < 8; ++wd) {
                uint32_t wbits = many ? cand[q][wd] : 0u;
                while (__builtin_amdgcn_ballot_w64(wbits != 0u) != 0) {  // block 32 wd + k sits in bit 31 - k
                    const int k32 = wbits ? __builtin_clz(wbits) : 0;
                    double bd_t = bd_m;
                    int code_t = code_m;
                    for (int k = 0; k < 16; ++k)
                        exact(16 * (32 * wd + k32) + k, code_t, bd_t);
                    if (wbits != 0u) {
                        bd_m = bd_t;
                        code_m = code_t;
                    }
                    wbits &= ~(0x80000000u >> k32);
                }
            }
            if (many) {
                code = code_m;
                bd = bd_m;
            }
        }
        const bool unsure = live[q] && (bad[q] || cnt < 1);
        if (__builtin_amdgcn_ballot_w64(unsure) != 0) {  // wave-uniform: the defining scan for this sub-chunk
            code = 0;
            bd = __builtin_huge_val();
            for (int c = 0; c < PQ12_CENTROIDS; ++c)
                exact(c, code, bd);
        }
        if (live[q])
            out[((((int64_t)b * Hkv + hkv) * n_new + t)) * PQ12_M + i] = (uint16_t)code;
    }
}

// ---------------------------------------------------------------------------------------------------
// A handful of tokens per KV head (one decoding step of a small batch): thread = CENTROID.  The filter kernel
// above would build 4096 rows and run both passes for a wavefront with a few live lanes; here the 1024 threads
// of a workgroup hold 4 centroids each in registers, evaluate the defining fp64 distances of the token at hand
// (ascending index per thread, strict "<") and the workgroup takes the lexicographic minimum of (distance,
// index): the lowest index among equal distances, as in the scan.  The floor is reading the codebooks once
// (64 MiB for K and V of 32 heads).  The code goes straight into the device layout — no staging, no packing
// kernels: a 12-bit field of a unit that other workgroups (K: the token's other subspaces) or nobody else in
// this call (V) writes, so it is cleared and set with two device-scope atomics per 32-bit word it touches;
// fields are disjoint, so the order of the workgroups does not matter.  Tokens beyond the capacity are not
// written (the length update flags them).
// ---------------------------------------------------------------------------------------------------
constexpr int FEW12_TOKENS = 16;  // capacity of the kernel
constexpr int FEW12_USED = 8;     // what the launcher gives it
constexpr int FEW12_WAVES = 16;

__global__ __launch_bounds__(FEW12_WAVES * 64) void pq12_encode_few_kernel(const __half *x0, const __half *x1,
                                                                          const __half *cb0, const __half *cb1,
                                                                          uint8_t *codes0, uint8_t *codes1,
                                                                          const int32_t *ctx_len, int B, int Hkv, int n_new,
                                                                          int64_t x_head_stride, int max_context,
                                                                          int64_t head_stride)
{
#pragma clang fp contract(off)
    static_assert(FEW12_TOKENS <= 64, "lane u fetches token u");
    __shared__ double red_d[FEW12_TOKENS][FEW12_WAVES];
    __shared__ int red_c[FEW12_TOKENS][FEW12_WAVES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int which = blockIdx.z;
    const int i = blockIdx.y;
    const int hkv = blockIdx.x;
    const int n_tok = B * n_new;  // <= FEW12_TOKENS
    const __half *x = which ? x1 : x0;
    const __half *cb = (which ? cb1 : cb0) + ((int64_t)hkv * PQ12_M + i) * PQ12_CENTROIDS * 4;
    uint8_t *codes = which ? codes1 : codes0;

    double c[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const u32x2e raw = *(const u32x2e *)(cb + (int64_t)(tid + 1024 * r) * 4);
        const f16x4 v = __builtin_bit_cast(f16x4, raw);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            c[r][j] = (double)(float)v[j];
    }
    // lane u < n_tok of every wavefront fetches token u's sub-vector
    const int u_mine = lane < n_tok ? lane : 0;
    const int b_mine = u_mine / n_new;
    const int t_mine = u_mine - b_mine * n_new;
    double x_mine[4];
    {
        const u32x2e raw = *(const u32x2e *)(x + ((((int64_t)b_mine * Hkv + hkv) * x_head_stride + t_mine) * PQ_HEAD_DIM + i * 4));
        const f16x4 v = __builtin_bit_cast(f16x4, raw);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            x_mine[j] = (double)(float)v[j];
    }

    for (int u = 0; u < n_tok; ++u) {
        double xv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xv[j] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x_mine[j]), u),
                                     __builtin_amdgcn_readlane(__double2loint(x_mine[j]), u));
        double bd = __builtin_huge_val();
        int bc = tid;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double dist = 0.0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double diff = xv[j] - c[r][j];
                dist = __builtin_fma(diff, diff, dist);
            }
            bc = dist < bd ? tid + 1024 * r : bc;  // ascending index inside the thread, strict "<"
            bd = __builtin_fmin(bd, dist);
        }
        wave_argmin(bd, bc);
        if (lane == 0) {
            red_d[u][wave] = bd;
            red_c[u][wave] = bc;
        }
    }
    __syncthreads();
    // wavefront u finishes token u: the 16 wavefronts' candidates sit in every row of 16 lanes
    if (wave < n_tok) {
        double d = red_d[wave][lane & (FEW12_WAVES - 1)];
        int cc = red_c[wave][lane & (FEW12_WAVES - 1)];
        wave_argmin(d, cc);
        if (lane == 0) {
            const int b = wave / n_new;
            const int t = wave - b * n_new;
            int p0 = ctx_len[b];
            p0 = p0 < 0 ? 0 : p0;
            const int64_t pos = (int64_t)p0 + t;
            if (pos < max_context) {
                int slot;
                const int64_t unit = which ? pq12_v_unit(pos, i, &slot) : pq12_k_unit(pos, i, &slot);
                unsigned int *w = (unsigned int *)(codes + ((int64_t)b * Hkv + hkv) * head_stride + unit);  // 3 words
                const int bit = 12 * slot;  // the field: bits bit .. bit + 11 of the 96
                const uint64_t field = (uint64_t)((uint32_t)cc & 0xfffu) << (bit & 31);
                const uint64_t mask = (uint64_t)0xfffu << (bit & 31);
                unsigned int *w0 = w + (bit >> 5);
                __hip_atomic_fetch_and(w0, ~(unsigned int)mask, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_fetch_or(w0, (unsigned int)field, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((mask >> 32) != 0) {  // the field runs into the next word
                    __hip_atomic_fetch_and(w0 + 1, ~(unsigned int)(mask >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_fetch_or(w0 + 1, (unsigned int)(field >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

// K units: one thread per (head, token j of the source, group of 8 subspaces)
__global__ void pq12_pack_k_kernel(const uint16_t *src, uint8_t *dst, const int32_t *pos0, int n, int Hkv, int max_context,
                                   int64_t head_stride, int64_t total)
{
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= total)
        return;
    const int g = (int)(x & 3);
    const int64_t j = (x >> 2) % n;
    const int64_t head = (x >> 2) / n;
    int64_t p0 = pos0 ? pos0[head / Hkv] : 0;
    p0 = p0 < 0 ? 0 : p0;
    const int64_t pos = p0 + j;
    if (pos >= max_context)
        return;
    uint32_t c[8], w[3];
#pragma unroll
    for (int s = 0; s < 8; ++s)
        c[s] = src[(head * n + j) * PQ12_M + 8 * g + s] & 0xfffu;
    pack8(c, w);
    int slot;
    uint32_t *d = (uint32_t *)(dst + head * head_stride + pq12_k_unit(pos, 8 * g, &slot));
    d[0] = w[0];
    d[1] = w[1];
    d[2] = w[2];
}

// V units: one thread per (head, 128-token block touched by the source, group of 4 subspaces, lane)
__global__ void pq12_pack_v_kernel(const uint16_t *src, uint8_t *dst, const int32_t *pos0, int n, int Hkv, int max_context,
                                   int64_t cap_padded, int64_t head_stride, int n_vb, int64_t total)
{
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= total)
        return;
    const int lane = (int)(x & 63);
    const int g = (int)((x >> 6) & 7);
    const int64_t vb_rel = (x >> 9) % n_vb;
    const int64_t head = (x >> 9) / n_vb;
    int64_t p0 = pos0 ? pos0[head / Hkv] : 0;
    p0 = p0 < 0 ? 0 : p0;
    const int64_t vblock = (p0 >> 7) + vb_rel;
    if (vblock * 128 >= cap_padded)
        return;
    const int sub = 4 * g + (lane & 3);
    bool any = false;
    int64_t jj[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int64_t tok = vblock * 128 + (lane >> 2) + 16 * k;
        const int64_t j = tok - p0;
        jj[k] = (j >= 0 && j < n && tok < max_context) ? j : -1;
        any = any || jj[k] >= 0;
    }
    if (!any)
        return;
    int slot;
    uint32_t *d = (uint32_t *)(dst + head * head_stride + pq12_v_unit(vblock * 128 + (lane >> 2), sub, &slot));
    uint32_t w[3] = {d[0], d[1], d[2]}, c[8];
    unpack8(w, c);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (jj[k] >= 0)
            c[k] = src[(head * n + jj[k]) * PQ12_M + sub] & 0xfffu;
    pack8(c, w);
    d[0] = w[0];
    d[1] = w[1];
    d[2] = w[2];
}

// one thread per code of the token-major tensor
__global__ void pq12_unpack_kernel(const uint8_t *packed, uint16_t *token_major, int kind, int n, int64_t head_stride,
                                   int64_t total)
{
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= total)
        return;
    const int i = (int)(x % PQ12_M);
    const int64_t t = (x / PQ12_M) % n;
    const int64_t head = x / ((int64_t)PQ12_M * n);
    int slot;
    const int64_t unit = kind == PQ_CODES_K ? pq12_k_unit(t, i, &slot) : pq12_v_unit(t, i, &slot);
    const uint8_t *b = packed + head * head_stride + unit + ((3 * slot) >> 1);
    const uint32_t two = (uint32_t)b[0] | ((uint32_t)b[1] << 8);
    token_major[x] = (uint16_t)((two >> (4 * (slot & 1))) & 0xfffu);
}

hipError_t launch_pack(const pq_attn_ctx *ctx, int kind, const uint16_t *src, int n, uint8_t *dst, const int32_t *pos0,
                       hipStream_t s)
{
    const int64_t heads = (int64_t)ctx->cfg.batch * ctx->cfg.n_kv_heads;
    const int64_t head_stride = ctx->cap_padded * PQ12_TOKEN_BYTES;
    if (n == 0)
        return hipSuccess;
    if (kind == PQ_CODES_K) {
        const int64_t total = heads * n * 4;
        hipLaunchKernelGGL(pq12_pack_k_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src, dst, pos0, n,
                           ctx->cfg.n_kv_heads, ctx->cfg.max_context, head_stride, total);
    } else {
        const int n_vb = ((n + 127) >> 7) + 1;
        const int64_t total = heads * n_vb * 512;
        hipLaunchKernelGGL(pq12_pack_v_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src, dst, pos0, n,
                           ctx->cfg.n_kv_heads, ctx->cfg.max_context, ctx->cap_padded, head_stride, n_vb, total);
    }
    return hipGetLastError();
}

}  // namespace

bool pq_config_is_12bit(const pq_attn_config *cfg) { return cfg->n_centroids == PQ12_CENTROIDS; }

hipError_t pq12_launch_pack_codes(const pq_attn_ctx *ctx, int kind, const uint16_t *token_major, int n_tokens,
                                  uint8_t *packed, bool unpack, hipStream_t s)
{
    if (!unpack)
        return launch_pack(ctx, kind, token_major, n_tokens, packed, nullptr, s);
    const int64_t heads = (int64_t)ctx->cfg.batch * ctx->cfg.n_kv_heads;
    const int64_t total = heads * n_tokens * PQ12_M;
    if (total == 0)
        return hipSuccess;
    hipLaunchKernelGGL(pq12_unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, packed,
                       const_cast<uint16_t *>(token_major), kind, n_tokens, ctx->cap_padded * PQ12_TOKEN_BYTES, total);
    return hipGetLastError();
}

hipError_t pq12_launch_encode_append(const pq_attn_ctx *ctx, const pq_encode_args &a, int64_t x_rows, int32_t *ctx_len,
                                     unsigned int *dev_err, hipStream_t s)
{
    const int64_t n_tok = (int64_t)a.B * a.n_new;  // tokens of a head over all sequences
    // measured, 32 heads, one new token per sequence: 1 sequence 17 us, 8 sequences 62 us with the kernel below
    // (6.6 us per token: fp64 arithmetic); 17 .. 64 sequences 74 .. 82 us with the split filter kernel
    if (n_tok <= FEW12_USED) {
        // a decoding step: encode and write the device layouts in one kernel, then the lengths
        hipLaunchKernelGGL(pq12_encode_few_kernel, dim3((unsigned)a.Hkv, PQ12_M, 2), dim3(FEW12_WAVES * 64), 0, s,
                           (const __half *)a.x[0], (const __half *)a.x[1], (const __half *)a.codebook[0],
                           (const __half *)a.codebook[1], a.codes[0], a.codes[1], a.ctx_len, a.B, a.Hkv, a.n_new, x_rows,
                           a.max_context, ctx->cap_padded * PQ12_TOKEN_BYTES);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        return pq_launch_bump_len(ctx_len, a.B, a.n_new, a.max_context, dev_err, s);
    } else if (n_tok <= 128) {
        // a decoding step of a batch: one sub-chunk per head, its centroids split over the workgroup's wavefronts
        const dim3 grid((unsigned)a.Hkv, PQ12_M, 2);
        if (n_tok > 64)
            hipLaunchKernelGGL((pq12_encode_fast_kernel<2, true>), grid, dim3(F12_WAVES * 64), 0, s, (const __half *)a.x[0],
                               (const __half *)a.x[1], (const __half *)a.codebook[0], (const __half *)a.codebook[1],
                               ctx->stage[0], ctx->stage[1], a.B, a.Hkv, a.n_new, 1, x_rows);
        else
            hipLaunchKernelGGL((pq12_encode_fast_kernel<1, true>), grid, dim3(F12_WAVES * 64), 0, s, (const __half *)a.x[0],
                               (const __half *)a.x[1], (const __half *)a.codebook[0], (const __half *)a.codebook[1],
                               ctx->stage[0], ctx->stage[1], a.B, a.Hkv, a.n_new, 1, x_rows);
    } else if (n_tok < ((int64_t)1 << 30)) {
        // matrix-core filter: 8 wavefronts per workgroup, each takes 64 NQ tokens of the head
        const int nq = n_tok > 64 * F12_WAVES ? 2 : 1;
        const int groups_per_head = (int)((n_tok + 64 * nq * F12_WAVES - 1) / (64 * nq * F12_WAVES));
        const dim3 grid((unsigned)(a.Hkv * groups_per_head), PQ12_M, 2);
        if (nq == 2)
            hipLaunchKernelGGL((pq12_encode_fast_kernel<2, false>), grid, dim3(F12_WAVES * 64), 0, s, (const __half *)a.x[0],
                               (const __half *)a.x[1], (const __half *)a.codebook[0], (const __half *)a.codebook[1],
                               ctx->stage[0], ctx->stage[1], a.B, a.Hkv, a.n_new, groups_per_head, x_rows);
        else
            hipLaunchKernelGGL((pq12_encode_fast_kernel<1, false>), grid, dim3(F12_WAVES * 64), 0, s, (const __half *)a.x[0],
                               (const __half *)a.x[1], (const __half *)a.codebook[0], (const __half *)a.codebook[1],
                               ctx->stage[0], ctx->stage[1], a.B, a.Hkv, a.n_new, groups_per_head, x_rows);
    } else {
        const int n_chunks = (a.n_new + 63) >> 6;
        const int groups_per_head = (a.B * n_chunks + E12_WAVES - 1) / E12_WAVES;
        const dim3 grid((unsigned)(a.Hkv * groups_per_head), PQ12_M, 2);
        hipLaunchKernelGGL(pq12_encode_kernel, grid, dim3(E12_WAVES * 64), 0, s, (const __half *)a.x[0],
                           (const __half *)a.x[1], (const __half *)a.codebook[0], (const __half *)a.codebook[1],
                           ctx->stage[0], ctx->stage[1], a.B, a.Hkv, a.n_new, groups_per_head, x_rows);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    e = launch_pack(ctx, PQ_CODES_K, ctx->stage[0], a.n_new, a.codes[0], a.ctx_len, s);
    if (e != hipSuccess)
        return e;
    e = launch_pack(ctx, PQ_CODES_V, ctx->stage[1], a.n_new, a.codes[1], a.ctx_len, s);
    if (e != hipSuccess)
        return e;
    // the lengths move only after both packing kernels have read the old ones (stream order)
    return pq_launch_bump_len(ctx_len, a.B, a.n_new, a.max_context, dev_err, s);
}

// ---------------------------------------------------------------------------------------------------
// Offline codebook training for 4096 centroids: the Lloyd iteration of pq_kmeans.hip with the assignment done
// by the encode kernel above (chunks of the samples, codes staged in the workspace) and the exact 64-bit
// integer member sums added straight to memory (a subspace has 4096 x 4 sums: they do not fit in LDS, and
// with that many addresses the atomics hardly collide).
// ---------------------------------------------------------------------------------------------------
namespace {

constexpr int KM12_CHUNK = 8192;  // samples per head and assignment launch

// one thread per (head, sample of the chunk, subspace)
__global__ void pq12_kmeans_accumulate_kernel(const __half *samples, const uint16_t *codes, unsigned long long *sums,
                                              unsigned int *counts, int64_t head_stride, int nc, int64_t total)
{
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= total)
        return;
    const int i = (int)(x & (PQ12_M - 1));
    const int64_t tok = (x >> 5) % nc;
    const int64_t head = (x >> 5) / nc;
    const uint32_t c = codes[x] & 0xfffu;
    const __half *v = samples + (head * head_stride + tok) * PQ_HEAD_DIM + i * 4;
    const int64_t e = (head * PQ12_M + i) * PQ12_CENTROIDS + c;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        // exact: an fp16 value times 2^24 is an integer below 2^41 in magnitude
        const long long fixed = (long long)(__half2float(v[j]) * 16777216.0f);
        atomicAdd(&sums[e * 4 + j], (unsigned long long)fixed);
    }
    atomicAdd(&counts[e], 1u);
}

}  // namespace

int64_t pq12_kmeans_workspace_bytes(const pq_attn_ctx *ctx)
{
    const int64_t n = (int64_t)ctx->cfg.n_kv_heads * PQ12_M * PQ12_CENTROIDS;
    return n * 4 * 8 + n * 4 + (int64_t)ctx->cfg.n_kv_heads * KM12_CHUNK * PQ12_M * 2;
}

hipError_t pq12_launch_kmeans(const pq_attn_ctx *ctx, const void *samples, int n_samples, void *codebook, int n_iters,
                              void *workspace, hipStream_t s)
{
    const int Hkv = ctx->cfg.n_kv_heads;
    const int64_t n = (int64_t)Hkv * PQ12_M * PQ12_CENTROIDS;
    unsigned long long *sums = (unsigned long long *)workspace;
    unsigned int *counts = (unsigned int *)(sums + n * 4);
    uint16_t *codes = (uint16_t *)(counts + n);
    hipError_t e = pq_launch_clear_words(workspace, (n * 4 * 8 + n * 4) / 4, s);
    if (e != hipSuccess)
        return e;
    for (int it = 0; it < n_iters; ++it) {
        for (int c0 = 0; c0 < n_samples; c0 += KM12_CHUNK) {
            const int nc = n_samples - c0 < KM12_CHUNK ? n_samples - c0 : KM12_CHUNK;
            const __half *x = (const __half *)samples + (int64_t)c0 * PQ_HEAD_DIM;
            // assignment = the encode's matrix-core filter (one sequence, grid.z = 1: only the first pointers are used)
            const int groups_per_head = (nc + 128 * F12_WAVES - 1) / (128 * F12_WAVES);
            hipLaunchKernelGGL((pq12_encode_fast_kernel<2, false>), dim3((unsigned)(Hkv * groups_per_head), PQ12_M, 1),
                               dim3(F12_WAVES * 64), 0, s, x, x, (const __half *)codebook, (const __half *)codebook, codes,
                               codes, 1, Hkv, nc, groups_per_head, (int64_t)n_samples);
            const int64_t total = (int64_t)Hkv * nc * PQ12_M;
            hipLaunchKernelGGL(pq12_kmeans_accumulate_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, codes,
                               sums, counts, (int64_t)n_samples, nc, total);
        }
        e = pq_launch_kmeans_update(codebook, sums, counts, n, 4, s);
        if (e != hipSuccess)
            return e;
    }
    return hipGetLastError();
}
