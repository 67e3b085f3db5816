// Decode attention over a KV cache quantized with 12-bit PQ codes (M = 32 subspaces of 4 dims, 4096
// centroids: Section IV-A) for GROUPED queries — 2..4 query heads per workgroup read one KV head — one
// fused kernel.
//
// Same result as the per-head 12-bit kernel (Eq. 7 = Eq. 6), different evaluation.  There every query head
// builds its own score tables and walks the KV head's codes by itself: G times the table refills and G times
// the LDS gathers, which are what bounds that kernel.  Here a KV head's codes are gathered ONCE for the
// group, from the CODEBOOKS (not from per-query tables), and the contraction over the query heads goes to
// the matrix cores.  A subspace of 4 dims is exactly the inner dimension of v_mfma_f32_4x4x4_16B_f16, so a
// gathered centroid (8 bytes) is an operand as it comes out of LDS:
//
//   score passes  8 slices of 4 subspaces: a slice of the KEY codebook [4][4096][4] fp16 (128 KiB) is
//                 copied to LDS.  Lane (quad s, row i) gathers the centroid of token s + 16 i of a
//                 64-token block: A = the quad's 4 tokens x 4 dims, B = the 4 query heads' slice of this
//                 subspace (lane j: head j), so D[token][head] lands with lane j holding head j's scores of
//                 the quad's 4 tokens — which is the A operand layout of the value passes, no transposition.
//                 One gather and one matrix instruction per (token, subspace) serve all heads.
//   softmax       all scores of the round exist before the first weight is needed: maximum per head over the
//                 workgroup (running maximum / rescale only between rounds), weights split into fp16 hi + lo
//                 (p = hi + lo to 2^-22 relative) in the registers that held the scores.
//   value passes  8 groups of 4 subspaces: the slice of the VALUE codebook goes to LDS; lane (s, j) gathers
//                 subspace j of the tokens s + 16 k of a 128-token block (its 12-byte unit), re-packs 4
//                 tokens x 4 dims into one B operand per dim (8 x v_perm) and accumulates
//                 D[head][lane's subspace, dim] += weights[head][4 tokens] x B — hi and lo — for all heads.
//                 The 16 token streams (quads) are summed at the end of each slice — DPP inside rows of 16
//                 lanes, a small LDS buffer across rows and wavefronts — into an fp32 output tile in LDS.
// The K and V code layouts are those of the per-head kernel (pq_internal.h); a K unit holds 8 subspaces and
// serves two consecutive score passes from registers, so each code byte still leaves HBM once.  Recent rows,
// split partials, ticket and merge follow the 8-bit grouped kernel.  What binds the kernel is not HBM but the
// 16 slices (2 MiB) every workgroup pulls out of L2 per round of tokens (see the round loop for the schedule).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_device_utils.h"

namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int GN = 8;                            // wavefronts per workgroup: 2 per SIMD, 256 registers each (a slice on
                                                 // its way takes 64 of them, the round's scores, weights and code units
                                                 // most of the rest; with 16 wavefronts of 128 registers the kernel
                                                 // spilled, and a reload from scratch waits for every request in flight)
constexpr int GH = 4;                            // rows of the 4x4x4 instruction = query heads per workgroup
constexpr int G12_TAB = 0;                       // 128 KiB: codebook slice [4 subspaces][4096][4] fp16
constexpr int G12_Q = 131072;                    // fp16 q [4][128] (heads beyond the group: zero rows)
constexpr int G12_O = G12_Q + GH * 256;          // float [4][128]: the scan's un-normalised output rows
constexpr int G12_WMAX = G12_O + GH * 512;       // float [8][4]: a round's maxima per wavefront and head
constexpr int G12_LW = G12_WMAX + GN * GH * 4;   // float [8][4]: weight sums per wavefront and head
constexpr int G12_RED = G12_LW + GN * GH * 4;    // float [8 wavefronts][4 rows of 16 lanes][16 values][4 subspaces]: a value
                                                 // pass's sums per wavefront and lane row, folded into the tile a phase later
constexpr int G12_FLAG = G12_RED + GN * 4 * 64 * 4;  // int: "this workgroup drew the last ticket"
constexpr int G12_BYTES = G12_FLAG + 16;
// wavefront partials of the recent rows float [8][4][PQ_PART_STRIDE] reuse the table once the scan is over
constexpr int G12_PART = G12_TAB;
static_assert(GN * GH * PQ_PART_STRIDE * 4 <= 131072, "partials fit in the table region");
static_assert(G12_BYTES <= 160 * 1024, "LDS budget of a gfx950 compute unit");

__device__ inline f16x4 f16x4_of(uint32_t lo, uint32_t hi)
{
    u32x2 v = {lo, hi};
    return __builtin_bit_cast(f16x4, v);
}

__device__ inline void unpack8g(const uint32_t w0, const uint32_t w1, const uint32_t w2, uint32_t (&c)[8])
{
    c[0] = w0 & 0xfffu;
    c[1] = (w0 >> 12) & 0xfffu;
    c[2] = ((w0 >> 24) | (w1 << 8)) & 0xfffu;
    c[3] = (w1 >> 4) & 0xfffu;
    c[4] = (w1 >> 16) & 0xfffu;
    c[5] = ((w1 >> 28) | (w2 << 4)) & 0xfffu;
    c[6] = (w2 >> 8) & 0xfffu;
    c[7] = w2 >> 20;
}

// sum / maximum over the 16 lanes of the wavefront that share lane % 4 (one head, or one subspace)
__device__ inline float sum_same_row_in_dpp_row(float x)
{
    x += dpp_move<0x124>(x);  // row_ror:4
    x += dpp_move<0x128>(x);  // row_ror:8
    return x;
}

__device__ inline float max_same_row(float x)
{
    x = fmaxf(x, dpp_move<0x124>(x));
    x = fmaxf(x, dpp_move<0x128>(x));
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}

// One 12-byte code unit: wave-uniform base (scalar registers) + this lane's 32-bit byte offset
template <bool NT> __device__ inline void load_unit(uint32_t (&dst)[3], const uint8_t *uniform_base, uint32_t lane_off)
{
    typedef __attribute__((address_space(1))) const char global_char;
    typedef __attribute__((address_space(1))) const uint32_t global_u32;
    uint64_t base = (uint64_t)uniform_base;
    asm("" : "+s"(base));  // stays a scalar base: the compiler does not fold it into a per-lane 64-bit address
    global_u32 *p = (global_u32 *)((global_char *)base + lane_off);
#pragma unroll
    for (int e = 0; e < 3; ++e)
        dst[e] = NT ? __builtin_nontemporal_load(p + e) : p[e];
}

constexpr int SLICE_VEC = 131072 / (GN * 64 * 16);  // 16-byte pieces of a slice per thread

// A 128 KiB codebook slice travels to the table region in two steps, a phase apart: requested into registers
// (16 x 16 bytes per thread, from L2 after the first workgroup of the XCD) as soon as the previous slice has been
// stored, and stored to LDS once every wavefront has left the gathers of the previous phase.
// PART / PARTS: the pieces PART * SLICE_VEC / PARTS .. of the slice (the requests of a slice are spread over the
// phase's scan, a few before each block: a wavefront that issues all 16 at once sits in front of the compute
// unit's address pipeline for most of a microsecond before its first gather)
template <int PART, int PARTS>
__device__ inline void slice_request(u32x4 (&t)[SLICE_VEC], const __half *slice, int tid)
{
    // the slice address is wave-uniform: kept in scalar registers, one 32-bit lane offset for all pieces (the
    // builtin returns a signed int: widen through uint32_t, or a low word with bit 31 set would sign-extend
    // into the high word)
    const uint64_t p = (uint64_t)slice;
    const uint32_t p_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
    const uint32_t p_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    typedef __attribute__((address_space(1))) const char global_char;  // a global, not a generic, address
    typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
    global_char *base = (global_char *)(((uint64_t)p_hi << 32) | (uint64_t)p_lo);
    const uint32_t off = (uint32_t)tid * 16u;
#pragma unroll
    for (int k = PART * (SLICE_VEC / PARTS); k < (PART + 1) * (SLICE_VEC / PARTS); ++k) {
        uint64_t piece = (uint64_t)base + (uint64_t)(k * (GN * 64 * 16));
        asm("" : "+s"(piece));  // a scalar base per piece + the common lane offset, not eight per-lane 64-bit addresses
        t[k] = *(global_u32x4 *)((global_char *)piece + off);
    }
}

__device__ inline void slice_store(lds_u8 *lbase, const u32x4 (&t)[SLICE_VEC], int tid)
{
#pragma unroll
    for (int k = 0; k < SLICE_VEC; ++k)
        *(lds_u32x4 *)(lbase + G12_TAB + (tid + k * (GN * 64)) * 16) = t[k];
}

// WAVE_VB: 128-token blocks per wavefront and round (8 score registers per lane each); a workgroup takes
// 8 WAVE_VB blocks per round.  READ_ONCE: one workgroup per (sequence, KV head, split) reads the codes, so
// they stream with the non-temporal hint; with more than 4 query heads per KV head several workgroups share
// the stream through their XCD's L2 and load normally.
template <int WAVE_VB, bool READ_ONCE>
__global__ __launch_bounds__(GN * 64) void pq12_decode_grouped_kernel(const pq_decode_args a)
{
    constexpr int ROUND_VB = GN * WAVE_VB;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[G12_BYTES];
    lds_u8 *lbase = (lds_u8 *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const uint32_t grid = gridDim.x;
    uint32_t logical = blockIdx.x;
    if ((grid & 7u) == 0)
        logical = (blockIdx.x & 7u) * (grid >> 3) + (blockIdx.x >> 3);
    const int S = a.S;
    // neighbours on an XCD: the splits of a (sequence, KV head, sub-group of G query heads), the sub-groups of the
    // KV head, then the same KV head of the other sequences (they stage the same codebook slices from L2)
    const int unit = (int)(logical / (uint32_t)S);
    const int split = (int)(logical - (uint32_t)unit * (uint32_t)S);
    const int n_sub = a.n_sub;
    const int hb = (int)((uint32_t)unit / (uint32_t)n_sub);  // hkv * B + b
    const int sub_group = unit - hb * n_sub;
    const int hkv = (int)((uint32_t)hb / (uint32_t)a.B);
    const int b = hb - hkv * a.B;
    const int bkv = b * a.Hkv + hkv;
    // the KV head's a.G query heads in n_sub sub-groups whose sizes differ by at most one: this workgroup's heads
    // are g_first .. g_first + G - 1, G = 2..4
    const int g_base = a.G / n_sub, g_rem = a.G - g_base * n_sub;
    const int G = g_base + (sub_group < g_rem ? 1 : 0);
    const int g_first = sub_group * g_base + (sub_group < g_rem ? sub_group : g_rem);
    const int bh0 = b * a.Hq + hkv * a.G + g_first;  // first query head of this workgroup

    int N = a.ctx_len[b];
    int R = (a.recent_k != nullptr && a.recent_len != nullptr) ? a.recent_len[b] : 0;
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    R = R < 0 ? 0 : (R > a.max_recent ? a.max_recent : R);
    const uint32_t nvb = (uint32_t)(N + 127) >> 7;  // 128-token blocks of the sequence
    const int vb0 = (int)(nvb * (uint32_t)split / (uint32_t)S);
    const int vb1 = (int)(nvb * (uint32_t)(split + 1) / (uint32_t)S);
    const int r0 = (int)((uint32_t)R * (uint32_t)split / (uint32_t)S);
    const int r1 = (int)((uint32_t)R * (uint32_t)(split + 1) / (uint32_t)S);

    const uint8_t *k_head = a.k_codes + (int64_t)bkv * a.head_stride;
    const uint8_t *v_head = a.v_codes + (int64_t)bkv * a.head_stride;
    const __half *kcb = (const __half *)a.kcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;
    const __half *vcb = (const __half *)a.vcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;

    // the group's queries (fp16 as they come: the products with fp16 centroids are exact in the fp32
    // accumulator; the softmax scale is applied to the finished score) and a zeroed output tile
    if (tid < 64) {
        u32x4 qraw = {0u, 0u, 0u, 0u};
        if (tid < 16 * G)
            qraw = *((const u32x4 *)((const __half *)a.q + (int64_t)bh0 * PQ_HEAD_DIM) + tid);
        *(lds_u32x4 *)(lbase + G12_Q + tid * 16) = qraw;
    }
    lds_f32 *o_lds = (lds_f32 *)(lbase + G12_O);
    lds_f32 *wmax = (lds_f32 *)(lbase + G12_WMAX);
    if (tid < GH * 128)
        o_lds[tid] = 0.f;

    const int quad = lane >> 2;  // the 4x4x4 block of this lane: a stream of tokens (token % 16)
    const int row = lane & 3;    // query head (as the holder of scores and weights); subspace of the group (value passes)
    // score passes: this lane gathers token quad + 16 row of a 64-token block
    // K units are requested lane = token (one contiguous 768-byte piece per wavefront and load) and handed to the
    // lane that gathers the token — lane (quad, row) takes token quad + 16 row — by a lane permutation when the
    // pass starts; requested in gather order, the 4 lanes of a quad touch 4 separate lines and the loads issue
    // several times slower
    const uint32_t unit_lane_off = (uint32_t)lane * 12u;
    const int k_src_lane4 = (quad + 16 * row) * 4;
    const uint32_t v_tab = (uint32_t)(G12_TAB + row * (PQ12_CENTROIDS * 8));

    float m_run[GH];           // running maxima, the same in every wavefront of the workgroup
    float l_lane = 0.f;        // this lane's share of head `row`'s weight sum
#pragma unroll
    for (int g = 0; g < GH; ++g)
        m_run[g] = NEG_BIG;

    // A value pass leaves, per wavefront and row of 16 lanes, the sums of its 64 outputs (4 heads x 4 subspaces x 4
    // dims) in LDS; after the next barrier 4 wavefronts fold the 32 partial sums of each output into the tile.
    lds_f32 *red = (lds_f32 *)(lbase + G12_RED);
    auto fold = [&](const int gv) {
        if (wave < 4) {  // output o = lane: value v = o / 4 (dim d = v / 4, head g = v % 4), subspace j = o % 4
            float sum = 0.f;
#pragma unroll
            for (int p = 0; p < GN; ++p)  // partials (wavefront, lane row) 8 wave .. 8 wave + 7
                sum += red[(wave * GN + p) * 64 + lane];
            const int v = lane >> 2, j = lane & 3;
            __hip_atomic_fetch_add((float *)(o_lds + (v & 3) * 128 + (4 * gv + j) * 4 + (v >> 2)), sum, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };

    // A round is 8 double phases: 4 groups of 8 key subspaces, then 4 pairs of value groups, each double phase two
    // phases over one table slice (4 subspaces) each.  Everything comes from memory ahead of its use:
    //   * the next slice is requested into registers during the scan of the current one, a quarter of its 16
    //     pieces in front of each block (a wavefront that issues all of them at once sits in front of the
    //     compute unit's address pipeline for most of a microsecond), and stored once everybody has left the
    //     current scan;
    //   * the code units of a double phase — 2 WAVE_VB of them either way: a K unit holds a token's 8 subspaces,
    //     V units of two groups belong to one double phase — are requested during the FIRST phase of the double
    //     phase before, and BEHIND that phase's slice requests: they come from HBM, loads return in order, and
    //     in front of the slice requests they hold the slice (L2 hits) back for a memory round trip.
    // Every request is unconditional and their number per phase is fixed, so the waits count exactly: the store of
    // a slice waits for the slice and not for the units requested behind it.
    u32x4 sl[SLICE_VEC];
    uint32_t un[2 * WAVE_VB][3];
    // double phase dp of the round that starts at block sb_: dp 0..3 = key unit group dp, 4..7 = value groups
    // 2 (dp - 4), + 1; dp = 8 is the next round's dp 0
    auto units_request = [&](int sb_, int dp, const int last_vb) {
        if (dp == 8) {  // wave-uniform selects, no branch
            sb_ += ROUND_VB;
            dp = 0;
        }
        const bool is_k = dp < 4;
#pragma unroll
        for (int jj = 0; jj < WAVE_VB; ++jj) {
            const int want = sb_ + wave + GN * jj;
            const int vb = want < last_vb ? want : last_vb;  // beyond the wavefront's blocks: a valid block, not used
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int64_t unit = is_k ? ((int64_t)(2 * vb + x) * 4 + dp) * 64 : ((int64_t)vb * 8 + 2 * (dp - 4) + x) * 64;
                load_unit<READ_ONCE>(un[2 * jj + x], (is_k ? k_head : v_head) + unit * 12, unit_lane_off);
            }
        }
    };
    // part jj of the next slice's requests, in front of block jj of the scan (pinned there)
    auto request_part = [&](const int jj, const __half *slice) {
        if (jj == 0) slice_request<0, WAVE_VB>(sl, slice, tid);
        if (jj == 1) slice_request<1 % WAVE_VB, WAVE_VB>(sl, slice, tid);
        if (jj == 2) slice_request<2 % WAVE_VB, WAVE_VB>(sl, slice, tid);
        if (jj == 3) slice_request<3 % WAVE_VB, WAVE_VB>(sl, slice, tid);
        __builtin_amdgcn_sched_barrier(0);
    };
    if (vb0 < vb1) {
        units_request(vb0, 0, vb1 - 1);
        slice_request<0, 1>(sl, kcb, tid);
    }

    for (int sb = vb0; sb < vb1; sb += ROUND_VB) {
        // wavefront w owns blocks sb + w + 8 jj, jj < n_jj
        const int left = vb1 - sb - wave;
        const int n_jj = left <= 0 ? 0 : (left + GN - 1) / GN < WAVE_VB ? (left + GN - 1) / GN : WAVE_VB;
        const int last_vb = vb1 - 1;
        f32x4 score[2 * WAVE_VB];     // element r: token quad + 16 r of the 64-token half block, head `row`
        u32x4 wt[2 * WAVE_VB];        // the same tokens' weights as A operands: fp16 hi (x, y) and lo (z, w)
#pragma unroll
        for (int e = 0; e < 2 * WAVE_VB; ++e)
            score[e] = f32x4{0.f, 0.f, 0.f, 0.f};

        // ---------------- score passes: 4 unit groups of 8 subspaces, two table slices of 4 subspaces each
#pragma nounroll
        for (int g = 0; g < 4; ++g) {
            // the units were requested lane = token; lane (quad, row) gathers token quad + 16 row
            uint32_t ku[2 * WAVE_VB][3];
#pragma unroll
            for (int e = 0; e < 2 * WAVE_VB; ++e)
#pragma unroll
                for (int x = 0; x < 3; ++x)
                    ku[e][x] = (uint32_t)__builtin_amdgcn_ds_bpermute(k_src_lane4, (int)un[e][x]);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                __syncthreads();  // the table region is free (and, the first time, the queries are in LDS)
                if (g == 0 && hf == 0 && sb > vb0)
                    fold(7);  // the previous round's last value pass
                slice_store(lbase, sl, tid);
                __syncthreads();
                const __half *next_slice = hf == 0   ? kcb + (int64_t)(8 * g + 4) * PQ12_CENTROIDS * 4
                                           : g < 3 ? kcb + (int64_t)(8 * g + 8) * PQ12_CENTROIDS * 4
                                                   : vcb;
                f16x4 qb[4];  // B operands: head `row`'s query slice of the 4 resident subspaces
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    qb[j] = __builtin_bit_cast(f16x4, *(lds_u32x2 *)(lbase + G12_Q + row * 256 + (8 * g + 4 * hf + j) * 8));
#pragma unroll
                for (int jj = 0; jj < WAVE_VB; ++jj) {
                    request_part(jj, next_slice);
                    if (jj >= n_jj)
                        continue;  // wave-uniform; `continue`, not `break`: the loop must unroll (registers are indexed by jj)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        uint32_t c[8];
                        unpack8g(ku[2 * jj + h][0], ku[2 * jj + h][1], ku[2 * jj + h][2], c);
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const u32x2 cv = *(lds_u32x2 *)(lbase + G12_TAB + j * (PQ12_CENTROIDS * 8) + c[4 * hf + j] * 8);
                            score[2 * jj + h] =
                                __builtin_amdgcn_mfma_f32_4x4x4f16(f16x4_of(cv.x, cv.y), qb[j], score[2 * jj + h], 0, 0, 0);
                        }
                    }
                }
                if (hf == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    units_request(sb, g + 1, last_vb);
                }
            }
        }

        // ---------------- softmax of the round, per head: the scores become fp16 hi / lo weights
        float mx = NEG_BIG;
#pragma unroll
        for (int jj = 0; jj < WAVE_VB; ++jj)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int tok = (sb + wave + GN * jj) * 128 + 64 * h + quad + 16 * r;
                    const bool valid = jj < n_jj && tok < N;
                    const float s = valid ? score[2 * jj + h][r] * a.scale_log2e : NEG_BIG;
                    score[2 * jj + h][r] = s;
                    mx = fmaxf(mx, s);
                }
        mx = max_same_row(mx);
        if (lane < GH)
            wmax[wave * GH + lane] = mx;
        __syncthreads();
        float alpha[GH];
#pragma unroll
        for (int g = 0; g < GH; ++g) {
            float mw = NEG_BIG;
#pragma unroll
            for (int w = 0; w < GN; ++w)
                mw = fmaxf(mw, wmax[w * GH + g]);
            const float m_new = fmaxf(m_run[g], mw);
            alpha[g] = __builtin_amdgcn_exp2f(m_run[g] - m_new);
            m_run[g] = m_new;
        }
        const float m_own = row == 0 ? m_run[0] : row == 1 ? m_run[1] : row == 2 ? m_run[2] : m_run[3];
        const float a_own = row == 0 ? alpha[0] : row == 1 ? alpha[1] : row == 2 ? alpha[2] : alpha[3];
        l_lane *= a_own;
        {  // the output tile of head wave / 2 follows the new maximum (nobody adds to it before the next barrier)
            const int hh = wave >> 1;
            const float a_h = hh == 0 ? alpha[0] : hh == 1 ? alpha[1] : hh == 2 ? alpha[2] : alpha[3];
            o_lds[tid] *= a_h;
        }
#pragma unroll
        for (int e = 0; e < 2 * WAVE_VB; ++e) {
            _Float16 hi[4], lo[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // an invalid token carries NEG_BIG; against a finite maximum that is weight 0, and a round whose
                // maximum is NEG_BIG itself has no valid token at all
                const float p = score[e][r] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(score[e][r] - m_own) : 0.f;
                l_lane += p;
                hi[r] = (_Float16)p;
                lo[r] = (_Float16)(p - (float)hi[r]);
            }
            const f16x4 vh = {hi[0], hi[1], hi[2], hi[3]}, vl = {lo[0], lo[1], lo[2], lo[3]};
            const u32x2 bh = __builtin_bit_cast(u32x2, vh), bl = __builtin_bit_cast(u32x2, vl);
            wt[e] = u32x4{bh.x, bh.y, bl.x, bl.y};
        }

        // ---------------- value passes: 4 pairs of groups of 4 subspaces
#pragma nounroll
        for (int u = 0; u < 4; ++u) {
            uint32_t vu[2 * WAVE_VB][3];
#pragma unroll
            for (int e = 0; e < 2 * WAVE_VB; ++e)
#pragma unroll
                for (int x = 0; x < 3; ++x)
                    vu[e][x] = un[e][x];
#pragma unroll
            for (int x2 = 0; x2 < 2; ++x2) {
                const int gv = 2 * u + x2;
                __syncthreads();  // the table region is free
                if (gv > 0)
                    fold(gv - 1);
                slice_store(lbase, sl, tid);
                __syncthreads();
                // after the last group: the next round's first slice (after the last round: requested, never used)
                const __half *next_slice = gv < 7 ? vcb + (int64_t)(4 * gv + 4) * PQ12_CENTROIDS * 4 : kcb;
                f32x4 acc[4];  // acc[d][g]: head g, dim d of subspace 4 gv + row, this quad's tokens
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < WAVE_VB; ++jj) {
                    request_part(jj, next_slice);
                    if (jj >= n_jj)
                        continue;
                    uint32_t c[8];
                    unpack8g(vu[2 * jj + x2][0], vu[2 * jj + x2][1], vu[2 * jj + x2][2], c);
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        u32x2 cv[4];  // tokens quad + 16 k of the half block, k = 0..3: dims (0, 1) and (2, 3)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            cv[k] = *(lds_u32x2 *)(lbase + v_tab + c[4 * h + k] * 8);
                        f16x4 B[4];  // per dim: the 4 tokens' values
                        B[0] = f16x4_of(__builtin_amdgcn_perm(cv[1].x, cv[0].x, 0x05040100u),
                                        __builtin_amdgcn_perm(cv[3].x, cv[2].x, 0x05040100u));
                        B[1] = f16x4_of(__builtin_amdgcn_perm(cv[1].x, cv[0].x, 0x07060302u),
                                        __builtin_amdgcn_perm(cv[3].x, cv[2].x, 0x07060302u));
                        B[2] = f16x4_of(__builtin_amdgcn_perm(cv[1].y, cv[0].y, 0x05040100u),
                                        __builtin_amdgcn_perm(cv[3].y, cv[2].y, 0x05040100u));
                        B[3] = f16x4_of(__builtin_amdgcn_perm(cv[1].y, cv[0].y, 0x07060302u),
                                        __builtin_amdgcn_perm(cv[3].y, cv[2].y, 0x07060302u));
                        const f16x4 Ahi = f16x4_of(wt[2 * jj + h].x, wt[2 * jj + h].y);
                        const f16x4 Alo = f16x4_of(wt[2 * jj + h].z, wt[2 * jj + h].w);
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            acc[d] = __builtin_amdgcn_mfma_f32_4x4x4f16(Ahi, B[d], acc[d], 0, 0, 0);
                            acc[d] = __builtin_amdgcn_mfma_f32_4x4x4f16(Alo, B[d], acc[d], 0, 0, 0);
                        }
                    }
                }
                if (x2 == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    units_request(sb, 4 + u + 1, last_vb);
                }
                // the 16 token streams: the 4 of a row of 16 lanes by DPP, the rows and wavefronts through LDS (see fold)
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int g = 0; g < GH; ++g) {
                        const float v = sum_same_row_in_dpp_row(acc[d][g]);
                        if ((lane & 12) == 0)
                            red[((wave * 4 + (lane >> 4)) * 16 + d * 4 + g) * 4 + row] = v;
                    }
            }
        }
    }
    if (vb0 < vb1) {
        __syncthreads();
        fold(7);
    }

    // ---------------- recent full-precision rows of this split, all heads of the group, per wavefront:
    // a wavefront's partial starts at the scan's maxima with nothing summed
    float m_w[GH], l_w[GH];
    f32x4 accx = {0.f, 0.f, 0.f, 0.f}, accy = {0.f, 0.f, 0.f, 0.f};  // element g: head g, dims 2 lane / 2 lane + 1
#pragma unroll
    for (int g = 0; g < GH; ++g) {
        m_w[g] = m_run[g];
        l_w[g] = 0.f;
    }
    if (vb0 >= vb1)
        __syncthreads();  // no round ran: the queries reach LDS here
    {
        const int64_t rbase = (int64_t)bkv * a.max_recent;
        constexpr int RBG = 4;  // rows per trip, their loads issued together
        for (int r = r0 + wave; r < r1; r += GN * RBG) {
            uint32_t kw[RBG], vw[RBG];
#pragma unroll
            for (int u = 0; u < RBG; ++u) {
                const int rr = r + u * GN < r1 ? r + u * GN : r;
                kw[u] = *((const uint32_t *)((const __half *)a.recent_k + (rbase + rr) * PQ_HEAD_DIM) + lane);
                vw[u] = *((const uint32_t *)((const __half *)a.recent_v + (rbase + rr) * PQ_HEAD_DIM) + lane);
            }
#pragma unroll
            for (int u = 0; u < RBG; ++u) {
                if (r + u * GN < r1) {  // wave-uniform
                    const __half2 kh = *(const __half2 *)&kw[u], vh = *(const __half2 *)&vw[u];
                    const float k0 = __low2float(kh), k1 = __high2float(kh), v0 = __low2float(vh), v1 = __high2float(vh);
#pragma unroll
                    for (int g = 0; g < GH; ++g) {
                        const uint32_t qw = *(lds_u32 *)(lbase + G12_Q + g * 256 + lane * 4);
                        const __half2 qh = *(const __half2 *)&qw;
                        const float s = wave_sum(fmaf(__low2float(qh), k0, __high2float(qh) * k1)) * a.scale_log2e;
                        const float m_new = fmaxf(m_w[g], s);
                        const float al = __builtin_amdgcn_exp2f(m_w[g] - m_new);
                        const float p = __builtin_amdgcn_exp2f(s - m_new);
                        l_w[g] = fmaf(l_w[g], al, p);
                        accx[g] = fmaf(accx[g], al, p * v0);
                        accy[g] = fmaf(accy[g], al, p * v1);
                        m_w[g] = m_new;
                    }
                }
            }
        }
    }

    // ---------------- merge inside the workgroup: the scan (maxima m_run, weight sums over all lanes, the
    // output tile) and the wavefronts' recent-row partials (they overwrite the table: wait for the scan's end)
    {
        float l = sum_same_row_in_dpp_row(l_lane);
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lane < GH)
            *((lds_f32 *)(lbase + G12_LW) + wave * GH + lane) = l;
    }
    __syncthreads();
    {
        lds_f32 *part = (lds_f32 *)(lbase + G12_PART) + wave * GH * PQ_PART_STRIDE;
#pragma unroll
        for (int g = 0; g < GH; ++g) {
            if (lane == 0) {
                part[g * PQ_PART_STRIDE] = m_w[g];
                part[g * PQ_PART_STRIDE + 1] = l_w[g];
            }
            part[g * PQ_PART_STRIDE + 4 + 2 * lane] = accx[g];
            part[g * PQ_PART_STRIDE + 5 + 2 * lane] = accy[g];
        }
    }
    __syncthreads();

    // Wavefront g (< G) finishes head g, then one ticket per workgroup; the workgroup that draws the last
    // ticket of the (sequence, KV head, sub-group) merges the splits (as in the 8-bit grouped kernel).
    typedef __attribute__((address_space(3))) int lds_i32;
    lds_i32 *last_flag = (lds_i32 *)(lbase + G12_FLAG);
    const int g = wave;
    if (g < G) {
        const lds_f32 *parts = (const lds_f32 *)(lbase + G12_PART);
        const lds_f32 *lw = (const lds_f32 *)(lbase + G12_LW);
        const float m_scan = g == 0 ? m_run[0] : g == 1 ? m_run[1] : g == 2 ? m_run[2] : m_run[3];
        float mx = m_scan;
#pragma unroll
        for (int w = 0; w < GN; ++w)
            mx = fmaxf(mx, parts[(w * GH + g) * PQ_PART_STRIDE]);
        const float f_scan = __builtin_amdgcn_exp2f(m_scan - mx);
        float l_scan = 0.f;
#pragma unroll
        for (int w = 0; w < GN; ++w)
            l_scan += lw[w * GH + g];
        float o0 = o_lds[g * 128 + 2 * lane] * f_scan, o1 = o_lds[g * 128 + 2 * lane + 1] * f_scan, l = l_scan * f_scan;
#pragma unroll
        for (int w = 0; w < GN; ++w) {
            const lds_f32 *pw = parts + (w * GH + g) * PQ_PART_STRIDE;
            const float f = __builtin_amdgcn_exp2f(pw[0] - mx);
            o0 = fmaf(pw[4 + 2 * lane], f, o0);
            o1 = fmaf(pw[5 + 2 * lane], f, o1);
            l = fmaf(pw[1], f, l);
        }
        if (S == 1) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            *(float2 *)(a.out + (int64_t)(bh0 + g) * PQ_HEAD_DIM + 2 * lane) = make_float2(o0 * inv, o1 * inv);
        } else {
            float *gpart = a.partials + ((int64_t)(bh0 + g) * S + split) * PQ_PART_STRIDE;
            // device-scope stores, complete (performed where every XCD sees them) before the barrier
            publish(gpart + 4 + 2 * lane, o0, o1);
            if (lane == 0)
                publish(gpart, mx, l);
            publish_wait();
        }
    }
    if (S == 1)
        return;
    __syncthreads();  // all G partials of this workgroup are published
    if (wave == 0) {
        unsigned int ticket = 0;
        if (lane == 0)
            ticket = __hip_atomic_fetch_add(a.tickets + bh0, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ticket = __builtin_amdgcn_readfirstlane(ticket);
        if (lane == 0)
            *last_flag = ticket == (unsigned int)(S - 1);
    }
    __syncthreads();
    if (!*last_flag || g >= G)
        return;
    asm volatile("" ::: "memory");  // the loads below stay behind the ticket in the instruction stream
    {
        const float *ps = a.partials + (int64_t)(bh0 + g) * S * PQ_PART_STRIDE;
        const float2 ml = lane < S ? fetch(ps + lane * PQ_PART_STRIDE) : make_float2(NEG_BIG, 0.f);
        const float mx = wave_max(ml.x);
        const float f_lane = __builtin_amdgcn_exp2f(ml.x - mx);
        const float l = wave_sum(ml.y * f_lane);
        float o0 = 0.f, o1 = 0.f;
        // four splits at a time, their loads issued together (loads beyond S repeat the last split with factor 0)
        for (int s0 = 0; s0 < S; s0 += 4) {
            float2 t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                t[u] = fetch(ps + (s0 + u < S ? s0 + u : S - 1) * PQ_PART_STRIDE + 4 + 2 * lane);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f_lane), (s0 + u) & 63));
                f = s0 + u < S ? f : 0.f;
                o0 = fmaf(t[u].x, f, o0);
                o1 = fmaf(t[u].y, f, o1);
            }
        }
        const float inv = l > 0.f ? 1.f / l : 0.f;
        *(float2 *)(a.out + (int64_t)(bh0 + g) * PQ_HEAD_DIM + 2 * lane) = make_float2(o0 * inv, o1 * inv);
    }
    if (wave == 0 && lane == 0)
        ticket_reset(a.tickets + bh0);
}

template <int WAVE_VB>
void launch_grouped12(const pq_decode_args &a, int grid, bool once, hipStream_t s)
{
    if (once)
        hipLaunchKernelGGL((pq12_decode_grouped_kernel<WAVE_VB, true>), dim3(grid), dim3(GN * 64), 0, s, a);
    else
        hipLaunchKernelGGL((pq12_decode_grouped_kernel<WAVE_VB, false>), dim3(grid), dim3(GN * 64), 0, s, a);
}

}  // namespace

// 12-bit contexts with 2 or more query heads per KV head take the kernel above (fp16 only, as all
// 12-bit contexts) — unless the work is small.  A workgroup of this kernel streams all 16 codebook slices (2 MiB)
// through its LDS per round, about 45 us whatever the length, while the per-head kernels' two-pass path (chosen
// when there are 5 or more compute units per (sequence, query head)) keeps one slice per workgroup: measured with
// 32 query / 8 KV heads, one sequence: 8K tokens 46 against 20 us, 32K 46 against 37 us, 64K 47 against 59 us,
// 128K 60 against 97 us; 16 query / 8 KV heads x 64K 48 against 40 us.  So the grouped kernel serves the shapes
// that would not decode in two passes (4 sequences x 32K: 59 against 121 us; 64 query / 8 KV heads x 32K: 48 against
// 71 us) and those with 1.5 M (query head, token) pairs of capacity or more.  A caller that asks for the two-pass
// path (n_splits < 0) keeps the per-head kernels.
bool pq12_config_uses_grouped_kernel(const pq_attn_config *cfg, int n_cu)
{
    const int g = cfg->n_kv_heads > 0 ? cfg->n_q_heads / cfg->n_kv_heads : 0;
    if (!pq_config_is_12bit(cfg) || cfg->n_splits < 0 || pq_grouped_heads_per_workgroup(g) == 0)
        return false;
    const int64_t heads = (int64_t)cfg->batch * cfg->n_q_heads;
    const bool two_pass_otherwise = cfg->n_splits == 0 && n_cu / heads >= 5;
    return !two_pass_otherwise || heads * cfg->max_context >= 1536 * 1024;
}

hipError_t pq12_launch_decode_grouped(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s)
{
    const int grid = a.B * a.Hkv * a.n_sub * a.S;
    const bool once = a.n_sub == 1;
    // blocks of 128 tokens per split at full capacity, per wavefront
    const int64_t per_wave = (ctx->cap_padded / 128 + (int64_t)a.S * GN - 1) / ((int64_t)a.S * GN);
    if (per_wave <= 1)
        launch_grouped12<1>(a, grid, once, s);
    else if (per_wave <= 2)
        launch_grouped12<2>(a, grid, once, s);
    else
        launch_grouped12<4>(a, grid, once, s);
    return hipGetLastError();
}
