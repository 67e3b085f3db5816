// Decode attention over a product-quantized KV cache for grouped queries (2..4 query heads
// per KV head, fp16, M = 64 subspaces of 2 dims or M = 32 of 4): one fused kernel per call.
//
// Same result as the per-head table kernel (Eq. 7 = Eq. 6), different evaluation.  With G
// query heads reading one KV head, per-head score tables cost G x 64 KiB of LDS and G times
// the gather and add work per code byte: the scan turns ALU/LDS bound at a fraction of the HBM
// rate.  Here the codes of a KV head are gathered ONCE and the contraction over the query
// heads — a genuine small dense product — goes to the matrix cores:
//
//   score pass  lane = token.  The K CODEBOOK image (not a per-query table) sits in LDS; a
//               lane gathers the centroids of its token, 4 subspaces (8 dims) per step, and
//               v_mfma_f32_4x4x4_16B_f16 multiplies, per quad of lanes, the 4 heads' query
//               slice (A, 4 heads x 4 dims, from LDS) with the quad's 4 tokens (B, 4 dims x 4
//               tokens): 32 instructions give all G scores of 64 tokens.  fp16 x fp16 products
//               are exact in the fp32 accumulator.  The instruction needs the 4 lanes of a quad
//               on the same dims, so the K code layout rotates by quad (PQ_K_SKEW_QUAD) and the
//               16 quads of a step work on 16 different groups of 4 columns.  Inside a quad,
//               lanes 2 and 3 gather their 4 subspaces two steps ahead of lanes 0 and 1 and
//               rotate the results back in registers: two lanes per column instead of four (a
//               2-way bank conflict, 4 cycles per gather; four lanes on one column cost 8, four
//               different orders 2 but twice the rotation work, and vector-ALU issue binds here).
//   softmax     per head: running maximum, moved (wave maximum, rescale) only when a block exceeds it
//               by a factor 2^8 in weight; the weights are split into an fp16 high and low part
//               (p = hi + lo to 2^-22 relative) and staged in LDS.
//   value pass  lane = subspace, as in the per-head kernel: one gather per code byte from the V
//               codebook image.  Four tokens' centroid pairs are re-packed (4 x v_perm) into
//               the B operands of the same 4x4x4 instruction, whose A operand holds the 4 heads'
//               weights of those 4 tokens: 4 instructions (x / y dims, hi / lo weights) per 4
//               tokens accumulate all G output rows; lane l ends up with dims 2l, 2l+1 of every
//               head.
// Vector-ALU work per code byte no longer grows with G; the per-head kernel remains the
// choice for G = 1 (its gathers are conflict-free) and serves every other shape.
//
// One workgroup = one (sequence, KV head, context split).  Schedule, block hand-out, recent
// rows, split merge and ticket protocol follow the per-head kernel.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_device_utils.h"

namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uint16_t lds_u16;

constexpr int GNW = 16;                      // wavefronts per workgroup (4 per SIMD: this kernel is bound by LDS and
                                             // instruction latency, not by HBM queues)
constexpr int GMAX = 4;                      // rows of the 4x4x4 instruction = query heads per KV head
constexpr int KIMG_OFF = 0;                  // fp16 K codebook image [256][256 bytes]
constexpr int VIMG_OFF = 65536;              // fp16 V codebook image [256][256 bytes]
// Rows of the two A-operand tables are padded by 8 bytes: the 4 lanes of a quad read the same
// offset of 4 different rows, and an unpadded row stride is a multiple of the bank count.
constexpr int Q_OFF = 131072;                // fp16 q, 4 rows of 256 bytes at q_row(g)
// Row offsets of q: in a score step the lanes of quad k read 16 bytes at 16 (U + k) of the 4 rows.
// The rows are a quarter of the bank cycle apart, so the 4 quads of a quarter-wavefront (16-byte
// reads are served 16 lanes at a time) cover the 64 banks once.
__host__ __device__ constexpr int q_row(int g) { return g * 320; }
constexpr int P_ROW = 128 + 8;               // bytes per head of staged weights
constexpr int PST_WAVE = 2 * GMAX * P_ROW;   // per wavefront: hi [4][64 (+4)] fp16, then lo likewise
constexpr int PST_OFF = Q_OFF + 1216;
static_assert(q_row(3) + 256 <= 1216, "q rows fit");
constexpr int GCTR_OFF = PST_OFF + GNW * PST_WAVE;  // uint32 block counter, uint32 "last ticket" flag
constexpr int GSMEM_BYTES = GCTR_OFF + 16;
// wavefront partials float [GNW][4][PQ_PART_STRIDE] reuse the K image once every wavefront has left the scan
constexpr int GPART_OFF = KIMG_OFF;
static_assert(GNW * GMAX * PQ_PART_STRIDE * 4 <= 65536, "partials fit in the K image");
static_assert(GSMEM_BYTES <= 160 * 1024, "LDS budget of a gfx950 compute unit");

__device__ inline f16x4 as_f16x4(uint32_t lo, uint32_t hi)
{
    u32x2 v = {lo, hi};
    return __builtin_bit_cast(f16x4, v);
}

// READ_ONCE: one workgroup per (sequence, KV head, split) reads the head's codes, so they stream with the
// non-temporal hint; with more than 4 query heads per KV head several workgroups (4 heads each) share the
// code stream through their XCD's L2 and load normally.
//
// M = 32 (subspaces of 4 dims) runs as 64 VIRTUAL subspaces of 2 dims: virtual subspace v is the dim pair v & 1 of
// real subspace v >> 1 and carries that subspace's code.  The packed codebook images are the same bytes either way
// ([256][128 dims] fp16), so only the code loads differ: half the bytes per token, one K code byte serves two of
// the four gathers of a score step, and two neighbouring lanes of the value pass share one V code stream.
template <bool READ_ONCE, int M>
__global__ __launch_bounds__(GNW * 64) void pq_decode_grouped_kernel(const pq_decode_args a)
{
    static_assert(M == 64 || M == 32, "64 subspaces of 2 dims or 32 of 4");
    constexpr int KVEC = M / 16;  // 16-byte vectors of K codes per lane and block
    constexpr int NW = GNW;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[GSMEM_BYTES];
    lds_u8 *lbase = (lds_u8 *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int S_grid = a.S;  // splits the grid was launched with (partials are laid out with this stride)
    // workgroups of one KV head are neighbours: (sequence, KV head, sub-group of G query heads, split)
    uint32_t unit_u, split_u;
    unit_and_split(blockIdx.x, gridDim.x, (uint32_t)S_grid, unit_u, split_u);
    const int unit = (int)unit_u, split = (int)split_u;
    const int n_sub = a.n_sub;                     // sub-groups per KV head
    // ... then the same KV head of the other sequences (same codebook images: once per XCD from memory)
    const int hb = (int)((uint32_t)unit / (uint32_t)n_sub);  // hkv * B + b
    const int sub_group = unit - hb * n_sub;
    const int hkv = (int)((uint32_t)hb / (uint32_t)a.B);
    const int b = hb - hkv * a.B;
    const int bkv = b * a.Hkv + hkv;
    // the KV head's a.G query heads in n_sub sub-groups whose sizes differ by at most one (the first a.G % n_sub take
    // one more): this workgroup's heads are g_first .. g_first + G - 1, G = 2..4
    const int g_base = a.G / n_sub, g_rem = a.G - g_base * n_sub;
    const int G = g_base + (sub_group < g_rem ? 1 : 0);
    const int g_first = sub_group * g_base + (sub_group < g_rem ? sub_group : g_rem);
    const int bh0 = b * a.Hq + hkv * a.G + g_first;  // first query head of this workgroup
    // The lengths are requested first and taken out of their registers only after the table loads
    // below have been issued.  The loads go through lane_zero(), which the compiler cannot see
    // through: a load from a wave-uniform address is otherwise made scalar on the spot, with a full
    // wait for each of the two — two serial memory round trips before the first table load.
    const int zero = lane_zero();
    const bool has_recent = a.recent_k != nullptr && a.recent_len != nullptr;
    const int n_vec = a.ctx_len[b + zero];
    const int r_vec = (has_recent ? a.recent_len : a.ctx_len)[b + zero];
    const float w_lane = (a.B > 1 && a.S > 1) ? batch_work_lane(a, has_recent, lane) : 0.f;  // one launched split: nothing to cap

    // ---- prologue: both codebook images and the group's queries; table loads first, bare
    // barrier, then the first code block (see the per-head kernel for why)
    constexpr int VPT = 8192 / (NW * 64);  // 16-byte vectors per thread for the two images
    u32x4 raw[VPT];
    {
        const u32x4 *ksrc = (const u32x4 *)((const __half *)a.kcb_packed + (int64_t)hkv * 256 * PQ_HEAD_DIM);
        const u32x4 *vsrc = (const u32x4 *)((const __half *)a.vcb_packed + (int64_t)hkv * 256 * PQ_HEAD_DIM);
#pragma unroll
        for (int v = 0; v < VPT / 2; ++v) {
            raw[v] = ksrc[tid + v * (NW * 64)];
            raw[VPT / 2 + v] = vsrc[tid + v * (NW * 64)];
        }
    }
    // q of the group: G x 128 fp16 = G x 16 vectors; heads beyond G are zero rows
    u32x4 qraw = {0u, 0u, 0u, 0u};
    if (tid < 16 * G)
        qraw = *((const u32x4 *)((const __half *)a.q + (int64_t)bh0 * PQ_HEAD_DIM) + tid);
    __builtin_amdgcn_s_barrier();

    int N = __builtin_amdgcn_readfirstlane(n_vec);
    int R = has_recent ? __builtin_amdgcn_readfirstlane(r_vec) : 0;
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    R = R < 0 ? 0 : (R > a.max_recent ? a.max_recent : R);
    const uint32_t nblk = (uint32_t)(N + 63) >> 6;
    // live splits follow the length (at least 4 blocks or 16 recent rows each); the others leave before the images
    // are staged
    uint32_t want = nblk / 4u > (uint32_t)R / 16u ? nblk / 4u : (uint32_t)R / 16u;  // ... or 16 recent rows
    if (a.B > 1 && a.S > 1) {  // ... and in a batch no more than the sequence's share of the compute units
        const uint32_t cap = live_split_cap(a, a.Hkv * a.n_sub, N + R, w_lane);
        want = want < cap ? want : cap;
    }
    const int S = (int)(want < 1u ? 1u : (want < (uint32_t)S_grid ? want : (uint32_t)S_grid));
    if (split >= S)
        return;
    const int blk0 = (int)(nblk * (uint32_t)split / (uint32_t)S);
    const int blk1 = (int)(nblk * (uint32_t)(split + 1) / (uint32_t)S);
    const int r0 = (int)((uint32_t)R * (uint32_t)split / (uint32_t)S);
    const int r1 = (int)((uint32_t)R * (uint32_t)(split + 1) / (uint32_t)S);
    const uint8_t *k_head = a.k_codes + (int64_t)bkv * a.head_stride;
    const uint8_t *v_head = a.v_codes + (int64_t)bkv * a.head_stride;

    // One K and one V buffer per wavefront, each refilled as soon as its pass is over: the V codes
    // of a block are requested when its score pass starts (the first block's: in the prologue), the K codes of
    // the next block when that score pass ends.  With 4 wavefronts per SIMD that is enough to keep the loads ahead.
    uint4 kbuf[KVEC], vbuf[4];
    // `live` false: a dead load by a wavefront that has run out of blocks (loads stay unconditional
    // so that the wait counts stay exact); all lanes then read the same 16 bytes, not 4 KiB.
    auto load_k = [&](uint4 (&dst)[KVEC], int blk_id, bool live) {
        const u32x4 *kp = (const u32x4 *)(k_head + (int64_t)blk_id * (64 * M)) + (live ? lane : 0);
        const int step = live ? 64 : 0;
#pragma unroll
        for (int j = 0; j < KVEC; ++j)
            dst[j] = load_codes<READ_ONCE>(kp + j * step);
    };
    auto load_v = [&](int blk_id) {  // 4 tiles of 16 tokens; this lane's (real) subspace in each
        const u32x4 *vp = (const u32x4 *)(v_head + (int64_t)blk_id * (64 * M)) + (M == 64 ? lane : lane >> 1);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            vbuf[j] = load_codes<READ_ONCE>(vp + j * M);
    };
    int blk = blk0 + wave;
    *(lds_u32 *)(lbase + GCTR_OFF) = (uint32_t)(blk0 + NW);
    const uint32_t ctr_addr = (uint32_t)(uintptr_t)(lbase + GCTR_OFF);
    load_k(kbuf, blk < blk1 ? blk : 0, blk < blk1);
    // The first block's V codes are requested here too: a wavefront scans only a handful of blocks, and a round
    // trip to memory in front of its first value pass is not amortised (measured on the 128K-token workload:
    // 35.7 -> 33.3 us on a box with slow memory round trips, no change on a faster one).
    load_v(blk < blk1 ? blk : 0);
    bool first_block = true;

#pragma unroll
    for (int v = 0; v < VPT / 2; ++v) {
        *(lds_u32x4 *)(lbase + KIMG_OFF + (tid + v * (NW * 64)) * 16) = raw[v];
        *(lds_u32x4 *)(lbase + VIMG_OFF + (tid + v * (NW * 64)) * 16) = raw[VPT / 2 + v];
    }
    if (tid < 64) {  // padded rows are 8-byte, not 16-byte, aligned: two 8-byte stores
        const u32x2 qlo = {qraw.x, qraw.y}, qhi = {qraw.z, qraw.w};
        *(lds_u32x2 *)(lbase + Q_OFF + q_row(tid >> 4) + (tid & 15) * 16) = qlo;
        *(lds_u32x2 *)(lbase + Q_OFF + q_row(tid >> 4) + (tid & 15) * 16 + 8) = qhi;
    }
    __syncthreads();

    const int quad = lane >> 2;  // the 4x4x4 block of this lane
    const int row = lane & 3;    // its row: query head as an A operand, token / dim as a B operand
    // score pass: column bytes, byte k of idx[r] = 4 * ((4r + k + 4 quad) % 64) = 16 * ((r + quad) % 16) + 4 k
    uint32_t idx[16];
#pragma unroll
    for (int r = 0; r < 16; ++r)
        idx[r] = 0x0c080400u + 0x10101010u * (uint32_t)((r + quad) & 15);
    // gather r of a step: this lane's (virtual) subspace kk = (r + 2 * (row / 2)) % 4 of the step -> address =
    // code << 8 | column.  M = 64: the step's word holds 4 codes, byte kk.  M = 32: a word holds two steps' 2 codes,
    // byte kk / 2 of the step's half (ksel[r][1] for odd steps).
    uint32_t ksel[4][2];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t kk = (uint32_t)(r + (row & 2)) & 3u;
        ksel[r][0] = 0x0c0c0000u | ((4u + (M == 64 ? kk : kk >> 1)) << 8) | kk;
        ksel[r][1] = 0x0c0c0000u | ((6u + (kk >> 1)) << 8) | kk;
    }
    const uint32_t rot2 = (row & 2) ? 0x07060504u : 0x03020100u;  // v_perm selector: first / second operand
    const uint32_t vcol = (uint32_t)(lane * 4) | ((VIMG_OFF >> 16) << 8);
    // A operands of the score pass at step U: q[row][4 sigma .. 4 sigma + 7], sigma = (2 U + 2 quad) % 32
    const uint32_t qa_base = (uint32_t)(Q_OFF + q_row(row));

    float m_run[GMAX], l_lane[GMAX];
    f32x4 accx = {0.f, 0.f, 0.f, 0.f}, accy = {0.f, 0.f, 0.f, 0.f};  // element g: head g, dims 2 lane / 2 lane + 1
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
        m_run[g] = NEG_BIG;
        l_lane[g] = 0.f;
    }
    lds_u8 *pst = lbase + PST_OFF + wave * PST_WAVE;  // hi at g * P_ROW + token * 2, lo at GMAX * P_ROW + the same

    auto process = [&](const int blk_id, const int next_id, const bool next_live) {
        // ---------------- score pass: sc[g] = q_g . K^_token for this lane's token
        // One step = one word of this lane's codes = the 4 subspaces 4 (U + quad) .. + 3 of its token.
        // The four lanes of a quad need the same subspaces; gathering them in the same order puts
        // four rows of one column, i.e. one bank, into every gather (8 cycles instead of 2).  Lanes
        // 2 and 3 therefore walk the four subspaces two steps ahead of lanes 0 and 1: two lanes per
        // column (4 cycles), and one register rotation by two brings their results back in order.
        // (Four different orders make the gathers conflict-free, but cost a second rotation stage —
        // 128 instead of 64 more vector instructions per block — and this kernel is bound by
        // vector-ALU issue: measured 38.6 us against 36.2 us.)
        f32x4 sc0 = {0.f, 0.f, 0.f, 0.f}, sc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int U = 0; U < 16; ++U) {
            const uint32_t w = M == 64 ? comp(kbuf[U >> 2], U & 3) : comp(kbuf[(U >> 3) % KVEC], (U >> 1) & 3);
            uint32_t got[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                got[r] = *(lds_u32 *)(lbase + __builtin_amdgcn_perm(w, idx[U], ksel[r][M == 64 ? 0 : U & 1]));
            // lanes 2 and 3 of the quad hold their four results rotated by two registers: rotate back
            // (v_perm as a two-way select with a per-lane selector)
            uint32_t c[4];
#pragma unroll
            for (int m = 0; m < 4; ++m)
                c[m] = __builtin_amdgcn_perm(got[(m + 2) & 3], got[m], rot2);
            const uint32_t sigma = (uint32_t)(2 * U + 2 * quad) & 31u;  // even: sigma + 1 does not wrap
            const f16x4 A0 = __builtin_bit_cast(f16x4, *(lds_u32x2 *)(lbase + qa_base + sigma * 8));
            const f16x4 A1 = __builtin_bit_cast(f16x4, *(lds_u32x2 *)(lbase + qa_base + sigma * 8 + 8));
            sc0 = __builtin_amdgcn_mfma_f32_4x4x4f16(A0, as_f16x4(c[0], c[1]), sc0, 0, 0, 0);
            sc1 = __builtin_amdgcn_mfma_f32_4x4x4f16(A1, as_f16x4(c[2], c[3]), sc1, 0, 0, 0);
        }
        load_k(kbuf, next_id, next_live);  // the score pass is done with the K codes of this block
        const bool valid = blk_id * 64 + lane < N;

        // ---------------- running softmax, one per head; weights staged as fp16 hi + lo
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            const float s = valid ? (sc0[g] + sc1[g]) * a.scale_log2e : NEG_BIG;
            // The reference maximum moves only when a score of the block exceeds it by more than 8 (a factor
            // 2^8 in weight; a wave-wide vote): weights stay below 2^8, far inside the range of the fp32 sums
            // and of the fp16 staging, and most blocks skip the wave-wide maximum and the rescaling.
            if (__builtin_amdgcn_ballot_w64(s > m_run[g] + 8.0f) != 0) {  // wave-uniform
                const float m_new = fmaxf(m_run[g], wave_max(s));
                const float alpha = __builtin_amdgcn_exp2f(m_run[g] - m_new);
                l_lane[g] *= alpha;
                accx[g] *= alpha;
                accy[g] *= alpha;
                m_run[g] = m_new;
            }
            const float p = valid ? __builtin_amdgcn_exp2f(s - m_run[g]) : 0.f;
            l_lane[g] += p;
            const _Float16 hi = (_Float16)p;
            const _Float16 lo = (_Float16)(p - (float)hi);
            *(lds_u16 *)(pst + g * P_ROW + lane * 2) = __builtin_bit_cast(uint16_t, hi);
            *(lds_u16 *)(pst + (GMAX + g) * P_ROW + lane * 2) = __builtin_bit_cast(uint16_t, lo);
        }
        __builtin_amdgcn_wave_barrier();

        // ---------------- value pass: 4 tokens per step
#pragma unroll
        for (int n = 0; n < 4; ++n) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t w = comp(vbuf[n], r);
                const int tok0 = 16 * n + 4 * r;
                uint32_t c[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t addr = __builtin_amdgcn_perm(w, vcol, 0x0c010000u | ((4 + k) << 8));
                    c[k] = *(lds_u32 *)(lbase + addr);
                }
                // B operands: this lane's x (then y) coordinate of the 4 tokens
                const f16x4 Bx = as_f16x4(__builtin_amdgcn_perm(c[1], c[0], 0x05040100u),
                                          __builtin_amdgcn_perm(c[3], c[2], 0x05040100u));
                const f16x4 By = as_f16x4(__builtin_amdgcn_perm(c[1], c[0], 0x07060302u),
                                          __builtin_amdgcn_perm(c[3], c[2], 0x07060302u));
                // A operands: weights of head `row` for the 4 tokens
                const f16x4 Ahi = __builtin_bit_cast(f16x4, *(lds_u32x2 *)(pst + row * P_ROW + tok0 * 2));
                const f16x4 Alo = __builtin_bit_cast(f16x4, *(lds_u32x2 *)(pst + (GMAX + row) * P_ROW + tok0 * 2));
                accx = __builtin_amdgcn_mfma_f32_4x4x4f16(Ahi, Bx, accx, 0, 0, 0);
                accy = __builtin_amdgcn_mfma_f32_4x4x4f16(Ahi, By, accy, 0, 0, 0);
                accx = __builtin_amdgcn_mfma_f32_4x4x4f16(Alo, Bx, accx, 0, 0, 0);
                accy = __builtin_amdgcn_mfma_f32_4x4x4f16(Alo, By, accy, 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    while (blk < blk1) {
        const int nb = lds_grab(ctr_addr);
        if (!first_block)  // wave-uniform
            load_v(blk);
        first_block = false;
        process(blk, nb < blk1 ? nb : blk, nb < blk1);
        blk = nb;
    }

    // ---------------- recent full-precision rows of this split, all heads of the group
    {
        const int64_t rbase = (int64_t)bkv * a.max_recent;
        // RBG rows per trip, their loads issued together (one memory round trip per trip, not per row); rows
        // beyond the range re-read the trip's first row and are skipped
        constexpr int RBG = 4;
        for (int r = r0 + wave; r < r1; r += NW * RBG) {
            uint32_t kw[RBG], vw[RBG];
#pragma unroll
            for (int u = 0; u < RBG; ++u) {
                const int rr = r + u * NW < r1 ? r + u * NW : r;
                kw[u] = *((const uint32_t *)((const __half *)a.recent_k + (rbase + rr) * PQ_HEAD_DIM) + lane);
                vw[u] = *((const uint32_t *)((const __half *)a.recent_v + (rbase + rr) * PQ_HEAD_DIM) + lane);
            }
#pragma unroll
            for (int u = 0; u < RBG; ++u) {
                if (r + u * NW < r1) {  // wave-uniform
                    const __half2 kh = *(const __half2 *)&kw[u], vh = *(const __half2 *)&vw[u];
                    const float k0 = __low2float(kh), k1 = __high2float(kh), v0 = __low2float(vh), v1 = __high2float(vh);
#pragma unroll
                    for (int g = 0; g < GMAX; ++g) {
                        // this lane's dims (2 lane, 2 lane + 1) of head g's query
                        const uint32_t qw = *(lds_u32 *)(lbase + Q_OFF + q_row(g) + lane * 4);
                        const __half2 qh = *(const __half2 *)&qw;
                        const float s = wave_sum(fmaf(__low2float(qh), k0, __high2float(qh) * k1)) * a.scale_log2e;
                        const float m_new = fmaxf(m_run[g], s);
                        const float alpha = __builtin_amdgcn_exp2f(m_run[g] - m_new);
                        const float p = __builtin_amdgcn_exp2f(s - m_new);
                        l_lane[g] = fmaf(l_lane[g], alpha, lane == 0 ? p : 0.f);
                        accx[g] = fmaf(accx[g], alpha, p * v0);
                        accy[g] = fmaf(accy[g], alpha, p * v1);
                        m_run[g] = m_new;
                    }
                }
            }
        }
    }

    // ---------------- merge the wavefronts of this workgroup (their partials overwrite the K image:
    // wait until nobody scans any more)
    __syncthreads();
    {
        lds_f32 *part = (lds_f32 *)(lbase + GPART_OFF) + wave * GMAX * PQ_PART_STRIDE;
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            const float l_w = wave_sum(l_lane[g]);
            if (lane == 0) {
                part[g * PQ_PART_STRIDE] = m_run[g];
                part[g * PQ_PART_STRIDE + 1] = l_w;
            }
            part[g * PQ_PART_STRIDE + 4 + 2 * lane] = accx[g];
            part[g * PQ_PART_STRIDE + 5 + 2 * lane] = accy[g];
        }
    }
    __syncthreads();

    // Wavefront g (< G) finishes head g: merges the workgroup's wavefronts, publishes the split
    // partial, and — in the workgroup that takes the last ticket of this (sequence, KV head) —
    // merges all splits and writes the output row.  One ticket per workgroup (wavefront 0),
    // between two barriers.
    typedef __attribute__((address_space(3))) int lds_i32;
    lds_i32 *last_flag = (lds_i32 *)(lbase + GCTR_OFF + 4);
    const int g = wave;
    if (g < G) {
        const lds_f32 *parts = (const lds_f32 *)(lbase + GPART_OFF);
        float mx = NEG_BIG;
#pragma unroll
        for (int w = 0; w < NW; ++w)
            mx = fmaxf(mx, parts[(w * GMAX + g) * PQ_PART_STRIDE]);
        float o0 = 0.f, o1 = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const lds_f32 *pw = parts + (w * GMAX + g) * PQ_PART_STRIDE;
            const float f = __builtin_amdgcn_exp2f(pw[0] - mx);
            o0 = fmaf(pw[4 + 2 * lane], f, o0);
            o1 = fmaf(pw[5 + 2 * lane], f, o1);
            l = fmaf(pw[1], f, l);
        }
        if (S == 1) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            *(float2 *)(a.out + (int64_t)(bh0 + g) * PQ_HEAD_DIM + 2 * lane) = make_float2(o0 * inv, o1 * inv);
        } else {
            float *gpart = a.partials + ((int64_t)(bh0 + g) * S_grid + split) * PQ_PART_STRIDE;
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
        // The other workgroups' partials, by device-scope loads issued after the ticket has returned: the first 32
        // splits' outputs together with the (maximum, weight sum) pairs, so that the merge costs one memory round
        // trip instead of three.  Loads of splits beyond S repeat the last split (unconditional loads from
        // wave-uniform bases); their factor is zero.
        const float *ps = a.partials + (int64_t)(bh0 + g) * S_grid * PQ_PART_STRIDE;
        float2 o[32];
#pragma unroll
        for (int u = 0; u < 32; ++u)
            o[u] = fetch(ps + (u < S ? u : S - 1) * PQ_PART_STRIDE + 4 + 2 * lane);
        const float2 ml = lane < S ? fetch(ps + lane * PQ_PART_STRIDE) : make_float2(NEG_BIG, 0.f);
        const float mx = wave_max(ml.x);
        const float f_lane = __builtin_amdgcn_exp2f(ml.x - mx);
        const float l = wave_sum(ml.y * f_lane);
        float o0 = 0.f, o1 = 0.f;
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f_lane), u));
            f = u < S ? f : 0.f;  // wave-uniform
            o0 = fmaf(o[u].x, f, o0);
            o1 = fmaf(o[u].y, f, o1);
        }
        // more than 32 splits (few heads, long contexts): four at a time
        for (int s0 = 32; s0 < S; s0 += 4) {
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

}  // namespace

// A KV head's g query heads are cut into ceil(g / 4) sub-groups (the matrix instruction has 4 rows), one workgroup
// each, sizes as equal as possible: 2..4 heads for every g >= 2 (5 = 3 + 2, 7 = 4 + 3, 10 = 4 + 3 + 3).
int pq_grouped_sub_groups(int g) { return g < 2 ? 0 : (g + GMAX - 1) / GMAX; }

// the largest sub-group; 0 for g = 1 (no grouped kernel)
int pq_grouped_heads_per_workgroup(int g)
{
    const int n = pq_grouped_sub_groups(g);
    return n == 0 ? 0 : (g + n - 1) / n;
}

bool pq_config_uses_grouped_kernel(const pq_attn_config *cfg)
{
    const int g = cfg->n_kv_heads > 0 ? cfg->n_q_heads / cfg->n_kv_heads : 0;
    return cfg->dtype == PQ_F16 && (cfg->n_subspaces == 64 || cfg->n_subspaces == 32) && cfg->n_centroids == 256 &&
           cfg->head_dim == PQ_HEAD_DIM &&
           pq_grouped_heads_per_workgroup(g) > 0;
}

hipError_t pq_launch_decode_grouped(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s)
{
    const int grid = a.B * a.Hkv * a.n_sub * a.S;
    const bool once = a.n_sub == 1;
    if (ctx->cfg.n_subspaces == 64) {
        if (once) hipLaunchKernelGGL((pq_decode_grouped_kernel<true, 64>), dim3(grid), dim3(GNW * 64), 0, s, a);
        else hipLaunchKernelGGL((pq_decode_grouped_kernel<false, 64>), dim3(grid), dim3(GNW * 64), 0, s, a);
    } else {
        if (once) hipLaunchKernelGGL((pq_decode_grouped_kernel<true, 32>), dim3(grid), dim3(GNW * 64), 0, s, a);
        else hipLaunchKernelGGL((pq_decode_grouped_kernel<false, 32>), dim3(grid), dim3(GNW * 64), 0, s, a);
    }
    return hipGetLastError();
}
