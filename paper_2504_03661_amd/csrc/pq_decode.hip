// Decode attention over a product-quantized KV cache: one fused kernel per call.
//
// What it computes (Eq. 7, equal to Eq. 6): for every (sequence b, query head hq)
//   s_t   = sum_i LUT[i][Delta_K[t][i]],  LUT[i][c] = scale * q^i . C_K^i[c]        (quantized tokens)
//   s_r   = scale * q . k_r                                                        (recent rows)
//   out   = sum_t p_t * (||_i C_V^i[Delta_V[t][i]]) + sum_r p_r * v_r,   p = softmax over all s
// with one shared maximum and normaliser, evaluated as split partials merged by
// online softmax (the "OlSoftmax" of Eq. 7; steps 1-4 of Section III-C).
//
// Mapping to gfx950.  One workgroup = one (b, hq, context split).  Its LDS holds
// the query's table LUT[c][i] (fp32, centroid-major, 64 KiB) and the head's value
// codebook (fp16, centroid-major, 64 KiB); both are built once in the prologue
// from the context's re-packed codebooks.  Each wavefront then streams 64-token
// blocks of codes on its own, with no workgroup barrier in the loop:
//   score pass  lane = token.  At step s lane l reads table column (s + l) % 64 of
//               row code: 64 lanes, 64 distinct columns, so the gather has no LDS
//               bank conflict for any code values.  The K code layout stores each
//               token's bytes pre-rotated so the lane's own 16-byte loads deliver
//               them in that order; the LDS address of a gather is one v_perm_b32
//               (code byte -> address bits 8..15, column byte -> bits 0..7).
//   softmax     wave maximum by DPP, running maximum / rescale per block, the
//               weights p_t go through a 256-byte LDS line so that the value pass
//               can read them as a broadcast.
//   value pass  lane = subspace (= output dims).  Lane i gathers centroid row
//               code from column i of the value codebook image: again 64 distinct
//               columns per gather; the fp16 pair is consumed by v_fma_mix.
// fp32 contexts: table and (fp32, 128 KiB) value codebook image take turns in LDS, the
// scan runs in chunks of two phases (see the scan loop).
// The recent full-precision rows are spread over the splits and folded into the
// same running softmax.  Partials of the wavefronts are merged in LDS, the
// workgroup's partial goes to global scratch, and the workgroup that takes the
// last ticket of its (b, hq) merges all splits and writes the output row.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <type_traits>

#include "pq_internal.h"
#include "pq_device_utils.h"

namespace {

constexpr int LUT_OFF = 0;           // float [256][64]
constexpr int VCB_OFF = 65536;       // fp16 image [256][256 bytes]
constexpr int PBUF_OFF = 131072;     // float [NW][64]
constexpr int PART_OFF = 131072 + 4096;  // float [NW][PQ_PART_STRIDE]
constexpr int CTR_OFF = PART_OFF + 16 * PQ_PART_STRIDE * 4;  // uint32: next unowned block of the split
constexpr int SMEM_BYTES = CTR_OFF + 16;
// fp32 contexts: the value codebook image is 128 KiB (256 rows of 512 bytes) and cannot sit next to the table, so
// a workgroup scans in chunks of F32_CHUNK blocks and two phases (see the scan below); the scores of a chunk wait
// in LDS between the phases
constexpr int F32_CHUNK = 64;        // blocks (of 64 tokens) per chunk
constexpr int SBUF_OFF = SMEM_BYTES; // float [F32_CHUNK][64]
constexpr int SMEM_BYTES_F32 = SBUF_OFF + F32_CHUNK * 256;
static_assert(SMEM_BYTES_F32 <= 160 * 1024, "LDS budget of a gfx950 compute unit");
template <int M, int DS, typename T, int NW, bool READ_ONCE>
__global__ __launch_bounds__(NW * 64) void pq_decode_kernel(const pq_decode_args a)
{
    static_assert(M * DS == PQ_HEAD_DIM, "head_dim 128 only");
    static_assert((M == 64 && DS == 2) || (M == 32 && DS == 4), "supported PQ shapes");
    constexpr bool F16 = sizeof(T) == 2;

    // The only LDS object of the kernel, so it sits at LDS address 0 and the
    // byte-assembled gather addresses below are used as they are.
    __shared__ __attribute__((aligned(1024))) unsigned char smem[F16 ? SMEM_BYTES : SMEM_BYTES_F32];
    lds_u8 *lbase = (lds_u8 *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which (sequence, query head, split) this workgroup owns.  Workgroups are
    // dealt round-robin to the 8 XCDs; un-deal them so that all splits of a head (and
    // all query heads of a KV group) sit on one XCD and share its L2 for the
    // codebooks and, with grouped queries, the code stream itself.
    const int S_grid = a.S;  // splits the grid was launched with (partials are laid out with this stride)
    // neighbours: the splits of a (sequence, query head), the query heads of its KV group, then the same
    // KV head of the other sequences (they load the same codebooks: once per XCD instead of once per sequence)
    uint32_t unit, split_u;
    unit_and_split(blockIdx.x, gridDim.x, (uint32_t)S_grid, unit, split_u);
    const int split = (int)split_u;
    const uint32_t bkv = unit / (uint32_t)a.G;          // hkv * B + b
    const int gq = (int)(unit - bkv * (uint32_t)a.G);
    const int hkv = (int)(bkv / (uint32_t)a.B);
    const int b = (int)(bkv - (uint32_t)hkv * (uint32_t)a.B);
    const int hq = hkv * a.G + gq;
    const int bh = b * a.Hq + hq;

    // The lengths are requested first and taken out of their registers only after the table loads
    // below have been issued.  The loads go through lane_zero(), which the compiler cannot see
    // through: a load from a wave-uniform address is otherwise made scalar on the spot, with a full
    // wait for each of the two — two serial memory round trips before the first table load.
    const int zero = lane_zero();
    const bool has_recent = a.recent_k != nullptr && a.recent_len != nullptr;
    const int n_vec = a.ctx_len[b + zero];
    const int r_vec = (has_recent ? a.recent_len : a.ctx_len)[b + zero];
    const float w_lane = (a.B > 1 && a.S > 1) ? batch_work_lane(a, has_recent, lane) : 0.f;  // one launched split: nothing to cap

    // ---- prologue: LUT[c][x] for x = 0..63 (for M = 32 columns x and x+32 hold the same
    // subspace), and the value codebook image.  Order matters at this time scale:
    //  1. every wavefront issues its table loads (they need nothing but the head index);
    //  2. a bare barrier, so that ALL table requests of the workgroup are queued in the
    //     compute unit's memory pipeline before ANY code request (the pipeline serves in
    //     order: a table request behind other wavefronts' code loads would arrive last);
    //  3. the sequence length is read, the split is cut, the first code block is requested;
    //  4. the tables are built while the codes stream in.
    constexpr int ROWS_PER_PASS = NW * 4;              // 16 threads cover one 64-column row
    constexpr int PASSES = 256 / ROWS_PER_PASS;
    constexpr int NV = 4 * DS * (int)sizeof(T) / 16;   // 16-byte vectors per 4 columns
    constexpr int VPT = 4096 / (NW * 64);              // codebook-image vectors per thread
    const int g = tid & 15;                            // columns 4g .. 4g+3
    const int row0 = tid >> 4;
    const int e0 = ((4 * g) & (M - 1)) * DS;           // first element of those columns in a row
    const char *kcb = (const char *)a.kcb_packed + (int64_t)hkv * 256 * PQ_HEAD_DIM * sizeof(T);
    u32x4 kraw[PASSES][NV];
    u32x4 qraw[NV];  // the query elements of columns 4g .. 4g+3 (converted after the barrier)
#pragma unroll
    for (int k = 0; k < PASSES; ++k)
#pragma unroll
        for (int v = 0; v < NV; ++v)
            kraw[k][v] = *(const u32x4 *)(kcb + ((row0 + k * ROWS_PER_PASS) * PQ_HEAD_DIM + e0) * sizeof(T) + v * 16);
    u32x4 vraw[VPT];
    if (F16) {
        const u32x4 *src = (const u32x4 *)((const __half *)a.vcb_packed + (int64_t)hkv * 256 * PQ_HEAD_DIM);
#pragma unroll
        for (int v = 0; v < VPT; ++v)
            vraw[v] = src[tid + v * (NW * 64)];
    }
#pragma unroll
    for (int v = 0; v < NV; ++v)
        qraw[v] = *(const u32x4 *)((const char *)a.q + (((int64_t)b * a.Hq + hq) * PQ_HEAD_DIM + e0) * sizeof(T) + v * 16);
    __builtin_amdgcn_s_barrier();

    int N = __builtin_amdgcn_readfirstlane(n_vec);
    int R = has_recent ? __builtin_amdgcn_readfirstlane(r_vec) : 0;
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    R = R < 0 ? 0 : (R > a.max_recent ? a.max_recent : R);
    // 32-bit unsigned arithmetic: the capacities are limited to 2^24 tokens and S to 64, and a
    // 64-bit division costs more instructions than the whole table build
    const uint32_t nblk = (uint32_t)(N + 63) >> 6;
    // The grid is sized for the capacity; the LIVE splits follow the length: a split scans at least 4 blocks
    // (or folds in at least 16 recent rows),
    // so a short sequence in a long cache uses the first few splits only and the others leave here, before
    // they build tables (every workgroup of the row computes the same count; the merge expects that many).
    uint32_t want = nblk / 4u > (uint32_t)R / 16u ? nblk / 4u : (uint32_t)R / 16u;  // ... or 16 recent rows
    if (a.B > 1 && a.S > 1) {  // ... and in a batch no more than the sequence's share of the compute units
        const uint32_t cap = live_split_cap(a, a.Hq, N + R, w_lane);
        want = want < cap ? want : cap;
    }
    const int S = (int)(want < 1u ? 1u : (want < (uint32_t)S_grid ? want : (uint32_t)S_grid));
    if (split >= S)
        return;
    const int blk0 = (int)(nblk * (uint32_t)split / (uint32_t)S);
    const int blk1 = (int)(nblk * (uint32_t)(split + 1) / (uint32_t)S);
    const int r0 = (int)((uint32_t)R * (uint32_t)split / (uint32_t)S);
    const int r1 = (int)((uint32_t)R * (uint32_t)(split + 1) / (uint32_t)S);

    const uint8_t *k_head = a.k_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;
    const uint8_t *v_head = a.v_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;

    // Code buffers of a wavefront.  Every code load is unconditional, so the compiler knows exactly
    // how many loads are in flight at each use and a wait for one buffer never drains another's
    // loads.  A wavefront that has run out of blocks issues a dead load instead (`live` false): all
    // lanes read the first 16 bytes of a block it has already read, one line instead of 4 KiB.
    //  M = 64 (8 KiB per block): one K and one V buffer, each refilled as soon as its pass is over
    //          — the V codes of a block are requested when its score pass starts, the K codes of
    //          the next block when that score pass ends.
    //  M = 32 (4 KiB per block): two K+V buffers, the whole next block loads during this one;
    //          the staggered scheme keeps too few bytes in flight for the smaller blocks
    //          (measured 417 us against 394 us at 16 x 32 heads x 64K).
    // Deeper queues than these were measured to be slower: HBM saturates with a few KiB in
    // flight per wavefront, more only lengthens the queue and with it the start-up and the drain.
    // READ_ONCE: one query head per KV head, so every code byte is read by exactly one workgroup,
    // once, and is loaded with the non-temporal hint (see load_codes).  With grouped queries the G
    // workgroups of a group share the code stream through their XCD's L2 and load normally.
    constexpr int NBUF = (M == 64 && F16) ? 1 : 2;  // fp32 contexts: two buffers, K codes in one phase, V codes in the other
    uint4 kbuf[NBUF][M / 16], vbuf[NBUF][M / 16];
    auto load_k = [&](uint4 (&dst)[M / 16], int blk_id, bool live) {
        const u32x4 *kp = (const u32x4 *)(k_head + (int64_t)blk_id * (64 * M)) + (live ? lane : 0);
        const int step = live ? 64 : 0;
#pragma unroll
        for (int j = 0; j < M / 16; ++j)
            dst[j] = load_codes<READ_ONCE>(kp + j * step);
    };
    auto load_v = [&](uint4 (&dst)[M / 16], int blk_id, bool live) {
        const u32x4 *vp = (const u32x4 *)(v_head + (int64_t)blk_id * (64 * M)) + (live ? lane : 0);
        const int step = live ? 64 : 0;
#pragma unroll
        for (int j = 0; j < M / 16; ++j)
            dst[j] = load_codes<READ_ONCE>(vp + j * step);
    };
    // Wavefront w starts with block blk0 + w; every later block of the split goes to whichever
    // wavefront asks next, so wavefronts that the memory system or the SIMD arbiter serve
    // faster scan more and all of them reach the merge together.  (Which wavefront sums which
    // block varies from run to run: outputs agree to fp32 rounding, not bit for bit.)
    int blk = blk0 + wave;
    *(lds_u32 *)(lbase + CTR_OFF) = (uint32_t)(blk0 + NW);  // same value from every thread: no branch
    const uint32_t ctr_addr = (uint32_t)(uintptr_t)(lbase + CTR_OFF);
    load_k(kbuf[0], blk < blk1 ? blk : 0, blk < blk1);
    if (F16 && NBUF == 2)
        load_v(vbuf[0], blk < blk1 ? blk : 0, blk < blk1);

    // ---- this lane's query sub-vector, pre-multiplied by scale * log2(e)
    const int sub = lane & (M - 1);
    float qs[DS];
#pragma unroll
    for (int j = 0; j < DS; ++j)
        qs[j] = elem<T>::ld(a.q, ((int64_t)b * a.Hq + hq) * PQ_HEAD_DIM + sub * DS + j) * a.scale_log2e;

    {
        float qv[4 * DS];
#pragma unroll
        for (int e = 0; e < 4 * DS; ++e)
            qv[e] = elem<T>::ld(&qraw[0], e) * a.scale_log2e;
#pragma unroll
        for (int k = 0; k < PASSES; ++k) {
            f32x4 ent;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float e = 0.f;
#pragma unroll
                for (int j = 0; j < DS; ++j)
                    e = fmaf(qv[u * DS + j], elem<T>::ld(&kraw[k][0], u * DS + j), e);
                ent[u] = e;
            }
            *(lds_f32x4 *)(lbase + LUT_OFF + (row0 + k * ROWS_PER_PASS) * 256 + g * 16) = ent;
        }
        if (F16) {
#pragma unroll
            for (int v = 0; v < VPT; ++v)
                *(lds_u32x4 *)(lbase + VCB_OFF + (tid + v * (NW * 64)) * 16) = vraw[v];
        }
    }
    __syncthreads();

    // column bytes of the score pass: byte k of idx[r] = 4 * ((4r + k + lane) % 64), the four bytes at once
    // (no byte of any intermediate exceeds 255, so nothing carries from byte to byte)
    uint32_t idx[M / 4];
#pragma unroll
    for (int r = 0; r < M / 4; ++r)
        idx[r] = (((uint32_t)(4 * r + lane) * 0x01010101u + 0x03020100u) & 0x3f3f3f3fu) << 2;
    // value pass: byte 0 = this lane's column offset in a 256-byte codebook row,
    // byte 1 = bits 16..23 of the codebook image's LDS address
    const uint32_t vcol = (uint32_t)(sub * (2 * DS)) | ((VCB_OFF >> 16) << 8);
    const int half_id = lane >> 5;  // M = 32: which of the two interleaved token streams

    float m_run = NEG_BIG;  // running maximum (wave-uniform)
    float l_lane = 0.f;     // this lane's share of the sum of weights
    float acc[DS];
#pragma unroll
    for (int j = 0; j < DS; ++j)
        acc[j] = 0.f;

    lds_u8 *pline = lbase + PBUF_OFF + wave * 256;

    auto process = [&](const uint4 (&kb)[M / 16], const uint4 (&vb)[M / 16], const int blk, auto &&after_score) {
        // ---------------- score pass
        float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < M / 4; ++r) {
            const uint32_t w = comp(kb[r >> 2], r & 3);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t sel = 0x0c0c0000u | ((4 + k) << 8) | k;
                const uint32_t addr = __builtin_amdgcn_perm(w, idx[r], sel);
                s4[k] += *(lds_f32 *)(lbase + addr);
            }
        }
        after_score();  // the score pass is done with this block's K codes
        const bool valid = blk * 64 + lane < N;
        const float s = valid ? (s4[0] + s4[1]) + (s4[2] + s4[3]) : NEG_BIG;

        // ---------------- running softmax
        float p;
        if constexpr (M == 32) {
            // M = 32 is close to the vector-ALU issue limit, so here the reference maximum moves only when a
            // score of the block exceeds it by more than 8 (a factor 2^8 in weight; a wave-wide vote): the
            // weights stay below 2^8, far inside the range of the fp32 sums, and nearly every block after the
            // first few skips the wave-wide maximum and the rescaling (16 x 32 heads x 64K: 350 -> 335 us).
            // At M = 64 the extra branch costs more than it saves (it makes the wait counts conservative).
            if (__builtin_amdgcn_ballot_w64(s > m_run + 8.0f) != 0) {  // wave-uniform
                const float m_new = fmaxf(m_run, wave_max(s));
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_lane *= alpha;
#pragma unroll
                for (int j = 0; j < DS; ++j)
                    acc[j] *= alpha;
                m_run = m_new;
            }
            p = valid ? __builtin_amdgcn_exp2f(s - m_run) : 0.f;
            l_lane += p;
        } else {
            const float m_new = fmaxf(m_run, wave_max(s));
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            p = valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
            l_lane = fmaf(l_lane, alpha, p);
#pragma unroll
            for (int j = 0; j < DS; ++j)
                acc[j] *= alpha;
            m_run = m_new;
        }
        *(lds_f32 *)(pline + lane * 4) = p;
        __builtin_amdgcn_wave_barrier();

        // ---------------- value pass
#pragma unroll
        for (int n = 0; n < M / 16; ++n) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t w = comp(vb[n], r);
                const int tok0 = (M == 64) ? (16 * n + 4 * r) : (32 * n + 16 * half_id + 4 * r);
                const f32x4 p4 = *(lds_f32x4 *)(pline + tok0 * 4);
                const float pk[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (F16) {
                        const uint32_t sel = 0x0c010000u | ((4 + k) << 8);
                        const uint32_t addr = __builtin_amdgcn_perm(w, vcol, sel);
                        if (DS == 2) {
                            const uint32_t cv = *(lds_u32 *)(lbase + addr);
                            const __half2 h = *(const __half2 *)&cv;
                            acc[0] = fmaf(pk[k], __low2float(h), acc[0]);
                            acc[1] = fmaf(pk[k], __high2float(h), acc[1]);
                        } else {
                            const u32x2 cv = *(lds_u32x2 *)(lbase + addr);
                            const uint32_t c0 = cv.x, c1 = cv.y;
                            const __half2 h0 = *(const __half2 *)&c0;
                            const __half2 h1 = *(const __half2 *)&c1;
                            acc[0] = fmaf(pk[k], __low2float(h0), acc[0]);
                            acc[1] = fmaf(pk[k], __high2float(h0), acc[1]);
                            acc[DS - 2] = fmaf(pk[k], __low2float(h1), acc[DS - 2]);
                            acc[DS - 1] = fmaf(pk[k], __high2float(h1), acc[DS - 1]);
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    if constexpr (!F16) {
        // fp32 contexts.  The table (64 KiB) and the fp32 value codebook image (128 KiB) do not fit LDS together, so
        // the split is scanned in chunks of F32_CHUNK blocks, each in two phases with the whole workgroup in step:
        //   phase 1  the table is resident; every wavefront scores its blocks of the chunk (block c0 + wave, then
        //            every NW-th) and leaves the raw scores in LDS;
        //   swap     the image of the value codebook replaces the table (read once more from L2);
        //   phase 2  the same blocks again: running softmax on the stored scores, then the value pass, whose
        //            gathers (8 or 16 bytes per lane, row = code, column = subspace) are conflict-free;
        //   before the next chunk the table is rebuilt from the key codebook.
        // A chunk moves 4096 tokens' codes (512 KiB at M = 64) for 256 KiB of codebook re-reads out of L2.
        constexpr int KV = M / 16;
        constexpr int IMG_VEC = 8192 / (NW * 64);  // 16-byte vectors of the image per thread
        const u32x4 *vimg = (const u32x4 *)((const float *)a.vcb_packed + (int64_t)hkv * 256 * PQ_HEAD_DIM);
        const uint32_t vcol32 = (uint32_t)(sub * DS * 4);
        // the table again, for the chunks after the first (the prologue's steps in one go)
        auto rebuild_table = [&]() {
#pragma unroll
            for (int k = 0; k < PASSES; ++k)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    kraw[k][v] = *(const u32x4 *)(kcb + ((row0 + k * ROWS_PER_PASS) * PQ_HEAD_DIM + e0) * sizeof(T) + v * 16);
#pragma unroll
            for (int v = 0; v < NV; ++v)
                qraw[v] = *(const u32x4 *)((const char *)a.q + (((int64_t)b * a.Hq + hq) * PQ_HEAD_DIM + e0) * sizeof(T) + v * 16);
            float qv[4 * DS];
#pragma unroll
            for (int e = 0; e < 4 * DS; ++e)
                qv[e] = elem<T>::ld(&qraw[0], e) * a.scale_log2e;
#pragma unroll
            for (int k = 0; k < PASSES; ++k) {
                f32x4 ent;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float e = 0.f;
#pragma unroll
                    for (int j = 0; j < DS; ++j)
                        e = fmaf(qv[u * DS + j], elem<T>::ld(&kraw[k][0], u * DS + j), e);
                    ent[u] = e;
                }
                *(lds_f32x4 *)(lbase + LUT_OFF + (row0 + k * ROWS_PER_PASS) * 256 + g * 16) = ent;
            }
        };
        auto score_block = [&](const uint4 (&kb)[KV], const int blk_id, const int c0) {
            float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < M / 4; ++r) {
                const uint32_t w = comp(kb[r >> 2], r & 3);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t sel = 0x0c0c0000u | ((4 + k) << 8) | k;
                    s4[k] += *(lds_f32 *)(lbase + __builtin_amdgcn_perm(w, idx[r], sel));
                }
            }
            const bool valid = blk_id * 64 + lane < N;
            *(lds_f32 *)(lbase + SBUF_OFF + ((blk_id - c0) * 64 + lane) * 4) =
                valid ? (s4[0] + s4[1]) + (s4[2] + s4[3]) : NEG_BIG;
        };
        auto value_block = [&](const uint4 (&vb)[KV], const int blk_id, const int c0) {
            const float s = *(lds_f32 *)(lbase + SBUF_OFF + ((blk_id - c0) * 64 + lane) * 4);
            const bool valid = blk_id * 64 + lane < N;
            const float m_new = fmaxf(m_run, wave_max(s));
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            const float p = valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
            l_lane = fmaf(l_lane, alpha, p);
#pragma unroll
            for (int j = 0; j < DS; ++j)
                acc[j] *= alpha;
            m_run = m_new;
            *(lds_f32 *)(pline + lane * 4) = p;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int n = 0; n < KV; ++n) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t w = comp(vb[n], r);
                    const int tok0 = (M == 64) ? (16 * n + 4 * r) : (32 * n + 16 * half_id + 4 * r);
                    const f32x4 p4 = *(lds_f32x4 *)(pline + tok0 * 4);
                    const float pk[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t addr = (((w >> (8 * k)) & 255u) << 9) | vcol32;  // image row = 512 bytes
                        if constexpr (DS == 2) {
                            const lds_f32 *cv = (const lds_f32 *)(lbase + addr);
                            const float c0v = cv[0], c1v = cv[1];
                            acc[0] = fmaf(pk[k], c0v, acc[0]);
                            acc[1] = fmaf(pk[k], c1v, acc[1]);
                        } else {
                            const f32x4 cv = *(lds_f32x4 *)(lbase + addr);
                            acc[0] = fmaf(pk[k], cv.x, acc[0]);
                            acc[1] = fmaf(pk[k], cv.y, acc[1]);
                            acc[DS - 2] = fmaf(pk[k], cv.z, acc[DS - 2]);
                            acc[DS - 1] = fmaf(pk[k], cv.w, acc[DS - 1]);
                        }
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        };
        for (int c0 = blk0; c0 < blk1; c0 += F32_CHUNK) {
            const int c1 = c0 + F32_CHUNK < blk1 ? c0 + F32_CHUNK : blk1;
            int cur = c0 + wave;
            if (c0 != blk0) {  // (the first chunk's table and first K codes come from the prologue)
                __syncthreads();  // the value pass of the previous chunk is over: the image may go
                load_k(kbuf[0], cur < c1 ? cur : c0, cur < c1);
                rebuild_table();
                __syncthreads();
            }
            // ---- phase 1: scores (two blocks per trip so that the buffers swap roles without copies)
            bool more = cur < c1;
            while (more) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (more) {
                        const int nb = cur + NW;
                        load_k(kbuf[j ^ 1], nb < c1 ? nb : cur, nb < c1);
                        score_block(kbuf[j], cur, c0);
                        cur = nb;
                        more = nb < c1;
                    }
                }
            }
            // ---- swap: the value codebook image over the table
            cur = c0 + wave;
            load_v(vbuf[0], cur < c1 ? cur : c0, cur < c1);
            __syncthreads();  // nobody reads the table any more
#pragma unroll
            for (int h = 0; h < IMG_VEC; h += 8) {
                u32x4 t[8];
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    t[v] = vimg[tid + (h + v) * (NW * 64)];
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    *(lds_u32x4 *)(lbase + (tid + (h + v) * (NW * 64)) * 16) = t[v];
            }
            __syncthreads();
            // ---- phase 2: softmax and value pass over the same blocks
            more = cur < c1;
            while (more) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (more) {
                        const int nb = cur + NW;
                        load_v(vbuf[j ^ 1], nb < c1 ? nb : cur, nb < c1);
                        value_block(vbuf[j], cur, c0);
                        cur = nb;
                        more = nb < c1;
                    }
                }
            }
        }
    } else if constexpr (NBUF == 1) {
        while (blk < blk1) {
            const int nb = lds_grab(ctr_addr);
            const int next_blk = nb < blk1 ? nb : blk;
            load_v(vbuf[0], blk, true);
            process(kbuf[0], vbuf[0], blk, [&]() { load_k(kbuf[0], next_blk, nb < blk1); });
            blk = nb;
        }
    } else {
        // two blocks per trip so that the buffers swap roles without register copies
        bool more = blk < blk1;
        while (more) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (more) {
                    const int nb = lds_grab(ctr_addr);
                    load_k(kbuf[j ^ 1], nb < blk1 ? nb : blk, nb < blk1);
                    load_v(vbuf[j ^ 1], nb < blk1 ? nb : blk, nb < blk1);
                    process(kbuf[j], vbuf[j], blk, []() {});
                    blk = nb;
                    more = nb < blk1;
                }
            }
        }
    }

    // ---------------- recent full-precision rows of this split (Eq. 7, second term)
    {
        // M = 32: only lanes 0..31 own output dims here (lanes 32..63 carry the second
        // token stream of the value pass and are merged below)
        const bool owner = (M == 64) || lane < 32;
        const int64_t rbase = ((int64_t)b * a.Hkv + hkv) * a.max_recent;
        // RB rows per trip: their loads go out together, so a wavefront with many rows (one split per head,
        // a few hundred recent rows) pays one memory round trip per RB rows instead of one per row.  Rows
        // beyond the range re-read the trip's first row and are skipped.  16 per trip when the wavefront has more
        // than 4 rows — with short sequences in a large batch the window is a large share of the work and its round
        // trips are not hidden by anything (256 x 32 heads x 1K tokens, 128 rows: 434 -> 363 us; 128 x 2K: 274 -> 253
        // us) — and 4 otherwise (the 14 dead loads of a 16-row trip cost 0.4 us on 1 x 32 heads x 32K, where a
        // wavefront has 2 rows).
        // (the rows wait in their registers as loaded — fp16 pairs — and are converted when used)
        constexpr int RW = DS * (int)sizeof(T) / 4;  // 32-bit words of a lane's DS elements
        auto rows = [&](auto rb_tag) {
            constexpr int RB = decltype(rb_tag)::value;
            for (int r = r0 + wave; r < r1; r += NW * RB) {
                uint32_t kw[RB][RW], vw[RB][RW];
#pragma unroll
                for (int u = 0; u < RB; ++u) {
                    const int rr = r + u * NW < r1 ? r + u * NW : r;
                    const uint32_t *kp = (const uint32_t *)((const T *)a.recent_k + (rbase + rr) * PQ_HEAD_DIM + sub * DS);
                    const uint32_t *vp = (const uint32_t *)((const T *)a.recent_v + (rbase + rr) * PQ_HEAD_DIM + sub * DS);
#pragma unroll
                    for (int x = 0; x < RW; ++x) {
                        kw[u][x] = owner ? kp[x] : 0u;
                        vw[u][x] = owner ? vp[x] : 0u;
                    }
                }
#pragma unroll
                for (int u = 0; u < RB; ++u) {
                    if (r + u * NW < r1) {  // wave-uniform
                        float dot = 0.f;
#pragma unroll
                        for (int j = 0; j < DS; ++j)
                            dot = fmaf(qs[j], elem<T>::ld(&kw[u][0], j), dot);
                        const float s = wave_sum(dot);
                        const float m_new = fmaxf(m_run, s);
                        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                        const float p = __builtin_amdgcn_exp2f(s - m_new);
                        l_lane = fmaf(l_lane, alpha, lane == 0 ? p : 0.f);
#pragma unroll
                        for (int j = 0; j < DS; ++j)
                            acc[j] = fmaf(acc[j], alpha, p * elem<T>::ld(&vw[u][0], j));
                        m_run = m_new;
                    }
                }
            }
        };
        // the larger trip: 16 rows for fp16 in the 8-wavefront kernel (32 registers), 8 in the 16-wavefront kernels
        // (128 registers per lane); fp32 contexts keep 4
        constexpr int RB_BIG = sizeof(T) == 2 ? (NW == 8 ? 16 : 8) : 4;
        if (RB_BIG > 4 && r1 - r0 > 4 * NW)  // workgroup-uniform
            rows(std::integral_constant<int, RB_BIG>{});
        else
            rows(std::integral_constant<int, 4>{});
    }

    // ---------------- merge the wavefronts of this workgroup
    {
        const float l_w = wave_sum(l_lane);
        if (M == 32) {
#pragma unroll
            for (int j = 0; j < DS; ++j)
                acc[j] += __shfl_xor(acc[j], 32);
        }
        lds_f32 *part = (lds_f32 *)(lbase + PART_OFF) + wave * PQ_PART_STRIDE;
        if (lane == 0) {
            part[0] = m_run;
            part[1] = l_w;
        }
        if (M == 64 || lane < 32) {
#pragma unroll
            for (int j = 0; j < DS; ++j)
                part[4 + sub * DS + j] = acc[j];
        }
    }
    __syncthreads();

    // From here on only wavefront 0 works: it merges the workgroup's wavefronts (lane l owns
    // output dims 2l, 2l+1), publishes the split partial and takes a ticket.
    if (wave != 0)
        return;
    float *gpart = a.partials + ((int64_t)bh * S_grid + split) * PQ_PART_STRIDE;
    float *orow = a.out + (int64_t)bh * PQ_HEAD_DIM;
    const lds_f32 *parts = (const lds_f32 *)(lbase + PART_OFF);
    float mx = NEG_BIG;
#pragma unroll
    for (int w = 0; w < NW; ++w)
        mx = fmaxf(mx, parts[w * PQ_PART_STRIDE]);
    float o0 = 0.f, o1 = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float f = __builtin_amdgcn_exp2f(parts[w * PQ_PART_STRIDE] - mx);
        o0 = fmaf(parts[w * PQ_PART_STRIDE + 4 + 2 * lane], f, o0);
        o1 = fmaf(parts[w * PQ_PART_STRIDE + 5 + 2 * lane], f, o1);
        l = fmaf(parts[w * PQ_PART_STRIDE + 1], f, l);
    }
    if (S == 1) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
        *(float2 *)(orow + 2 * lane) = make_float2(o0 * inv, o1 * inv);
        return;
    }
    // The partial is published with device-scope stores (they are performed at the memory all
    // XCDs share, not left dirty in this XCD's L2), so the only thing the ticket has to wait for
    // is their completion; a release fence would add a whole-L2 write-back (about 1.8 us).
    publish(gpart + 4 + 2 * lane, o0, o1);
    if (lane == 0)
        publish(gpart, mx, l);
    publish_wait();

    // ---------------- the workgroup that takes the last ticket of this (b, hq) merges the
    // splits (flash-decoding style) and leaves the ticket counter at zero for the next call
    unsigned int ticket = 0;
    if (lane == 0)
        ticket = __hip_atomic_fetch_add(a.tickets + bh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != (unsigned int)(S - 1))
        return;
    asm volatile("" ::: "memory");  // the loads below stay behind the ticket in the instruction stream
    // the other splits' partials: device-scope loads, issued after the ticket has returned
    const float *ps = a.partials + (int64_t)bh * S_grid * PQ_PART_STRIDE;
    // Lane s holds (maximum, weight sum) of split s.  The first eight splits' output loads are issued
    // together with that load, so the merge costs one memory round trip for up to eight splits.
    float2 o[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
        o[u] = u < S ? fetch(ps + u * PQ_PART_STRIDE + 4 + 2 * lane) : make_float2(0.f, 0.f);
    const float2 ml = lane < S ? fetch(ps + lane * PQ_PART_STRIDE) : make_float2(NEG_BIG, 0.f);
    mx = wave_max(ml.x);
    const float f_lane = __builtin_amdgcn_exp2f(ml.x - mx);
    l = wave_sum(ml.y * f_lane);
    o0 = o1 = 0.f;
    for (int s0 = 0;;) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f_lane), (s0 + u) & 63));
            o0 = fmaf(o[u].x, f, o0);
            o1 = fmaf(o[u].y, f, o1);
        }
        s0 += 8;
        if (s0 >= S)
            break;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            o[u] = s0 + u < S ? fetch(ps + (s0 + u) * PQ_PART_STRIDE + 4 + 2 * lane) : make_float2(0.f, 0.f);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    *(float2 *)(orow + 2 * lane) = make_float2(o0 * inv, o1 * inv);
    if (lane == 0)
        ticket_reset(a.tickets + bh);
}

template <int M, int DS, typename T, int NW, bool READ_ONCE>
hipError_t launch(const pq_decode_args &a, hipStream_t s)
{
    const int grid = a.B * a.Hq * a.S;
    hipLaunchKernelGGL((pq_decode_kernel<M, DS, T, NW, READ_ONCE>), dim3(grid), dim3(NW * 64), 0, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t pq_launch_decode(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s)
{
    const bool f16 = ctx->cfg.dtype == PQ_F16;
    // Wavefronts per workgroup.  With one query head per KV head the scan is bound by HBM; at
    // M = 64 (8 KiB per block) 8 wavefronts — less data in flight, shorter queues — measured
    // fastest, at M = 32 (4 KiB per block) 16 do (16 x 32 heads x 64K: 355 us against 381 us).
    // With grouped queries every code byte is scored by G workgroups out of one XCD's L2, the scan
    // is bound by the vector ALU and LDS, and 16 wavefronts (4 per SIMD) hide their latencies
    // better (79 us against 86 us at 32 query heads over 8 KV heads, 128K context).
    const bool shared = ctx->group > 1;
    if (ctx->cfg.n_subspaces == 64) {
        if (shared)
            return f16 ? launch<64, 2, __half, 16, false>(a, s) : launch<64, 2, float, 16, false>(a, s);
        return f16 ? launch<64, 2, __half, 8, true>(a, s) : launch<64, 2, float, 8, true>(a, s);
    }
    if (shared)
        return f16 ? launch<32, 4, __half, 16, false>(a, s) : launch<32, 4, float, 16, false>(a, s);
    return f16 ? launch<32, 4, __half, 16, true>(a, s) : launch<32, 4, float, 16, true>(a, s);
}
