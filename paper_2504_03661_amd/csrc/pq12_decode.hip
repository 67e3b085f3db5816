// Decode attention over a KV cache quantized with 12-bit PQ codes (M = 32 subspaces of 4 dims, 4096
// centroids per subspace: the paper's 3-bit-per-dimension setting, Section IV-A), one fused kernel.
//
// Same result as the 8-bit kernels (Eq. 7 = Eq. 6: tables q^i . (C_K^i)^T sampled by the key codes, one
// softmax shared with the full-precision rows, values aggregated through C_V by the value codes), but
// the tables no longer fit: 32 x 4096 fp32 table entries are 512 KiB, the fp16 value codebook 1 MiB, the
// LDS of a compute unit 160 KiB.  So a workgroup walks the SUBSPACES in groups, with one 128 KiB table
// region in LDS that is refilled per group, and keeps what must survive from group to group — the
// partial scores of its tokens — in registers: a wavefront owns up to 16 blocks of 128 tokens (32
// scores per lane), a workgroup up to 32K tokens per round.
//
//   score passes   4 groups of 8 subspaces: build the group's table [8][4096] fp32 from the key codebook
//                  (L2) and the query, then every wavefront adds, for each of its blocks (lane = token),
//                  the 8 sampled entries per token to that token's score register;
//   softmax        all scores of the round are known: maximum over the workgroup, running maximum /
//                  rescale only between rounds, weights replace the scores in their registers;
//   value passes   8 groups of 4 subspaces: copy the group's slice of the value codebook (128 KiB) to
//                  LDS; a wavefront then takes its blocks one by one: the block's 128 weights go to a
//                  line of LDS that only this wavefront uses, and lane = (subspace of the group, one of
//                  16 token streams) gathers the 8-byte centroid of its subspace for every 16th token and
//                  accumulates weight x centroid; the 16 streams are summed once, at the end.
// The code tensors are group-major (pq_internal.h) so that every pass streams exactly its own bytes:
// each code byte still comes from HBM once, and is loaded with the non-temporal hint: the stream then leaves
// the codebooks — 2 MiB per head, read again by every launch — in the memory-side cache instead of pushing
// them out (8 sequences x 32 heads x 32K: 236 -> 198 us).  Table traffic is 2 MiB of codebook per workgroup and round
// from L2.  Gathers from a [subspace][code] table hit random banks (no layout can avoid that for
// random codes): LDS, not HBM, bounds this kernel.  The recent rows, the split merge and the ticket
// protocol are those of the 8-bit kernel.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "pq_internal.h"
#include "pq_device_utils.h"

namespace {

constexpr int NW12 = 16;
constexpr int RB12 = 4;                               // recent rows a wavefront loads together
constexpr int TAB_OFF = 0;                            // 128 KiB: score table [8][4096] fp32 / value image [4][4096][4] fp16
constexpr int P_OFF = 131072;                         // float [16][128]: weights of the block a wavefront works on
constexpr int Q12_OFF = P_OFF + NW12 * 512;           // float [128]: query x scale x log2(e)
constexpr int WMAX_OFF = Q12_OFF + 512;               // float [16]
constexpr int PART12_OFF = WMAX_OFF + 64;             // float [16][PQ_PART_STRIDE]
constexpr int SMEM12_BYTES = PART12_OFF + NW12 * PQ_PART_STRIDE * 4;
static_assert(SMEM12_BYTES <= 160 * 1024, "LDS budget of a gfx950 compute unit");

__device__ inline void unpack8(const uint32_t w0, const uint32_t w1, const uint32_t w2, uint32_t (&c)[8])
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

__device__ inline float dot4(const f32x4 &q, uint32_t lo, uint32_t hi)
{
    const __half2 a = *(const __half2 *)&lo, b = *(const __half2 *)&hi;
    float e = q.x * __low2float(a);
    e = fmaf(q.y, __high2float(a), e);
    e = fmaf(q.z, __low2float(b), e);
    return fmaf(q.w, __high2float(b), e);
}

// WAVE_VB: 128-token blocks per wavefront and round (two score registers per lane each); a workgroup
// takes 16 WAVE_VB blocks per round.  16 (32K tokens per round) keeps the table refills rare on long
// splits; short splits use a leaner instantiation.
template <int WAVE_VB>
__global__ __launch_bounds__(NW12 * 64) void pq12_decode_kernel(const pq_decode_args a)
{
    constexpr int ROUND_VB = NW12 * WAVE_VB;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM12_BYTES];
    lds_u8 *lbase = (lds_u8 *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const uint32_t grid = gridDim.x;
    uint32_t logical = blockIdx.x;
    if ((grid & 7u) == 0)
        logical = (blockIdx.x & 7u) * (grid >> 3) + (blockIdx.x >> 3);
    const int S = a.S;
    // Neighbouring workgroups (one XCD): the splits of a (sequence, head), then the same head of the other
    // sequences — they refill their table region from the same 2 MiB of codebooks, which then come from the
    // XCD's L2 instead of once per sequence from memory.
    const int unit = (int)(logical / (uint32_t)S);
    const int split = (int)(logical - (uint32_t)unit * (uint32_t)S);
    const int hq = (int)((uint32_t)unit / (uint32_t)a.B);
    const int b = unit - hq * a.B;
    const int bh = b * a.Hq + hq;
    const int hkv = (int)((uint32_t)hq / (uint32_t)a.G);

    int N = a.ctx_len[b];
    int R = (a.recent_k != nullptr && a.recent_len != nullptr) ? a.recent_len[b] : 0;
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    R = R < 0 ? 0 : (R > a.max_recent ? a.max_recent : R);
    const uint32_t nvb = (uint32_t)(N + 127) >> 7;  // 128-token blocks of the sequence
    const int vb0 = (int)(nvb * (uint32_t)split / (uint32_t)S);
    const int vb1 = (int)(nvb * (uint32_t)(split + 1) / (uint32_t)S);
    const int r0 = (int)((uint32_t)R * (uint32_t)split / (uint32_t)S);
    const int r1 = (int)((uint32_t)R * (uint32_t)(split + 1) / (uint32_t)S);

    const uint8_t *k_head = a.k_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;
    const uint8_t *v_head = a.v_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;
    const __half *kcb = (const __half *)a.kcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;
    const __half *vcb = (const __half *)a.vcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;

    lds_f32 *qs = (lds_f32 *)(lbase + Q12_OFF);
    lds_f32 *pw = (lds_f32 *)(lbase + P_OFF);
    lds_f32 *wmax = (lds_f32 *)(lbase + WMAX_OFF);
    if (tid < PQ_HEAD_DIM)
        qs[tid] = __half2float(((const __half *)a.q)[((int64_t)b * a.Hq + hq) * PQ_HEAD_DIM + tid]) * a.scale_log2e;

    float m_run = NEG_BIG;  // running maximum, the same in every wavefront of the workgroup
    float l_lane = 0.f;
    float acc[8][4];
#pragma unroll
    for (int g = 0; g < 8; ++g)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[g][j] = 0.f;

    const uint32_t *k_units = (const uint32_t *)k_head + lane * 3;
    const uint32_t *v_units = (const uint32_t *)v_head + lane * 3;
    lds_f32 *pline = pw + wave * 128;

    for (int sb = vb0; sb < vb1; sb += ROUND_VB) {
        // wavefront w owns blocks sb + w + 16 jj, jj < n_jj (128 tokens each: two score registers per lane)
        const int left = vb1 - sb - wave;
        const int n_jj = left <= 0 ? 0 : (left + NW12 - 1) / NW12 < WAVE_VB ? (left + NW12 - 1) / NW12 : WAVE_VB;
        const int last_vb = vb1 - 1;  // loads beyond the wavefront's blocks re-read a valid block and are not used
        float score[2 * WAVE_VB];
#pragma unroll
        for (int e = 0; e < 2 * WAVE_VB; ++e)
            score[e] = 0.f;

        // ---------------- score passes: 4 groups of 8 subspaces
        for (int g = 0; g < 4; ++g) {
            // the first block's codes are requested before the table is built
            uint32_t cur[6], nxt[6];
            {
                const int vb = sb + wave < last_vb ? sb + wave : last_vb;
                const uint32_t *u = k_units + (((int64_t)(2 * vb) * 4 + g) * 64) * 3;
#pragma unroll
                for (int e = 0; e < 3; ++e) {
                    cur[e] = __builtin_nontemporal_load(u + (e));
                    cur[3 + e] = __builtin_nontemporal_load(u + (4 * 64 * 3 + e));  // the second 64-token block of the 128-token block
                }
            }
            __syncthreads();  // the table region is free (and, the first time, the query is in LDS)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int sub = 8 * g + i;
                const u32x4 *src = (const u32x4 *)(kcb + ((int64_t)sub * PQ12_CENTROIDS + 4 * tid) * 4);
                const u32x4 c01 = src[0], c23 = src[1];  // centroids 4 tid .. 4 tid + 3, four fp16 each
                const f32x4 q4 = *(lds_f32x4 *)(lbase + Q12_OFF + sub * 16);
                f32x4 ent;
                ent.x = dot4(q4, c01.x, c01.y);
                ent.y = dot4(q4, c01.z, c01.w);
                ent.z = dot4(q4, c23.x, c23.y);
                ent.w = dot4(q4, c23.z, c23.w);
                *(lds_f32x4 *)(lbase + TAB_OFF + (i * PQ12_CENTROIDS + 4 * tid) * 4) = ent;
            }
            __syncthreads();
#pragma unroll
            for (int jj = 0; jj < WAVE_VB; ++jj) {
                if (jj >= n_jj)
                    continue;  // wave-uniform; `continue`, not `break`: the loop must unroll (registers are indexed by jj)
                {
                    const int want = sb + wave + NW12 * (jj + 1);
                    const int vb = want < last_vb ? want : last_vb;
                    const uint32_t *u = k_units + (((int64_t)(2 * vb) * 4 + g) * 64) * 3;
#pragma unroll
                    for (int e = 0; e < 3; ++e) {
                        nxt[e] = __builtin_nontemporal_load(u + (e));
                        nxt[3 + e] = __builtin_nontemporal_load(u + (4 * 64 * 3 + e));
                    }
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint32_t c[8];
                    unpack8(cur[3 * h], cur[3 * h + 1], cur[3 * h + 2], c);
                    float sum = 0.f;
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8)
                        sum += *(lds_f32 *)(lbase + TAB_OFF + (s8 * PQ12_CENTROIDS + c[s8]) * 4);
                    score[2 * jj + h] += sum;
                }
#pragma unroll
                for (int e = 0; e < 6; ++e)
                    cur[e] = nxt[e];
            }
        }

        // ---------------- softmax of the round: the scores become weights
        float mx = NEG_BIG;
#pragma unroll
        for (int jj = 0; jj < WAVE_VB; ++jj)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tok = (sb + wave + NW12 * jj) * 128 + 64 * h + lane;
                const bool valid = jj < n_jj && tok < N;
                score[2 * jj + h] = valid ? score[2 * jj + h] : NEG_BIG;
                mx = fmaxf(mx, score[2 * jj + h]);
            }
        mx = wave_max(mx);
        if (lane == 0)
            wmax[wave] = mx;
        __syncthreads();
        const float m_new = fmaxf(m_run, wave_max(wmax[lane & 15]));
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_lane *= alpha;
#pragma unroll
        for (int g = 0; g < 8; ++g)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[g][j] *= alpha;
#pragma unroll
        for (int e = 0; e < 2 * WAVE_VB; ++e) {
            // an invalid token carries NEG_BIG; against a finite maximum that is weight 0, and a round whose
            // maximum is NEG_BIG itself has no valid token at all
            const float p = score[e] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(score[e] - m_new) : 0.f;
            l_lane += p;
            score[e] = p;
        }
        m_run = m_new;

        // ---------------- value passes: 8 groups of 4 subspaces
        for (int g = 0; g < 8; ++g) {
            uint32_t cur[3], nxt[3];
            {
                const int vb = sb + wave < last_vb ? sb + wave : last_vb;
                const uint32_t *u = v_units + (((int64_t)vb * 8 + g) * 64) * 3;
#pragma unroll
                for (int e = 0; e < 3; ++e)
                    cur[e] = __builtin_nontemporal_load(u + (e));
            }
            __syncthreads();  // the table region is free
            {
                const u32x4 *src = (const u32x4 *)(vcb + (int64_t)(4 * g) * PQ12_CENTROIDS * 4);
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    *(lds_u32x4 *)(lbase + TAB_OFF + (tid + k * (NW12 * 64)) * 16) = src[tid + k * (NW12 * 64)];
            }
            __syncthreads();
#pragma unroll
            for (int jj = 0; jj < WAVE_VB; ++jj) {
                if (jj >= n_jj)
                    continue;  // wave-uniform; `continue`, not `break`: the loop must unroll (registers are indexed by jj)
                {
                    const int want = sb + wave + NW12 * (jj + 1);
                    const int vb = want < last_vb ? want : last_vb;
                    const uint32_t *u = v_units + (((int64_t)vb * 8 + g) * 64) * 3;
#pragma unroll
                    for (int e = 0; e < 3; ++e)
                        nxt[e] = __builtin_nontemporal_load(u + (e));
                }
                // this block's 128 weights to the wavefront's own line
                __builtin_amdgcn_wave_barrier();
                pline[lane] = score[2 * jj];
                pline[64 + lane] = score[2 * jj + 1];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                uint32_t c[8];
                unpack8(cur[0], cur[1], cur[2], c);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float p = pline[(lane >> 2) + 16 * k];
                    const u32x2 cv = *(lds_u32x2 *)(lbase + TAB_OFF + ((lane & 3) * PQ12_CENTROIDS + c[k]) * 8);
                    const uint32_t lo = cv.x, hi = cv.y;
                    const __half2 h0 = *(const __half2 *)&lo, h1 = *(const __half2 *)&hi;
                    acc[g][0] = fmaf(p, __low2float(h0), acc[g][0]);
                    acc[g][1] = fmaf(p, __high2float(h0), acc[g][1]);
                    acc[g][2] = fmaf(p, __low2float(h1), acc[g][2]);
                    acc[g][3] = fmaf(p, __high2float(h1), acc[g][3]);
                }
#pragma unroll
                for (int e = 0; e < 3; ++e)
                    cur[e] = nxt[e];
            }
        }
    }

    // ---------------- sum the 16 token streams (lanes with equal lane % 4), then lane l owns dims 2l, 2l + 1
    lds_f32 *part = (lds_f32 *)(lbase + PART12_OFF) + wave * PQ_PART_STRIDE;
#pragma unroll
    for (int g = 0; g < 8; ++g)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v = acc[g][j];
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 4)
                part[4 + (4 * g + lane) * 4 + j] = v;
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    float o0 = part[4 + 2 * lane], o1 = part[5 + 2 * lane];
    __syncthreads();  // every wavefront has left the chunk loop: the query in LDS is still needed, the rest is free

    // ---------------- recent full-precision rows of this split (Eq. 7, second term), per wavefront
    {
        const float q0 = qs[2 * lane], q1 = qs[2 * lane + 1];
        const int64_t rbase = ((int64_t)b * a.Hkv + hkv) * a.max_recent;
        // RB12 rows per trip, their loads issued together (one memory round trip per trip, not per row); rows
        // beyond the range re-read the trip's first row and are skipped
        for (int r = r0 + wave; r < r1; r += NW12 * RB12) {
            __half2 kk[RB12], vv[RB12];
#pragma unroll
            for (int u = 0; u < RB12; ++u) {
                const int rr = r + u * NW12 < r1 ? r + u * NW12 : r;
                kk[u] = *((const __half2 *)((const __half *)a.recent_k + (rbase + rr) * PQ_HEAD_DIM) + lane);
                vv[u] = *((const __half2 *)((const __half *)a.recent_v + (rbase + rr) * PQ_HEAD_DIM) + lane);
            }
#pragma unroll
            for (int u = 0; u < RB12; ++u) {
                if (r + u * NW12 < r1) {  // wave-uniform
                    const float s = wave_sum(fmaf(q0, __low2float(kk[u]), q1 * __high2float(kk[u])));
                    const float m_new = fmaxf(m_run, s);
                    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                    const float p = __builtin_amdgcn_exp2f(s - m_new);
                    l_lane = fmaf(l_lane, alpha, lane == 0 ? p : 0.f);
                    o0 = fmaf(o0, alpha, p * __low2float(vv[u]));
                    o1 = fmaf(o1, alpha, p * __high2float(vv[u]));
                    m_run = m_new;
                }
            }
        }
    }

    // ---------------- merge the wavefronts, publish the split, merge the splits (as in the 8-bit kernel)
    {
        const float l_w = wave_sum(l_lane);
        if (lane == 0) {
            part[0] = m_run;
            part[1] = l_w;
        }
        part[4 + 2 * lane] = o0;
        part[5 + 2 * lane] = o1;
    }
    __syncthreads();
    if (wave != 0)
        return;
    float *gpart = a.partials + ((int64_t)bh * S + split) * PQ_PART_STRIDE;
    float *orow = a.out + (int64_t)bh * PQ_HEAD_DIM;
    const lds_f32 *parts = (const lds_f32 *)(lbase + PART12_OFF);
    float mx = NEG_BIG;
#pragma unroll
    for (int w = 0; w < NW12; ++w)
        mx = fmaxf(mx, parts[w * PQ_PART_STRIDE]);
    float l = 0.f;
    o0 = o1 = 0.f;
#pragma unroll
    for (int w = 0; w < NW12; ++w) {
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
    // device-scope stores, complete before the ticket; device-scope loads after it (see the 8-bit kernel)
    publish(gpart + 4 + 2 * lane, o0, o1);
    if (lane == 0)
        publish(gpart, mx, l);
    publish_wait();
    unsigned int ticket = 0;
    if (lane == 0)
        ticket = __hip_atomic_fetch_add(a.tickets + bh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != (unsigned int)(S - 1))
        return;
    asm volatile("" ::: "memory");  // the loads below stay behind the ticket in the instruction stream
    const float *ps = a.partials + (int64_t)bh * S * PQ_PART_STRIDE;
    const float2 ml = lane < S ? fetch(ps + lane * PQ_PART_STRIDE) : make_float2(NEG_BIG, 0.f);
    mx = wave_max(ml.x);
    const float f_lane = __builtin_amdgcn_exp2f(ml.x - mx);
    l = wave_sum(ml.y * f_lane);
    o0 = o1 = 0.f;
    for (int s = 0; s < S; ++s) {
        const float2 o = fetch(ps + s * PQ_PART_STRIDE + 4 + 2 * lane);
        const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f_lane), s & 63));
        o0 = fmaf(o.x, f, o0);
        o1 = fmaf(o.y, f, o1);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    *(float2 *)(orow + 2 * lane) = make_float2(o0 * inv, o1 * inv);
    if (lane == 0)
        ticket_reset(a.tickets + bh);
}


// ---------------------------------------------------------------------------------
// Two-pass path for few (sequence, query head) pairs.
//
// The fused kernel above splits a head's TOKENS over workgroups, and every workgroup streams all of the
// head's tables (1.5 MiB) through its LDS: with few heads and therefore many splits per head the table
// refills, not the codes, are most of the bytes a compute unit moves (1 x 32 heads x 32K: 1.5 MiB of tables
// against 0.4 MB of codes per workgroup).  Here the SUBSPACES are split instead, so that a workgroup loads
// one table region once and keeps it:
//   pass 1  one workgroup per (sequence, query head, group of 8 subspaces, token range): builds the
//           group's score table [8][4096] from the key codebook and the query, streams the group's key
//           units and writes, per token, the sum of its 8 sampled entries — a partial score — to memory
//           (4 floats per token and query head);
//   pass 2  one workgroup per (sequence, query head, group of 4 subspaces, token range): keeps the group's
//           slice of the value codebook in LDS, adds the 4 partial scores of a token, runs the running
//           softmax (every group of a head computes the same maximum and weight sum) and accumulates the
//           16 output dims of its subspaces.  With one token range per head the row is written directly;
//           otherwise the ranges are merged as in the fused kernel, behind one ticket per head.
// Each code byte still comes from HBM once; the partial scores cost 16 bytes per token and query head
// written and read back (pass 2 finds them in the memory-side cache).
// ---------------------------------------------------------------------------------
constexpr int W2_OFF = 131072;                 // pass 2: float [16][NB2][128] weights of the blocks a wavefront works on
constexpr int NB2 = 2;                         // pass 2: 128-token blocks a wavefront works on together
constexpr int Q2_OFF = W2_OFF + NW12 * NB2 * 512;  // float [128]: query x scale x log2(e)
constexpr int PART2_OFF = Q2_OFF + 512;        // pass 2: float [16][24]: maximum, weight sum, 2 unused, 16 dims
constexpr int PART2_STRIDE = 24;
constexpr int SMEM2_BYTES = PART2_OFF + NW12 * PART2_STRIDE * 4;
constexpr int PF2 = 1;                         // 128-token blocks a wavefront requests ahead (3 measured slower: 46 against 44 us)
static_assert(SMEM2_BYTES <= 160 * 1024, "LDS budget of a gfx950 compute unit");

__device__ inline uint32_t undeal(uint32_t id, uint32_t grid)
{
    // consecutive logical ids on one XCD (workgroups are dealt to the 8 XCDs round-robin)
    return (grid & 7u) == 0 ? (id & 7u) * (grid >> 3) + (id >> 3) : id;
}

__global__ __launch_bounds__(NW12 * 64) void pq12_scores_kernel(const pq_decode_args a, float *scores, const int TS)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM2_BYTES];
    lds_u8 *lbase = (lds_u8 *)smem;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const uint32_t logical = undeal(blockIdx.x, gridDim.x);
    const int bh = (int)(logical / (uint32_t)(4 * TS));
    const int rem = (int)(logical - (uint32_t)bh * (uint32_t)(4 * TS));
    const int g = rem / TS;
    const int ts = rem - g * TS;
    const int b = (int)((uint32_t)bh / (uint32_t)a.Hq);
    const int hq = bh - b * a.Hq;
    const int hkv = (int)((uint32_t)hq / (uint32_t)a.G);

    // Order of the prologue (as in the 8-bit kernels): everything that needs only the head index is requested
    // first — the length (through an index the compiler cannot prove uniform, so that the load stays in flight
    // instead of becoming a scalar load with a wait on the spot), the query, the first half of the codebook
    // slice — then the length is taken out of its register, the range is cut and the first codes are requested.
    const int zero = lane_zero();
    const int n_vec = a.ctx_len[b + zero];
    const __half *kcb = (const __half *)a.kcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;
    const float q_mine = tid < PQ_HEAD_DIM ? __half2float(((const __half *)a.q)[(int64_t)bh * PQ_HEAD_DIM + tid]) : 0.f;
    u32x4 craw[4][2];  // centroids 4 tid .. 4 tid + 3 of four subspaces, four fp16 each
    auto load_centroids = [&](int i0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4 *src = (const u32x4 *)(kcb + ((int64_t)(8 * g + i0 + i) * PQ12_CENTROIDS + 4 * tid) * 4);
            craw[i][0] = src[0];
            craw[i][1] = src[1];
        }
    };
    auto build_rows = [&](int i0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x4 q4 = *(lds_f32x4 *)(lbase + Q2_OFF + (8 * g + i0 + i) * 16);
            f32x4 ent;
            ent.x = dot4(q4, craw[i][0].x, craw[i][0].y);
            ent.y = dot4(q4, craw[i][0].z, craw[i][0].w);
            ent.z = dot4(q4, craw[i][1].x, craw[i][1].y);
            ent.w = dot4(q4, craw[i][1].z, craw[i][1].w);
            *(lds_f32x4 *)(lbase + TAB_OFF + ((i0 + i) * PQ12_CENTROIDS + 4 * tid) * 4) = ent;
        }
    };
    load_centroids(0);

    int N = __builtin_amdgcn_readfirstlane(n_vec);
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    const uint32_t nvb = (uint32_t)(N + 127) >> 7;
    const int vb0 = (int)(nvb * (uint32_t)ts / (uint32_t)TS);
    const int vb1 = (int)(nvb * (uint32_t)(ts + 1) / (uint32_t)TS);
    if (vb0 >= vb1)
        return;  // workgroup-uniform

    const uint8_t *k_head = a.k_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;
    const uint32_t *k_units = (const uint32_t *)k_head + lane * 3;
    const int64_t cap = a.head_stride / PQ12_TOKEN_BYTES;  // tokens per row of partial scores
    float *row = scores + ((int64_t)bh * 4 + g) * cap;

    // the first blocks' codes are requested before the table is built; PF2 blocks per wavefront stay in flight
    const int last_vb = vb1 - 1;
    uint32_t un[PF2][6];
    auto load_units = [&](uint32_t (&dst)[6], int vb) {
        const uint32_t *u = k_units + (((int64_t)(2 * (vb < last_vb ? vb : last_vb)) * 4 + g) * 64) * 3;
#pragma unroll
        for (int e = 0; e < 3; ++e) {
            dst[e] = __builtin_nontemporal_load(u + (e));
            dst[3 + e] = __builtin_nontemporal_load(u + (4 * 64 * 3 + e));  // the second 64-token block of the 128-token block
        }
    };
#pragma unroll
    for (int d = 0; d < PF2; ++d)
        load_units(un[d], vb0 + wave + NW12 * d);

    if (tid < PQ_HEAD_DIM)
        *(lds_f32 *)(lbase + Q2_OFF + tid * 4) = q_mine * a.scale_log2e;
    __syncthreads();
    build_rows(0);
    load_centroids(4);
    build_rows(4);
    __syncthreads();

    for (int vb = vb0 + wave; vb < vb1;) {
#pragma unroll
        for (int d = 0; d < PF2; ++d) {
            if (vb < vb1) {  // wave-uniform
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint32_t c[8];
                    unpack8(un[d][3 * h], un[d][3 * h + 1], un[d][3 * h + 2], c);
                    float t[8];
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8)
                        t[s8] = *(lds_f32 *)(lbase + TAB_OFF + (s8 * PQ12_CENTROIDS + c[s8]) * 4);
                    row[(int64_t)vb * 128 + 64 * h + lane] =
                        ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
                }
                load_units(un[d], vb + NW12 * PF2);
                vb += NW12;
            }
        }
    }
}

__global__ __launch_bounds__(NW12 * 64) void pq12_values_kernel(const pq_decode_args a, const float *scores, const int TS)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM2_BYTES];
    lds_u8 *lbase = (lds_u8 *)smem;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const uint32_t logical = undeal(blockIdx.x, gridDim.x);
    const int bh = (int)(logical / (uint32_t)(8 * TS));
    const int rem = (int)(logical - (uint32_t)bh * (uint32_t)(8 * TS));
    const int g = rem / TS;
    const int ts = rem - g * TS;
    const int b = (int)((uint32_t)bh / (uint32_t)a.Hq);
    const int hq = bh - b * a.Hq;
    const int hkv = (int)((uint32_t)hq / (uint32_t)a.G);

    // Order of the prologue: lengths (kept in flight, see pass 1), the table slice and the query are requested
    // first; then the range is cut, and this wavefront's first recent rows and code blocks are requested.
    const int zero = lane_zero();
    const bool has_recent = a.recent_k != nullptr && a.recent_len != nullptr;
    const int n_vec = a.ctx_len[b + zero];
    const int r_vec = (has_recent ? a.recent_len : a.ctx_len)[b + zero];
    const __half *vcb = (const __half *)a.vcb_packed + (int64_t)hkv * PQ12_M * PQ12_CENTROIDS * 4;
    u32x4 raw[8];
    {
        const u32x4 *src = (const u32x4 *)(vcb + (int64_t)(4 * g) * PQ12_CENTROIDS * 4);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            raw[k] = src[tid + k * (NW12 * 64)];
    }
    const float q_mine = tid < PQ_HEAD_DIM ? __half2float(((const __half *)a.q)[(int64_t)bh * PQ_HEAD_DIM + tid]) : 0.f;

    int N = __builtin_amdgcn_readfirstlane(n_vec);
    int R = has_recent ? __builtin_amdgcn_readfirstlane(r_vec) : 0;
    N = N < 0 ? 0 : (N > a.max_context ? a.max_context : N);
    R = R < 0 ? 0 : (R > a.max_recent ? a.max_recent : R);
    const uint32_t nvb = (uint32_t)(N + 127) >> 7;
    const int vb0 = (int)(nvb * (uint32_t)ts / (uint32_t)TS);
    const int vb1 = (int)(nvb * (uint32_t)(ts + 1) / (uint32_t)TS);
    const int r0 = (int)((uint32_t)R * (uint32_t)ts / (uint32_t)TS);
    const int r1 = (int)((uint32_t)R * (uint32_t)(ts + 1) / (uint32_t)TS);

    const uint8_t *v_head = a.v_codes + ((int64_t)b * a.Hkv + hkv) * a.head_stride;
    const uint32_t *v_units = (const uint32_t *)v_head + lane * 3;
    const int64_t cap = a.head_stride / PQ12_TOKEN_BYTES;
    const float *rows = scores + (int64_t)bh * 4 * cap;
    const int64_t rbase = ((int64_t)b * a.Hkv + hkv) * a.max_recent;

    // recent rows of this wavefront: RB12 per trip, their loads issued together; rows beyond the range re-read
    // the trip's first row and are skipped.  The first trip's rows are requested here, behind the table.
    __half2 kk[RB12];
    float vv[RB12];
    auto load_recent = [&](int r) {
#pragma unroll
        for (int u = 0; u < RB12; ++u) {
            const int rr = r + u * NW12 < r1 ? r + u * NW12 : r;
            kk[u] = *((const __half2 *)((const __half *)a.recent_k + (rbase + rr) * PQ_HEAD_DIM) + lane);
            vv[u] = lane < 16 ? __half2float(((const __half *)a.recent_v)[(rbase + rr) * PQ_HEAD_DIM + 16 * g + lane]) : 0.f;
        }
    };
    if (r0 + wave < r1)
        load_recent(r0 + wave);

    // the first blocks' partial scores and codes
    const int last_vb = vb1 > vb0 ? vb1 - 1 : 0;
    float sc[NB2][8];
    uint32_t un[NB2][3];
    auto load_block = [&](float (&scd)[8], uint32_t (&und)[3], int vb_want) {
        const int vb = vb_want < last_vb ? vb_want : last_vb;
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
            scd[2 * kg] = rows[kg * cap + (int64_t)vb * 128 + lane];
            scd[2 * kg + 1] = rows[kg * cap + (int64_t)vb * 128 + 64 + lane];
        }
        const uint32_t *u = v_units + (((int64_t)vb * 8 + g) * 64) * 3;
#pragma unroll
        for (int e = 0; e < 3; ++e)
            und[e] = __builtin_nontemporal_load(u + (e));
    };
    if (vb1 > vb0) {
#pragma unroll
        for (int e = 0; e < NB2; ++e)
            load_block(sc[e], un[e], vb0 + wave + NW12 * e);
    }

    if (tid < PQ_HEAD_DIM)
        *(lds_f32 *)(lbase + Q2_OFF + tid * 4) = q_mine * a.scale_log2e;
#pragma unroll
    for (int k = 0; k < 8; ++k)
        *(lds_u32x4 *)(lbase + TAB_OFF + (tid + k * (NW12 * 64)) * 16) = raw[k];
    __syncthreads();

    float m_run = NEG_BIG;  // this wavefront's reference maximum
    float l_lane = 0.f;
    // ---------------- recent full-precision rows of this token range first (their data arrived with the table):
    // every group scores them, each adds its own dims; lane l < 16 owns dim 16 g + l
    float o_rec = 0.f;
    {
        const float q0 = *(lds_f32 *)(lbase + Q2_OFF + lane * 8), q1 = *(lds_f32 *)(lbase + Q2_OFF + lane * 8 + 4);
        for (int r = r0 + wave; r < r1; r += NW12 * RB12) {
#pragma unroll
            for (int u = 0; u < RB12; ++u) {
                if (r + u * NW12 < r1) {  // wave-uniform
                    const float sr = wave_sum(fmaf(q0, __low2float(kk[u]), q1 * __high2float(kk[u])));
                    const float m_new = fmaxf(m_run, sr);
                    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                    const float pr = __builtin_amdgcn_exp2f(sr - m_new);
                    l_lane = fmaf(l_lane, alpha, lane == 0 ? pr : 0.f);
                    o_rec = fmaf(o_rec, alpha, pr * vv[u]);
                    m_run = m_new;
                }
            }
            if (r + NW12 * RB12 < r1)
                load_recent(r + NW12 * RB12);
        }
    }
    float acc[NB2][4];
#pragma unroll
    for (int e = 0; e < NB2; ++e)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[e][j] = 0.f;
    lds_f32 *pline = (lds_f32 *)(lbase + W2_OFF) + wave * (NB2 * 128);
    // A wavefront takes NB2 blocks per trip (vb, vb + 16, ...) and works on them together: their gathers and
    // multiply-adds are independent, which hides the LDS latency that one block at a time leaves exposed.  A
    // block beyond the range counts as empty (its loads re-read the last block).
    for (int vb = vb0 + wave; vb < vb1; vb += NW12 * NB2) {
        float s[NB2][2], p[NB2][2];
        float smax = NEG_BIG;
#pragma unroll
        for (int e = 0; e < NB2; ++e)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int vbe = vb + NW12 * e;
                const bool valid = vbe < vb1 && vbe * 128 + 64 * h + lane < N;
                s[e][h] = valid ? (sc[e][h] + sc[e][2 + h]) + (sc[e][4 + h] + sc[e][6 + h]) : NEG_BIG;
                smax = fmaxf(smax, s[e][h]);
            }
        // the registers of this trip's loads are free again: request the next trip's blocks now, a whole trip ahead
        uint32_t c[NB2][8];
#pragma unroll
        for (int e = 0; e < NB2; ++e) {
            unpack8(un[e][0], un[e][1], un[e][2], c[e]);
            load_block(sc[e], un[e], vb + NW12 * (NB2 + e));
        }
        // the reference maximum moves only when a score exceeds it by more than 8 (2^8 in weight)
        if (__builtin_amdgcn_ballot_w64(smax > m_run + 8.0f) != 0) {  // wave-uniform
            const float m_new = fmaxf(m_run, wave_max(smax));
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            l_lane *= alpha;
            o_rec *= alpha;
#pragma unroll
            for (int e = 0; e < NB2; ++e)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[e][j] *= alpha;
            m_run = m_new;
        }
#pragma unroll
        for (int e = 0; e < NB2; ++e)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                p[e][h] = s[e][h] > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(s[e][h] - m_run) : 0.f;
                l_lane += p[e][h];
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int e = 0; e < NB2; ++e) {
            pline[e * 128 + lane] = p[e][0];
            pline[e * 128 + 64 + lane] = p[e][1];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int e = 0; e < NB2; ++e) {
                const float pk = pline[e * 128 + (lane >> 2) + 16 * k];
                const u32x2 cv = *(lds_u32x2 *)(lbase + TAB_OFF + ((lane & 3) * PQ12_CENTROIDS + c[e][k]) * 8);
                const uint32_t lo = cv.x, hi = cv.y;
                const __half2 h0 = *(const __half2 *)&lo, h1 = *(const __half2 *)&hi;
                acc[e][0] = fmaf(pk, __low2float(h0), acc[e][0]);
                acc[e][1] = fmaf(pk, __high2float(h0), acc[e][1]);
                acc[e][2] = fmaf(pk, __low2float(h1), acc[e][2]);
                acc[e][3] = fmaf(pk, __high2float(h1), acc[e][3]);
            }
    }

    // ---------------- sum the 16 token streams (lanes with equal lane % 4); then lane l < 16 owns dim 16 g + l
    lds_f32 *part = (lds_f32 *)(lbase + PART2_OFF) + wave * PART2_STRIDE;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[0][j];
#pragma unroll
        for (int e = 1; e < NB2; ++e)
            v += acc[e][j];
        v += __shfl_xor(v, 4);
        v += __shfl_xor(v, 8);
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        if (lane < 4)
            part[4 + lane * 4 + j] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float o = (lane < 16 ? part[4 + lane] : 0.f) + o_rec;
    {
        const float l_w = wave_sum(l_lane);
        if (lane == 0) {
            part[0] = m_run;
            part[1] = l_w;
        }
        if (lane < 16)
            part[4 + lane] = o;
    }
    __syncthreads();
    if (wave != 0)
        return;

    // ---------------- wavefront 0 merges the workgroup: lane l < 8 takes dims 16 g + 2 l, + 1
    const lds_f32 *parts = (const lds_f32 *)(lbase + PART2_OFF);
    float mx = NEG_BIG;
#pragma unroll
    for (int w = 0; w < NW12; ++w)
        mx = fmaxf(mx, parts[w * PART2_STRIDE]);
    float l = 0.f, o0 = 0.f, o1 = 0.f;
    const int dl = lane < 8 ? lane : 0;
#pragma unroll
    for (int w = 0; w < NW12; ++w) {
        const float f = __builtin_amdgcn_exp2f(parts[w * PART2_STRIDE] - mx);
        o0 = fmaf(parts[w * PART2_STRIDE + 4 + 2 * dl], f, o0);
        o1 = fmaf(parts[w * PART2_STRIDE + 5 + 2 * dl], f, o1);
        l = fmaf(parts[w * PART2_STRIDE + 1], f, l);
    }
    float *orow = a.out + (int64_t)bh * PQ_HEAD_DIM;
    if (TS == 1) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
        if (lane < 8)
            *(float2 *)(orow + 16 * g + 2 * lane) = make_float2(o0 * inv, o1 * inv);
        return;
    }
    // Several token ranges: publish this range's 16 dims (and, from group 0, its maximum and weight sum, which
    // every group of the range computes alike), then one ticket per head counts the 8 TS workgroups; the last
    // one merges the ranges.  Device-scope stores complete before the ticket, device-scope loads follow it.
    float *gpart = a.partials + ((int64_t)bh * TS + ts) * PQ_PART_STRIDE;
    if (lane < 8)
        publish(gpart + 4 + 16 * g + 2 * lane, o0, o1);
    if (g == 0 && lane == 0)
        publish(gpart, mx, l);
    publish_wait();
    unsigned int ticket = 0;
    if (lane == 0)
        ticket = __hip_atomic_fetch_add(a.tickets + bh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != (unsigned int)(8 * TS - 1))
        return;
    asm volatile("" ::: "memory");  // the loads below stay behind the ticket in the instruction stream
    const float *ps = a.partials + (int64_t)bh * TS * PQ_PART_STRIDE;
    const float2 ml = lane < TS ? fetch(ps + lane * PQ_PART_STRIDE) : make_float2(NEG_BIG, 0.f);
    mx = wave_max(ml.x);
    const float f_lane = __builtin_amdgcn_exp2f(ml.x - mx);
    l = wave_sum(ml.y * f_lane);
    o0 = o1 = 0.f;
    for (int s = 0; s < TS; ++s) {
        const float2 os = fetch(ps + s * PQ_PART_STRIDE + 4 + 2 * lane);
        const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f_lane), s & 63));
        o0 = fmaf(os.x, f, o0);
        o1 = fmaf(os.y, f, o1);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    *(float2 *)(orow + 2 * lane) = make_float2(o0 * inv, o1 * inv);
    if (lane == 0)
        ticket_reset(a.tickets + bh);
}

}  // namespace

hipError_t pq12_launch_decode(const pq_attn_ctx *ctx, const pq_decode_args &a, hipStream_t s)
{
    if (ctx->scores12 != nullptr) {
        // two passes: a.S is the number of token ranges of pass 2; pass 1 has half as many workgroups per
        // range (4 groups against 8), so it takes twice the ranges where the context is long enough
        const int64_t nvb = ctx->cap_padded / 128;
        int ts1 = 2 * a.S;
        if ((int64_t)ts1 * 16 > nvb)
            ts1 = a.S;
        hipLaunchKernelGGL(pq12_scores_kernel, dim3(a.B * a.Hq * 4 * ts1), dim3(NW12 * 64), 0, s, a, ctx->scores12, ts1);
        hipLaunchKernelGGL(pq12_values_kernel, dim3(a.B * a.Hq * 8 * a.S), dim3(NW12 * 64), 0, s, a, ctx->scores12, a.S);
        return hipGetLastError();
    }
    const int grid = a.B * a.Hq * a.S;
    // blocks of 128 tokens per split at full capacity, per wavefront
    const int64_t per_wave = (ctx->cap_padded / 128 + (int64_t)a.S * NW12 - 1) / ((int64_t)a.S * NW12);
    if (per_wave <= 2)
        hipLaunchKernelGGL(pq12_decode_kernel<2>, dim3(grid), dim3(NW12 * 64), 0, s, a);
    else if (per_wave <= 6)
        hipLaunchKernelGGL(pq12_decode_kernel<6>, dim3(grid), dim3(NW12 * 64), 0, s, a);
    else
        hipLaunchKernelGGL(pq12_decode_kernel<16>, dim3(grid), dim3(NW12 * 64), 0, s, a);
    return hipGetLastError();
}
