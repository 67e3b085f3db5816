// Nearest centroid of fp16 sub-vectors among 256 fp16 centroids: matrix-core filter + fp64 decision.
// Shared by the encode kernel and the k-means assignment; the argument, the error bound and the fall-back are
// described in pq_encode.hip.  Everything here works on ONE wavefront (lane = token of a 64-token sub-chunk, NQ
// sub-chunks at a time) and on two LDS arrays the caller owns: the A rows of the 256 centroids (pq_filter_row_bytes
// each) and their fp64 copy.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pq_filter_constants.h"

namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4e __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2e __attribute__((ext_vector_type(2)));

template <int DS> constexpr int pq_filter_row_bytes() { return DS == 2 ? 8 : 16; }  // ds coordinates, h, l (, 0, 0)

// A row and fp64 copy of centroid c (src: its ds fp16 coordinates); updates the running maxima of |c|^2 / 2 and
// |c_j|, and `bad` when |c|^2 / 2 does not split into two fp16
template <int DS>
__device__ inline void pq_filter_build_row(const __half *src, unsigned char *arow_c, double *cb_c, float &n_max, float &c_max,
                                           bool &bad)
{
    constexpr int ROW = pq_filter_row_bytes<DS>();
    float n = 0.f;
    _Float16 row[ROW / 2];
#pragma unroll
    for (int j = 0; j < DS; ++j) {
        const _Float16 v = __builtin_bit_cast(_Float16, src[j]);
        const float f = (float)v;
        cb_c[j] = (double)f;
        row[j] = v;
        n += f * f;  // exact squares; the sum is rounded (covered by the bound)
        c_max = fmaxf(c_max, fabsf(f));
    }
    const float h = 0.5f * n;
    const _Float16 hh = (_Float16)h;
    const _Float16 hl = (_Float16)(h - (float)hh);
    row[DS] = hh;
    row[DS + 1] = hl;
    if (DS == 4)
        row[6] = row[7] = (_Float16)0.f;
    bad |= !(h < 60000.f);
    n_max = fmaxf(n_max, h);
    __builtin_memcpy(arow_c, row, ROW);
}

// codes of this lane's NQ tokens (xv: their fp16 sub-vectors; dead lanes pass any finite values and live = false)
template <int DS, int NQ>
__device__ inline void pq_filter_codes(const unsigned char *arow, const double *cb, const float n_max, const float c_max,
                                       const bool cb_bad, const _Float16 (&xin)[NQ][DS], const bool (&live)[NQ], int (&codes)[NQ])
{
#pragma clang fp contract(off)
    constexpr int ROW = pq_filter_row_bytes<DS>();
    const int lane = threadIdx.x & 63;
    bool bad[NQ];
    double xd[NQ][DS];
    f16x4 bop[NQ];
    f32x4e off4[NQ];
    float tau[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        float x1 = 0.f, x2 = 0.f;
        bad[q] = cb_bad;
        _Float16 xv[4] = {(_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f};
#pragma unroll
        for (int j = 0; j < DS; ++j) {
            const _Float16 v = xin[q][j];
            const float f = (float)v;
            xd[q][j] = (double)f;
            xv[j] = -v;
            x1 += fabsf(f);
            x2 += f * f;
        }
        bop[q] = f16x4{xv[0], xv[1], xv[2], xv[3]};
        {
            // keep the negated operand in its registers (the compiler otherwise redoes the negation per use)
            u32x2e w = __builtin_bit_cast(u32x2e, bop[q]);
            asm volatile("" : "+v"(w));
            bop[q] = __builtin_bit_cast(f16x4, w);
        }
        // off: |x|^2/2 with half a per cent on top, plus the same again as tau and a floor, so that every
        // computed value stays above zero; T = N + X C + off; tau = 2^-18.3 T + 2^-22
        const float t0 = n_max + x1 * c_max + PQ_FILTER_X2_FACTOR * x2;
        float off = PQ_FILTER_X2_FACTOR * x2 + 2.0f * (PQ_FILTER_TAU_REL * (2.0f * t0) + PQ_FILTER_TAU_ABS);
        tau[q] = PQ_FILTER_TAU_REL * (t0 + off) + PQ_FILTER_TAU_ABS;
        off += tau[q];
        off4[q] = f32x4e{off, off, off, off};
        bad[q] |= !(off < 1.0e30f);
    }
    const f16x4 ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)0.f, (_Float16)0.f};
    const unsigned char *my_row = arow + (lane & 3) * ROW;
    auto values = [&](int m, int q) -> f32x4e {
        if (DS == 2) {
            const f16x4 A = *(const f16x4 *)(my_row + m * (4 * ROW));
            return __builtin_amdgcn_mfma_f32_4x4x4f16(A, bop[q], off4[q], 0, 0, 0);
        }
        const f16x4 A1 = *(const f16x4 *)(my_row + m * (4 * ROW));
        const f16x4 A2 = *(const f16x4 *)(my_row + m * (4 * ROW) + 8);
        return __builtin_amdgcn_mfma_f32_4x4x4f16(A2, ones, __builtin_amdgcn_mfma_f32_4x4x4f16(A1, bop[q], off4[q], 0, 0, 0), 0, 0, 0);
    };

    // ---- pass 1: smallest computed value per token (positive floats order like their bit patterns)
    int best[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
        best[q] = 0x7f800000;
    for (int m = 0; m < 64; ++m) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const f32x4e d = values(m, q);
            best[q] = min(min(best[q], __float_as_int(d[0])), __float_as_int(d[1]));
            best[q] = min(min(best[q], __float_as_int(d[2])), __float_as_int(d[3]));
        }
    }
    // ---- pass 2: candidate groups, one bit per group.  The C operand becomes off - (best + tau): a computed value
    // is then negative exactly where it lies within tau of the best one, so the sign bit IS the candidate flag —
    // OR over the group's 4 values, shifted into the mask by one v_alignbit (group g lands in bit 63 - g).
    // The rounding differs from pass 1's (another C), within the same bound e; the minimiser's value comes out
    // <= 2 e - tau + (the two roundings of best + tau - off, <= 2^-23 T) < 0, so it is marked.
    uint32_t cand_lo[NQ], cand_hi[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const float b = __int_as_float(best[q]);
        bad[q] |= !(b > 0.f && b < 1.0e30f);                   // the offset did not keep the values positive and finite
        const float d = off4[q][0] - (b + tau[q]);
        off4[q] = f32x4e{d, d, d, d};
        cand_lo[q] = 0u;
        cand_hi[q] = 0u;
    }
#pragma unroll 4
    for (int m = 0; m < 32; ++m) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const f32x4e d = values(m, q);
            const uint32_t any = (__float_as_uint(d[0]) | __float_as_uint(d[1])) | (__float_as_uint(d[2]) | __float_as_uint(d[3]));
            cand_lo[q] = __builtin_amdgcn_alignbit(cand_lo[q], any, 31);
        }
    }
#pragma unroll 4
    for (int m = 0; m < 32; ++m) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const f32x4e d = values(m + 32, q);
            const uint32_t any = (__float_as_uint(d[0]) | __float_as_uint(d[1])) | (__float_as_uint(d[2]) | __float_as_uint(d[3]));
            cand_hi[q] = __builtin_amdgcn_alignbit(cand_hi[q], any, 31);
        }
    }
    int cnt[NQ], first[NQ], last[NQ];
    bool two = false;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const uint64_t cand = ((uint64_t)cand_lo[q] << 32) | cand_hi[q];
        cnt[q] = __builtin_popcountll(cand);
        first[q] = cand ? __builtin_clzll(cand) : 0;
        last[q] = cand ? 63 - __builtin_ctzll(cand) : 0;
        two |= live[q] && cnt[q] == 2;
    }
    two = __builtin_amdgcn_ballot_w64(two) != 0;  // wave-uniform: some token has a second candidate group

    // ---- refine / full scan
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        int code = 0;
        double bd = __builtin_huge_val();
        auto take = [&](int c) {
            double dist = 0.0;
#pragma unroll
            for (int j = 0; j < DS; ++j) {
                const double diff = xd[q][j] - cb[c * DS + j];
                dist = __builtin_fma(diff, diff, dist);
            }
            code = dist < bd ? c : code;  // strict: the lowest index among equal distances stays
            bd = __builtin_fmin(bd, dist);
        };
#pragma unroll
        for (int k = 0; k < 4; ++k)  // ascending centroid index: the first group ...
            take(4 * first[q] + k);
        if (two) {
#pragma unroll
            for (int k = 0; k < 4; ++k)  // ... then the last one (the same group again where there is only one)
                take(4 * last[q] + k);
        }
        // more than two candidate groups (a cluster of near-ties, a token far outside the codebook's range): the
        // lane walks all of its marked groups, ascending — the nearest centroid and every tie lie in them
        const bool many = live[q] && !bad[q] && cnt[q] > 2;
        if (__builtin_amdgcn_ballot_w64(many) != 0) {  // wave-uniform
            const int code_12 = code;
            const double bd_12 = bd;
            code = 0;
            bd = __builtin_huge_val();
            uint64_t left = many ? ((uint64_t)cand_lo[q] << 32) | cand_hi[q] : 0;  // group g sits in bit 63 - g
            while (__builtin_amdgcn_ballot_w64(left != 0) != 0) {
                const int g = left ? __builtin_clzll(left) : 0;
                const int code_before = code;
                const double bd_before = bd;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    take(4 * g + k);
                if (left == 0) {  // this lane had nothing left: keep what it had
                    code = code_before;
                    bd = bd_before;
                }
                left &= ~(0x8000000000000000ull >> g);
            }
            if (!many) {
                code = code_12;
                bd = bd_12;
            }
        }
        const bool unsure = live[q] && (bad[q] || cnt[q] < 1);
        if (__builtin_amdgcn_ballot_w64(unsure) != 0) {  // wave-uniform: the defining scan for this sub-chunk
            code = 0;
            bd = __builtin_huge_val();
            for (int c = 0; c < 256; ++c) {
                double dist = 0.0;
#pragma unroll
                for (int j = 0; j < DS; ++j) {
                    const double diff = xd[q][j] - cb[c * DS + j];
                    dist = __builtin_fma(diff, diff, dist);
                }
                code = dist < bd ? c : code;
                bd = __builtin_fmin(bd, dist);
            }
        }
        codes[q] = code;
    }
}

}  // namespace
