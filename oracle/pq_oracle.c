/*
 * CPU oracle for decode attention over a product-quantized KV cache and for the
 * nearest-centroid encode that fills it.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is plain, slow, double
 * precision, and shares no code, header, table or helper with the GPU library.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it computes is the plain definition, not the fast evaluation:
 *
 *   decode  (Eq. 5, then Eq. 6 evaluated as Eq. 1 for a single query):
 *           every cached token is de-quantized by gathering one centroid per
 *           subspace and concatenating them; the recent full-precision rows are
 *           appended; the output is ordinary softmax attention of the query over
 *           those rows (two passes: maximum, then exp / sum).  No look-up table,
 *           no splitting, no online softmax: Eq. 7 is an algebraic identity with
 *           Eq. 6, so the plain form is the reference for it.
 *
 *   encode  (Eq. 4 read with Section II-C's "assigned to the nearest centroid"):
 *           for each sub-vector the index of the centroid at the smallest squared
 *           Euclidean distance, equal distances going to the lowest index.  The paper
 *           fixes no rounding; the distance is evaluated in IEEE double, left to right:
 *           dist = 0, then for j = 0 .. ds-1  dist = fma(x_j - c_j, x_j - c_j, dist)
 *           (each difference rounded once, each fused multiply-add rounded once;
 *           nothing else may be contracted: build with -ffp-contract=off).  For fp16
 *           inputs every difference is exact, and while distances stay below 32 so is
 *           every sum: the code is then the exact-arithmetic nearest centroid.  Beyond
 *           that it is the nearest centroid up to two roundings of 2^-53 relative.
 *
 * Pins (tests that hold it to something other than itself): brute-force
 * attention with library softmax on tiny inputs, codebooks that contain the
 * source vectors (exact dense attention), softmax weights summing to one, q = 0
 * giving the mean of the value rows, single-token and all-equal-code closed
 * forms, permutation and code/recent exchange invariance, GQA as replicated MHA,
 * the table-sum form of Eq. 7 in double; for encode a library vector quantizer,
 * duplicated centroids, exact hits, and exact integer arithmetic (fp16 values as
 * integers x 2^-24) on large magnitudes, near-midpoint tokens, subnormals and ties.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Width of a centroid index.  The 8-bit settings (256 centroids) store one byte per code; the
 * paper's 12-bit setting (M = 32, 4096 centroids per subspace; Section IV-A, footnote on the
 * (M, nbits) pairs) needs 16.  pq_oracle16.c compiles this file a second time with 16-bit codes
 * and the function names suffixed _u16; nothing else differs. */
#ifndef PQ_CODE_T
#define PQ_CODE_T uint8_t
#define PQ_NAME(n) n
#endif
#define PQ_MAX_CENTROIDS (1 << (8 * (int)sizeof(PQ_CODE_T)))

/* Eq. 5: de-quantize n tokens of one KV head.
 *   codes    [n][M]            one centroid index per subspace
 *   codebook [M][C][ds]        centroids of this head
 *   out      [n][M*ds]         concatenation over subspaces of the gathered centroids */
void PQ_NAME(oracle_pq_dequantize)(const PQ_CODE_T *codes, const double *codebook, int64_t n, int M, int C, int ds,
                          double *out)
{
    const int d = M * ds;
    for (int64_t t = 0; t < n; ++t)
        for (int i = 0; i < M; ++i) {
            const int c = codes[t * M + i];
            for (int j = 0; j < ds; ++j)
                out[t * d + i * ds + j] = codebook[((int64_t)i * C + c) * ds + j];
        }
}

/* Eq. 1 for one query row: out = softmax(scale * q K^T) V over n rows of width d.
 * weights (optional, length n) receives the softmax weights.  n == 0 gives zeros. */
void PQ_NAME(oracle_dense_attention)(const double *q, const double *keys, const double *values, int64_t n, int d,
                            double scale, double *out, double *weights)
{
    for (int k = 0; k < d; ++k)
        out[k] = 0.0;
    if (n <= 0)
        return;
    double *s = (double *)malloc((size_t)n * sizeof(double));
    double smax = -INFINITY;
    for (int64_t t = 0; t < n; ++t) {
        double dot = 0.0;
        for (int k = 0; k < d; ++k)
            dot += q[k] * keys[t * d + k];
        s[t] = scale * dot;
        if (s[t] > smax)
            smax = s[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        s[t] = exp(s[t] - smax);
        denom += s[t];
    }
    for (int64_t t = 0; t < n; ++t) {
        const double p = s[t] / denom;
        if (weights)
            weights[t] = p;
        for (int k = 0; k < d; ++k)
            out[k] += p * values[t * d + k];
    }
    free(s);
}

/* Eq. 6 for every (sequence, query head) — or only for the listed pairs.
 *
 *   q           [B][Hq][d]
 *   k_codes     [B][Hkv][ctx_cap][M]   v_codes likewise
 *   ctx_len     [B]                    quantized tokens of each sequence
 *   k_codebook  [Hkv][M][C][ds]        v_codebook likewise (shared by the batch)
 *   recent_k    [B][Hkv][rec_cap][d]   recent_v likewise; may be NULL (no window)
 *   recent_len  [B]                    may be NULL (all zero)
 *   pairs       [n_pairs][2] (b, hq)   NULL: all B*Hq pairs; the listed pairs must be distinct
 *                                      (each output row is accumulated by one thread)
 *   out         [B][Hq][d]             rows not listed in `pairs` are left alone
 *   weight_sum  optional [B][Hq]       sum of the softmax weights (an invariant: 1)
 *
 * Query head hq reads KV head hq / (Hq / Hkv).  A sequence with no token at all
 * gives a row of zeros.  Returns 0, or -1 on a shape error / failed allocation. */
int PQ_NAME(oracle_pq_decode)(int B, int Hq, int Hkv, int d, int M, int C, const double *q, const PQ_CODE_T *k_codes,
                     const PQ_CODE_T *v_codes, int64_t ctx_cap, const int32_t *ctx_len, const double *k_codebook,
                     const double *v_codebook, const double *recent_k, const double *recent_v, int64_t rec_cap,
                     const int32_t *recent_len, double scale, const int32_t *pairs, int64_t n_pairs, double *out,
                     double *weight_sum)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || M <= 0 || d % M || Hq % Hkv || C <= 0 || C > PQ_MAX_CENTROIDS)
        return -1;
    const int ds = d / M;
    const int G = Hq / Hkv;
    const int64_t total = pairs ? n_pairs : (int64_t)B * Hq;
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < total; ++w) {
        const int b = pairs ? pairs[2 * w] : (int)(w / Hq);
        const int hq = pairs ? pairs[2 * w + 1] : (int)(w % Hq);
        const int hkv = hq / G;
        const int64_t N = ctx_len[b];
        const int64_t R = (recent_k && recent_len) ? recent_len[b] : 0;
        const int64_t n = N + R;
        double *o = out + ((int64_t)b * Hq + hq) * d;
        if (n == 0) {
            memset(o, 0, (size_t)d * sizeof(double));
            if (weight_sum)
                weight_sum[(int64_t)b * Hq + hq] = 0.0;
            continue;
        }
        double *keys = (double *)malloc((size_t)n * d * sizeof(double));
        double *vals = (double *)malloc((size_t)n * d * sizeof(double));
        double *wts = (double *)malloc((size_t)n * sizeof(double));
        if (!keys || !vals || !wts) {
#pragma omp atomic write
            failed = 1;
            free(keys);
            free(vals);
            free(wts);
            continue;
        }
        const int64_t head = (int64_t)b * Hkv + hkv;
        PQ_NAME(oracle_pq_dequantize)(k_codes + head * ctx_cap * M, k_codebook + (int64_t)hkv * M * C * ds, N, M, C, ds,
                             keys);
        PQ_NAME(oracle_pq_dequantize)(v_codes + head * ctx_cap * M, v_codebook + (int64_t)hkv * M * C * ds, N, M, C, ds,
                             vals);
        if (R > 0) {
            memcpy(keys + N * d, recent_k + head * rec_cap * d, (size_t)R * d * sizeof(double));
            memcpy(vals + N * d, recent_v + head * rec_cap * d, (size_t)R * d * sizeof(double));
        }
        PQ_NAME(oracle_dense_attention)(q + ((int64_t)b * Hq + hq) * d, keys, vals, n, d, scale, o, wts);
        if (weight_sum) {
            double sum = 0.0;
            for (int64_t t = 0; t < n; ++t)
                sum += wts[t];
            weight_sum[(int64_t)b * Hq + hq] = sum;
        }
        free(keys);
        free(vals);
        free(wts);
    }
    return failed ? -1 : 0;
}

/* Eq. 4: nearest-centroid codes of n vectors of one head.
 *   x        [n][M*ds]
 *   codebook [M][C][ds]
 *   codes    [n][M]
 * The scan starts at centroid 0 and replaces the best only on a strictly smaller
 * distance, so equal distances keep the lowest index. */
void PQ_NAME(oracle_pq_encode_head)(const double *x, const double *codebook, int64_t n, int M, int C, int ds,
                           PQ_CODE_T *codes)
{
    const int d = M * ds;
    for (int64_t t = 0; t < n; ++t)
        for (int i = 0; i < M; ++i) {
            int best = 0;
            double best_dist = 0.0;
            for (int c = 0; c < C; ++c) {
                double dist = 0.0;
                for (int j = 0; j < ds; ++j) {
                    const double diff = x[t * d + i * ds + j] - codebook[((int64_t)i * C + c) * ds + j];
                    dist = fma(diff, diff, dist);
                }
                if (c == 0 || dist < best_dist) {
                    best = c;
                    best_dist = dist;
                }
            }
            codes[t * M + i] = (PQ_CODE_T)best;
        }
}

/* Encode n_new vectors per (sequence, KV head).
 *   x        [B][Hkv][n_new][d]
 *   codebook [Hkv][M][C][ds]
 *   codes    [B][Hkv][n_new][M] */
int PQ_NAME(oracle_pq_encode)(int B, int Hkv, int d, int M, int C, int64_t n_new, const double *x, const double *codebook,
                     PQ_CODE_T *codes)
{
    if (B <= 0 || Hkv <= 0 || M <= 0 || d % M || C <= 0 || C > PQ_MAX_CENTROIDS || n_new < 0)
        return -1;
    const int ds = d / M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < (int64_t)B * Hkv; ++w) {
        const int hkv = (int)(w % Hkv);
        PQ_NAME(oracle_pq_encode_head)(x + w * n_new * d, codebook + (int64_t)hkv * M * C * ds, n_new, M, C, ds,
                              codes + w * n_new * M);
    }
    return 0;
}

int PQ_NAME(oracle_num_threads)(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* Limits the threads later calls use (n <= 0: back to the default of the OpenMP runtime's environment). */
void PQ_NAME(oracle_set_num_threads)(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n > 0 ? n : omp_get_num_procs());
#else
    (void)n;
#endif
}
