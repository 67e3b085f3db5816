// Constants of the matrix-core nearest-centroid filter, in one place: the 8-bit and the 12-bit encode kernels
// include this file and the host-side bound test parses it, so the three cannot drift apart.
//
// Per token, with X1 = sum |x_j|, X2 = sum x_j^2, N = max |c|^2 / 2 and C = max |c_j| over the codebook:
//   T0  = N + X1 C + PQ_FILTER_X2_FACTOR X2
//   off = PQ_FILTER_X2_FACTOR X2 + 2 (PQ_FILTER_TAU_REL (2 T0) + PQ_FILTER_TAU_ABS)   (keeps every value positive)
//   tau = PQ_FILTER_TAU_REL (T0 + off) + PQ_FILTER_TAU_ABS                              (candidate threshold)
// PQ_FILTER_TAU_REL = 2^-18.3 is 1.3 x twice the worst-case relative error of the fp32 sums (2^-19.7 of the summed
// magnitudes even if every addition truncated); PQ_FILTER_TAU_ABS = 2^-22 is a floor for tiny magnitudes.
#pragma once

#define PQ_FILTER_X2_FACTOR 0.5025f
#define PQ_FILTER_TAU_REL 3.1e-06f
#define PQ_FILTER_TAU_ABS 2.4e-07f
