/* The CPU oracle of pq_oracle.c once more, for 16-bit centroid indices (the 12-bit setting with 4096
 * centroids per subspace): same source, same arithmetic, function names suffixed _u16.
 * TEST INFRASTRUCTURE, NOT A PRODUCT PATH. */
#define PQ_CODE_T uint16_t
#define PQ_NAME(n) n##_u16
#include "pq_oracle.c"
