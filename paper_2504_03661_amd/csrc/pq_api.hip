// C ABI of libpq_attn: argument checks, context life cycle, launch plumbing.
// Every step of the path runs in the kernels; this file only validates and launches.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "pq_internal.h"

// Scratch of pq_attn_decode_noalloc: one array per GPU the library runs on, held until the process ends.
//   [0, 2 MiB)           centroid-major image of the K codebooks      (PQ_NOALLOC_CODEBOOK_BYTES)
//   [2 MiB, 4 MiB)       the same for V
//   then                 split partials [PQ_NOALLOC_MAX_ROWS][PQ_PART_STRIDE] fp32
//   then                 tickets [PQ_NOALLOC_MAX_ROWS] uint32
// In host code the array's name is a stand-in, not a device address: host code uses the pointer that
// hipGetSymbolAddress returns for the current device.
#define PQ_NOALLOC_PARTIALS_OFF (2 * (size_t)PQ_NOALLOC_CODEBOOK_BYTES)
#define PQ_NOALLOC_TICKETS_OFF (PQ_NOALLOC_PARTIALS_OFF + (size_t)PQ_NOALLOC_MAX_ROWS * PQ_PART_STRIDE * sizeof(float))
#define PQ_NOALLOC_SCRATCH_BYTES (PQ_NOALLOC_TICKETS_OFF + (size_t)PQ_NOALLOC_MAX_ROWS * sizeof(unsigned int))
static __device__ __align__(256) unsigned char scratch[PQ_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr float LOG2E = 1.44269504088896340736f;

// per device: the address of that GPU's copy of `scratch` and its compute-unit count, looked up once
constexpr int MAX_DEVICES = 64;
struct noalloc_device {
    unsigned char *ptr = nullptr;
    int n_cu = 0;
};
noalloc_device g_noalloc[MAX_DEVICES];
std::mutex g_noalloc_mutex;

// the caller has made `dev` current
int noalloc_lookup(int dev, noalloc_device *out)
{
    if (dev < 0 || dev >= MAX_DEVICES)
        return PQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (g_noalloc[dev].ptr == nullptr) {
        void *p = nullptr;
        int n_cu = 0;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) {
            (void)hipGetLastError();
            return PQ_ERR_HIP;
        }
        g_noalloc[dev].n_cu = n_cu;
        g_noalloc[dev].ptr = (unsigned char *)p;
    }
    *out = g_noalloc[dev];
    return PQ_OK;
}

struct device_guard {
    int prev = -1;
    bool ok = false;
    explicit device_guard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess)
            return;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
    }
    ~device_guard()
    {
        if (ok && prev >= 0)
            (void)hipSetDevice(prev);
    }
};

int validate(const pq_attn_config *c)
{
    if (c == nullptr)
        return PQ_ERR_NULL;
    if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->n_subspaces <= 0 ||
        c->n_centroids <= 0 || c->max_context <= 0 || c->max_recent < 0 || c->device < 0 || c->reserved != 0)
        return PQ_ERR_SHAPE;
    // a negative split count is the 12-bit contexts' request for the two-pass decode with that many token ranges
    if (c->n_splits < 0 && c->n_centroids != PQ12_CENTROIDS)
        return PQ_ERR_SHAPE;
    if (c->n_q_heads % c->n_kv_heads != 0 || c->head_dim % c->n_subspaces != 0)
        return PQ_ERR_SHAPE;
    if (c->dtype != PQ_F16 && c->dtype != PQ_F32)
        return PQ_ERR_SHAPE;
    if (c->head_dim != PQ_HEAD_DIM || (c->n_subspaces != 64 && c->n_subspaces != 32))
        return PQ_ERR_UNSUPPORTED;
    // 8-bit codes, or the 12-bit setting: 32 subspaces x 4096 centroids, fp16
    if (c->n_centroids != 256 && !(c->n_centroids == PQ12_CENTROIDS && c->n_subspaces == PQ12_M && c->dtype == PQ_F16))
        return PQ_ERR_UNSUPPORTED;
    if (c->n_splits > PQ_MAX_SPLITS || c->n_splits < -PQ_MAX_SPLITS || c->max_context > PQ_MAX_TOKENS || c->max_recent > PQ_MAX_TOKENS)
        return PQ_ERR_UNSUPPORTED;
    if ((int64_t)c->batch * c->n_q_heads * PQ_MAX_SPLITS > (int64_t)1 << 30)
        return PQ_ERR_UNSUPPORTED;
    return PQ_OK;
}

int64_t padded_capacity(const pq_attn_config *c)
{
    const int64_t block = pq_config_is_12bit(c) ? 128 : 64;
    return ((int64_t)c->max_context + block - 1) / block * block;
}

// bytes of one token in one code tensor
int64_t token_bytes(const pq_attn_config *c) { return pq_config_is_12bit(c) ? PQ12_TOKEN_BYTES : c->n_subspaces; }

// Splits per (sequence, head): a workgroup's tables take most of a compute unit's LDS, so one
// workgroup is resident per CU at a time and the grid should fill the chip exactly once —
// measured: 32 heads x 8 splits 34 us, x 6 splits 35 us, x 12 splits 44 us; 96 heads x 2 splits
// (192 workgroups) 98 us against 126 us for 3 splits (288 workgroups, a second partial round).
// Hence the largest split count whose grid still fits the chip, but never so many that a
// split has less than a block per wavefront.
int choose_splits(const pq_attn_config *c, int n_cu)
{
    // the grouped-query kernel runs one workgroup per (sequence, KV head, split)
    const int g = c->n_q_heads / c->n_kv_heads;
    const bool grouped12 = pq12_config_uses_grouped_kernel(c, n_cu);
    const int64_t heads = (int64_t)c->batch * (pq_config_uses_grouped_kernel(c) || grouped12
                                                   ? c->n_kv_heads * pq_grouped_sub_groups(g)
                                                   : c->n_q_heads);
    int64_t s = n_cu / heads;
    const int64_t blocks = padded_capacity(c) / 64;
    // 8-bit kernels: at least 4 blocks of 64 tokens per split — short contexts gain more from the parallelism
    // than they lose to idle wavefronts (32 heads x 1K tokens: 11.1 us with one split, 8.2 us with four; 2K: 11.3
    // -> 8.8; 4K: 10.9 -> 9.6); 12-bit kernel: at least one 4096-token chunk (grouped queries: 2048 tokens, one
    // 128-token block per wavefront)
    const int64_t per_split = grouped12 ? 32 : pq_config_is_12bit(c) ? 64 : 4;
    const int64_t max_by_work = blocks / per_split > 0 ? blocks / per_split : 1;
    if (s > max_by_work)
        s = max_by_work;
    if (s > PQ_MAX_SPLITS)
        s = PQ_MAX_SPLITS;
    if (s < 1)
        s = 1;
    return (int)s;
}

// Codebook pointers passed to an entry point are registered there and then: the context copies them on the
// stream (its own natural-layout copy for the encode kernels, the centroid-major image for the decode
// kernels) and never looks at the caller's tensors again.  NULL, NULL means "the registered ones".
int ensure_codebooks(pq_attn_ctx *ctx, const void *k, const void *v, hipStream_t s)
{
    if (k == nullptr && v == nullptr)
        return ctx->registered ? PQ_OK : PQ_ERR_NULL;
    if (k == nullptr || v == nullptr)
        return PQ_ERR_NULL;
    if (pq_config_is_12bit(&ctx->cfg)) {
        // the 12-bit kernels read the natural layout [Hkv][M][4096][ds]: one plain copy serves both paths
        const int64_t bytes = (int64_t)ctx->cfg.n_kv_heads * PQ12_M * PQ12_CENTROIDS * 4 * sizeof(uint16_t);
        if (pq_launch_copy16(k, ctx->kcb_packed, bytes, s) != hipSuccess ||
            pq_launch_copy16(v, ctx->vcb_packed, bytes, s) != hipSuccess)
            return PQ_ERR_HIP;
    } else {
        if (pq_launch_pack_codebook(ctx, k, ctx->kcb_packed, ctx->kcb_natural, s) != hipSuccess)
            return PQ_ERR_HIP;
        if (pq_launch_pack_codebook(ctx, v, ctx->vcb_packed, ctx->vcb_natural, s) != hipSuccess)
            return PQ_ERR_HIP;
    }
    ctx->registered = true;
    return PQ_OK;
}

// Tokens per (sequence, KV head) the staging buffers of a 12-bit context hold: the whole capacity when that is
// small, otherwise what 8 MiB per tensor give (an append of more tokens runs as several chunks), at least 64.
int32_t stage_tokens_for(const pq_attn_config *c)
{
    const int64_t heads = (int64_t)c->batch * c->n_kv_heads;
    int64_t t = ((int64_t)8 << 20) / (heads * PQ12_M * (int64_t)sizeof(uint16_t));
    if (t < 64)
        t = 64;
    if (t > c->max_context)
        t = c->max_context;
    return (int32_t)t;
}

int launch_decode(const pq_attn_ctx *ctx, const void *q, const uint8_t *k_codes, const uint8_t *v_codes,
                  const int32_t *ctx_len, const void *recent_k, const void *recent_v, const int32_t *recent_len, float scale,
                  float *out, hipStream_t s)
{
    pq_decode_args a;
    a.q = q;
    a.k_codes = k_codes;
    a.v_codes = v_codes;
    a.ctx_len = ctx_len;
    a.kcb_packed = ctx->kcb_packed;
    a.vcb_packed = ctx->vcb_packed;
    a.recent_k = recent_k;
    a.recent_v = recent_v;
    a.recent_len = recent_k ? recent_len : nullptr;
    a.out = out;
    a.partials = ctx->partials;
    a.tickets = ctx->tickets;
    a.scale_log2e = scale * LOG2E;
    a.B = ctx->cfg.batch;
    a.Hq = ctx->cfg.n_q_heads;
    a.Hkv = ctx->cfg.n_kv_heads;
    a.G = ctx->group;
    a.Gs = ctx->k_skew == PQ_K_SKEW_QUAD || ctx->grouped12 ? pq_grouped_heads_per_workgroup(ctx->group) : 0;
    a.n_sub = ctx->k_skew == PQ_K_SKEW_QUAD || ctx->grouped12 ? pq_grouped_sub_groups(ctx->group) : 0;
    a.S = ctx->n_splits;
    a.max_context = ctx->cfg.max_context;
    a.max_recent = ctx->cfg.max_recent;
    a.n_cu = ctx->n_cu;
    a.head_stride = ctx->cap_padded * token_bytes(&ctx->cfg);
    const hipError_t e = ctx->grouped12                  ? pq12_launch_decode_grouped(ctx, a, s)
                         : pq_config_is_12bit(&ctx->cfg) ? pq12_launch_decode(ctx, a, s)
                         : ctx->k_skew == PQ_K_SKEW_QUAD ? pq_launch_decode_grouped(ctx, a, s)
                                                         : pq_launch_decode(ctx, a, s);
    return e == hipSuccess ? PQ_OK : PQ_ERR_HIP;
}

void free_ctx(pq_attn_ctx *ctx)
{
    if (ctx->kcb_packed) (void)hipFree(ctx->kcb_packed);
    if (ctx->vcb_packed) (void)hipFree(ctx->vcb_packed);
    if (ctx->kcb_natural && ctx->kcb_natural != ctx->kcb_packed) (void)hipFree(ctx->kcb_natural);
    if (ctx->vcb_natural && ctx->vcb_natural != ctx->vcb_packed) (void)hipFree(ctx->vcb_natural);
    if (ctx->partials) (void)hipFree(ctx->partials);
    if (ctx->tickets) (void)hipFree(ctx->tickets);
    if (ctx->dev_err) (void)hipFree(ctx->dev_err);
    if (ctx->scores12) (void)hipFree(ctx->scores12);
    if (ctx->stage[0]) (void)hipFree(ctx->stage[0]);
    if (ctx->stage[1]) (void)hipFree(ctx->stage[1]);
    delete ctx;
}

}  // namespace

extern "C" {

int pq_attn_validate_config(const pq_attn_config *cfg) { return validate(cfg); }

int64_t pq_attn_codes_bytes(const pq_attn_config *cfg)
{
    const int rc = validate(cfg);
    if (rc != PQ_OK)
        return rc;
    return (int64_t)cfg->batch * cfg->n_kv_heads * padded_capacity(cfg) * token_bytes(cfg);
}

int pq_attn_create(const pq_attn_config *cfg, pq_attn_ctx **out)
{
    if (out == nullptr)
        return PQ_ERR_NULL;
    const int rc = validate(cfg);
    if (rc != PQ_OK)
        return rc;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || cfg->device >= n_dev) {
        (void)hipGetLastError();
        return PQ_ERR_HIP;
    }
    device_guard guard(cfg->device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg->device) != hipSuccess)
        return PQ_ERR_HIP;

    pq_attn_ctx *ctx = new (std::nothrow) pq_attn_ctx();
    if (ctx == nullptr)
        return PQ_ERR_ALLOC;
    ctx->cfg = *cfg;
    ctx->ds = cfg->head_dim / cfg->n_subspaces;
    ctx->group = cfg->n_q_heads / cfg->n_kv_heads;
    ctx->cap_padded = padded_capacity(cfg);
    ctx->elem_bytes = cfg->dtype == PQ_F16 ? 2 : 4;
    ctx->k_skew = pq_config_uses_grouped_kernel(cfg) ? PQ_K_SKEW_QUAD : PQ_K_SKEW_LANE;
    ctx->n_cu = prop.multiProcessorCount;
    ctx->grouped12 = pq12_config_uses_grouped_kernel(cfg, prop.multiProcessorCount);
    ctx->n_splits = cfg->n_splits > 0 ? cfg->n_splits : choose_splits(cfg, prop.multiProcessorCount);
    // 12-bit contexts with few (sequence, query head) pairs decode in two passes (split by subspace group, see
    // pq12_decode.hip): chosen when there are 5 or more compute units per (sequence, head) pair, whatever the context
    // length (measured with 32 heads: one sequence 21 against 47 us at 1K tokens, 32 against 56 us at 16K, 45 against
    // 64 us at 32K; two sequences at 32K 87 against 84 us, four 182 against 164 us), or on request
    bool two_pass = false;
    const int64_t cus_per_head = prop.multiProcessorCount / ((int64_t)cfg->batch * cfg->n_q_heads);
    if (pq_config_is_12bit(cfg) && !ctx->grouped12 && (cfg->n_splits < 0 || (cfg->n_splits == 0 && cus_per_head >= 5))) {
        two_pass = true;
        const int64_t n_bh8 = (int64_t)cfg->batch * cfg->n_q_heads * 8;
        int64_t ts = cfg->n_splits < 0 ? -cfg->n_splits : prop.multiProcessorCount / n_bh8;
        const int64_t by_work = ctx->cap_padded / 128 / 16;  // at least one 128-token block per wavefront
        if (cfg->n_splits == 0 && ts > by_work)
            ts = by_work;
        ctx->n_splits = (int)(ts < 1 ? 1 : (ts > PQ_MAX_SPLITS ? PQ_MAX_SPLITS : ts));
    }

    const size_t cb_bytes = (size_t)cfg->n_kv_heads * cfg->n_centroids * PQ_HEAD_DIM * ctx->elem_bytes;
    const size_t n_bh = (size_t)cfg->batch * cfg->n_q_heads;
    const size_t part_bytes = n_bh * ctx->n_splits * PQ_PART_STRIDE * sizeof(float);
    bool ok = hipMalloc(&ctx->kcb_packed, cb_bytes) == hipSuccess;
    ok = ok && hipMalloc(&ctx->vcb_packed, cb_bytes) == hipSuccess;
    ok = ok && hipMalloc((void **)&ctx->partials, part_bytes) == hipSuccess;
    ok = ok && hipMalloc((void **)&ctx->tickets, n_bh * sizeof(unsigned int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&ctx->dev_err, 2 * sizeof(unsigned int)) == hipSuccess;  // [1]: probe sink
    if (two_pass)  // partial scores [B*Hq][4 groups][capacity]
        ok = ok && hipMalloc((void **)&ctx->scores12, n_bh * 4 * (size_t)ctx->cap_padded * sizeof(float)) == hipSuccess;
    if (pq_config_is_12bit(cfg)) {
        ctx->kcb_natural = ctx->kcb_packed;
        ctx->vcb_natural = ctx->vcb_packed;
        ctx->stage_tokens = stage_tokens_for(cfg);
        const size_t st_bytes = (size_t)cfg->batch * cfg->n_kv_heads * ctx->stage_tokens * PQ12_M * sizeof(uint16_t);
        ok = ok && hipMalloc((void **)&ctx->stage[0], st_bytes) == hipSuccess;
        ok = ok && hipMalloc((void **)&ctx->stage[1], st_bytes) == hipSuccess;
    } else {
        ok = ok && hipMalloc(&ctx->kcb_natural, cb_bytes) == hipSuccess;
        ok = ok && hipMalloc(&ctx->vcb_natural, cb_bytes) == hipSuccess;
    }
    if (!ok) {
        (void)hipGetLastError();
        free_ctx(ctx);
        return PQ_ERR_ALLOC;
    }
    ok = hipMemset(ctx->tickets, 0, n_bh * sizeof(unsigned int)) == hipSuccess;
    ok = ok && hipMemset(ctx->dev_err, 0, 2 * sizeof(unsigned int)) == hipSuccess;
    ok = ok && hipMemset(ctx->partials, 0, part_bytes) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        free_ctx(ctx);
        return PQ_ERR_HIP;
    }
    *out = ctx;
    return PQ_OK;
}

int pq_attn_destroy(pq_attn_ctx *ctx)
{
    if (ctx == nullptr)
        return PQ_ERR_NULL;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    const bool ok = hipDeviceSynchronize() == hipSuccess;
    free_ctx(ctx);
    return ok ? PQ_OK : PQ_ERR_HIP;
}

int pq_attn_n_splits(const pq_attn_ctx *ctx) { return ctx ? ctx->n_splits : PQ_ERR_NULL; }

int pq_attn_n_passes(const pq_attn_ctx *ctx) { return ctx ? (ctx->scores12 ? 2 : 1) : PQ_ERR_NULL; }

int pq_attn_heads_per_workgroup(const pq_attn_ctx *ctx)
{
    if (ctx == nullptr)
        return PQ_ERR_NULL;
    return ctx->k_skew == PQ_K_SKEW_QUAD || ctx->grouped12 ? pq_grouped_heads_per_workgroup(ctx->group) : 1;
}

int pq_attn_set_codebooks(pq_attn_ctx *ctx, const void *k_codebook, const void *v_codebook, void *hip_stream)
{
    if (ctx == nullptr || k_codebook == nullptr || v_codebook == nullptr)
        return PQ_ERR_NULL;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    return ensure_codebooks(ctx, k_codebook, v_codebook, (hipStream_t)hip_stream);
}

int pq_attn_decode(pq_attn_ctx *ctx, const void *q, const uint8_t *k_codes, const uint8_t *v_codes,
                   const int32_t *ctx_len, const void *k_codebook, const void *v_codebook, const void *recent_k,
                   const void *recent_v, const int32_t *recent_len, float scale, float *out, void *hip_stream)
{
    if (ctx == nullptr || q == nullptr || k_codes == nullptr || v_codes == nullptr || ctx_len == nullptr ||
        out == nullptr)
        return PQ_ERR_NULL;
    if ((recent_k == nullptr) != (recent_v == nullptr))
        return PQ_ERR_NULL;
    if (recent_k != nullptr && ctx->cfg.max_recent == 0)
        return PQ_ERR_SHAPE;
    if (!(fabsf(scale) <= 3.0e38f))  // NaN or infinite
        return PQ_ERR_SHAPE;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    hipStream_t s = (hipStream_t)hip_stream;
    const int rc = ensure_codebooks(ctx, k_codebook, v_codebook, s);
    if (rc != PQ_OK)
        return rc;

    return launch_decode(ctx, q, k_codes, v_codes, ctx_len, recent_k, recent_v, recent_len, scale, out, s);
}

int pq_attn_decode_noalloc(const pq_attn_config *cfg, const void *q, const uint8_t *k_codes, const uint8_t *v_codes,
                           const int32_t *ctx_len, const void *k_codebook, const void *v_codebook, const void *recent_k,
                           const void *recent_v, const int32_t *recent_len, float scale, float *out, void *hip_stream)
{
    if (cfg == nullptr || q == nullptr || k_codes == nullptr || v_codes == nullptr || ctx_len == nullptr ||
        k_codebook == nullptr || v_codebook == nullptr || out == nullptr)
        return PQ_ERR_NULL;
    const int rc = validate(cfg);
    if (rc != PQ_OK)
        return rc;
    if ((recent_k == nullptr) != (recent_v == nullptr))
        return PQ_ERR_NULL;
    if (recent_k != nullptr && cfg->max_recent == 0)
        return PQ_ERR_SHAPE;
    if (!(fabsf(scale) <= 3.0e38f))
        return PQ_ERR_SHAPE;
    if (pq_config_is_12bit(cfg))
        return PQ_ERR_UNSUPPORTED;  // 1.5 MiB of tables per head and a per-token score buffer: not in a modest array
    // limits of the static scratch
    const size_t elem = cfg->dtype == PQ_F16 ? 2 : 4;
    const int64_t rows = (int64_t)cfg->batch * cfg->n_q_heads;
    if ((size_t)cfg->n_kv_heads * 256 * PQ_HEAD_DIM * elem > PQ_NOALLOC_CODEBOOK_BYTES || rows > PQ_NOALLOC_MAX_ROWS ||
        (cfg->n_splits > 0 && rows * cfg->n_splits > PQ_NOALLOC_MAX_ROWS))
        return PQ_ERR_CAPACITY;
    device_guard guard(cfg->device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    noalloc_device dev;
    const int lrc = noalloc_lookup(cfg->device, &dev);
    if (lrc != PQ_OK)
        return lrc;

    // a context on the stack whose buffers are pieces of this GPU's scratch array
    pq_attn_ctx ctx{};
    ctx.cfg = *cfg;
    ctx.ds = cfg->head_dim / cfg->n_subspaces;
    ctx.group = cfg->n_q_heads / cfg->n_kv_heads;
    ctx.cap_padded = padded_capacity(cfg);
    ctx.elem_bytes = elem;
    ctx.k_skew = pq_config_uses_grouped_kernel(cfg) ? PQ_K_SKEW_QUAD : PQ_K_SKEW_LANE;
    ctx.n_cu = dev.n_cu;
    int64_t splits = cfg->n_splits > 0 ? cfg->n_splits : choose_splits(cfg, dev.n_cu);
    if (rows * splits > PQ_NOALLOC_MAX_ROWS)
        splits = PQ_NOALLOC_MAX_ROWS / rows;
    ctx.n_splits = (int)splits;
    ctx.kcb_packed = dev.ptr;
    ctx.vcb_packed = dev.ptr + PQ_NOALLOC_CODEBOOK_BYTES;
    ctx.partials = (float *)(dev.ptr + PQ_NOALLOC_PARTIALS_OFF);
    ctx.tickets = (unsigned int *)(dev.ptr + PQ_NOALLOC_TICKETS_OFF);
    hipStream_t s = (hipStream_t)hip_stream;
    if (pq_launch_pack_codebook(&ctx, k_codebook, ctx.kcb_packed, nullptr, s) != hipSuccess ||
        pq_launch_pack_codebook(&ctx, v_codebook, ctx.vcb_packed, nullptr, s) != hipSuccess)
        return PQ_ERR_HIP;
    // the tickets must start at zero; the array keeps whatever the last call on this GPU left (a fill kernel,
    // not a memset: this call may be recorded into a HIP graph)
    if (pq_launch_clear_words(ctx.tickets, rows, s) != hipSuccess)
        return PQ_ERR_HIP;
    return launch_decode(&ctx, q, k_codes, v_codes, ctx_len, recent_k, recent_v, recent_len, scale, out, s);
}

int pq_encode_append(pq_attn_ctx *ctx, const void *new_k, const void *new_v, int32_t n_new, const void *k_codebook,
                     const void *v_codebook, uint8_t *k_codes, uint8_t *v_codes, int32_t *ctx_len, void *hip_stream)
{
    if (ctx == nullptr || new_k == nullptr || new_v == nullptr || k_codes == nullptr || v_codes == nullptr ||
        ctx_len == nullptr)
        return PQ_ERR_NULL;
    if (n_new <= 0 || n_new > ctx->cfg.max_context)
        return PQ_ERR_CAPACITY;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    hipStream_t s = (hipStream_t)hip_stream;
    // keeps the decode path's packed copy in step with the codebooks used to encode
    const int rc = ensure_codebooks(ctx, k_codebook, v_codebook, s);
    if (rc != PQ_OK)
        return rc;

    pq_encode_args a;
    a.x[0] = new_k;
    a.x[1] = new_v;
    a.codebook[0] = ctx->kcb_natural;  // the context's own copies, never the caller's tensors
    a.codebook[1] = ctx->vcb_natural;
    a.codes[0] = k_codes;
    a.codes[1] = v_codes;
    a.ctx_len = ctx_len;
    a.B = ctx->cfg.batch;
    a.Hkv = ctx->cfg.n_kv_heads;
    a.n_new = n_new;
    a.max_context = ctx->cfg.max_context;
    a.k_skew = ctx->k_skew;
    a.head_stride = ctx->cap_padded * token_bytes(&ctx->cfg);
    if (pq_config_is_12bit(&ctx->cfg)) {
        // codes are staged token-major (uint16) and packed by a second kernel; the staging buffers were sized at
        // creation, a longer append goes through them in chunks (each chunk: encode, pack, advance the lengths)
        for (int32_t t0 = 0; t0 < n_new; t0 += ctx->stage_tokens) {
            a.n_new = n_new - t0 < ctx->stage_tokens ? n_new - t0 : ctx->stage_tokens;
            a.x[0] = (const char *)new_k + (int64_t)t0 * PQ_HEAD_DIM * sizeof(uint16_t);
            a.x[1] = (const char *)new_v + (int64_t)t0 * PQ_HEAD_DIM * sizeof(uint16_t);
            if (pq12_launch_encode_append(ctx, a, n_new, ctx_len, ctx->dev_err, s) != hipSuccess)
                return PQ_ERR_HIP;
        }
        return PQ_OK;
    }
    return pq_launch_encode(ctx, a, ctx_len, ctx->dev_err, s) == hipSuccess ? PQ_OK : PQ_ERR_HIP;
}

static int pack_common(pq_attn_ctx *ctx, int32_t kind, const void *token_major, int32_t n_tokens, uint8_t *packed,
                       bool unpack, void *hip_stream)
{
    if (ctx == nullptr || token_major == nullptr || packed == nullptr)
        return PQ_ERR_NULL;
    if (kind != PQ_CODES_K && kind != PQ_CODES_V)
        return PQ_ERR_SHAPE;
    if (n_tokens < 0)
        return PQ_ERR_SHAPE;
    if (n_tokens > ctx->cfg.max_context)
        return PQ_ERR_CAPACITY;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    const hipError_t e =
        pq_config_is_12bit(&ctx->cfg)
            ? pq12_launch_pack_codes(ctx, kind, (const uint16_t *)token_major, n_tokens, packed, unpack, (hipStream_t)hip_stream)
            : pq_launch_pack_codes(ctx, kind, (const uint8_t *)token_major, n_tokens, packed, unpack, (hipStream_t)hip_stream);
    return e == hipSuccess ? PQ_OK : PQ_ERR_HIP;
}

int pq_pack_codes(pq_attn_ctx *ctx, int32_t kind, const void *token_major, int32_t n_tokens, uint8_t *packed,
                  void *hip_stream)
{
    return pack_common(ctx, kind, token_major, n_tokens, packed, false, hip_stream);
}

int pq_unpack_codes(pq_attn_ctx *ctx, int32_t kind, const uint8_t *packed, int32_t n_tokens, void *token_major,
                    void *hip_stream)
{
    return pack_common(ctx, kind, token_major, n_tokens, const_cast<uint8_t *>(packed), true, hip_stream);
}

int64_t pq_kmeans_workspace_bytes(const pq_attn_ctx *ctx)
{
    if (ctx == nullptr)
        return PQ_ERR_NULL;
    if (ctx->cfg.dtype != PQ_F16)
        return PQ_ERR_UNSUPPORTED;
    return pq_kmeans_accumulator_bytes(ctx);
}

int pq_kmeans_fit(pq_attn_ctx *ctx, const void *samples, int32_t n_samples, void *codebook, int32_t n_iters,
                  void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    if (ctx == nullptr || samples == nullptr || codebook == nullptr || workspace == nullptr)
        return PQ_ERR_NULL;
    if (ctx->cfg.dtype != PQ_F16)
        return PQ_ERR_UNSUPPORTED;
    if (n_samples < 1 || n_iters < 1 || ((uintptr_t)workspace & 7) != 0)
        return PQ_ERR_SHAPE;
    if (n_samples > (1 << 20) || workspace_bytes < pq_kmeans_accumulator_bytes(ctx))
        return PQ_ERR_CAPACITY;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    return pq_launch_kmeans(ctx, samples, n_samples, codebook, n_iters, workspace, (hipStream_t)hip_stream) == hipSuccess
               ? PQ_OK
               : PQ_ERR_HIP;
}

int pq_stream_read_probe(pq_attn_ctx *ctx, const void *src, int64_t bytes, void *hip_stream)
{
    if (ctx == nullptr || src == nullptr)
        return PQ_ERR_NULL;
    if (bytes < 16 || (bytes & 15) != 0 || ((uintptr_t)src & 15) != 0)
        return PQ_ERR_SHAPE;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    return pq_launch_stream_read(src, bytes, ctx->dev_err + 1, (hipStream_t)hip_stream) == hipSuccess ? PQ_OK : PQ_ERR_HIP;
}

int pq_attn_device_error(pq_attn_ctx *ctx, uint32_t *flags)
{
    if (ctx == nullptr || flags == nullptr)
        return PQ_ERR_NULL;
    device_guard guard(ctx->cfg.device);
    if (!guard.ok)
        return PQ_ERR_HIP;
    unsigned int v = 0;
    if (hipDeviceSynchronize() != hipSuccess)
        return PQ_ERR_HIP;
    if (hipMemcpy(&v, ctx->dev_err, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess)
        return PQ_ERR_HIP;
    if (v != 0 && hipMemset(ctx->dev_err, 0, sizeof(v)) != hipSuccess)
        return PQ_ERR_HIP;
    *flags = v;
    return PQ_OK;
}

const char *pq_status_string(int status)
{
    switch (status) {
    case PQ_OK: return "ok";
    case PQ_ERR_NULL: return "a required pointer is NULL";
    case PQ_ERR_SHAPE: return "inconsistent sizes";
    case PQ_ERR_UNSUPPORTED: return "shape not supported by this build";
    case PQ_ERR_CAPACITY: return "capacity exceeded";
    case PQ_ERR_HIP: return "HIP runtime error";
    case PQ_ERR_ALLOC: return "allocation failed";
    default: return "unknown status";
    }
}

}  // extern "C"
