// C ABI of the HashAttention decode library: argument checks, scratch
// ownership, launch-shape choices.  All arithmetic is in the kernels.
#include "../../include/hashattn.h"
#include "kernels.hpp"

#include <climits>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

struct hashattn_ctx {
    hashattn_config cfg;
    int device;
    int group;
    // TOPK scratch
    int32_t* blk_cum;
    int32_t blocks_pitch;
    int32_t topk_path;            // 0: chosen per call; 1: always two launches; 2: one launch whenever the shape allows
    uint4* frags;                 // bf16 weight fragments of the matrix-core key encoder, per KV head
    uint32_t* append_done;        // two-word block counter of the decode-time append kernel (see finish_append)
    int32_t* append_fault_host;   // pinned host word an append launch raises when it finds that counter inconsistent
    int32_t* append_fault_dev;    // the device's address of the same word
    int64_t frag_bytes;
    // split partials shared by GATHER-ATT and the dense kernel
    float* part;
    int64_t part_floats;
    int64_t scratch_bytes;
    char err[256];
};

namespace {

constexpr int kMinUnit = 256;          // tokens per wave unit: one 16-byte load per lane
constexpr int kMaxUnit = 2048;
constexpr int kMaxSplits = 256;

thread_local char g_create_err[256] = "";     // last failure of a call without a context, per host thread

hashattn_status fail(hashattn_ctx* ctx, hashattn_status st, const char* fmt, ...)
{
    char* dst = ctx ? ctx->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return st;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool pow2_width(int w) { return w == 32 || w == 64 || w == 128 || w == 256; }

hashattn_status check_mlp(hashattn_ctx* ctx, const hashattn_mlp* m, int n_heads, const char* what)
{
    if (!m) return fail(ctx, HASHATTN_INVALID_ARG, "%s: mapping network is NULL", what);
    if (m->n_heads != n_heads)
        return fail(ctx, HASHATTN_INVALID_ARG, "%s: network has %d heads, expected %d", what, m->n_heads, n_heads);
    if (m->n_layers < 1 || m->n_layers > 3)
        return fail(ctx, HASHATTN_UNSUPPORTED, "%s: n_layers %d not in 1..3", what, m->n_layers);
    if (m->dims[0] != ha::kHeadDim || m->dims[m->n_layers] != ctx->cfg.bits)
        return fail(ctx, HASHATTN_UNSUPPORTED, "%s: network must map 128 inputs to %d outputs (the context's bits)", what, ctx->cfg.bits);
    for (int l = 1; l < m->n_layers; ++l)
        if (!pow2_width(m->dims[l]))
            return fail(ctx, HASHATTN_UNSUPPORTED, "%s: hidden width %d not in {32,64,128,256}", what, m->dims[l]);
    for (int l = 0; l < m->n_layers; ++l) {
        if (!m->W[l]) return fail(ctx, HASHATTN_INVALID_ARG, "%s: W[%d] is NULL", what, l);
        if (!aligned(m->W[l], 16)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: W[%d] not 16-byte aligned", what, l);
        if (m->bias[l] && !aligned(m->bias[l], 4))
            return fail(ctx, HASHATTN_INVALID_ARG, "%s: bias[%d] not 4-byte aligned", what, l);
    }
    return HASHATTN_OK;
}

ha::MlpView view_of(const hashattn_mlp* m)
{
    ha::MlpView v{};
    v.n_layers = m->n_layers;
    for (int i = 0; i < 5; ++i) v.dims[i] = m->dims[i];
    for (int i = 0; i < 4; ++i) { v.W[i] = i < m->n_layers ? m->W[i] : nullptr; v.bias[i] = i < m->n_layers ? m->bias[i] : nullptr; }
    return v;
}

// ctx may be NULL (the entry point without a context): the message then goes to the thread's buffer.
hashattn_status check_cache(hashattn_ctx* ctx, const hashattn_config& cfg, const hashattn_kv* kv, int batch, bool need_codes,
                            const char* what)
{
    if (!kv) return fail(ctx, HASHATTN_INVALID_ARG, "%s: cache is NULL", what);
    if (batch < 1) return fail(ctx, HASHATTN_INVALID_ARG, "%s: batch %d < 1", what, batch);
    if (batch > cfg.max_batch)
        return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "%s: batch %d exceeds max_batch %d", what, batch, cfg.max_batch);
    if (!kv->k || !kv->v || !kv->seq_lens) return fail(ctx, HASHATTN_INVALID_ARG, "%s: k, v or seq_lens is NULL", what);
    if (need_codes && !kv->codes) return fail(ctx, HASHATTN_INVALID_ARG, "%s: codes is NULL", what);
    if (!aligned(kv->k, 16) || !aligned(kv->v, 16)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: k/v not 16-byte aligned", what);
    if (kv->codes && !aligned(kv->codes, 16)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: codes not 16-byte aligned", what);
    if (!aligned(kv->seq_lens, 4)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: seq_lens not 4-byte aligned", what);
    if (kv->max_seq_len < 0) return fail(ctx, HASHATTN_INVALID_ARG, "%s: max_seq_len %d < 0", what, kv->max_seq_len);
    if (kv->max_seq_len > cfg.max_context)
        return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "%s: max_seq_len %d exceeds max_context %lld", what,
                    kv->max_seq_len, (long long)cfg.max_context);
    if (cfg.page_size == 0) {
        if (kv->page_table) return fail(ctx, HASHATTN_INVALID_ARG, "%s: page_table given to a contiguous context", what);
        if (kv->n_max < 1 || (kv->n_max & 3)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: n_max %lld must be a positive multiple of 4", what, (long long)kv->n_max);
        if (kv->max_seq_len > kv->n_max) return fail(ctx, HASHATTN_INVALID_ARG, "%s: max_seq_len %d exceeds n_max %lld", what, kv->max_seq_len, (long long)kv->n_max);
    } else {
        if (!kv->page_table) return fail(ctx, HASHATTN_INVALID_ARG, "%s: page_table is NULL in a paged context", what);
        if (!aligned(kv->page_table, 4)) return fail(ctx, HASHATTN_INVALID_ARG, "%s: page_table not 4-byte aligned", what);
        if (kv->max_pages_per_seq < 1 || kv->n_pages < 1) return fail(ctx, HASHATTN_INVALID_ARG, "%s: max_pages_per_seq and n_pages must be >= 1", what);
        if ((int64_t)kv->max_seq_len > (int64_t)kv->max_pages_per_seq * ha::kPage)
            return fail(ctx, HASHATTN_INVALID_ARG, "%s: max_seq_len %d exceeds the page table's reach", what, kv->max_seq_len);
    }
    return HASHATTN_OK;
}

hashattn_status check_cache(hashattn_ctx* ctx, const hashattn_kv* kv, int batch, bool need_codes, const char* what)
{
    return check_cache(ctx, ctx->cfg, kv, batch, need_codes, what);
}

ha::KvView view_of(int n_kv_heads, const hashattn_kv* kv)
{
    ha::KvView v{};
    v.k = static_cast<const uint16_t*>(kv->k);
    v.v = static_cast<const uint16_t*>(kv->v);
    v.codes = kv->codes;
    v.page_table = kv->page_table;
    v.seq_lens = kv->seq_lens;
    v.n_max = kv->n_max;
    v.max_pages_per_seq = kv->max_pages_per_seq;
    v.n_kv_heads = n_kv_heads;
    return v;
}

ha::KvView view_of(const hashattn_ctx* ctx, const hashattn_kv* kv) { return view_of(ctx->cfg.n_kv_heads, kv); }

// Tokens per wave unit of SCORE/TOPK: small units fill the chip at short contexts, larger ones
// keep the number of blocks (and of per-block tables every block has to sum) down at long contexts.
// `mixed`: the caller gave a k per sequence, so lengths differ; a block is sized by the longest
// sequence and mostly idle for a short one, hence the smaller cap.
int pick_unit_tokens(const hashattn_ctx* ctx, int batch, int max_seq_len, bool mixed, int* waves_per_block)
{
    const int64_t lanes = (int64_t)batch * ctx->cfg.n_kv_heads;
    const bool wide = ctx->cfg.bits > 32;
    const int cap = (mixed || wide) ? kMaxUnit / 2 : kMaxUnit;      // wide codes: units of at most 1024
    const int hard_cap = wide ? kMaxUnit / 2 : kMaxUnit;
    auto pick = [&](int wpb) {
        auto blocks = [&](int u) { return (max_seq_len + (int64_t)u * wpb - 1) / ((int64_t)u * wpb); };
        int unit = kMinUnit;
        // up to about one block per CU keeps the per-block tables short
        while (unit < cap && lanes * blocks(unit) > 256) unit *= 2;
        // units of 2048 tokens (two chunks per wave in the select, 92 registers: two 8-wave blocks per CU) only
        // where units of 1024 (75 registers: three blocks per CU) would mean more than 2048 blocks (few pairs at a very
        // long context take 16-wave blocks instead, below)
        if (unit == kMaxUnit && !wide && lanes > 16 && lanes * blocks(kMaxUnit / 2) <= 2048) unit = kMaxUnit / 2;
        // never more blocks per sequence than the scratch pitch
        while (unit < hard_cap && blocks(unit) > ctx->blocks_pitch) unit *= 2;
        return unit;
    };
    // Blocks of 8 waves: two share a CU and one's table prologue overlaps the other's scoring.  With few
    // (sequence, KV head) pairs and a very long context that would mean units of 2048 tokens (two chunks
    // per wave in the select); blocks of 16 waves with units of 1024 measured faster there.
    int wpb = ha::kTopkWavesPerBlock;
    int unit = pick(wpb);
    if (!wide && !mixed && lanes <= 16 && unit == kMaxUnit && ctx->group <= 4) {   // 8 heads per group: a 16-wave block would spill
        wpb = 16;
        unit = pick(wpb);
    }
    *waves_per_block = wpb;
    return unit;
}

// SCORE + TOPK in one launch (a block per sequence and query head) or in two (blocks per KV head and piece of
// the sequence).  One launch wins while its blocks, each as long as the sequence, all fit on the chip's 256
// compute units at once, two to a unit (measured at 2K to 32K tokens: ahead up to 512 blocks, behind at 1024).
bool one_launch_topk(const hashattn_ctx* ctx, int batch, int max_seq_len)
{
    if (ctx->cfg.bits != ha::kBits || max_seq_len > ha::score_topk_one_block_limit() || ctx->topk_path == 1) return false;
    if (ctx->topk_path == 2) return true;
    return (int64_t)batch * ctx->cfg.n_q_heads <= 512;
}

// Split shape for the attention kernels: `total` tokens per (sequence, head), `lanes` independent
// (sequence, head) pairs that share the launch.  About a thousand blocks fill the chip; pieces of
// at most `max_chunk` tokens keep a batch of mixed lengths balanced (the grid is sized by the
// longest list, blocks past the end of a shorter one exit at once).
void pick_splits(int64_t part_floats, int n_q_heads, int64_t lanes, int64_t total, int batch, int64_t max_chunk, int* chunk,
                 int* n_splits)
{
    int64_t cap = part_floats / ((int64_t)batch * n_q_heads * ha::kPartStride);
    if (cap > kMaxSplits) cap = kMaxSplits;
    if (cap < 1) cap = 1;
    const int64_t target = 1024, min_chunk = 64;
    int64_t want = (target + lanes - 1) / lanes;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    int64_t c = (total + want - 1) / want;
    c = (c + 63) / 64 * 64;                                    // whole 64-row iterations
    if (c > max_chunk) c = max_chunk;
    if (c < min_chunk) c = min_chunk;
    int64_t s = (total + c - 1) / c;
    if (s < 1) s = 1;
    while (s > cap) { c *= 2; s = (total + c - 1) / c; }
    *chunk = (int)c;
    *n_splits = (int)s;
}

hashattn_status hip_fail(hashattn_ctx* ctx, hipError_t e, const char* what)
{
    return fail(ctx, HASHATTN_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

// An append launch found its block counter in a state that no completed launch leaves behind (see
// finish_append) and said so in pinned host memory: the sequence lengths of the caches it served may be
// wrong, so every later call on the context is refused.
hashattn_status check_append_state(hashattn_ctx* ctx, const char* what)
{
    const int32_t seen = *static_cast<volatile int32_t*>(ctx->append_fault_host);
    if (seen == 0) return HASHATTN_OK;
    return fail(ctx, HASHATTN_HIP_ERROR,
                "%s: an earlier decode-time append counted block number %d, beyond its grid: a launch before it did "
                "not run to its end and sequence lengths may not have advanced once; destroy this context and check the caches",
                what, seen);
}

}  // namespace

extern "C" {

hashattn_status hashattn_create(hashattn_ctx** out, const hashattn_config* cfg)
{
    if (!out || !cfg) return fail(nullptr, HASHATTN_INVALID_ARG, "create: NULL argument");
    *out = nullptr;
    if (cfg->head_dim != ha::kHeadDim) return fail(nullptr, HASHATTN_UNSUPPORTED, "create: head_dim %d, only 128 is supported", cfg->head_dim);
    if (cfg->bits != 32 && cfg->bits != 64 && cfg->bits != 128 && cfg->bits != 256 && cfg->bits != 512)
        return fail(nullptr, HASHATTN_UNSUPPORTED, "create: bits %d not in {32,64,128,256,512}", cfg->bits);
    if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads)
        return fail(nullptr, HASHATTN_INVALID_ARG, "create: n_q_heads %d must be a positive multiple of n_kv_heads %d", cfg->n_q_heads, cfg->n_kv_heads);
    const int group = cfg->n_q_heads / cfg->n_kv_heads;
    if (group != 1 && group != 2 && group != 4 && group != 8)
        return fail(nullptr, HASHATTN_UNSUPPORTED, "create: group size %d not in {1,2,4,8}", group);
    if (cfg->page_size != 0 && cfg->page_size != ha::kPage)
        return fail(nullptr, HASHATTN_UNSUPPORTED, "create: page_size %d, only 0 (contiguous) or 16", cfg->page_size);
    if (cfg->max_batch < 1 || cfg->max_batch > 65535) return fail(nullptr, HASHATTN_INVALID_ARG, "create: max_batch %d not in 1..65535", cfg->max_batch);
    const int64_t context_limit = (int64_t)ha::kMaxTopkBlocks * ha::kTopkWavesPerBlock *
                                  (cfg->bits > 32 ? kMaxUnit / 2 : kMaxUnit);       // 4 Mi tokens (2 Mi with wide codes)
    if (cfg->max_context < 1 || cfg->max_context > context_limit)
        return fail(nullptr, HASHATTN_INVALID_ARG, "create: max_context %lld not in 1..%lld", (long long)cfg->max_context,
                    (long long)context_limit);
    if (cfg->max_k < 1 || cfg->max_k > (int64_t)1 << 30)
        return fail(nullptr, HASHATTN_INVALID_ARG, "create: max_k %lld not in 1..2^30", (long long)cfg->max_k);
    if (cfg->n_kv_heads > 65535) return fail(nullptr, HASHATTN_INVALID_ARG, "create: n_kv_heads too large");

    hashattn_ctx* ctx = new (std::nothrow) hashattn_ctx();
    if (!ctx) return fail(nullptr, HASHATTN_HIP_ERROR, "create: out of host memory");
    ctx->cfg = *cfg;
    ctx->group = group;
    ctx->err[0] = 0;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) { delete ctx; return fail(nullptr, HASHATTN_HIP_ERROR, "create: hipGetDevice: %s", hipGetErrorString(e)); }

    const int64_t bh = (int64_t)cfg->max_batch * cfg->n_q_heads;
    // per-block score tables: one block per 8 units of at least 256 tokens, at most kMaxTopkBlocks per sequence
    int64_t pitch = (cfg->max_context + (int64_t)kMinUnit * ha::kTopkWavesPerBlock - 1) / ((int64_t)kMinUnit * ha::kTopkWavesPerBlock);
    if (pitch > ha::kMaxTopkBlocks) pitch = ha::kMaxTopkBlocks;
    ctx->blocks_pitch = (int32_t)pitch;
    const int64_t hist_bytes = bh * pitch * (cfg->bits + 2) * (int64_t)sizeof(int32_t);   // rows C(0..bits) and a zero
    int64_t splits = (cfg->max_context + 63) / 64;               // dense needs more splits than gather
    int64_t want = 8192 / bh; if (want < 16) want = 16;
    if (splits > want) splits = want;
    if (splits > kMaxSplits) splits = kMaxSplits;
    ctx->part_floats = bh * splits * ha::kPartStride;
    const int64_t part_bytes = ctx->part_floats * (int64_t)sizeof(float);
    ctx->frag_bytes = (int64_t)cfg->n_kv_heads * ha::encode_mfma_scratch_bytes_per_head();
    ctx->scratch_bytes = hist_bytes + part_bytes + ctx->frag_bytes;

    if ((e = hipMalloc(reinterpret_cast<void**>(&ctx->blk_cum), hist_bytes)) != hipSuccess ||
        (e = hipMalloc(reinterpret_cast<void**>(&ctx->part), part_bytes)) != hipSuccess ||
        (e = hipMalloc(reinterpret_cast<void**>(&ctx->frags), ctx->frag_bytes)) != hipSuccess ||
        (e = hipMalloc(reinterpret_cast<void**>(&ctx->append_done), 256)) != hipSuccess ||
        (e = hipMemset(ctx->append_done, 0, 256)) != hipSuccess ||
        (e = hipHostMalloc(reinterpret_cast<void**>(&ctx->append_fault_host), 64, hipHostMallocMapped)) != hipSuccess ||
        (e = hipHostGetDevicePointer(reinterpret_cast<void**>(&ctx->append_fault_dev), ctx->append_fault_host, 0)) != hipSuccess ||
        (e = hipDeviceSynchronize()) != hipSuccess) {      // the counter is zero before any stream uses it
        const long long wanted = (long long)ctx->scratch_bytes;
        hashattn_destroy(ctx);
        return fail(nullptr, HASHATTN_HIP_ERROR, "create: allocating %lld scratch bytes: %s", wanted, hipGetErrorString(e));
    }
    *ctx->append_fault_host = 0;
    if ((e = ha::setup_encode_bulk()) != hipSuccess || (e = ha::setup_encode_mfma()) != hipSuccess) {
        hashattn_destroy(ctx);
        return fail(nullptr, HASHATTN_HIP_ERROR, "create: raising the LDS limit of the key encoder: %s", hipGetErrorString(e));
    }
    if ((e = cfg->bits == ha::kBits ? ha::setup_score_topk(group) : ha::setup_score_topk_wide(group, cfg->bits / ha::kBits)) != hipSuccess) {
        hashattn_destroy(ctx);
        return fail(nullptr, HASHATTN_HIP_ERROR, "create: raising the LDS limit of the TOPK kernels: %s", hipGetErrorString(e));
    }
    *out = ctx;
    return HASHATTN_OK;
}

hashattn_status hashattn_destroy(hashattn_ctx* ctx)
{
    if (!ctx) return HASHATTN_OK;
    if (ctx->blk_cum) (void)hipFree(ctx->blk_cum);
    if (ctx->part) (void)hipFree(ctx->part);
    if (ctx->frags) (void)hipFree(ctx->frags);
    if (ctx->append_done) (void)hipFree(ctx->append_done);
    if (ctx->append_fault_host) (void)hipHostFree(ctx->append_fault_host);
    delete ctx;
    return HASHATTN_OK;
}

const char* hashattn_last_error(const hashattn_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

int64_t hashattn_scratch_bytes(const hashattn_ctx* ctx) { return ctx ? ctx->scratch_bytes : 0; }

hashattn_status hashattn_selftest_set_append_counter(hashattn_ctx* ctx, int32_t value, void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (value < 0) return fail(ctx, HASHATTN_INVALID_ARG, "selftest_set_append_counter: value %d < 0", value);
    const hipError_t e = ha::launch_set_append_counter(ctx->append_done, (uint32_t)value, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "selftest_set_append_counter");
}

hashattn_status hashattn_selftest_set_topk_path(hashattn_ctx* ctx, int32_t path)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (path < 0 || path > 2) return fail(ctx, HASHATTN_INVALID_ARG, "selftest_set_topk_path: path %d is not 0, 1 or 2", path);
    ctx->topk_path = path;
    return HASHATTN_OK;
}

hashattn_status hashattn_encode_keys(hashattn_ctx* ctx, const hashattn_mlp* phi_kv, const void* k_new,
                                     const void* v_new, int32_t batch, int64_t n_new, hashattn_kv* cache,
                                     void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (hashattn_status s = check_append_state(ctx, "encode_keys")) return s;
    if (hashattn_status s = check_mlp(ctx, phi_kv, ctx->cfg.n_kv_heads, "encode_keys")) return s;
    if (hashattn_status s = check_cache(ctx, cache, batch, true, "encode_keys")) return s;
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(ctx, HASHATTN_INVALID_ARG, "encode_keys: k_new and v_new must both be given (append) or both NULL (in place)");
    if (n_new < 1) return fail(ctx, HASHATTN_INVALID_ARG, "encode_keys: n_new %lld < 1", (long long)n_new);
    const bool paged = ctx->cfg.page_size != 0;
    if (k_new) {
        if (!aligned(k_new, 16) || !aligned(v_new, 16)) return fail(ctx, HASHATTN_INVALID_ARG, "encode_keys: k_new/v_new not 16-byte aligned");
        const int64_t room = paged ? (int64_t)cache->max_pages_per_seq * ha::kPage : cache->n_max;
        if ((int64_t)cache->max_seq_len + n_new > room)
            return fail(ctx, HASHATTN_INVALID_ARG, "encode_keys: appending %lld tokens to max_seq_len %d exceeds the cache capacity %lld",
                        (long long)n_new, cache->max_seq_len, (long long)room);
        if ((int64_t)cache->max_seq_len + n_new > ctx->cfg.max_context)
            return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "encode_keys: append would exceed max_context %lld", (long long)ctx->cfg.max_context);
    }
    const ha::EncodeScratch enc{ctx->frags, ha::encode_mfma_scratch_bytes_per_head() / 16, ctx->append_done,
                                ctx->append_fault_dev};
    const hipError_t e = ha::launch_encode_keys(view_of(phi_kv), view_of(ctx, cache), paged,
                                                static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                                                batch, n_new, cache->max_seq_len, &enc, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "encode_keys");
    if (k_new) cache->max_seq_len += (int32_t)n_new;
    return HASHATTN_OK;
}

hashattn_status hashattn_encode_query(hashattn_ctx* ctx, const hashattn_mlp* phi_q, const void* q, int32_t batch,
                                      uint32_t* q_codes, void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (hashattn_status s = check_append_state(ctx, "encode_query")) return s;
    if (hashattn_status s = check_mlp(ctx, phi_q, ctx->cfg.n_q_heads, "encode_query")) return s;
    if (!q || !q_codes) return fail(ctx, HASHATTN_INVALID_ARG, "encode_query: q or q_codes is NULL");
    if (!aligned(q, 16) || !aligned(q_codes, 4)) return fail(ctx, HASHATTN_INVALID_ARG, "encode_query: q needs 16-byte, q_codes 4-byte alignment");
    if (batch < 1) return fail(ctx, HASHATTN_INVALID_ARG, "encode_query: batch %d < 1", batch);
    if (batch > ctx->cfg.max_batch) return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "encode_query: batch %d exceeds max_batch %d", batch, ctx->cfg.max_batch);
    const hipError_t e = ha::launch_encode_query(view_of(phi_q), static_cast<const uint16_t*>(q), batch,
                                                 ctx->cfg.n_q_heads, q_codes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "encode_query");
}

hashattn_status hashattn_score_topk_window(hashattn_ctx* ctx, const uint32_t* q_codes, const hashattn_kv* cache,
                                           int32_t batch, const int32_t* k_per_seq, int32_t k_max, int32_t n_sink,
                                           int32_t n_local, int32_t* idx, int32_t* count, uint8_t* threshold,
                                           void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (hashattn_status s = check_append_state(ctx, "score_topk")) return s;
    if (hashattn_status s = check_cache(ctx, cache, batch, true, "score_topk")) return s;
    if (!q_codes || !idx || !count) return fail(ctx, HASHATTN_INVALID_ARG, "score_topk: q_codes, idx or count is NULL");
    if (!aligned(q_codes, 4) || !aligned(idx, 4) || !aligned(count, 4) || (k_per_seq && !aligned(k_per_seq, 4)))
        return fail(ctx, HASHATTN_INVALID_ARG, "score_topk: 4-byte alignment required");
    if (k_max < 1) return fail(ctx, HASHATTN_INVALID_ARG, "score_topk: k_max %d < 1", k_max);
    if (n_sink < 0 || n_local < 0) return fail(ctx, HASHATTN_INVALID_ARG, "score_topk: n_sink %d or n_local %d is negative", n_sink, n_local);
    if ((int64_t)k_max + n_sink + n_local > ctx->cfg.max_k)
        return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "score_topk: k_max + n_sink + n_local = %lld exceeds max_k %lld",
                    (long long)k_max + n_sink + n_local, (long long)ctx->cfg.max_k);
    const ha::TopkScratch sc{ctx->blk_cum, ctx->blocks_pitch};
    int wpb = 0;
    const int unit = pick_unit_tokens(ctx, batch, cache->max_seq_len, k_per_seq != nullptr, &wpb);
    const ha::TopkCall call{q_codes, k_per_seq, k_max, n_sink, n_local, batch, ctx->cfg.n_q_heads, cache->max_seq_len,
                            wpb, idx, count, threshold};
    if (one_launch_topk(ctx, batch, cache->max_seq_len)) {
        const hipError_t e1 = ha::launch_score_topk_one_block(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group, call,
                                                              nullptr, nullptr, static_cast<hipStream_t>(stream));
        return e1 == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e1, "score_topk");
    }
    const hipError_t e = ctx->cfg.bits == ha::kBits
        ? ha::launch_score_topk(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group, call, unit, sc,
                                static_cast<hipStream_t>(stream))
        : ha::launch_score_topk_wide(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group, ctx->cfg.bits / ha::kBits,
                                     call, unit, sc, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "score_topk");
}

hashattn_status hashattn_score_topk(hashattn_ctx* ctx, const uint32_t* q_codes, const hashattn_kv* cache,
                                    int32_t batch, const int32_t* k_per_seq, int32_t k_max, int32_t* idx,
                                    int32_t* count, uint8_t* threshold, void* stream)
{
    return hashattn_score_topk_window(ctx, q_codes, cache, batch, k_per_seq, k_max, 0, 0, idx, count, threshold, stream);
}

hashattn_status hashattn_encode_score_topk(hashattn_ctx* ctx, const hashattn_mlp* phi_q, const void* q,
                                           const hashattn_kv* cache, int32_t batch, const int32_t* k_per_seq,
                                           int32_t k_max, int32_t n_sink, int32_t n_local, uint32_t* q_codes,
                                           int32_t* idx, int32_t* count, uint8_t* threshold, void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    // one launch when the shape allows it and the mapping is one the kernel has; every argument is then
    // checked here as the two calls would check it
    const bool one = phi_q && cache && one_launch_topk(ctx, batch, cache->max_seq_len) && phi_q->n_layers >= 1 &&
                     phi_q->n_layers <= 4 && ha::one_block_can_encode(view_of(phi_q));
    if (!one) {
        if (hashattn_status s = hashattn_encode_query(ctx, phi_q, q, batch, q_codes, stream)) return s;
        return hashattn_score_topk_window(ctx, q_codes, cache, batch, k_per_seq, k_max, n_sink, n_local, idx, count,
                                          threshold, stream);
    }
    if (hashattn_status s = check_append_state(ctx, "encode_score_topk")) return s;
    if (hashattn_status s = check_mlp(ctx, phi_q, ctx->cfg.n_q_heads, "encode_score_topk")) return s;
    if (hashattn_status s = check_cache(ctx, cache, batch, true, "encode_score_topk")) return s;
    if (!q || !q_codes || !idx || !count) return fail(ctx, HASHATTN_INVALID_ARG, "encode_score_topk: q, q_codes, idx or count is NULL");
    if (!aligned(q, 16) || !aligned(q_codes, 4) || !aligned(idx, 4) || !aligned(count, 4) || (k_per_seq && !aligned(k_per_seq, 4)))
        return fail(ctx, HASHATTN_INVALID_ARG, "encode_score_topk: q needs 16-byte alignment, the integer arrays 4-byte");
    if (k_max < 1) return fail(ctx, HASHATTN_INVALID_ARG, "encode_score_topk: k_max %d < 1", k_max);
    if (n_sink < 0 || n_local < 0) return fail(ctx, HASHATTN_INVALID_ARG, "encode_score_topk: n_sink %d or n_local %d is negative", n_sink, n_local);
    if ((int64_t)k_max + n_sink + n_local > ctx->cfg.max_k)
        return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "encode_score_topk: k_max + n_sink + n_local = %lld exceeds max_k %lld",
                    (long long)k_max + n_sink + n_local, (long long)ctx->cfg.max_k);
    const ha::TopkCall call{q_codes, k_per_seq, k_max, n_sink, n_local, batch, ctx->cfg.n_q_heads, cache->max_seq_len,
                            0, idx, count, threshold};
    const ha::MlpView phi = view_of(phi_q);
    const hipError_t e = ha::launch_score_topk_one_block(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group, call, &phi,
                                                         static_cast<const uint16_t*>(q), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "encode_score_topk");
}

hashattn_status hashattn_decode_step(hashattn_ctx* ctx, const hashattn_mlp* phi_kv, const void* k_new, const void* v_new,
                                     const hashattn_mlp* phi_q, const void* q, hashattn_kv* cache, int32_t batch,
                                     const int32_t* k_per_seq, int32_t k_max, int32_t n_sink, int32_t n_local, float scale,
                                     uint32_t* q_codes, int32_t* idx, int32_t* count, uint8_t* threshold, void* out,
                                     void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(ctx, HASHATTN_INVALID_ARG, "decode_step: k_new and v_new must both be given (append) or both NULL");
    bool encoded = false;
    if (k_new) {
        // the append and the query encoding share a launch when both mappings have the same fixed shape and
        // the query encoding is not going to be folded into the SCORE + TOPK launch anyway
        const bool share = phi_kv && phi_q && cache && q && q_codes && ctx->cfg.bits == ha::kBits &&
                           phi_kv->n_layers >= 1 && phi_kv->n_layers <= 4 && phi_q->n_layers >= 1 && phi_q->n_layers <= 4 &&
                           ha::encode_step_supported(view_of(phi_kv), view_of(phi_q)) &&
                           !one_launch_topk(ctx, batch, cache->max_seq_len + 1);
        if (!share) {
            if (hashattn_status s = hashattn_encode_keys(ctx, phi_kv, k_new, v_new, batch, 1, cache, stream)) return s;
        } else {
            if (hashattn_status s = check_append_state(ctx, "decode_step")) return s;
            if (hashattn_status s = check_mlp(ctx, phi_kv, ctx->cfg.n_kv_heads, "decode_step")) return s;
            if (hashattn_status s = check_mlp(ctx, phi_q, ctx->cfg.n_q_heads, "decode_step")) return s;
            if (hashattn_status s = check_cache(ctx, cache, batch, true, "decode_step")) return s;
            if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(q, 16) || !aligned(q_codes, 4))
                return fail(ctx, HASHATTN_INVALID_ARG, "decode_step: k_new, v_new and q need 16-byte, q_codes 4-byte alignment");
            const bool paged = ctx->cfg.page_size != 0;
            const int64_t room = paged ? (int64_t)cache->max_pages_per_seq * ha::kPage : cache->n_max;
            if ((int64_t)cache->max_seq_len + 1 > room)
                return fail(ctx, HASHATTN_INVALID_ARG, "decode_step: appending a token to max_seq_len %d exceeds the cache capacity %lld",
                            cache->max_seq_len, (long long)room);
            if ((int64_t)cache->max_seq_len + 1 > ctx->cfg.max_context)
                return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "decode_step: append would exceed max_context %lld", (long long)ctx->cfg.max_context);
            const ha::EncodeScratch enc{ctx->frags, ha::encode_mfma_scratch_bytes_per_head() / 16, ctx->append_done,
                                        ctx->append_fault_dev};
            const hipError_t e = ha::launch_encode_step(view_of(phi_kv), view_of(phi_q), view_of(ctx, cache), paged,
                                                        ctx->cfg.n_q_heads, static_cast<const uint16_t*>(k_new),
                                                        static_cast<const uint16_t*>(v_new), static_cast<const uint16_t*>(q), batch,
                                                        q_codes, cache->max_seq_len, enc, static_cast<hipStream_t>(stream));
            if (e != hipSuccess) return hip_fail(ctx, e, "decode_step");
            cache->max_seq_len += 1;
            encoded = true;
        }
    }
    if (encoded) {
        if (hashattn_status s = hashattn_score_topk_window(ctx, q_codes, cache, batch, k_per_seq, k_max, n_sink, n_local, idx,
                                                           count, threshold, stream))
            return s;
    } else {
        if (hashattn_status s = hashattn_encode_score_topk(ctx, phi_q, q, cache, batch, k_per_seq, k_max, n_sink, n_local,
                                                           q_codes, idx, count, threshold, stream))
            return s;
    }
    return hashattn_gather_attend(ctx, q, cache, idx, count, batch, k_max + n_sink + n_local, scale, out, stream);
}

hashattn_status hashattn_gather_attend(hashattn_ctx* ctx, const void* q, const hashattn_kv* cache, const int32_t* idx,
                                       const int32_t* count, int32_t batch, int32_t k_max, float scale, void* out,
                                       void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (hashattn_status s = check_append_state(ctx, "gather_attend")) return s;
    if (hashattn_status s = check_cache(ctx, cache, batch, false, "gather_attend")) return s;
    if (!q || !idx || !count || !out) return fail(ctx, HASHATTN_INVALID_ARG, "gather_attend: q, idx, count or out is NULL");
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(idx, 4) || !aligned(count, 4))
        return fail(ctx, HASHATTN_INVALID_ARG, "gather_attend: q/out need 16-byte, idx/count 4-byte alignment");
    if (k_max < 1) return fail(ctx, HASHATTN_INVALID_ARG, "gather_attend: k_max %d < 1", k_max);
    if (k_max > ctx->cfg.max_k) return fail(ctx, HASHATTN_SCRATCH_TOO_SMALL, "gather_attend: k_max %d exceeds max_k %lld", k_max, (long long)ctx->cfg.max_k);
    if (!(scale == scale)) return fail(ctx, HASHATTN_INVALID_ARG, "gather_attend: scale is NaN");
    int chunk, n_splits;
    // pieces of at most 512 rows; twice that measured 2 % faster with many lists of equal length (16 sequences
    // of 131072 tokens) and 3 % slower on a paged batch of mixed lengths, where it leaves too few pieces
    // to balance, so paged caches keep 512
    const int64_t lists = (int64_t)batch * ctx->cfg.n_q_heads;
    const int64_t max_rows = lists >= 256 && ctx->cfg.page_size == 0 ? 1024 : 512;
    pick_splits(ctx->part_floats, ctx->cfg.n_q_heads, lists, k_max, batch, max_rows, &chunk, &n_splits);
    const hipError_t e = ha::launch_gather_attend(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group,
                                                  static_cast<const uint16_t*>(q), idx, count, batch, ctx->cfg.n_q_heads,
                                                  k_max, chunk, n_splits, scale, ctx->part, static_cast<uint16_t*>(out),
                                                  static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "gather_attend");
}

hashattn_status hashattn_gather_attend_noalloc(int32_t n_q_heads, int32_t n_kv_heads, int32_t page_size, const void* q,
                                               const hashattn_kv* cache, const int32_t* idx, const int32_t* count,
                                               int32_t batch, int32_t k_max, float scale, void* out, void* stream)
{
    const char* what = "gather_attend_noalloc";
    if (n_kv_heads < 1 || n_kv_heads > 65535 || n_q_heads < 1 || n_q_heads % n_kv_heads)
        return fail(nullptr, HASHATTN_INVALID_ARG, "%s: n_q_heads %d must be a positive multiple of n_kv_heads %d", what, n_q_heads, n_kv_heads);
    const int group = n_q_heads / n_kv_heads;
    if (group != 1 && group != 2 && group != 4 && group != 8)
        return fail(nullptr, HASHATTN_UNSUPPORTED, "%s: group size %d not in {1,2,4,8}", what, group);
    if (page_size != 0 && page_size != ha::kPage)
        return fail(nullptr, HASHATTN_UNSUPPORTED, "%s: page_size %d, only 0 (contiguous) or 16", what, page_size);
    hashattn_config cfg{};
    cfg.n_q_heads = n_q_heads; cfg.n_kv_heads = n_kv_heads; cfg.page_size = page_size;
    cfg.max_batch = 65535; cfg.max_context = INT32_MAX;
    if (hashattn_status s = check_cache(nullptr, cfg, cache, batch, false, what)) return s;
    if (!q || !idx || !count || !out) return fail(nullptr, HASHATTN_INVALID_ARG, "%s: q, idx, count or out is NULL", what);
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(idx, 4) || !aligned(count, 4))
        return fail(nullptr, HASHATTN_INVALID_ARG, "%s: q/out need 16-byte, idx/count 4-byte alignment", what);
    if (k_max < 1) return fail(nullptr, HASHATTN_INVALID_ARG, "%s: k_max %d < 1", what, k_max);
    if (!(scale == scale)) return fail(nullptr, HASHATTN_INVALID_ARG, "%s: scale is NaN", what);
    float* part = nullptr;
    int64_t part_floats = 0;
    if (hipError_t e = ha::static_partials(&part, &part_floats); e != hipSuccess)
        return fail(nullptr, HASHATTN_HIP_ERROR, "%s: address of the static scratch array: %s", what, hipGetErrorString(e));
    // one split partial per (sequence, head) is the least the split kernels need
    const int64_t heads = (int64_t)batch * n_q_heads;
    if (heads * ha::kPartStride > part_floats)
        return fail(nullptr, HASHATTN_SCRATCH_TOO_SMALL,
                    "%s: batch %d x %d query heads = %lld (sequence, head) pairs exceeds the %lld the static scratch of %lld bytes holds",
                    what, batch, n_q_heads, (long long)heads, (long long)(part_floats / ha::kPartStride),
                    (long long)(part_floats * (int64_t)sizeof(float)));
    int chunk, n_splits;
    pick_splits(part_floats, n_q_heads, heads, k_max, batch, 512, &chunk, &n_splits);
    const hipError_t e = ha::launch_gather_attend(view_of(n_kv_heads, cache), page_size != 0, group,
                                                  static_cast<const uint16_t*>(q), idx, count, batch, n_q_heads, k_max, chunk,
                                                  n_splits, scale, part, static_cast<uint16_t*>(out),
                                                  static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : fail(nullptr, HASHATTN_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

hashattn_status hashattn_dense_attend(hashattn_ctx* ctx, const void* q, const hashattn_kv* cache, int32_t batch,
                                      float scale, void* out, void* stream)
{
    if (!ctx) return HASHATTN_INVALID_ARG;
    if (hashattn_status s = check_append_state(ctx, "dense_attend")) return s;
    if (hashattn_status s = check_cache(ctx, cache, batch, false, "dense_attend")) return s;
    if (!q || !out) return fail(ctx, HASHATTN_INVALID_ARG, "dense_attend: q or out is NULL");
    if (!aligned(q, 16) || !aligned(out, 16)) return fail(ctx, HASHATTN_INVALID_ARG, "dense_attend: q/out need 16-byte alignment");
    if (!(scale == scale)) return fail(ctx, HASHATTN_INVALID_ARG, "dense_attend: scale is NaN");
    int chunk, n_splits;
    const int64_t total = cache->max_seq_len > 0 ? cache->max_seq_len : 1;
    const int64_t lanes = (int64_t)batch * ctx->cfg.n_kv_heads;
    pick_splits(ctx->part_floats, ctx->cfg.n_q_heads, lanes, total, batch, lanes > 128 ? 4096 : 16384, &chunk, &n_splits);   // measured on C2 / C4 shapes
    const hipError_t e = ha::launch_dense_attend(view_of(ctx, cache), ctx->cfg.page_size != 0, ctx->group,
                                                 static_cast<const uint16_t*>(q), batch, ctx->cfg.n_q_heads,
                                                 cache->max_seq_len, chunk, n_splits, scale, ctx->part,
                                                 static_cast<uint16_t*>(out), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HASHATTN_OK : hip_fail(ctx, e, "dense_attend");
}

}  // extern "C"
