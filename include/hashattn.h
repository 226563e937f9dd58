/*
 * hashattn.h - C ABI of the MI355X (gfx950) HashAttention decode library.
 *
 * One decode layer-step of HashAttention (arxiv 2412.14468, section 4):
 *     [append new token]  ->  encode query  ->  SCORE  ->  TOPK  ->  GATHER-ATT
 *
 * Conventions that hold for every call
 *   - "dev" pointers are DEVICE pointers owned by the caller.  The library
 *     never frees, reallocates or keeps them after the call returns.  "host"
 *     pointers are ordinary host memory.  Structs are passed by host pointer
 *     and may hold device pointers; they are read during the call only.
 *   - Work is enqueued on the caller's HIP stream (`stream`, a hipStream_t
 *     passed as void*; NULL = the default stream) and the call returns without
 *     synchronising.  Nothing is copied to the host.
 *   - A context owns only the library's scratch memory (histograms, offsets,
 *     split partials), sized at creation from the max_* fields.  Calls that
 *     use one context must not overlap in time (same stream, or ordered
 *     streams): they share that scratch.
 *   - Errors are return codes; arguments are checked on the host before any
 *     launch, so a call that returns an error has enqueued nothing.
 *     hashattn_last_error() gives a readable message for the last failure on
 *     that context (or of hashattn_create when ctx == NULL).
 *   - bf16 tensors are 16-bit brain floats; head_dim is 128; codes have 32
 *     bits unless the context is created for wider signatures (below).  Query
 *     head h uses KV head h / (n_q_heads / n_kv_heads).
 *   - Bit order of a code: output unit j of the mapping network is bit j
 *     (least significant bit = unit 0); bit = 1 iff the activation is > 0
 *     (phi(x) = relu(sign(F(x))), section 4.1, eq. 2; sign(0) gives 0).
 *   - Token t of sequence b, KV head h lives at row
 *       contiguous:  (b * n_kv_heads + h) * n_max + t
 *       paged:       (page_table[b][t / page_size] * n_kv_heads + h) * page_size + t % page_size
 *     in k, v (rows of head_dim bf16) and in codes (one uint32 per row).
 *   - Wider signatures (the paper's ablation on the number of bits; its SCORE
 *     latency table lists 64 to 512 bits): with bits = b = 32 W in the config,
 *     a code is W consecutive uint32 (codes hold W words per row, q_codes
 *     [batch][n_q_heads][W]); output unit j of the mapping is bit j % 32 of
 *     word j / 32; the score of a token is b - bitcount(xor), 0..b; the
 *     mapping networks end in b outputs (hidden layers stay within 256
 *     units); `threshold` is stored as min(T, 255); max_context is at most
 *     2 Mi tokens.  Everything else reads as for 32 bits.
 */
#ifndef HASHATTN_H
#define HASHATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hashattn_ctx hashattn_ctx;

typedef int32_t hashattn_status;
enum {
    HASHATTN_OK = 0,
    HASHATTN_INVALID_ARG = 1,       /* NULL pointer, bad size, misalignment, limit exceeded */
    HASHATTN_UNSUPPORTED = 2,       /* shape the kernels are not written for */
    HASHATTN_SCRATCH_TOO_SMALL = 3, /* call exceeds the max_* the context was created with */
    HASHATTN_HIP_ERROR = 4          /* a HIP runtime call failed */
};

/* Limits and shape of the attention layer a context serves. */
typedef struct {
    int32_t head_dim;      /* must be 128 */
    int32_t n_q_heads;     /* multiple of n_kv_heads; group size 1, 2, 4 or 8 */
    int32_t n_kv_heads;
    int32_t bits;          /* signature width b: 32, 64, 128, 256 or 512 (see "Wider signatures") */
    int32_t page_size;     /* 0 = contiguous KV cache, 16 = paged */
    int32_t max_batch;
    int64_t max_context;   /* largest sequence length any call will see */
    int64_t max_k;         /* largest k any call will ask for */
} hashattn_config;

/* Mapping network F of phi (section 4.1, eq. 2): n_layers weight matrices with
 * SiLU between them and no activation before the sign.  Layer l maps dims[l]
 * inputs to dims[l+1] outputs as y = x W (+ bias).  dims[0] = 128; a hidden
 * width is 32, 64, 128 or 256; dims[n_layers] = the context's `bits`.  One
 * network per head.  Other shapes are refused with HASHATTN_UNSUPPORTED. */
typedef struct {
    int32_t n_heads;
    int32_t n_layers;         /* 1, 2 or 3 */
    int32_t dims[5];
    const float* W[4];        /* dev fp32, [n_heads][dims[l]][dims[l+1]] row-major */
    const float* bias[4];     /* dev fp32, [n_heads][dims[l+1]], or NULL */
} hashattn_mlp;

/* KV cache with its key-code store (32 bits per token per KV head, section 4.1
 * "Implementation").  All device memory belongs to the caller. */
typedef struct {
    void* k;                  /* dev bf16: contiguous [B][H_kv][n_max][128] | paged [P][H_kv][16][128] */
    void* v;                  /* dev bf16, same layout */
    uint32_t* codes;          /* dev: contiguous [B][H_kv][n_max] | paged [P][H_kv][16] */
    const int32_t* page_table;/* dev [B][max_pages_per_seq] physical page ids; paged only, else NULL */
    int32_t* seq_lens;        /* dev [B] current length of every sequence */
    int64_t n_max;            /* contiguous: row capacity per (b, head), a multiple of 4; paged: ignored */
    int64_t n_pages;          /* paged: number of physical pages P; contiguous: ignored */
    int32_t max_pages_per_seq;/* paged only */
    int32_t max_seq_len;      /* HOST upper bound on seq_lens[*] valid for this call (sizes the grids);
                                 hashattn_encode_keys in append mode adds n_new to it.  Calls recorded
                                 into a HIP graph keep the bound they were captured with: the device
                                 lengths advance on every replay, this host field does not, so a caller
                                 that replays appends captures with a bound that covers all replays
                                 and keeps the field up to date itself */
} hashattn_kv;

/* Create / destroy a context on the current HIP device.  Allocates scratch
 * with hipMalloc (a few MB for the Llama-3.1-8B shape at 512K context). */
hashattn_status hashattn_create(hashattn_ctx** ctx, const hashattn_config* cfg);
hashattn_status hashattn_destroy(hashattn_ctx* ctx);
const char* hashattn_last_error(const hashattn_ctx* ctx);
/* Bytes of device scratch the context holds. */
int64_t hashattn_scratch_bytes(const hashattn_ctx* ctx);
/* For tests of the consistency check described at hashattn_encode_keys: leaves
 * the append kernel's block counter, on `stream`, as a launch that stopped
 * after `value` of its blocks would (>= 0; 0 is the normal state).  Not needed
 * by any caller of the path. */
hashattn_status hashattn_selftest_set_append_counter(hashattn_ctx* ctx, int32_t value, void* stream);
/* For tests: SCORE + TOPK has a one-launch form for short contexts and few
 * (sequence, head) pairs and a two-launch form for everything else, with
 * identical results.  path 0 (the default) lets every call choose, 1 always
 * takes two launches, 2 takes one launch whenever the context length allows
 * it (at most 32768 tokens, 32-bit signatures).  Host state only. */
hashattn_status hashattn_selftest_set_topk_path(hashattn_ctx* ctx, int32_t path);

/* Key signatures phi_int,kv(k), computed when a token enters the KV cache and
 * stored beside it (section 4.1, "Implementation" paragraph; phi_kv reads the
 * key vector only).
 *   append mode (k_new, v_new != NULL): k_new, v_new are dev bf16
 *     [batch][H_kv][n_new][128].  For every sequence b the n_new rows are
 *     written at positions seq_lens[b] .. seq_lens[b]+n_new-1 of the cache
 *     together with their codes, then seq_lens[b] += n_new (on the device) and
 *     cache->max_seq_len += n_new (on the host).  Needs max_seq_len + n_new <=
 *     n_max (contiguous) or <= max_pages_per_seq * 16 (paged; the page table
 *     must already map the new positions).
 *   in-place mode (k_new == NULL, v_new == NULL): the rows are already in the
 *     cache; the codes of the last min(n_new, seq_lens[b]) tokens of every
 *     sequence are recomputed from the cached keys.  seq_lens is unchanged.
 *     n_new = max_seq_len rebuilds the whole store (prefill).
 * The decode-time append (few rows) moves the lengths from inside its one
 * kernel, through a block counter in the context's scratch that every launch
 * must find complete.  A launch that finds it otherwise (an earlier append
 * on this context did not run to its end) reports it: from then on every call
 * on the context returns HASHATTN_HIP_ERROR and hashattn_last_error() says why. */
hashattn_status hashattn_encode_keys(hashattn_ctx* ctx, const hashattn_mlp* phi_kv,
                                     const void* k_new, const void* v_new,
                                     int32_t batch, int64_t n_new,
                                     hashattn_kv* cache, void* stream);

/* Query signatures phi_int,q(q) (section 4.1, eq. 2), one network per query head.
 *   q        dev bf16 [batch][n_q_heads][128]
 *   q_codes  dev uint32 [batch][n_q_heads] (output) */
hashattn_status hashattn_encode_query(hashattn_ctx* ctx, const hashattn_mlp* phi_q,
                                      const void* q, int32_t batch,
                                      uint32_t* q_codes, void* stream);

/* SCORE + TOPK (section 4; section 4.1, eq. 1).  The score of token i for
 * query head h is the Hamming similarity 32 - bitcount(q_code XOR k_code_i),
 * which orders tokens exactly as -Hamming distance does.  For every (b, h) the
 * k_eff = min(k_b, seq_lens[b]) best tokens are selected; among equal scores
 * the lower token index wins.
 *   q_codes    dev uint32 [batch][n_q_heads]
 *   k_per_seq  dev int32 [batch], or NULL for k_max everywhere
 *   k_max      host upper bound on every k_b (>= 1, <= max_k); row pitch of idx
 *   idx        dev int32 [batch][n_q_heads][k_max] (output): logical token ids,
 *              ascending; slots >= count are left untouched
 *   count      dev int32 [batch][n_q_heads] (output): k_eff (0 for an empty sequence)
 *   threshold  dev uint8 [batch][n_q_heads] (output) or NULL: smallest selected score */
hashattn_status hashattn_score_topk(hashattn_ctx* ctx, const uint32_t* q_codes,
                                    const hashattn_kv* cache, int32_t batch,
                                    const int32_t* k_per_seq, int32_t k_max,
                                    int32_t* idx, int32_t* count, uint8_t* threshold,
                                    void* stream);

/* SCORE + TOPK with always-kept tokens (section 5, "Baselines and setup": the
 * first and the most recent tokens are always in context and the token budget
 * counts only the tokens retrieved besides them).  With lo = min(n_sink, N) and
 * hi = max(lo, N - n_local), N = seq_lens[b], the index set of (b, h) is
 *   {0 .. lo-1}  u  the min(k_b, hi - lo) best tokens of [lo, hi)  u  {hi .. N-1},
 * ascending; the always-kept tokens are not scored.  n_sink = n_local = 0 is
 * hashattn_score_topk.  Arguments as there, except:
 *   n_sink, n_local  host, >= 0; k_max + n_sink + n_local <= max_k
 *   idx        dev int32 [batch][n_q_heads][k_max + n_sink + n_local]
 *   count      lo + min(k_b, hi - lo) + (N - hi)
 *   threshold  smallest retrieved score (0 when nothing is retrieved)
 * Pass k_max + n_sink + n_local as k_max to hashattn_gather_attend. */
hashattn_status hashattn_score_topk_window(hashattn_ctx* ctx, const uint32_t* q_codes,
                                           const hashattn_kv* cache, int32_t batch,
                                           const int32_t* k_per_seq, int32_t k_max,
                                           int32_t n_sink, int32_t n_local,
                                           int32_t* idx, int32_t* count, uint8_t* threshold,
                                           void* stream);

/* ENCODE-Q, SCORE and TOPK in one call (section 4: eq. 2 for the query, eq. 1
 * for the scores, the standard top-k over them): q_codes[b][h] is the code of
 * q[b][h] under phi_q as hashattn_encode_query computes it, and idx, count
 * and threshold are what hashattn_score_topk_window gives for those codes.
 * With at most 512 (sequence, query head) pairs, max_seq_len <= 32768, 32-bit
 * signatures and a mapping of 2 or 3 layers of width 128 this is one kernel
 * launch instead of three, which is most of the time of a decode step at
 * batch 1 and a short context; any other shape runs the two calls one after
 * the other.  In the one-launch form the partial sums of a layer are added in
 * another order than in hashattn_encode_query, so a bit of q_codes whose
 * activation is within float rounding of zero can differ between the two.
 *   q        dev bf16 [batch][n_q_heads][128] (input)
 *   q_codes  dev uint32 [batch][n_q_heads] (output)
 * Everything else as in hashattn_score_topk_window. */
hashattn_status hashattn_encode_score_topk(hashattn_ctx* ctx, const hashattn_mlp* phi_q, const void* q,
                                           const hashattn_kv* cache, int32_t batch,
                                           const int32_t* k_per_seq, int32_t k_max,
                                           int32_t n_sink, int32_t n_local, uint32_t* q_codes,
                                           int32_t* idx, int32_t* count, uint8_t* threshold,
                                           void* stream);

/* One decode step of a layer in one call (section 4; section 4.1): [the new
 * token enters the cache as in hashattn_encode_keys with n_new = 1,] the query
 * is encoded, scored against every cached key (the new one included), the
 * top-k tokens are selected as in hashattn_score_topk_window, and GATHER-ATT
 * runs over them.  The results are those of the separate calls in that order;
 * the call exists so that the library can share launches between the steps
 * (append and query encoding in one launch when both mappings have one of the
 * shapes 128 -> 32, 128 -> 128 -> 32, 128 -> 128 -> 128 -> 32; query encoding,
 * SCORE and TOPK in one launch for short contexts, see
 * hashattn_encode_score_topk).
 *   k_new, v_new  dev bf16 [batch][H_kv][128], or both NULL: nothing is appended
 *                 and phi_kv is not read
 *   cache         as in hashattn_encode_keys: seq_lens and max_seq_len advance
 *                 by one when a token is appended
 *   scale         softmax scale, 1 / sqrt(128) for section 3.1's attention
 *   q_codes, idx, count, threshold   outputs as in hashattn_encode_score_topk
 *   out           dev bf16 [batch][n_q_heads][128]
 * Errors as in the separate calls; a step that fails after the append has been
 * launched leaves the token appended. */
hashattn_status hashattn_decode_step(hashattn_ctx* ctx, const hashattn_mlp* phi_kv, const void* k_new,
                                     const void* v_new, const hashattn_mlp* phi_q, const void* q,
                                     hashattn_kv* cache, int32_t batch, const int32_t* k_per_seq,
                                     int32_t k_max, int32_t n_sink, int32_t n_local, float scale,
                                     uint32_t* q_codes, int32_t* idx, int32_t* count, uint8_t* threshold,
                                     void* out, void* stream);

/* GATHER-ATT (section 4): softmax attention over the selected tokens only,
 *   out[b][h] = sum_{i in I} softmax_i(scale * <q, k_i>) v_i,
 * normalised over the selected tokens, fp32 accumulation, bf16 result.
 *   q      dev bf16 [batch][n_q_heads][128]
 *   idx    dev int32 [batch][n_q_heads][k_max]: logical token ids, unique and
 *          < seq_lens[b] (not checked on the device)
 *   count  dev int32 [batch][n_q_heads]: entries of idx in use (<= k_max);
 *          0 gives a zero output row
 *   scale  softmax scale, 1/sqrt(128) for SDPA (section 3.1)
 *   out    dev bf16 [batch][n_q_heads][128] (output) */
hashattn_status hashattn_gather_attend(hashattn_ctx* ctx, const void* q,
                                       const hashattn_kv* cache, const int32_t* idx,
                                       const int32_t* count, int32_t batch, int32_t k_max,
                                       float scale, void* out, void* stream);

/* hashattn_gather_attend for callers that cannot allocate device memory or hold
 * a context: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same computation, arguments and kernels as
 * hashattn_gather_attend, with the layer shape passed directly (n_q_heads a
 * multiple of n_kv_heads with group size 1, 2, 4 or 8; page_size 0 or 16;
 * head_dim 128).  The split partials go to a static device array of 8 MiB that
 * the library holds on every GPU it runs on until the process ends; the call
 * allocates and frees nothing (its first call on a device looks up that
 * array's address).  Limit: batch * n_q_heads <= 15887 (one partial of 528
 * bytes per (sequence, head) at least); beyond it the call returns
 * HASHATTN_SCRATCH_TOO_SMALL and enqueues nothing.  All calls on one GPU share
 * the array: calls that may overlap in time (different streams) race; calls on
 * one stream, or ordered streams, are safe.  Nothing in the array has to be
 * cleared between calls (every partial that is read was written by the same
 * call).  Errors are read with hashattn_last_error(NULL) on the calling thread. */
hashattn_status hashattn_gather_attend_noalloc(int32_t n_q_heads, int32_t n_kv_heads, int32_t page_size,
                                               const void* q, const hashattn_kv* cache,
                                               const int32_t* idx, const int32_t* count,
                                               int32_t batch, int32_t k_max, float scale,
                                               void* out, void* stream);

/* Dense single-query SDPA over all seq_lens[b] tokens (section 3.1), GQA-aware
 * (K/V rows are read once per KV head).  The in-house dense decode kernel the
 * sparse path is compared against; same q/out layout as hashattn_gather_attend. */
hashattn_status hashattn_dense_attend(hashattn_ctx* ctx, const void* q,
                                      const hashattn_kv* cache, int32_t batch,
                                      float scale, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HASHATTN_H */
