// Host-side launchers of the HashAttention kernels.  Each launcher assumes its
// arguments were validated by the C ABI layer and enqueues on `stream`.
#pragma once
#include "common.hpp"

namespace ha {

// Mapping network on the device side (weights are caller-owned device memory).
struct MlpView {
    int32_t n_layers;
    int32_t dims[5];
    const float* W[4];
    const float* bias[4];
};

struct TopkScratch {
    int32_t* blk_cum;      // [B][Hq][blocks_pitch][34]: per block of 8 units, #{score >= s}
    int32_t blocks_pitch;
};

hipError_t launch_encode_query(const MlpView& phi, const uint16_t* q, int batch, int n_heads,
                               uint32_t* q_codes, hipStream_t stream);

// Scratch of the key encoders: bf16 weight fragments of every KV head for the matrix-core bulk kernel
// (frags == nullptr: vector kernels only), the two-word block counter of the decode-time append
// (blocks counted so far, and that count when the current launch began) and the word of pinned host
// memory that an append launch raises when it finds the counter in a state no completed launch
// leaves behind.
struct EncodeScratch {
    uint4* frags;
    int64_t quads_per_head;        // 16-byte units per head
    uint32_t* append_done;
    int32_t* append_fault;         // device address of the host word
};

hipError_t launch_encode_keys(const MlpView& phi, const KvView& kv, bool paged,
                              const uint16_t* k_new, const uint16_t* v_new,
                              int batch, int64_t n_new, int max_seq_len, const EncodeScratch* sc,
                              hipStream_t stream);
// The decode step's append (one token per sequence: rows, key code, lengths) and its query encoding in one
// launch, for mappings of one of the fixed shapes of the vector kernels, the same for keys and queries.
bool encode_step_supported(const MlpView& phi_kv, const MlpView& phi_q);
hipError_t launch_encode_step(const MlpView& phi_kv, const MlpView& phi_q, const KvView& kv, bool paged, int n_q_heads,
                              const uint16_t* k_new, const uint16_t* v_new, const uint16_t* q, int batch,
                              uint32_t* q_codes, int max_seq_len, const EncodeScratch& sc, hipStream_t stream);

hipError_t setup_encode_bulk();
hipError_t launch_set_append_counter(uint32_t* state, uint32_t value, hipStream_t stream);

int64_t encode_mfma_scratch_bytes_per_head();
bool encode_mfma_supported(const MlpView& phi);
hipError_t setup_encode_mfma();
hipError_t launch_encode_bulk_mfma(const MlpView& phi, const KvView& kv, bool paged, int batch, int64_t span,
                                   int64_t n_new, int max_seq_len, int from_end, const EncodeScratch& sc,
                                   hipStream_t stream);

hipError_t setup_score_topk(int group);

// Arguments of one SCORE + TOPK call.  The first n_sink and the last n_local tokens of every sequence
// are always selected; k counts the tokens retrieved between them; idx rows have
// k_max + n_sink + n_local entries.
struct TopkCall {
    const uint32_t* q_codes;
    const int32_t* k_per_seq;
    int32_t k_max, n_sink, n_local;
    int32_t batch, n_q_heads, max_seq_len;
    int32_t waves_per_block;      // 8 or 16 units per block (32-bit signatures; wider ones always use 8)
    int32_t* idx;
    int32_t* count;
    uint8_t* threshold;
};

hipError_t launch_score_topk(const KvView& kv, bool paged, int group, const TopkCall& call, int unit_tokens,
                             const TopkScratch& sc, hipStream_t stream);
// SCORE + TOPK in one launch, one block per (sequence, query head), for max_seq_len up to the limit.  With a
// query mapping `phi` that one_block_can_encode accepts and the query vectors `q`, the blocks compute the
// query codes first and write them to call.q_codes; with phi = NULL they read call.q_codes.
int score_topk_one_block_limit();
bool one_block_can_encode(const MlpView& phi);
hipError_t launch_score_topk_one_block(const KvView& kv, bool paged, int group, const TopkCall& call, const MlpView* phi,
                                       const uint16_t* q, hipStream_t stream);

// Signatures of 32 * words bits (words = 2, 4, 8, 16): codes and q_codes carry a trailing axis of
// `words`, blk_cum rows have 32 * words + 2 ints, unit_tokens is at most 1024.
hipError_t setup_score_topk_wide(int group, int words);
hipError_t launch_score_topk_wide(const KvView& kv, bool paged, int group, int words, const TopkCall& call,
                                  int unit_tokens, const TopkScratch& sc, hipStream_t stream);

hipError_t launch_gather_attend(const KvView& kv, bool paged, int group, const uint16_t* q,
                                const int32_t* idx, const int32_t* count, int batch, int n_q_heads,
                                int k_max, int chunk, int n_splits, float scale, float* part,
                                uint16_t* out, hipStream_t stream);

// The library's static split-partials array on the current device (for the entry point that allocates nothing).
hipError_t static_partials(float** ptr, int64_t* n_floats);

hipError_t launch_dense_attend(const KvView& kv, bool paged, int group, const uint16_t* q,
                               int batch, int n_q_heads, int max_seq_len, int chunk, int n_splits,
                               float scale, float* part, uint16_t* out, hipStream_t stream);

}  // namespace ha
