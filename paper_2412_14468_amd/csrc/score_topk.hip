// SCORE + TOPK (section 4; section 4.1, eq. 1) for gfx950.
//
// The score of a token is the Hamming similarity 32 - popcount(q_code ^ k_code),
// an integer in 0..32, so top-k is a 33-bin counting select in two launches:
//   1. score_hist   every wave streams one "unit" (a contiguous run of tokens) of
//                   one KV head's uint32 codes, scores it for the G query heads of
//                   the group and counts scores per head in LDS.  Per unit it stores
//                   the cumulative counts C_u(s) = #{score >= s}; per block it adds
//                   its counts to the head's global histogram (integer atomics).
//   2. topk_select  every block first derives, per head, the threshold T (largest T
//                   with #{score >= T} >= k) from the global histogram, the tie quota
//                   r = k - #{score > T}, and the number of selected tokens in the
//                   units before its own (sums over two rows of the per-unit table, in
//                   unit order, so ties go to the lower token index).  Each wave then
//                   re-reads its unit, recomputes the scores and writes the selected
//                   token ids at offset + rank, ranks coming from wave ballots in token
//                   order.  The result is ascending by index and does not depend on
//                   the order in which waves run.
// The global histogram must be zero when a call starts: the block of topk_select that
// takes the last ticket (all blocks have read the histogram by then) clears it again.
// Scores never go to HBM; the codes are read twice (the second read mostly from
// L2 / Infinity Cache).  All loads of a unit are issued before the first is used.
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kAllTies = 0x7fffffff;
constexpr int kCopies = 4;            // LDS histogram copies per wave (by lane & 3): fewer same-address adds
constexpr int kChunk = 4 * 4 * kWave; // tokens a wave loads at once: four 16-byte loads per lane

template <bool PAGED>
__device__ __forceinline__ void load_chunk(const KvView& c, int b, int kvh, int base, int t_end, int lane,
                                           uint4 (&cw)[4])
{
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int t0 = base + it * 4 * kWave + lane * 4;
        cw[it] = make_uint4(0u, 0u, 0u, 0u);
        if (t0 < t_end) cw[it] = *reinterpret_cast<const uint4*>(c.codes + row_of<PAGED>(c, b, kvh, t0));
    }
}

template <int G, bool PAGED>
__global__ __launch_bounds__(256) void score_hist_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                         int n_q_heads, int n_cap, int unit_tokens, int units_pitch,
                                                         uint16_t* __restrict__ unit_cum, int32_t* __restrict__ ghist)
{
    __shared__ unsigned hist[4][kCopies][G * kBins];
    __shared__ unsigned wsum[4][G * kBins];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int unit = blockIdx.x * 4 + wave;
    const int n = min(c.seq_lens[b], n_cap);   // n_cap: the host's bound that sized grid and scratch
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    const bool active = t_begin < n;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);

    uint4 cw[4];
    if (active) load_chunk<PAGED>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    uint32_t qc[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform((int)q_codes[(int64_t)b * n_q_heads + kvh * G + j]);
    for (int i = lane; i < kCopies * G * kBins; i += kWave) (&hist[wave][0][0])[i] = 0u;
    __syncthreads();

    if (active) {
        unsigned* mine = hist[wave][lane & (kCopies - 1)];
        for (int base = (int)t_begin; base < t_end; base += kChunk) {
            uint4 nx[4];
            const bool more = base + kChunk < t_end;
            if (more) load_chunk<PAGED>(c, b, kvh, base + kChunk, t_end, lane, nx);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int t0 = base + it * 4 * kWave + lane * 4;
                const uint32_t w[4] = {cw[it].x, cw[it].y, cw[it].z, cw[it].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (t0 + e < t_end) {
#pragma unroll
                        for (int j = 0; j < G; ++j)
                            atomicAdd(&mine[j * kBins + kBits - __popc(w[e] ^ qc[j])], 1u);
                    }
                }
            }
            if (more) {
#pragma unroll
                for (int it = 0; it < 4; ++it) cw[it] = nx[it];
            }
        }
    }
    __syncthreads();

    // per unit: cumulative counts C_u(s) = #{score >= s}; lanes 0..32 hold the bins of one head
#pragma unroll
    for (int j = 0; j < G; ++j) {
        int h = 0;
        if (lane < kBins) {
#pragma unroll
            for (int cp = 0; cp < kCopies; ++cp) h += (int)hist[wave][cp][j * kBins + lane];
            wsum[wave][j * kBins + lane] = (unsigned)h;
        }
        const int incl = wave_incl_scan_i32(h);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (active && lane < kBins) {
            const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
            unit_cum[(bh * kBins + lane) * units_pitch + unit] = (uint16_t)(total - incl + h);
        }
    }
    __syncthreads();
    // per block: add the counts of its four units to the head's global histogram
    for (int i = tid; i < G * kBins; i += 256) {
        const int v = (int)(wsum[0][i] + wsum[1][i] + wsum[2][i] + wsum[3][i]);
        if (v) {
            const int j = i / kBins, s = i - j * kBins;
            atomicAdd(&ghist[((int64_t)b * n_q_heads + kvh * G + j) * kBins + s], v);
        }
    }
}

// Per-head selection parameters shared by the four waves of a block.
struct HeadSel {
    int T;            // threshold; kBins when nothing is selected
    int r;            // tokens taken from the tie bucket (score == T)
    int gt_before;    // #{score > T} in the units before the block's first unit
    int ge_before;    // #{score >= T} in the units before the block's first unit
    int gt_unit[4];   // the same two counts for the block's own four units
    int ge_unit[4];
};

template <int G, bool PAGED>
__global__ __launch_bounds__(256) void topk_select_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                          const int32_t* __restrict__ k_per_seq, int k_max,
                                                          int n_q_heads, int n_cap, int unit_tokens, int units_pitch,
                                                          const uint16_t* __restrict__ unit_cum,
                                                          int32_t* __restrict__ ghist, int32_t* __restrict__ tickets,
                                                          int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                          uint8_t* __restrict__ threshold)
{
    __shared__ HeadSel sel[G];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int unit0 = blockIdx.x * 4, unit = unit0 + wave;
    const int n = min(c.seq_lens[b], n_cap);
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    const bool active = t_begin < n;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);
    int k = k_per_seq ? k_per_seq[b] : k_max;
    k = max(0, min(k, min(k_max, n)));

    uint4 cw[4];
    if (active) load_chunk<PAGED>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    uint32_t qc[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform((int)q_codes[(int64_t)b * n_q_heads + kvh * G + j]);

    // ---- selection parameters: wave w works them out for heads w, w + 4, ...
    for (int j = wave; j < G; j += 4) {
        const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
        const int g = lane < kBins ? ghist[bh * kBins + lane] : 0;
        const int incl = wave_incl_scan_i32(g);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        const int cum = total - incl + g;                 // #{score >= lane}; 0 for lanes >= 33
        int T = kBins, r = 0;
        if (k > 0) {
            const uint64_t ge_k = __ballot(lane < kBins && cum >= k);   // lane 0 is set: cum(0) = n >= k
            T = 63 - __clzll((long long)(ge_k | 1ull));
            r = k - __shfl(cum, T + 1, kWave);            // cum(33) = 0
        }
        // selected-token counts of the units before this block, and of its own four units
        int gt = 0, ge = 0, gtu = 0, geu = 0;
        if (k > 0) {
            const uint16_t* row_ge = unit_cum + (bh * kBins + T) * units_pitch;
            const uint16_t* row_gt = row_ge + units_pitch;               // row T + 1 (not stored for T = 32)
            for (int u = lane; u < unit0; u += kWave) {
                ge += row_ge[u];
                if (T < kBits) gt += row_gt[u];
            }
            const int n_units = (n + unit_tokens - 1) / unit_tokens;
            if (lane < 4 && unit0 + lane < n_units) {
                geu = row_ge[unit0 + lane];
                if (T < kBits) gtu = row_gt[unit0 + lane];
            }
        }
        gt = wave_sum_i32(gt);
        ge = wave_sum_i32(ge);
        if (lane < 4) { sel[j].gt_unit[lane] = gtu; sel[j].ge_unit[lane] = geu; }
        if (lane == 0) {
            sel[j].T = T;
            sel[j].r = r;
            sel[j].gt_before = gt;
            sel[j].ge_before = ge;
            if (blockIdx.x == 0) {
                count[bh] = k;
                if (threshold) threshold[bh] = (uint8_t)(k > 0 ? T : 0);
            }
        }
    }
    __syncthreads();

    // ---- compaction of this wave's unit
    if (active && k > 0) {
        int T[G], pos[G], quota[G], ties_seen[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            int gt = sel[j].gt_before, ge = sel[j].ge_before;
            for (int w = 0; w < wave; ++w) { gt += sel[j].gt_unit[w]; ge += sel[j].ge_unit[w]; }
            const int eq_before = ge - gt, eq_unit = sel[j].ge_unit[wave] - sel[j].gt_unit[wave];
            const int r = sel[j].r;
            const int left = r - eq_before;           // quota still open when this unit starts
            T[j] = uniform(sel[j].T);
            pos[j] = uniform(gt + min(eq_before, r));
            quota[j] = uniform(left >= eq_unit ? kAllTies : max(left, 0));
            ties_seen[j] = 0;
        }
        for (int base = (int)t_begin; base < t_end; base += kChunk) {
            uint4 nx[4];
            const bool more = base + kChunk < t_end;
            if (more) load_chunk<PAGED>(c, b, kvh, base + kChunk, t_end, lane, nx);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int t0 = base + it * 4 * kWave + lane * 4;
                if (base + it * 4 * kWave >= t_end) break;             // uniform over the wave
                const uint32_t w[4] = {cw[it].x, cw[it].y, cw[it].z, cw[it].w};
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    int s[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[e] = (t0 + e < t_end) ? kBits - __popc(w[e] ^ qc[j]) : -1;
                    bool take[4];
                    if (quota[j] == kAllTies) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) take[e] = s[e] >= T[j];
                    } else if (quota[j] == 0) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) take[e] = s[e] > T[j];
                    } else {
                        // the unit where the tie quota runs out: rank the ties in token order
                        int before = ties_seen[j], all = 0;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint64_t m = __ballot(s[e] == T[j]);
                            before += lanes_below(m);
                            all += __popcll(m);
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bool tie = s[e] == T[j];
                            take[e] = s[e] > T[j] || (tie && before < quota[j]);
                            before += tie ? 1 : 0;
                        }
                        ties_seen[j] += all;
                    }
                    int rank = pos[j], all = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint64_t m = __ballot(take[e]);
                        rank += lanes_below(m);
                        all += __popcll(m);
                    }
                    int32_t* out = idx + ((int64_t)b * n_q_heads + kvh * G + j) * k_max;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (take[e]) {
                            if (rank < k_max) out[rank] = t0 + e;
                            ++rank;
                        }
                    }
                    pos[j] += all;
                }
            }
            if (more) {
#pragma unroll
                for (int it = 0; it < 4; ++it) cw[it] = nx[it];
            }
        }
    }

    // ---- the block that takes the last ticket clears the group's global histograms for the next call
    // (every block read them before the barrier above, so nobody needs them any more)
    if (wave == 0) {
        int t = 0;
        if (lane == 0) t = atomicAdd(&tickets[(int64_t)b * gridDim.y + kvh], 1);
        t = uniform(t);
        if (t == (int)gridDim.x - 1) {
            for (int i = lane; i < G * kBins; i += kWave)
                ghist[((int64_t)b * n_q_heads + kvh * G) * kBins + i] = 0;
            if (lane == 0) tickets[(int64_t)b * gridDim.y + kvh] = 0;
        }
    }
}

template <int G>
hipError_t launch_g(const KvView& kv, bool paged, const uint32_t* q_codes, int batch, int n_q_heads,
                    const int32_t* k_per_seq, int k_max, int max_seq_len, int unit_tokens,
                    const TopkScratch& sc, int32_t* idx, int32_t* count, uint8_t* threshold,
                    hipStream_t stream)
{
    int n_units = (max_seq_len + unit_tokens - 1) / unit_tokens;
    if (n_units < 1) n_units = 1;                 // one block per group still reports count = 0
    const dim3 grid((n_units + 3) / 4, kv.n_kv_heads, batch), block(256);
    if (paged) {
        score_hist_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                sc.units_pitch, sc.unit_cum, sc.ghist);
        topk_select_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, k_per_seq, k_max, n_q_heads, max_seq_len,
                                                                 unit_tokens, sc.units_pitch, sc.unit_cum, sc.ghist,
                                                                 sc.tickets, idx, count, threshold);
    } else {
        score_hist_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                 sc.units_pitch, sc.unit_cum, sc.ghist);
        topk_select_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, k_per_seq, k_max, n_q_heads, max_seq_len,
                                                                  unit_tokens, sc.units_pitch, sc.unit_cum, sc.ghist,
                                                                  sc.tickets, idx, count, threshold);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_score_topk(const KvView& kv, bool paged, int group, const uint32_t* q_codes,
                             int batch, int n_q_heads, const int32_t* k_per_seq, int k_max,
                             int max_seq_len, int unit_tokens, const TopkScratch& sc,
                             int32_t* idx, int32_t* count, uint8_t* threshold, hipStream_t stream)
{
    switch (group) {
    case 1: return launch_g<1>(kv, paged, q_codes, batch, n_q_heads, k_per_seq, k_max, max_seq_len,
                               unit_tokens, sc, idx, count, threshold, stream);
    case 2: return launch_g<2>(kv, paged, q_codes, batch, n_q_heads, k_per_seq, k_max, max_seq_len,
                               unit_tokens, sc, idx, count, threshold, stream);
    case 4: return launch_g<4>(kv, paged, q_codes, batch, n_q_heads, k_per_seq, k_max, max_seq_len,
                               unit_tokens, sc, idx, count, threshold, stream);
    case 8: return launch_g<8>(kv, paged, q_codes, batch, n_q_heads, k_per_seq, k_max, max_seq_len,
                               unit_tokens, sc, idx, count, threshold, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ha
