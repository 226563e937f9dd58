// SCORE + TOPK (section 4; section 4.1, eq. 1) for gfx950.
//
// The score of a token is the Hamming similarity 32 - popcount(q_code ^ k_code),
// an integer in 0..32, so top-k is a 33-bin counting select:
//   1. score_hist   every wave streams one "unit" (a contiguous run of tokens) of
//                   one KV head's uint32 codes, scores it for the G query heads of
//                   the group and counts scores per head in LDS; the per-unit
//                   histograms go to scratch.
//   2. topk_scan    one block per (sequence, query head): totals per bin, the
//                   threshold T (largest T with #{score >= T} >= k), the tie quota
//                   r = k - #{score > T}, and per unit the output offset and the
//                   part of the quota that falls inside it (exclusive scans in
//                   unit order, so ties go to the lower token index).
//   3. topk_compact every wave re-reads its unit, recomputes the scores and writes
//                   the selected token ids at offset + rank, ranks coming from wave
//                   ballots in token order.  The result is ascending by index and
//                   does not depend on the order in which waves run.
// Scores never go to HBM; the codes are read twice (the second read mostly from
// L2 / Infinity Cache).
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kAllTies = 0x7fffffff;

template <int G, bool PAGED>
__global__ __launch_bounds__(256) void score_hist_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                         int n_q_heads, int n_cap, int unit_tokens, int units_pitch,
                                                         uint16_t* __restrict__ unit_hist)
{
    __shared__ unsigned hist[4][G * kBins];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int unit = blockIdx.x * 4 + wave;
    const int n = min(c.seq_lens[b], n_cap);   // n_cap: the host's bound that sized grid and scratch
    for (int i = lane; i < G * kBins; i += kWave) hist[wave][i] = 0u;
    __syncthreads();

    const int64_t t_begin = (int64_t)unit * unit_tokens;
    const bool active = t_begin < n;
    if (active) {
        uint32_t qc[G];
#pragma unroll
        for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform((int)q_codes[(int64_t)b * n_q_heads + kvh * G + j]);
        const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);
        for (int t0 = (int)t_begin + lane * 4; t0 < t_end; t0 += 4 * kWave) {
            const uint4 cw = *reinterpret_cast<const uint4*>(c.codes + row_of<PAGED>(c, b, kvh, t0));
            const uint32_t w[4] = {cw.x, cw.y, cw.z, cw.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (t0 + e < t_end) {
#pragma unroll
                    for (int j = 0; j < G; ++j)
                        atomicAdd(&hist[wave][j * kBins + kBits - __popc(w[e] ^ qc[j])], 1u);
                }
            }
        }
    }
    __syncthreads();
    if (active) {
        for (int i = lane; i < G * kBins; i += kWave) {
            const int j = i / kBins, s = i - j * kBins;
            const int64_t hq = (int64_t)b * n_q_heads + kvh * G + j;
            unit_hist[(hq * kBins + s) * units_pitch + unit] = (uint16_t)hist[wave][i];
        }
    }
}

// One block per (sequence, query head).  The head's [33][n_units] histogram tile is staged in LDS
// with one round of 16-byte loads; everything after that reads LDS only.
// lds_pitch: row pitch of the tile in uint16, a multiple of 8 and >= the number of units in use.
__global__ __launch_bounds__(256) void topk_scan_kernel(const int32_t* __restrict__ seq_lens,
                                                        const int32_t* __restrict__ k_per_seq, int k_max,
                                                        int n_q_heads, int n_cap, int unit_tokens, int units_pitch,
                                                        int lds_pitch, const uint16_t* __restrict__ unit_hist,
                                                        int2* __restrict__ unit_off, int2* __restrict__ sel,
                                                        int32_t* __restrict__ count, uint8_t* __restrict__ threshold)
{
    extern __shared__ uint16_t tile[];          // [kBins][lds_pitch]
    __shared__ int total[kBins];
    __shared__ int s_T, s_r;
    __shared__ int wave_gt[4], wave_eq[4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int hq = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * n_q_heads + hq;
    const int n = min(seq_lens[b], n_cap);
    int k = k_per_seq ? k_per_seq[b] : k_max;
    k = max(0, min(k, min(k_max, n)));
    if (k == 0) {                       // uniform over the block
        if (tid == 0) {
            count[bh] = 0;
            sel[bh] = make_int2(kBins, 0);
            if (threshold) threshold[bh] = 0;
        }
        return;
    }
    const int n_units = (n + unit_tokens - 1) / unit_tokens;
    const uint16_t* h = unit_hist + bh * kBins * units_pitch;
    {
        const int vec_per_row = (n_units + 7) >> 3;            // 8 counts per 16-byte load
        for (int v = tid; v < kBins * vec_per_row; v += 256) {
            const int s = v / vec_per_row, cvec = v - s * vec_per_row;
            *reinterpret_cast<uint4*>(tile + s * lds_pitch + cvec * 8) =
                *reinterpret_cast<const uint4*>(h + (int64_t)s * units_pitch + cvec * 8);
        }
    }
    __syncthreads();

    for (int s = wave; s < kBins; s += 4) {
        int acc = 0;
        for (int u = lane; u < n_units; u += kWave) acc += tile[s * lds_pitch + u];
        acc = wave_sum_i32(acc);
        if (lane == 0) total[s] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        int T = kBits, at_least = total[kBits];
        while (at_least < k && T > 0) { --T; at_least += total[T]; }
        s_T = T;
        s_r = k - (at_least - total[T]);        // taken from the tie bucket, >= 1
        count[bh] = k;
        sel[bh] = make_int2(T, 0);
        if (threshold) threshold[bh] = (uint8_t)T;
    }
    __syncthreads();
    const int T = s_T, r = s_r;

    // exclusive scan over units of (#score > T, #score == T); each thread owns a run of units
    const int per = (n_units + 255) / 256;
    const int u0 = tid * per, u1 = min(n_units, u0 + per);
    int my_gt = 0, my_eq = 0;
    for (int u = u0; u < u1; ++u) {
        for (int s = T + 1; s < kBins; ++s) my_gt += tile[s * lds_pitch + u];
        my_eq += tile[T * lds_pitch + u];
    }
    int inc_gt = my_gt, inc_eq = my_eq;         // inclusive scan inside the wave
    for (int o = 1; o < kWave; o <<= 1) {
        const int a = __shfl_up(inc_gt, o, kWave), e = __shfl_up(inc_eq, o, kWave);
        if (lane >= o) { inc_gt += a; inc_eq += e; }
    }
    if (lane == kWave - 1) { wave_gt[wave] = inc_gt; wave_eq[wave] = inc_eq; }
    __syncthreads();
    int run_gt = inc_gt - my_gt, run_eq = inc_eq - my_eq;
    for (int w = 0; w < wave; ++w) { run_gt += wave_gt[w]; run_eq += wave_eq[w]; }

    int2* off = unit_off + bh * units_pitch;
    for (int u = u0; u < u1; ++u) {
        int gt = 0;
        for (int s = T + 1; s < kBins; ++s) gt += tile[s * lds_pitch + u];
        const int eq = tile[T * lds_pitch + u];
        const int left = r - run_eq;            // quota still open when this unit starts
        const int quota = left >= eq ? kAllTies : max(left, 0);
        off[u] = make_int2(run_gt + min(run_eq, r), quota);
        run_gt += gt;
        run_eq += eq;
    }
}

template <int G, bool PAGED>
__global__ __launch_bounds__(256) void topk_compact_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                           int n_q_heads, int n_cap, int unit_tokens, int units_pitch,
                                                           const int2* __restrict__ unit_off,
                                                           const int2* __restrict__ sel, int k_max,
                                                           int32_t* __restrict__ idx)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int unit = blockIdx.x * 4 + wave;
    const int n = min(c.seq_lens[b], n_cap);
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    if (t_begin >= n) return;                   // whole wave leaves; the kernel has no barrier
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);

    uint32_t qc[G];
    int T[G], pos[G], quota[G], ties_seen[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
        qc[j] = (uint32_t)uniform((int)q_codes[bh]);
        T[j] = uniform(sel[bh].x);              // 33 when nothing is to be selected
        const int2 o = T[j] < kBins ? unit_off[bh * units_pitch + unit] : make_int2(0, 0);
        pos[j] = uniform(o.x);
        quota[j] = uniform(o.y);
        ties_seen[j] = 0;
    }

    for (int base = (int)t_begin; base < t_end; base += 4 * kWave) {
        const int t0 = base + lane * 4;
        uint4 cw = make_uint4(0u, 0u, 0u, 0u);
        if (t0 < t_end) cw = *reinterpret_cast<const uint4*>(c.codes + row_of<PAGED>(c, b, kvh, t0));
        const uint32_t w[4] = {cw.x, cw.y, cw.z, cw.w};
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
}

template <int G>
hipError_t launch_g(const KvView& kv, bool paged, const uint32_t* q_codes, int batch, int n_q_heads,
                    const int32_t* k_per_seq, int k_max, int max_seq_len, int unit_tokens,
                    const TopkScratch& sc, int32_t* idx, int32_t* count, uint8_t* threshold,
                    hipStream_t stream)
{
    const int n_units = (max_seq_len + unit_tokens - 1) / unit_tokens;
    const dim3 grid((n_units + 3) / 4, kv.n_kv_heads, batch), block(256);
    if (n_units > 0) {
        if (paged)
            score_hist_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                    sc.units_pitch, sc.unit_hist);
        else
            score_hist_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                     sc.units_pitch, sc.unit_hist);
    }
    const int lds_pitch = ((n_units > 0 ? n_units : 1) + 7) / 8 * 8;
    const size_t lds_bytes = sizeof(uint16_t) * kBins * (size_t)lds_pitch;      // <= 64 KiB: n_units <= kMaxScanUnits
    topk_scan_kernel<<<dim3(n_q_heads, batch), block, lds_bytes, stream>>>(kv.seq_lens, k_per_seq, k_max, n_q_heads,
                                                                            max_seq_len, unit_tokens, sc.units_pitch,
                                                                            lds_pitch, sc.unit_hist, sc.unit_off, sc.sel,
                                                                            count, threshold);
    if (n_units > 0) {
        if (paged)
            topk_compact_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                      sc.units_pitch, sc.unit_off, sc.sel,
                                                                      k_max, idx);
        else
            topk_compact_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                       sc.units_pitch, sc.unit_off, sc.sel,
                                                                       k_max, idx);
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
