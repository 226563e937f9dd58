// SCORE + TOPK (section 4; section 4.1, eq. 1) for gfx950.
//
// The score of a token is the Hamming similarity 32 - popcount(q_code ^ k_code),
// an integer in 0..32, so top-k is a 33-bin counting select in two launches.
// A sequence is cut into "units" (contiguous runs of tokens, one per wave); a block
// of 16 waves owns 16 consecutive units of one KV head and serves the G query heads
// of its group from one read of the codes.
//   1. score_hist   every wave scores its unit for the G heads and counts scores per
//                   head in LDS; the cumulative counts C(s) = #{score >= s} are stored
//                   per unit and per block (one coalesced row per head each).
//   2. topk_select  every block sums the per-block rows of its heads to get the
//                   threshold T (largest T with #{score >= T} >= k) and the tie quota
//                   r = k - #{score > T}; rows T and T + 1 of the blocks before it and of
//                   its own units give every wave its first output slot and its share of
//                   the quota (block and unit order = token order, so ties go to the lower
//                   token index).  Each wave then re-scores its unit into per-lane bit
//                   masks and writes the selected token ids at offset + rank, ranks
//                   coming from packed wave prefix sums in token order.  The result is
//                   ascending by index and does not depend on the order in which waves
//                   or blocks run.
// Scores never go to HBM; the codes are read twice (the second read mostly from
// L2 / Infinity Cache).  All loads of a unit are issued before the first is used.
// Nothing persists between calls.
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kAllTies = 0x7fffffff;
constexpr int kCopies = 4;            // LDS histogram copies per wave (by lane & 3): fewer same-address adds
constexpr int kChunk = 4 * 4 * kWave; // tokens a wave loads at once: four 16-byte loads per lane
constexpr int kWpb = kTopkWavesPerBlock;
constexpr int kThreads = kWpb * kWave;

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

// Tables written by score_hist and read by topk_select; a row holds #{score >= s} for s = 0..32 and
// a zero in slot 33, so that "row[T + 1]" is valid for T = 32:
//   blk_cum:  [B][Hq][blocks_pitch][34] ints, one row per block of 16 units
//   unit_cum: [B][Hq][blocks_pitch * 16][34] uint16, one row per unit
template <int G, bool PAGED>
__global__ __launch_bounds__(kThreads) void score_hist_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                              int n_q_heads, int n_cap, int unit_tokens,
                                                              int blocks_pitch, int32_t* __restrict__ blk_cum,
                                                              uint16_t* __restrict__ unit_cum)
{
    __shared__ unsigned hist[kWpb][kCopies][G * kBins];
    __shared__ int bsum[G * kBins];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);      // block index inside the sequence
    const int unit = bx * kWpb + wave;
    const int n = min(c.seq_lens[b], n_cap);   // n_cap: the host's bound that sized grid and scratch
    if ((int64_t)bx * kWpb * unit_tokens >= n) return;      // whole block beyond the sequence
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    const bool active = t_begin < n;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);

    uint4 cw[4];
    if (active) load_chunk<PAGED>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    uint32_t qc[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform((int)q_codes[(int64_t)b * n_q_heads + kvh * G + j]);
    for (int i = lane; i < kCopies * G * kBins; i += kWave) (&hist[wave][0][0])[i] = 0u;
    for (int i = tid; i < G * kBins; i += kThreads) bsum[i] = 0;
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
    // per unit: cumulative counts per head by a wave scan (lanes 0..32 hold the bins, lane 33 the zero slot)
#pragma unroll
    for (int j = 0; j < G; ++j) {
        int h = 0;
        if (lane < kBins) {
#pragma unroll
            for (int cp = 0; cp < kCopies; ++cp) h += (int)hist[wave][cp][j * kBins + lane];
            if (h) atomicAdd(&bsum[j * kBins + lane], h);
        }
        const int incl = wave_incl_scan_i32(h);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (active && lane < kCumRow) {
            const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
            unit_cum[(bh * blocks_pitch * kWpb + unit) * kCumRow + lane] = (uint16_t)(total - incl + h);
        }
    }
    __syncthreads();
    // per block: the same from the block's summed counts
    for (int j = wave; j < G; j += kWpb) {
        const int h = lane < kBins ? bsum[j * kBins + lane] : 0;
        const int incl = wave_incl_scan_i32(h);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (lane < kCumRow) {
            const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
            blk_cum[(bh * blocks_pitch + bx) * kCumRow + lane] = total - incl + h;
        }
    }
}

// Mask of one lane's tokens of a chunk (bit it * 4 + e, it < NIT) whose Hamming distance to qc is <= lim.
template <int NIT>
__device__ __forceinline__ unsigned near_mask(const uint4 (&cw)[4], uint32_t qc, int lim)
{
    unsigned m = 0;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const uint32_t w[4] = {cw[it].x, cw[it].y, cw[it].z, cw[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) m |= (unsigned)((int)__popc(w[e] ^ qc) <= lim) << (it * 4 + e);
    }
    return m;
}

template <int NIT>
__device__ __forceinline__ unsigned equal_mask(const uint4 (&cw)[4], uint32_t qc, int dist)
{
    unsigned m = 0;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const uint32_t w[4] = {cw[it].x, cw[it].y, cw[it].z, cw[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) m |= (unsigned)((int)__popc(w[e] ^ qc) == dist) << (it * 4 + e);
    }
    return m;
}

// Lane-exclusive prefix counts of the 4-bit groups of m (NIT of them) over the wave, and the wave totals.
// Two 16-bit fields per register, so one scan serves two groups (a group holds at most 256).
template <int NIT>
__device__ __forceinline__ void group_ranks(unsigned m, int (&excl)[4], int (&total)[4])
{
    const int c0 = __popc(m & 0xfu), c1 = __popc(m & 0xf0u);
    const int i01 = wave_incl_scan_i32(c0 | (c1 << 16));
    const int t01 = __builtin_amdgcn_readlane(i01, 63);
    excl[0] = (i01 & 0xffff) - c0;
    excl[1] = (int)((unsigned)i01 >> 16) - c1;
    total[0] = t01 & 0xffff;
    total[1] = (int)((unsigned)t01 >> 16);
    excl[2] = excl[3] = total[2] = total[3] = 0;
    if constexpr (NIT > 2) {
        const int c2 = __popc(m & 0xf00u), c3 = __popc(m & 0xf000u);
        const int i23 = wave_incl_scan_i32(c2 | (c3 << 16));
        const int t23 = __builtin_amdgcn_readlane(i23, 63);
        excl[2] = (i23 & 0xffff) - c2;
        excl[3] = (int)((unsigned)i23 >> 16) - c3;
        total[2] = t23 & 0xffff;
        total[3] = (int)((unsigned)t23 >> 16);
    }
}

// Compaction of one chunk (NIT groups of 256 tokens starting at `base`) of one wave for its G heads.
template <int G, int NIT>
__device__ __forceinline__ void compact_chunk(const uint4 (&cw)[4], int base, int t_end, int lane,
                                              const uint32_t (&qc)[G], const int (&lim)[G], const int (&quota)[G],
                                              int (&pos)[G], int (&ties_seen)[G], int32_t* __restrict__ idx0,
                                              int k_max)
{
    unsigned valid = 0xffffu;                             // tokens of this lane that exist
    if (base + NIT * 4 * kWave > t_end) {                 // ragged last chunk (uniform over the wave)
        valid = 0;
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                valid |= (unsigned)(base + it * 4 * kWave + lane * 4 + e < t_end) << (it * 4 + e);
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        unsigned m = near_mask<NIT>(cw, qc[j], lim[j]) & valid;
        if (quota[j] != kAllTies && quota[j] != 0) {
            // the unit where the tie quota runs out: ties are ranked in token order
            const unsigned ties = equal_mask<NIT>(cw, qc[j], lim[j] + 1) & valid;
            int ex[4], tt[4];
            group_ranks<NIT>(ties, ex, tt);
            int before_group = ties_seen[j];
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                int rank = before_group + ex[it];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned bit = 1u << (it * 4 + e);
                    if (ties & bit) {
                        if (rank < quota[j]) m |= bit;
                        ++rank;
                    }
                }
                before_group += tt[it];
            }
            ties_seen[j] = before_group;
        }
        int ex[4], tt[4];
        group_ranks<NIT>(m, ex, tt);
        int32_t* out = idx0 + (int64_t)j * k_max;
        int group_start = pos[j];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            int rank = group_start + ex[it];
            const int t0 = base + it * 4 * kWave + lane * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (m & (1u << (it * 4 + e))) {
                    if (rank < k_max) out[rank] = t0 + e;
                    ++rank;
                }
            }
            group_start += tt[it];
        }
        pos[j] = group_start;
    }
}

template <int G, bool PAGED>
__global__ __launch_bounds__(kThreads) void topk_select_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                               const int32_t* __restrict__ k_per_seq, int k_max,
                                                               int n_q_heads, int n_cap, int unit_tokens,
                                                               int blocks_pitch, const int32_t* __restrict__ blk_cum,
                                                               const uint16_t* __restrict__ unit_cum,
                                                               int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                               uint8_t* __restrict__ threshold)
{
    constexpr int kRowsPerPass = kThreads / kCumRow;           // 30 table rows are read side by side
    __shared__ int tot[G * kCumRow];
    __shared__ int2 upos[kWpb][G];                             // per wave and head: {first output slot, tie quota}
    __shared__ int thr[G];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);      // block index inside the sequence
    const int unit0 = bx * kWpb, unit = unit0 + wave;
    const int64_t bh0 = (int64_t)b * n_q_heads + kvh * G;
    const int nb_cap = gridDim.x;                              // blocks the host launched per sequence

    // ---- everything that does not depend on another load is requested first
    const int n_raw = c.seq_lens[b];
    const int k_raw = k_per_seq ? k_per_seq[b] : k_max;
    const int srow = tid / kCumRow, scol = tid - srow * kCumRow;
    int tv[G][2];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int blk = srow + u * kRowsPerPass;
            tv[j][u] = 0;
            if (srow < kRowsPerPass && blk < nb_cap)
                tv[j][u] = blk_cum[((bh0 + j) * blocks_pitch + blk) * kCumRow + scol];
        }
    uint32_t qc[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform((int)q_codes[bh0 + j]);
    for (int i = tid; i < G * kCumRow; i += kThreads) tot[i] = 0;

    const int n = min(n_raw, n_cap);
    const int k = max(0, min(k_raw, min(k_max, n)));
    const int block_tokens = kWpb * unit_tokens;
    if (bx > 0 && ((int64_t)bx * block_tokens >= n || k == 0)) return;   // block 0 reports the counts
    const int n_blocks = (n + block_tokens - 1) / block_tokens;
    const int n_units = (n + unit_tokens - 1) / unit_tokens;
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    const bool active = t_begin < n && k > 0;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);
    uint4 cw[4];
    if (active) load_chunk<PAGED>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    __syncthreads();

    // ---- whole-sequence cumulative counts per head: sum of the per-block rows (stale rows of blocks
    // beyond the sequence are dropped here)
    if (srow < kRowsPerPass) {
#pragma unroll
        for (int j = 0; j < G; ++j) {
            int v = 0;
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (srow + u * kRowsPerPass < n_blocks) v += tv[j][u];
            for (int blk = srow + 2 * kRowsPerPass; blk < n_blocks; blk += kRowsPerPass)      // very long contexts
                v += blk_cum[((bh0 + j) * blocks_pitch + blk) * kCumRow + scol];
            if (v) atomicAdd(&tot[j * kCumRow + scol], v);
        }
    }
    __syncthreads();

    // ---- selection parameters: wave j works them out for head j and for the 16 units of the block
    for (int j = wave; j < G; j += kWpb) {
        const int64_t bh = bh0 + j;
        const int32_t* tab = blk_cum + bh * blocks_pitch * kCumRow;
        const uint16_t* utab = unit_cum + bh * blocks_pitch * kWpb * kCumRow;
        const int cum = lane < kCumRow ? tot[j * kCumRow + lane] : 0;   // #{score >= lane} over the sequence
        int T = kBins, r = 0, gt = 0, ge = 0, ugt = 0, uge = 0;
        if (k > 0) {
            const uint64_t ge_k = __ballot(lane < kBins && cum >= k);   // lane 0 is set: cum(0) = n >= k
            T = 63 - __clzll((long long)(ge_k | 1ull));
            r = k - __shfl(cum, T + 1, kWave);                          // slot 33 holds 0
            for (int blk = lane; blk < bx; blk += kWave) {
                ge += tab[blk * kCumRow + T];
                gt += tab[blk * kCumRow + T + 1];
            }
            if (lane < kWpb && unit0 + lane < n_units) {
                uge = utab[(int64_t)(unit0 + lane) * kCumRow + T];
                ugt = utab[(int64_t)(unit0 + lane) * kCumRow + T + 1];
            }
        }
        gt = wave_sum_i32(gt);
        ge = wave_sum_i32(ge);
        const int ueq = uge - ugt;
        const int gt_start = gt + wave_incl_scan_i32(ugt) - ugt;        // #{score > T} before unit `lane`
        const int eq_start = (ge - gt) + wave_incl_scan_i32(ueq) - ueq; // #{score == T} before unit `lane`
        if (lane < kWpb) {
            const int left = r - eq_start;                              // tie quota still open at this unit
            upos[lane][j] = make_int2(gt_start + min(eq_start, r), left >= ueq ? kAllTies : max(left, 0));
        }
        if (lane == 0) {
            thr[j] = T;
            if (bx == 0) {
                count[bh] = k;
                if (threshold) threshold[bh] = (uint8_t)(k > 0 ? T : 0);
            }
        }
    }
    __syncthreads();
    if (!active) return;

    // ---- compaction of this wave's unit
    int lim[G], pos[G], quota[G], ties_seen[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int T = uniform(thr[j]);
        const int2 u = upos[wave][j];
        pos[j] = uniform(u.x);
        quota[j] = uniform(u.y);
        // score >= T (all ties taken) or score > T, as a bound on the Hamming distance 32 - score
        lim[j] = quota[j] == kAllTies ? kBits - T : kBits - T - 1;
        ties_seen[j] = 0;
    }
    for (int base = (int)t_begin; base < t_end; base += kChunk) {
        if (base != (int)t_begin) load_chunk<PAGED>(c, b, kvh, base, t_end, lane, cw);
        const int groups = (min(t_end - base, kChunk) + 4 * kWave - 1) / (4 * kWave);     // uniform over the wave
        int32_t* idx0 = idx + bh0 * k_max;
        if (groups == 1)
            compact_chunk<G, 1>(cw, base, t_end, lane, qc, lim, quota, pos, ties_seen, idx0, k_max);
        else if (groups == 2)
            compact_chunk<G, 2>(cw, base, t_end, lane, qc, lim, quota, pos, ties_seen, idx0, k_max);
        else
            compact_chunk<G, 4>(cw, base, t_end, lane, qc, lim, quota, pos, ties_seen, idx0, k_max);
    }
}

template <int G>
hipError_t launch_g(const KvView& kv, bool paged, const uint32_t* q_codes, int batch, int n_q_heads,
                    const int32_t* k_per_seq, int k_max, int max_seq_len, int unit_tokens,
                    const TopkScratch& sc, int32_t* idx, int32_t* count, uint8_t* threshold,
                    hipStream_t stream)
{
    const int64_t block_tokens = (int64_t)kWpb * unit_tokens;
    int n_blocks = (int)((max_seq_len + block_tokens - 1) / block_tokens);
    if (n_blocks < 1) n_blocks = 1;               // block 0 of every group still reports count = 0
    const dim3 grid(n_blocks, kv.n_kv_heads, batch), block(kThreads);
    if (paged) {
        score_hist_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                sc.blocks_pitch, sc.blk_cum, sc.unit_cum);
        topk_select_kernel<G, true><<<grid, block, 0, stream>>>(kv, q_codes, k_per_seq, k_max, n_q_heads, max_seq_len,
                                                                 unit_tokens, sc.blocks_pitch, sc.blk_cum, sc.unit_cum, idx, count,
                                                                 threshold);
    } else {
        score_hist_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, n_q_heads, max_seq_len, unit_tokens,
                                                                 sc.blocks_pitch, sc.blk_cum, sc.unit_cum);
        topk_select_kernel<G, false><<<grid, block, 0, stream>>>(kv, q_codes, k_per_seq, k_max, n_q_heads, max_seq_len,
                                                                  unit_tokens, sc.blocks_pitch, sc.blk_cum, sc.unit_cum, idx, count,
                                                                  threshold);
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
