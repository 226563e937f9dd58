// SCORE + TOPK (section 4; section 4.1, eq. 1) for gfx950.
//
// The score of a token is the Hamming similarity 32 - popcount(q_code ^ k_code),
// an integer in 0..32, so top-k is a 33-bin counting select in two launches.
// A sequence is cut into "units" (contiguous runs of tokens, one per wave); a block
// of 8 (or 16) waves owns as many consecutive units of one KV head and serves the G query heads
// of its group from one read of the codes.
//   1. score_hist   every wave scores its unit for the G heads and counts scores per
//                   head in one LDS histogram per block.  A bin has 32 copies, picked
//                   by lane, so the 64 adds of a wave instruction fall on 32 different
//                   banks whatever the scores are (with the copies of a bin side by
//                   side the adds of a wave cost about 2 LDS passes; with a histogram
//                   per wave and 4 copies per bin they cost about 10).  The cumulative
//                   counts C(s) = #{score >= s} of the block go to one row per head.
//   2. topk_select  every block sums the rows of its heads to get the threshold T
//                   (largest T with C(T) >= k) and the tie quota r = k - C(T + 1); rows
//                   T and T + 1 of the blocks before it give its first output slot and
//                   its share of the quota (block order = token order, so ties go to the
//                   lower token index).  Each wave re-scores its unit into one bit mask
//                   per lane and head, the waves of the block exchange their counts
//                   through LDS, and each wave writes the selected token ids at
//                   offset + rank.  For that the codes are first moved through LDS so
//                   that a lane holds consecutive tokens: the rank of a token is then
//                   the lane's prefix count plus the bits below it, one wave prefix sum
//                   serves two heads, and the ids of a lane leave in a loop over its set
//                   bits.  The result is ascending by index and does not depend on the
//                   order in which waves or blocks run.
// Scores never go to HBM; the codes are read twice (the second read mostly from
// L2 / Infinity Cache).  All loads of a unit are issued before the first is used.
// Nothing persists between calls.
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kAllTies = 0x7fffffff;
constexpr int kBinCopies = 32;        // LDS copies of a histogram bin, one per bank
constexpr int kChunk = 4 * 4 * kWave; // most tokens a wave handles at once: four 16-byte loads per lane

// Which (sequence, KV head, block inside the sequence) a workgroup takes.  Contiguous cache: a 3-D grid
// (block, head, sequence), the block index rotated by head and sequence so that the blocks of mixed-length
// batches spread over the XCDs.  Paged cache: the codes of a page are [head][16 tokens], 64 bytes per head,
// so a 128-byte line holds the same tokens of two neighbouring heads; fetched by blocks on different XCDs
// (each with its own L2) every line would cross from memory twice (measured: 2.0 x the code bytes).  There the
// grid is 1-D and laid out so that the two heads of a pair take workgroup numbers 8 apart: workgroups go to
// the eight XCDs round-robin, so both land on the same XCD, a few dispatch slots from each other, and the
// second finds the line in that L2.  Number w = 16 q + 8 p + r (p = head parity, r < 8) takes work item
// 8 q + r of the list (sequence, block, head pair), pairs fastest.  False: nothing to do (padding).
template <bool PAGED>
__device__ __forceinline__ bool block_coords(int nb_cap, int n_kv_heads, int batch, int& b, int& kvh, int& bx)
{
    if constexpr (PAGED) {
        if (n_kv_heads & 1) {                               // no pairs: plain order, heads fastest
            const int item = blockIdx.x;
            if (item >= nb_cap * n_kv_heads * batch) return false;
            kvh = item % n_kv_heads;
            const int t = item / n_kv_heads;
            b = t / nb_cap;
            bx = (t - b * nb_cap + b) % nb_cap;
            return true;
        }
        const int w = blockIdx.x, pairs = n_kv_heads >> 1;
        const int item = (w >> 4) * 8 + (w & 7);
        if (item >= nb_cap * pairs * batch) return false;
        kvh = 2 * (item % pairs) + ((w >> 3) & 1);
        const int t = item / pairs;
        b = t / nb_cap;
        bx = (t - b * nb_cap + b) % nb_cap;                 // rotated by the sequence: block 0, which every sequence has, is not always on the same XCDs
        return true;
    } else {
        b = blockIdx.z;
        kvh = blockIdx.y;
        bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);
        return true;
    }
}

// NIT 16-byte loads per lane, coalesced: load `it` of lane L holds tokens base + it * 256 + 4 L .. + 3.
// Needs base < t_end.  Pieces past t_end repeat the last piece before it instead of being skipped
// (callers mask by token index), so the loads are unconditional and the compiler can wait for them
// one by one.
template <bool PAGED, int NIT>
__device__ __forceinline__ void load_chunk(const KvView& c, int b, int kvh, int base, int t_end, int lane,
                                           uint4 (&cw)[NIT])
{
    const int last = (t_end - 1) & ~3;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int t0 = min(base + it * 4 * kWave + lane * 4, last);
        cw[it] = *reinterpret_cast<const uint4*>(c.codes + row_of<PAGED>(c, b, kvh, t0));
    }
}

// CHECKED: only tokens t with lo <= t < hi are counted.  nqc: the complemented query codes, so that the
// bit count of the xor is the score itself (three instructions and one LDS add per token and head:
// xor, count, shift-or into the address).
template <int G, bool CHECKED>
__device__ __forceinline__ void count_chunk(const uint4 (&cw)[4], int base, int lo, int hi, int lane,
                                            const uint32_t (&nqc)[G], unsigned* mine)
{
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int t0 = base + it * 4 * kWave + lane * 4;
        const uint32_t w[4] = {cw[it].x, cw[it].y, cw[it].z, cw[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (!CHECKED || (t0 + e >= lo && t0 + e < hi)) {
#pragma unroll
                for (int j = 0; j < G; ++j)       // score = popcount of the agreeing bits
                    atomicAdd(&mine[(j * kBins + __popc(w[e] ^ nqc[j])) * kBinCopies], 1u);
            }
        }
    }
}

// Table written by score_hist and read by topk_select; a row holds #{score >= s} for s = 0..32 and
// a zero in slot 33, so that "row[T + 1]" is valid for T = 32:
//   blk_cum:  [B][Hq][blocks_pitch][34] ints, one row per block of 8 units
// WPB: waves (units) per block, 8 or 16.
template <int G, bool PAGED, int WPB>
__global__ __launch_bounds__(WPB * kWave) void score_hist_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                              int n_q_heads, int n_cap, int unit_tokens,
                                                              int n_sink, int n_local, int speculate, int nb_cap, int batch,
                                                              int blocks_pitch, int32_t* __restrict__ blk_cum)
{
    __shared__ __attribute__((aligned(16))) unsigned hist[G * kBins * kBinCopies];   // [head][score][copy]
    __shared__ int bsum[G * kBins];
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;    // wave: scalar, so are the token ranges
    int b, kvh, bx;                                                     // bx: block index inside the sequence
    if (!block_coords<PAGED>(nb_cap, c.n_kv_heads, batch, b, kvh, bx)) return;
    const int unit = bx * WPB + wave;
    const int64_t t_begin = (int64_t)unit * unit_tokens;
    // loads complete in issue order: the few small ones go first, so that waiting for them does not
    // mean waiting for the codes
    int qraw[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qraw[j] = (int)q_codes[(int64_t)b * n_q_heads + kvh * G + j];
    const int n_raw = c.seq_lens[b];
    uint4 cw[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) cw[it] = make_uint4(0u, 0u, 0u, 0u);     // element by element: keeps the array in registers
    // contiguous cache: rows up to the host's bound n_cap exist whatever the sequence length is, so
    // the first loads need not wait for it (what lies past the length is masked out below).  Not in a
    // batch of mixed lengths (speculate == 0): there most blocks of a short sequence lie beyond its end,
    // and a block that has asked for codes cannot leave before they have arrived.
    const bool early = !PAGED && speculate != 0;
    if (early && t_begin < n_cap)
        load_chunk<PAGED, 4>(c, b, kvh, (int)t_begin, (int)min((int64_t)n_cap, t_begin + unit_tokens), lane, cw);
    const int n = min(n_raw, n_cap);           // n_cap: the host's bound that sized grid and scratch
    if ((int64_t)bx * WPB * unit_tokens >= n) return;      // whole block beyond the sequence
    const bool active = t_begin < n;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);   // always-kept tokens [0, lo) and [hi, n) are not scored
    if (!early && active) load_chunk<PAGED, 4>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    uint32_t qc[G];                                        // complemented (see count_chunk); made uniform after the
#pragma unroll                                             // complement so that it stays one
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform(~qraw[j]);
    for (int i = tid; i < G * kBins * kBinCopies; i += (WPB * kWave)) hist[i] = 0u;
    __syncthreads();

    if (active) {
        unsigned* mine = hist + (lane & (kBinCopies - 1));
        for (int base = (int)t_begin; base < t_end; base += kChunk) {
            uint4 nx[4];
            const bool more = base + kChunk < t_end;
            if (more) load_chunk<PAGED, 4>(c, b, kvh, base + kChunk, t_end, lane, nx);
            if (base >= lo && base + kChunk <= min(t_end, hi)) count_chunk<G, false>(cw, base, lo, hi, lane, qc, mine);
            else count_chunk<G, true>(cw, base, lo, min(t_end, hi), lane, qc, mine);   // ragged end, window edges
            if (more) {
#pragma unroll
                for (int it = 0; it < 4; ++it) cw[it] = nx[it];
            }
        }
    }
    __syncthreads();
    // the 32 copies of a bin: four threads add eight each, then across the quad
    for (int row = tid >> 2; row < G * kBins; row += (WPB * kWave) / 4) {
        const uint4* p = reinterpret_cast<const uint4*>(hist + row * kBinCopies + (tid & 3) * 8);
        const uint4 a = p[0], d = p[1];
        int s = (int)((a.x + a.y) + (a.z + a.w) + (d.x + d.y) + (d.z + d.w));
        s += dpp_i<0xB1>(s);    // quad_perm:[1,0,3,2]
        s += dpp_i<0x4E>(s);    // quad_perm:[2,3,0,1]
        if ((tid & 3) == 0) bsum[row] = s;
    }
    __syncthreads();
    // cumulative counts per head by a wave scan (lanes 0..32 hold the bins, lane 33 the zero slot)
    for (int j = wave; j < G; j += WPB) {
        const int h = lane < kBins ? bsum[j * kBins + lane] : 0;
        const int incl = wave_incl_scan_i32(h);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (lane < kCumRow) {
            const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
            blk_cum[(bh * blocks_pitch + bx) * kCumRow + lane] = total - incl + h;
        }
    }
}

// Bit p of the result (p < TPL): token p of the lane has Hamming distance <= lim to qc; the bits from
// TPL up are set.  popcount + bias has its top bit set exactly when the distance exceeds lim, and
// one funnel shift moves that bit into the mask: three instructions per token and head.
template <int TPL>
__device__ __forceinline__ unsigned within_mask(const uint32_t (&w)[TPL], uint32_t qc, int lim)
{
    const unsigned bias = 0x7fffffffu - (unsigned)lim;       // lim is in -2..32
    unsigned m = 0;
#pragma unroll
    for (int p = TPL - 1; p >= 0; --p) {
        unsigned d;                                          // popcount(w ^ qc) + bias: the count instruction adds its second operand
        asm("v_xor_b32 %0, %2, %1\n\tv_bcnt_u32_b32 %0, %0, %3" : "=&v"(d) : "v"(w[p]), "s"(qc), "s"(bias));
        m = __builtin_amdgcn_alignbit(m, d, 31);             // (m << 1) | top bit of d
    }
    return ~m;
}

template <int TPL>
__device__ __forceinline__ unsigned equal_mask(const uint32_t (&w)[TPL], uint32_t qc, int dist)
{
    unsigned m = 0;
#pragma unroll
    for (int p = TPL - 1; p >= 0; --p) m = (m << 1) | (unsigned)((int)__popc(w[p] ^ qc) == dist);
    return m;
}

__device__ __forceinline__ void wave_lds_order()
{
    // LDS accesses of one wave execute in program order; this only keeps the compiler from
    // moving them across the point where lanes read what other lanes of the wave wrote
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// From the coalesced load layout to runs: afterwards lane L holds tokens base + L * TPL .. + TPL - 1
// (TPL = 4 NIT) in w.  `stage` is the wave's own LDS area of 64 * NIT 16-byte slots.
template <int NIT>
__device__ __forceinline__ void to_lane_runs(const uint4 (&cw)[NIT], uint4* stage, int lane, uint32_t (&w)[NIT * 4])
{
    if constexpr (NIT == 1) {
        w[0] = cw[0].x; w[1] = cw[0].y; w[2] = cw[0].z; w[3] = cw[0].w;
    } else {
        wave_lds_order();                            // earlier reads of the area are done
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int piece = it * kWave + lane;     // 4-token piece index inside the chunk
            stage[piece] = cw[it];              // piece p of the chunk belongs to lane p / NIT
        }
        wave_lds_order();
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const uint4 x = stage[lane * NIT + i];
            w[4 * i] = x.x; w[4 * i + 1] = x.y; w[4 * i + 2] = x.z; w[4 * i + 3] = x.w;
        }
    }
}

// NIT: 16-byte loads per lane and chunk (unit_tokens = 256 NIT for NIT < 4); NCH: chunks of 1024
// tokens per unit (unit_tokens = 1024 NCH, NIT = 4).
template <int G, bool PAGED, int NIT, int NCH, int WPB>
__global__ __launch_bounds__(WPB * kWave) void topk_select_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                               const int32_t* __restrict__ k_per_seq, int k_max,
                                                               int n_sink, int n_local, int pitch, int speculate,
                                                               int nb_cap, int batch,
                                                               int n_q_heads, int n_cap, int blocks_pitch,
                                                               const int32_t* __restrict__ blk_cum,
                                                               int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                               uint8_t* __restrict__ threshold)
{
    constexpr int kTpl = 4 * NIT;                              // tokens per lane and chunk
    constexpr int kChunkTokens = kTpl * kWave;
    constexpr int kUnitTokens = kChunkTokens * NCH;
    constexpr int kBlockTokens = kUnitTokens * WPB;
    constexpr int kRowsPerPass = (WPB * kWave) / kCumRow;           // 30 table rows are read side by side
    constexpr int kPairs = (G + 1) / 2;                        // two heads share a packed wave sum / scan
    extern __shared__ uint4 stage_all[];                       // NIT > 1: 64 * NIT slots per wave
    __shared__ int tot[G * kCumRow], bef[G * kCumRow], own[G * kCumRow];   // cumulative counts: sequence, blocks before this one, this block
    __shared__ int thr[G], posb[G], quotab[G];                 // per head: T, first output slot and tie quota of the block
    __shared__ int wcnt[WPB][kPairs], weq[WPB][kPairs];      // per wave: selected / tied tokens, two heads per int
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;    // wave: scalar, so are the token ranges
    int b, kvh, bx;                                            // bx: block index inside the sequence; nb_cap blocks launched per sequence
    if (!block_coords<PAGED>(nb_cap, c.n_kv_heads, batch, b, kvh, bx)) return;
    const int64_t bh0 = (int64_t)b * n_q_heads + kvh * G;

    // ---- everything that does not depend on another load is requested first; in a batch of mixed
    // lengths (speculate == 0) the length comes before that, over the scalar path, so that a block
    // beyond the end of a short sequence leaves without waiting for anything else
    const int n_raw = c.seq_lens[b];
    const int k_raw = k_per_seq ? k_per_seq[b] : k_max;
    constexpr int kBlockTokensEarly = 4 * NIT * kWave * NCH * WPB;
    if (!speculate && bx > 0 && (int64_t)bx * kBlockTokensEarly >= min(n_raw, n_cap)) return;
    const int srow = tid / kCumRow, scol = tid - srow * kCumRow;
    constexpr int kPrefetch = 3;                                // passes of table rows requested up front
    int tv[G][kPrefetch];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) {
            const int blk = srow + u * kRowsPerPass;
            tv[j][u] = 0;
            if (srow < kRowsPerPass && blk < nb_cap)
                tv[j][u] = blk_cum[((bh0 + j) * blocks_pitch + blk) * kCumRow + scol];
        }
    int qraw[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qraw[j] = (int)q_codes[bh0 + j];
    // the codes go last: loads complete in issue order, and nothing before the scoring needs them
    const int64_t t_begin = ((int64_t)bx * WPB + wave) * kUnitTokens;
    uint4 cw[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) cw[it] = make_uint4(0u, 0u, 0u, 0u);   // element by element: keeps the array in registers
    const bool early = !PAGED && speculate != 0;     // contiguous cache: no need to wait for the sequence length (see score_hist)
    if (early && t_begin < n_cap)
        load_chunk<PAGED, NIT>(c, b, kvh, (int)t_begin, (int)min((int64_t)n_cap, t_begin + kUnitTokens), lane, cw);
    uint32_t qc[G];
#pragma unroll
    for (int j = 0; j < G; ++j) qc[j] = (uint32_t)uniform(qraw[j]);
    for (int i = tid; i < G * kCumRow; i += (WPB * kWave)) tot[i] = bef[i] = own[i] = 0;

    const int n = min(n_raw, n_cap);
    // the first `lo` and the tokens from `hi` on are always taken; k counts the tokens retrieved in between
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);
    const int k = max(0, min(k_raw, min(k_max, hi - lo)));
    const bool nothing = k == 0 && lo == 0 && hi == n;
    if (bx > 0 && ((int64_t)bx * kBlockTokens >= n || nothing)) return;   // block 0 reports the counts
    const int n_blocks = (n + kBlockTokens - 1) / kBlockTokens;
    const bool active = t_begin < n && !nothing;
    const int t_end = (int)min((int64_t)n, t_begin + kUnitTokens);
    if (!early && active) load_chunk<PAGED, NIT>(c, b, kvh, (int)t_begin, t_end, lane, cw);
    __syncthreads();

    // ---- cumulative counts per head from the per-block rows, in one trip to memory: over the whole
    // sequence, over the blocks before this one, and this block's own row (stale rows of blocks beyond
    // the sequence are dropped here)
    if (srow < kRowsPerPass) {
#pragma unroll
        for (int j = 0; j < G; ++j) {
            int v = 0, vb = 0;
            auto take = [&](int blk, int x) {
                v += x;
                if (blk < bx) vb += x;
                if (blk == bx) own[j * kCumRow + scol] = x;
            };
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u)
                if (srow + u * kRowsPerPass < n_blocks) take(srow + u * kRowsPerPass, tv[j][u]);
            for (int blk = srow + kPrefetch * kRowsPerPass; blk < n_blocks; blk += kRowsPerPass)   // very long contexts
                take(blk, blk_cum[((bh0 + j) * blocks_pitch + blk) * kCumRow + scol]);
            if (v) atomicAdd(&tot[j * kCumRow + scol], v);
            if (vb) atomicAdd(&bef[j * kCumRow + scol], vb);
        }
    }
    __syncthreads();

    // ---- selection parameters: wave j works them out for head j
    for (int j = wave; j < G; j += WPB) {
        const int64_t bh = bh0 + j;
        const int cum = lane < kCumRow ? tot[j * kCumRow + lane] : 0;   // #{score >= lane} over the sequence
        int T = kBins, r = 0, gt = 0, ge = 0, own_gt = 0, own_ge = 0;
        if (k > 0) {
            const uint64_t ge_k = __ballot(lane < kBins && cum >= k);   // lane 0 is set: cum(0) = n >= k
            T = 63 - __clzll((long long)(ge_k | 1ull));
            r = k - __shfl(cum, T + 1, kWave);                          // slot 33 holds 0
            ge = bef[j * kCumRow + T];                                  // #{score >= T} before this block
            gt = bef[j * kCumRow + T + 1];
            own_ge = own[j * kCumRow + T];
            own_gt = own[j * kCumRow + T + 1];
        }
        if (lane == 0) {
            const int eq_before = ge - gt, own_eq = own_ge - own_gt;    // #{score == T} before / inside this block
            const int left = r - eq_before;                             // tie quota still open at this block
            const int bs = (int)min((int64_t)n, (int64_t)bx * kBlockTokens);   // always-kept tokens before this block
            thr[j] = T;
            posb[j] = gt + min(eq_before, r) + min(lo, bs) + max(0, bs - hi);
            quotab[j] = left >= own_eq ? kAllTies : max(left, 0);
            if (bx == 0) {
                count[bh] = lo + k + (n - hi);
                if (threshold) threshold[bh] = (uint8_t)(k > 0 ? T : 0);
            }
        }
    }
    __syncthreads();

    // ---- every wave: masks of the tokens to take (score > T, or >= T where the whole block's ties
    // fit the quota) and, for a head whose quota ends inside this block, of its ties
    uint4* stage = stage_all + wave * (kWave * NIT);
    unsigned sel[NCH][G], tie[NCH][G];
    int lim[G], quota[G];
    bool any_partial = false;
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int T = uniform(thr[j]);
        quota[j] = uniform(quotab[j]);
        lim[j] = quota[j] == kAllTies ? kBits - T : kBits - T - 1;      // bound on the Hamming distance 32 - score
        any_partial |= quota[j] != kAllTies && quota[j] != 0;
    }
    int csum[kPairs], esum[kPairs];
#pragma unroll
    for (int pr = 0; pr < kPairs; ++pr) csum[pr] = esum[pr] = 0;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
        for (int j = 0; j < G; ++j) sel[ch][j] = tie[ch][j] = 0u;
        const int cbase = (int)t_begin + ch * kChunkTokens;
        if (active && cbase < t_end) {                                  // uniform over the wave
            uint32_t w[kTpl];
            to_lane_runs<NIT>(cw, stage, lane, w);
            if (ch + 1 < NCH && cbase + kChunkTokens < t_end)           // next chunk: on its way while this one is scored
                load_chunk<PAGED, NIT>(c, b, kvh, cbase + kChunkTokens, t_end, lane, cw);
            const int first = cbase + lane * kTpl;                          // first token of this lane's run
            auto below = [&](int t) { return (1u << max(0, min(t - first, kTpl))) - 1u; };   // bits of tokens < t
            const unsigned valid = below(t_end);
            const unsigned scored = below(hi) & ~below(lo) & valid;         // tokens that compete for the budget
            const unsigned kept = valid & ~scored;                          // always-kept tokens
#pragma unroll
            for (int j = 0; j < G; ++j) {
                sel[ch][j] = (within_mask<kTpl>(w, qc[j], lim[j]) & scored) | kept;
                if (any_partial && quota[j] != kAllTies && quota[j] != 0)
                    tie[ch][j] = equal_mask<kTpl>(w, qc[j], lim[j] + 1) & scored;
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            csum[j >> 1] += __popc(sel[ch][j]) << (16 * (j & 1));
            esum[j >> 1] += __popc(tie[ch][j]) << (16 * (j & 1));
        }
    }
#pragma unroll
    for (int pr = 0; pr < kPairs; ++pr) {
        const int cs = wave_sum_i32(csum[pr]);
        const int es = any_partial ? wave_sum_i32(esum[pr]) : 0;
        if (lane == 0) { wcnt[wave][pr] = cs; weq[wave][pr] = es; }
    }
    __syncthreads();
    if (!active) return;

    // ---- first output slot of this wave per head; resolve a quota that ends inside the block
    int start[G];
#pragma unroll
    for (int pr = 0; pr < kPairs; ++pr) {
        const int before2 = wave_sum_i32(lane < wave ? wcnt[lane][pr] : 0);
        const int eqb2 = any_partial ? wave_sum_i32(lane < wave ? weq[lane][pr] : 0) : 0;
        const int own2 = any_partial ? weq[wave][pr] : 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = 2 * pr + h;
            if (j >= G) break;
            const int before = (before2 >> (16 * h)) & 0xffff;
            start[j] = uniform(posb[j]) + before;
            if (quota[j] != kAllTies && quota[j] != 0) {
                const int eq_before = (eqb2 >> (16 * h)) & 0xffff, own = (own2 >> (16 * h)) & 0xffff;
                const int left = quota[j] - eq_before;                  // quota still open at this wave
                start[j] += min(eq_before, quota[j]);
                if (left >= own) {
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) sel[ch][j] |= tie[ch][j];
                } else if (left > 0) {                                  // ties are ranked in token order
                    int seen = 0;
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {
                        const int mine = __popc(tie[ch][j]);
                        const int incl = wave_incl_scan_i32(mine);
                        const int take = max(0, min(mine, left - seen - (incl - mine)));
                        sel[ch][j] |= lowest_bits(tie[ch][j], take);
                        seen += __builtin_amdgcn_readlane(incl, 63);
                    }
                }
            }
        }
    }

    // ---- ranks in token order and the ids
    int32_t* idx0 = idx + bh0 * pitch;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int first = (int)t_begin + ch * kChunkTokens + lane * kTpl;
#pragma unroll
        for (int pr = 0; pr < kPairs; ++pr) {
            const int j0 = 2 * pr, j1 = 2 * pr + 1;
            const int c0 = __popc(sel[ch][j0]), c1 = j1 < G ? __popc(sel[ch][j1 < G ? j1 : j0]) : 0;
            const int incl = wave_incl_scan_i32(c0 | (c1 << 16));
            const int total = __builtin_amdgcn_readlane(incl, 63);
            emit_ids(sel[ch][j0], start[j0] + (incl & 0xffff) - c0, first, pitch, idx0 + (int64_t)j0 * pitch);
            start[j0] += total & 0xffff;
            if (j1 < G) {
                const int jj = j1 < G ? j1 : j0;
                emit_ids(sel[ch][jj], start[jj] + (int)((unsigned)incl >> 16) - c1, first, pitch, idx0 + (int64_t)jj * pitch);
                start[jj] += (int)((unsigned)total >> 16);
            }
        }
    }
}

template <int G, bool PAGED, int NIT, int NCH, int WPB>
hipError_t select_variant(bool setup_only, const KvView& kv, const TopkCall& a, const TopkScratch& sc, dim3 grid,
                          int blocks_per_seq, hipStream_t stream)
{
    constexpr int lds = NIT > 1 ? WPB * kWave * NIT * (int)sizeof(uint4) : 0;
    if (setup_only)
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&topk_select_kernel<G, PAGED, NIT, NCH, WPB>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    topk_select_kernel<G, PAGED, NIT, NCH, WPB><<<grid, dim3(WPB * kWave), lds, stream>>>(
        kv, a.q_codes, a.k_per_seq, a.k_max, a.n_sink, a.n_local, a.k_max + a.n_sink + a.n_local,
        a.k_per_seq == nullptr, blocks_per_seq, a.batch, a.n_q_heads,
        a.max_seq_len, sc.blocks_pitch, sc.blk_cum, a.idx, a.count, a.threshold);
    return hipSuccess;
}

template <int G, bool PAGED, int WPB>
hipError_t select_by_unit(bool setup_only, int unit_tokens, const KvView& kv, const TopkCall& a, const TopkScratch& sc,
                          dim3 grid, int blocks_per_seq, hipStream_t stream)
{
    switch (unit_tokens) {
    case 256: return select_variant<G, PAGED, 1, 1, WPB>(setup_only, kv, a, sc, grid, blocks_per_seq, stream);
    case 512: return select_variant<G, PAGED, 2, 1, WPB>(setup_only, kv, a, sc, grid, blocks_per_seq, stream);
    case 1024: return select_variant<G, PAGED, 4, 1, WPB>(setup_only, kv, a, sc, grid, blocks_per_seq, stream);
    case 2048: return select_variant<G, PAGED, 4, 2, WPB>(setup_only, kv, a, sc, grid, blocks_per_seq, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int G, bool PAGED, int WPB>
hipError_t launch_gpw(bool setup_only, const KvView& kv, const TopkCall& a, int unit_tokens, const TopkScratch& sc,
                      hipStream_t stream)
{
    if (setup_only) {
        for (int unit = 256; unit <= 2048; unit *= 2)
            if (hipError_t e = select_by_unit<G, PAGED, WPB>(true, unit, kv, a, sc, dim3(1), 1, stream); e != hipSuccess) return e;
        return hipSuccess;
    }
    const int64_t block_tokens = (int64_t)WPB * unit_tokens;
    int n_blocks = (int)((a.max_seq_len + block_tokens - 1) / block_tokens);
    if (n_blocks < 1) n_blocks = 1;               // block 0 of every group still reports count = 0
    // contiguous: (block, head, sequence); paged: 1-D, head pairs eight workgroup numbers apart (block_coords)
    dim3 grid(n_blocks, kv.n_kv_heads, a.batch);
    if constexpr (PAGED) {
        const int64_t n_kv = kv.n_kv_heads;
        const int64_t items = (n_kv & 1) ? (int64_t)n_blocks * n_kv * a.batch : (int64_t)n_blocks * (n_kv / 2) * a.batch;
        const int64_t groups = (n_kv & 1) ? items : (items + 7) / 8 * 16;
        if (groups > 0x7fffffff) return hipErrorInvalidValue;
        grid = dim3((unsigned)groups);
    }
    const dim3 block(WPB * kWave);
    // a k per sequence means lengths differ: blocks then wait for their sequence's length before any other load
    score_hist_kernel<G, PAGED, WPB><<<grid, block, 0, stream>>>(kv, a.q_codes, a.n_q_heads, a.max_seq_len, unit_tokens,
                                                             a.n_sink, a.n_local, a.k_per_seq == nullptr, n_blocks, a.batch,
                                                             sc.blocks_pitch, sc.blk_cum);
    if (hipError_t e = select_by_unit<G, PAGED, WPB>(false, unit_tokens, kv, a, sc, grid, n_blocks, stream); e != hipSuccess) return e;
    return hipGetLastError();
}

template <int G, bool PAGED>
hipError_t launch_gp(bool setup_only, const KvView& kv, const TopkCall& a, int unit_tokens, const TopkScratch& sc,
                     hipStream_t stream)
{
    if (setup_only) {
        if (hipError_t e = launch_gpw<G, PAGED, 8>(true, kv, a, unit_tokens, sc, stream); e != hipSuccess) return e;
        return launch_gpw<G, PAGED, 16>(true, kv, a, unit_tokens, sc, stream);
    }
    return a.waves_per_block == 16 ? launch_gpw<G, PAGED, 16>(false, kv, a, unit_tokens, sc, stream)
                                   : launch_gpw<G, PAGED, 8>(false, kv, a, unit_tokens, sc, stream);
}

template <int G>
hipError_t launch_g(bool setup_only, const KvView& kv, bool paged, const TopkCall& a, int unit_tokens,
                    const TopkScratch& sc, hipStream_t stream)
{
    if (setup_only) {
        if (hipError_t e = launch_gp<G, false>(true, kv, a, unit_tokens, sc, stream); e != hipSuccess) return e;
        return launch_gp<G, true>(true, kv, a, unit_tokens, sc, stream);
    }
    return paged ? launch_gp<G, true>(false, kv, a, unit_tokens, sc, stream)
                 : launch_gp<G, false>(false, kv, a, unit_tokens, sc, stream);
}

hipError_t dispatch_group(bool setup_only, const KvView& kv, bool paged, int group, const TopkCall& a,
                          int unit_tokens, const TopkScratch& sc, hipStream_t stream)
{
    switch (group) {
    case 1: return launch_g<1>(setup_only, kv, paged, a, unit_tokens, sc, stream);
    case 2: return launch_g<2>(setup_only, kv, paged, a, unit_tokens, sc, stream);
    case 4: return launch_g<4>(setup_only, kv, paged, a, unit_tokens, sc, stream);
    case 8: return launch_g<8>(setup_only, kv, paged, a, unit_tokens, sc, stream);
    default: return hipErrorInvalidValue;
    }
}


// ---------------------------------------------------------------------------------------------------
// One launch for short contexts.  With few (sequence, head) pairs and a context of a few ten thousand
// tokens the two kernels above are launch and round-trip latency: tables written, a kernel boundary, the
// tables and the codes fetched again.  Here one block of 16 waves owns a whole (sequence, query head): a wave
// keeps its unit's codes in registers (NCH chunks of 1024 tokens), counts the scores into a histogram of its
// own in LDS, and leaves its 33 bin counts in a table of the block; after the one block barrier every wave
// reads the table, works out T, the tie quota and its own first output slot (waves are in token order), and
// emits its ids from the registers it still holds.  The KV head's codes are read by each of its query
// heads' blocks (from L2 after the first), which costs less than a second launch.
// NL > 0: the block also maps its query vector to the code first (eq. 2; NL layers 128 -> 128 (-> 128) -> 32
// with SiLU between them), with the codes of the keys already on their way, and leaves the code in q_codes:
// ENCODE-Q, SCORE and TOPK in one launch.  The 1024 threads split a layer's inputs eight ways (32 ways for
// the last layer) and add the parts in a fixed order, so the code does not depend on timing; the order is
// not that of the stand-alone query encoder, so a bit whose activation is within rounding of zero may differ
// from it.
constexpr int kOneWaves = 16;
constexpr int kOneLdsPerWave = kBins * kBinCopies * (int)sizeof(unsigned);   // histogram, later the staging area (4096 B) of to_lane_runs
static_assert(kOneLdsPerWave >= 4 * kWave * (int)sizeof(uint4), "the staging area of a wave lies inside its histogram");

template <bool PAGED, int NCH, int NL>
__global__ __launch_bounds__(kOneWaves * kWave) void score_topk_one_block_kernel(
    KvView c, MlpView phi, const uint16_t* __restrict__ q, uint32_t* __restrict__ q_codes,
    const int32_t* __restrict__ k_per_seq, int k_max, int n_sink,
    int n_local, int pitch, int n_q_heads, int group, int n_cap, int32_t* __restrict__ idx,
    int32_t* __restrict__ count, uint8_t* __restrict__ threshold)
{
    constexpr int kTpl = 16, kChunkTokens = kTpl * kWave, kUnitTokens = kChunkTokens * NCH;
    extern __shared__ uint4 lds_all[];                          // kOneLdsPerWave bytes per wave
    __shared__ int wbins[kOneWaves][kCumRow];                   // per wave: #{score == s}, slot 33 = 0
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;
    // workgroups go to the eight XCDs round-robin: numbering the heads KV head first puts the query heads of a
    // group n_kv_heads numbers apart, on one XCD when that is a multiple of eight, so that the group's codes
    // come from memory once and from that XCD's L2 afterwards
    const int n_kv_heads = n_q_heads / group;
    const int kvh = blockIdx.x % n_kv_heads, h = kvh * group + blockIdx.x / n_kv_heads, b = blockIdx.y;
    const int64_t bh = (int64_t)b * n_q_heads + h;
    unsigned* whist = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(lds_all) + wave * kOneLdsPerWave);

    // ---- requests in the order their answers are needed (loads complete in issue order): query vector and
    // mapping weights, lengths, then the codes
    constexpr int kHid = 128;                                   // hidden width and input width of the mapping
    __shared__ float mlp_in[2][kHid];
    __shared__ float mlp_red[kOneWaves * kWave];
    __shared__ uint32_t q_code_of_block;
    const int mj = tid & (kHid - 1), mp = tid >> 7;             // hidden layers: output mj, inputs 16 mp .. 16 mp + 15
    const int lj = tid & (kBits - 1), lp = tid >> 5;            // last layer: output lj, inputs 4 lp .. 4 lp + 3
    float w_hid[NL > 0 ? NL - 1 : 1][16], w_last[4];
    int qraw = 0;
    if constexpr (NL == 0) {
        qraw = (int)q_codes[bh];
    } else {
        if (tid < kHid / 2) {
            const uint32_t two = reinterpret_cast<const uint32_t*>(q)[bh * (kHid / 2) + tid];
            mlp_in[0][2 * tid] = bf16_lo(two);
            mlp_in[0][2 * tid + 1] = bf16_hi(two);
        }
#pragma unroll
        for (int l = 0; l < NL - 1; ++l) {
            const float* W = phi.W[l] + (int64_t)h * kHid * kHid;
#pragma unroll
            for (int i = 0; i < 16; ++i) w_hid[l][i] = W[(mp * 16 + i) * kHid + mj];
        }
        const float* W = phi.W[NL - 1] + (int64_t)h * kHid * kBits;
#pragma unroll
        for (int i = 0; i < 4; ++i) w_last[i] = W[(lp * 4 + i) * kBits + lj];
    }
    const int n_raw = c.seq_lens[b];
    const int k_raw = k_per_seq ? k_per_seq[b] : k_max;
    const int t_begin = wave * kUnitTokens;
    uint4 cw[NCH][4];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
        for (int it = 0; it < 4; ++it) cw[ch][it] = make_uint4(0u, 0u, 0u, 0u);
    constexpr bool early = !PAGED;         // contiguous cache: rows up to n_cap exist, no need to wait for the length
    if (early) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
            if (t_begin + ch * kChunkTokens < n_cap)
                load_chunk<PAGED, 4>(c, b, kvh, t_begin + ch * kChunkTokens, min(n_cap, t_begin + kUnitTokens), lane, cw[ch]);
    }
    for (int i = lane; i < kBins * kBinCopies; i += kWave) whist[i] = 0u;
    const int n = min(n_raw, n_cap);
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);
    const int k = max(0, min(k_raw, min(k_max, hi - lo)));
    const bool nothing = k == 0 && lo == 0 && hi == n;
    const bool active = t_begin < n && !nothing;
    const int t_end = min(n, t_begin + kUnitTokens);
    if (!early && active) {
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
            if (t_begin + ch * kChunkTokens < t_end)
                load_chunk<PAGED, 4>(c, b, kvh, t_begin + ch * kChunkTokens, t_end, lane, cw[ch]);
    }
    if constexpr (NL > 0) {
        // ---- the query's code (eq. 2)
        __syncthreads();
#pragma unroll
        for (int l = 0; l < NL - 1; ++l) {
            const float* in = mlp_in[l & 1];
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc = fmaf(in[mp * 16 + i], w_hid[l][i], acc);
            mlp_red[mp * kHid + mj] = acc;
            __syncthreads();
            if (tid < kHid) {
                float z = 0.f;
#pragma unroll
                for (int pp = 0; pp < kOneWaves * kWave / kHid; ++pp) z += mlp_red[pp * kHid + tid];
                if (phi.bias[l]) z += phi.bias[l][(int64_t)h * kHid + tid];
                mlp_in[(l + 1) & 1][tid] = silu(z);
            }
            __syncthreads();
        }
        const float* in = mlp_in[(NL - 1) & 1];
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fmaf(in[lp * 4 + i], w_last[i], acc);
        mlp_red[lp * kBits + lj] = acc;
        __syncthreads();
        if (wave == 0) {
            float z = 0.f;
            if (lane < kBits) {
#pragma unroll
                for (int pp = 0; pp < kOneWaves * kWave / kBits; ++pp) z += mlp_red[pp * kBits + lane];
                if (phi.bias[NL - 1]) z += phi.bias[NL - 1][(int64_t)h * kBits + lane];
            }
            const uint32_t code = (uint32_t)__ballot(lane < kBits && z > 0.f);     // output unit j is bit j
            if (lane == 0) {
                q_code_of_block = code;
                q_codes[bh] = code;
            }
        }
        __syncthreads();
        qraw = (int)q_code_of_block;
    }
    const uint32_t qc = (uint32_t)uniform(qraw);
    const uint32_t nqc[1] = {(uint32_t)uniform(~qraw)};
    wave_lds_order();

    // ---- the wave's histogram, then its 33 bin counts
    if (active) {
        unsigned* mine = whist + (lane & (kBinCopies - 1));
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int base = t_begin + ch * kChunkTokens;
            if (base < t_end) {
                if (base >= lo && base + kChunkTokens <= min(t_end, hi)) count_chunk<1, false>(cw[ch], base, lo, hi, lane, nqc, mine);
                else count_chunk<1, true>(cw[ch], base, lo, min(t_end, hi), lane, nqc, mine);
            }
        }
    }
    wave_lds_order();
    for (int row0 = 0; row0 < kCumRow; row0 += 8) {             // eight lanes add the 32 copies of a bin
        const int row = row0 + (lane >> 3);
        int s = 0;
        if (row < kBins) {
            const uint4 x = *reinterpret_cast<const uint4*>(whist + row * kBinCopies + (lane & 7) * 4);
            s = (int)((x.x + x.y) + (x.z + x.w));
        }
        s += dpp_i<0xB1>(s);    // quad_perm:[1,0,3,2]
        s += dpp_i<0x4E>(s);    // quad_perm:[2,3,0,1]
        s += __shfl_xor(s, 4, kWave);
        if ((lane & 7) == 0 && row < kCumRow) wbins[wave][row] = s;
    }
    __syncthreads();

    // ---- every wave: counts over the sequence, before itself, its own; T, quota, first slot
    int tot = 0, bef = 0, own = 0;
    if (lane < kCumRow) {
#pragma unroll
        for (int w = 0; w < kOneWaves; ++w) {
            const int v = wbins[w][lane];
            tot += v;
            if (w < wave) bef += v;
            if (w == wave) own = v;
        }
    }
    const int tot_incl = wave_incl_scan_i32(tot), bef_incl = wave_incl_scan_i32(bef);
    const int cum = __builtin_amdgcn_readlane(tot_incl, 63) - tot_incl + tot;        // #{score >= lane} over the sequence
    const int cum_bef = __builtin_amdgcn_readlane(bef_incl, 63) - bef_incl + bef;    // the same over the waves before this one
    int T = kBins, r = 0, gt = 0, eq_before = 0, own_eq = 0;
    if (k > 0) {
        const uint64_t ge_k = __ballot(lane < kBins && cum >= k);
        T = 63 - __clzll((long long)(ge_k | 1ull));
        r = k - __shfl(cum, T + 1, kWave);                      // slot 33 holds 0
        gt = __shfl(cum_bef, T + 1, kWave);
        eq_before = __shfl(bef, T, kWave);
        own_eq = __shfl(own, T, kWave);
    }
    T = uniform(T);
    const int left = uniform(r - eq_before);                    // tie quota still open at this wave
    const int quota = left >= own_eq ? kAllTies : max(left, 0);
    const int lim = quota == kAllTies ? kBits - T : kBits - T - 1;   // bound on the Hamming distance 32 - score
    const bool partial = quota != kAllTies && quota != 0;
    const int ws = min(n, t_begin);                             // always-kept tokens before this wave
    int start = uniform(gt + min(eq_before, r) + min(lo, ws) + max(0, ws - hi));
    if (tid == 0) {
        count[bh] = lo + k + (n - hi);
        if (threshold) threshold[bh] = (uint8_t)(k > 0 ? T : 0);
    }
    if (!active) return;

    // ---- masks from the codes still in registers, ties ranked in token order, ids
    uint4* stage = reinterpret_cast<uint4*>(whist);
    unsigned sel[NCH], tie[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        sel[ch] = tie[ch] = 0u;
        const int cbase = t_begin + ch * kChunkTokens;
        if (cbase < t_end) {
            uint32_t w[kTpl];
            to_lane_runs<4>(cw[ch], stage, lane, w);
            const int first = cbase + lane * kTpl;
            auto below = [&](int t) { return (1u << max(0, min(t - first, kTpl))) - 1u; };
            const unsigned valid = below(t_end);
            const unsigned scored = below(hi) & ~below(lo) & valid;
            sel[ch] = (within_mask<kTpl>(w, qc, lim) & scored) | (valid & ~scored);
            if (partial) tie[ch] = equal_mask<kTpl>(w, qc, lim + 1) & scored;
        }
    }
    if (partial) {
        int seen = 0;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int mine = __popc(tie[ch]);
            const int incl = wave_incl_scan_i32(mine);
            const int take = max(0, min(mine, quota - seen - (incl - mine)));
            sel[ch] |= lowest_bits(tie[ch], take);
            seen += __builtin_amdgcn_readlane(incl, 63);
        }
    }
    int32_t* out = idx + bh * pitch;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int c0 = __popc(sel[ch]);
        const int incl = wave_incl_scan_i32(c0);
        emit_ids(sel[ch], start + incl - c0, t_begin + ch * kChunkTokens + lane * kTpl, pitch, out);
        start += __builtin_amdgcn_readlane(incl, 63);
    }
}

// What the one-launch kernel is to encode with: nothing (q_codes are given), or a query mapping of 2 or 3 layers.
struct OneBlockEncode {
    int n_layers = 0;
    MlpView phi{};
    const uint16_t* q = nullptr;
};

template <bool PAGED, int NCH, int NL>
hipError_t one_block_variant(bool setup_only, const KvView& kv, int group, const TopkCall& a, const OneBlockEncode& enc,
                             hipStream_t stream)
{
    constexpr int lds = kOneWaves * kOneLdsPerWave;
    if (setup_only)
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&score_topk_one_block_kernel<PAGED, NCH, NL>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    score_topk_one_block_kernel<PAGED, NCH, NL><<<dim3(a.n_q_heads, a.batch), dim3(kOneWaves * kWave), lds, stream>>>(
        kv, enc.phi, enc.q, const_cast<uint32_t*>(a.q_codes), a.k_per_seq, a.k_max, a.n_sink, a.n_local,
        a.k_max + a.n_sink + a.n_local, a.n_q_heads, group, a.max_seq_len, a.idx, a.count, a.threshold);
    return hipGetLastError();
}

template <bool PAGED, int NCH>
hipError_t one_block_by_layers(bool setup_only, const KvView& kv, int group, const TopkCall& a, const OneBlockEncode& enc,
                               hipStream_t stream)
{
    if (setup_only) {
        if (hipError_t e = one_block_variant<PAGED, NCH, 0>(true, kv, group, a, enc, stream); e != hipSuccess) return e;
        if (hipError_t e = one_block_variant<PAGED, NCH, 2>(true, kv, group, a, enc, stream); e != hipSuccess) return e;
        return one_block_variant<PAGED, NCH, 3>(true, kv, group, a, enc, stream);
    }
    switch (enc.n_layers) {
    case 0: return one_block_variant<PAGED, NCH, 0>(false, kv, group, a, enc, stream);
    case 2: return one_block_variant<PAGED, NCH, 2>(false, kv, group, a, enc, stream);
    case 3: return one_block_variant<PAGED, NCH, 3>(false, kv, group, a, enc, stream);
    default: return hipErrorInvalidValue;
    }
}

template <bool PAGED>
hipError_t one_block_by_length(bool setup_only, const KvView& kv, int group, const TopkCall& a, const OneBlockEncode& enc,
                               hipStream_t stream)
{
    if (setup_only) {
        if (hipError_t e = one_block_by_layers<PAGED, 1>(true, kv, group, a, enc, stream); e != hipSuccess) return e;
        return one_block_by_layers<PAGED, 2>(true, kv, group, a, enc, stream);
    }
    return a.max_seq_len <= kOneWaves * 1024 ? one_block_by_layers<PAGED, 1>(false, kv, group, a, enc, stream)
                                             : one_block_by_layers<PAGED, 2>(false, kv, group, a, enc, stream);
}

}  // namespace

// Raises the dynamic LDS limit of the select kernels of this group size (their staging area reaches
// 64 KiB); called once when a context is created, never on the launch path.
hipError_t setup_score_topk(int group)
{
    if (hipError_t e = one_block_by_length<false>(true, KvView{}, group, TopkCall{}, OneBlockEncode{}, nullptr); e != hipSuccess) return e;
    if (hipError_t e = one_block_by_length<true>(true, KvView{}, group, TopkCall{}, OneBlockEncode{}, nullptr); e != hipSuccess) return e;
    return dispatch_group(true, KvView{}, false, group, TopkCall{}, 0, TopkScratch{}, nullptr);
}

// Most tokens per sequence the one-launch path takes: 16 waves with two chunks of 1024 tokens each.
int score_topk_one_block_limit() { return kOneWaves * 2 * 1024; }

bool one_block_can_encode(const MlpView& phi)
{
    if (phi.n_layers != 2 && phi.n_layers != 3) return false;
    for (int l = 0; l < phi.n_layers; ++l)
        if (phi.dims[l] != 128) return false;
    return phi.dims[phi.n_layers] == kBits;
}

hipError_t launch_score_topk_one_block(const KvView& kv, bool paged, int group, const TopkCall& call, const MlpView* phi,
                                       const uint16_t* q, hipStream_t stream)
{
    if (call.max_seq_len > score_topk_one_block_limit()) return hipErrorInvalidValue;
    OneBlockEncode enc;
    if (phi) {
        if (!one_block_can_encode(*phi) || !q) return hipErrorInvalidValue;
        enc.n_layers = phi->n_layers;
        enc.phi = *phi;
        enc.q = q;
    }
    return paged ? one_block_by_length<true>(false, kv, group, call, enc, stream)
                 : one_block_by_length<false>(false, kv, group, call, enc, stream);
}

hipError_t launch_score_topk(const KvView& kv, bool paged, int group, const TopkCall& call, int unit_tokens,
                             const TopkScratch& sc, hipStream_t stream)
{
    return dispatch_group(false, kv, paged, group, call, unit_tokens, sc, stream);
}

}  // namespace ha
