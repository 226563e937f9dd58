// SCORE + TOPK for signatures wider than 32 bits (b = 32 W bits, W = 2, 4, 8, 16; the bit-width
// ablation of section 5.3 and the SCORE latency table of the appendix) for gfx950.
//
// Same two launches and the same tables as the 32-bit kernels (score_topk.hip): a block of 8
// waves owns 8 consecutive units of one KV head and serves its G query heads; score_hist leaves
// one row of cumulative counts C(s) = #{score >= s}, s = 0..b, per block and head; topk_select
// sums the rows, finds the threshold T and the tie quota, and writes the ids in token order.
// What differs: a code is W words, the score b - sum of popcounts has b + 1 values, and a lane
// handles one token at a time (a wave walks its unit 64 tokens per step), so that ranks come
// straight from wave ballots:
//   - the query words sit in LDS and are read as broadcasts (G W words do not fit scalar registers
//     for the larger shapes); popcount accumulates in the instruction's add operand;
//   - the select makes two passes over per-step ballot masks instead of two passes over the codes:
//     the first pass scores the unit once, keeps for every 64-token step and head the masks
//     "score > T" and "score == T" in LDS and counts them; after the waves of the block have
//     exchanged their counts, the second pass gives every lane a run of consecutive tokens, cut out
//     of those masks, and ranks and stores the ids as the 32-bit select does (ties in token order
//     against the wave's share of the quota).
// Units are 256, 512 or 1024 tokens (16 steps of masks per wave at most).
// For W = 2 and 4 with up to eight 16-byte loads per lane the select is the 32-bit one carried over
// (topk_select_runs_kernel, further down); the step-mask select serves the rest.
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kAllTies = 0x7fffffff;
constexpr int kWpb = kTopkWavesPerBlock;
constexpr int kThreads = kWpb * kWave;
constexpr int kMaxSteps = 16;                 // 64-token steps per unit: units of at most 1024 tokens
// steps whose codes are in flight ahead of the one being scored (a ring of registers)
__host__ __device__ constexpr int depth_of(int W) { return W <= 4 ? 4 : 2; }

__host__ __device__ constexpr int bins_of(int W) { return 32 * W + 1; }
// LDS histogram copies per bin: as many as fit about 32 KiB, a power of two, at most 32
__host__ __device__ constexpr int copies_of(int G, int W)
{
    int c = 32;
    while (c > 1 && G * bins_of(W) * c > 8192) c /= 2;
    return c;
}

template <int W>
struct CodeWords {
    uint32_t w[W];
};

// the W words of token t (one lane, one token); pointer arithmetic in words
template <bool PAGED, int W>
__device__ __forceinline__ CodeWords<W> load_code(const KvView& c, int b, int kvh, int t)
{
    CodeWords<W> r;
    const uint32_t* p = c.codes + row_of<PAGED>(c, b, kvh, t) * W;
    if constexpr (W == 2) {
        const uint2 x = *reinterpret_cast<const uint2*>(p);
        r.w[0] = x.x; r.w[1] = x.y;
    } else {
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            const uint4 x = reinterpret_cast<const uint4*>(p)[i];
            r.w[4 * i] = x.x; r.w[4 * i + 1] = x.y; r.w[4 * i + 2] = x.z; r.w[4 * i + 3] = x.w;
        }
    }
    return r;
}

// similarity b - Hamming distance = number of agreeing bits
template <int W>
__device__ __forceinline__ int similarity(const CodeWords<W>& k, const uint32_t* __restrict__ q)
{
    int s = 0;
#pragma unroll
    for (int i = 0; i < W; ++i) s += __popc(~(k.w[i] ^ q[i]));
    return s;
}

// blk_cum rows have 32 W + 2 ints: C(0..b) and a zero, so that "row[T + 1]" is valid for T = b
template <int G, bool PAGED, int W>
__global__ __launch_bounds__(kThreads) void score_hist_wide_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                                   int n_q_heads, int n_cap, int unit_tokens,
                                                                   int n_sink, int n_local, int blocks_pitch,
                                                                   int32_t* __restrict__ blk_cum)
{
    constexpr int kBinsW = bins_of(W), kRow = kBinsW + 1, kCopiesW = copies_of(G, W);
    constexpr int kPerLane = (kRow + kWave - 1) / kWave;          // bins a lane owns in the final scan
    __shared__ unsigned hist[G * kBinsW * kCopiesW];                 // [head][score][copy]
    __shared__ int bsum[G * kRow];
    __shared__ uint32_t qs[G * W];
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);
    const int n = min(c.seq_lens[b], n_cap);
    if ((int64_t)bx * kWpb * unit_tokens >= n) return;
    const int64_t t_begin = ((int64_t)bx * kWpb + wave) * unit_tokens;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);       // only tokens in [lo, hi) are scored
    for (int i = tid; i < G * kBinsW * kCopiesW; i += kThreads) hist[i] = 0u;
    for (int i = tid; i < G * kRow; i += kThreads) bsum[i] = 0;
    if (tid < G * W) qs[tid] = q_codes[((int64_t)b * n_q_heads + kvh * G) * W + tid];
    __syncthreads();

    unsigned* mine = hist + (lane & (kCopiesW - 1));
    const int s_end = min(t_end, hi);                               // scored tokens of this unit: [max(t_begin, lo), s_end)
    // The loads are unconditional (a token past the unit's end repeats the last one, and what is outside
    // the scored range is masked where it is counted): loads under a per-lane condition would make the
    // wave wait for all of them at every step instead of for the oldest only.
    const bool active = t_begin < t_end;                             // uniform over the wave
    auto fetch = [&](int t) {
        CodeWords<W> r;
#pragma unroll
        for (int i = 0; i < W; ++i) r.w[i] = 0u;
        if (active) r = load_code<PAGED, W>(c, b, kvh, min(t, t_end - 1));
        return r;
    };
    constexpr int kDepth = depth_of(W);
    CodeWords<W> ring[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) ring[d] = fetch((int)t_begin + d * kWave + lane);
    for (int64_t base = t_begin; base < t_end; base += kDepth * kWave) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int t = (int)base + d * kWave + lane;
            const CodeWords<W> cur = ring[d];
            ring[d] = load_code<PAGED, W>(c, b, kvh, min(t + kDepth * kWave, t_end - 1));   // refill: kDepth steps ahead
            if (t >= lo && t < s_end) {
#pragma unroll
                for (int j = 0; j < G; ++j)
                    atomicAdd(&mine[(j * kBinsW + similarity<W>(cur, qs + j * W)) * kCopiesW], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < G * kBinsW; i += kThreads) {
        int s = 0;
#pragma unroll
        for (int cp = 0; cp < kCopiesW; ++cp) s += (int)hist[i * kCopiesW + cp];
        bsum[(i / kBinsW) * kRow + i % kBinsW] = s;
    }
    __syncthreads();
    // cumulative counts from the top: lane L owns bins L * kPerLane .. + kPerLane - 1 of head `wave`
    for (int j = wave; j < G; j += kWpb) {
        int h[kPerLane], mine_sum = 0;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int s = lane * kPerLane + i;
            h[i] = s < kBinsW ? bsum[j * kRow + s] : 0;
            mine_sum += h[i];
        }
        const int incl = wave_incl_scan_i32(mine_sum);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        int above = total - incl;                                  // counts of all bins owned by higher lanes
        const int64_t bh = (int64_t)b * n_q_heads + kvh * G + j;
        int32_t* row = blk_cum + (bh * blocks_pitch + bx) * kRow;
#pragma unroll
        for (int i = kPerLane - 1; i >= 0; --i) {
            const int s = lane * kPerLane + i;
            above += h[i];
            if (s < kRow) row[s] = above;                          // slot b + 1 gets 0
        }
    }
}

// Selection parameters of a block, per head, from the per-block rows of cumulative counts (one trip to
// memory, one thread per (head, score)): the threshold thr[j] (largest score s with C(s) >= k), the
// block's first output slot posb[j] and its tie quota quotab[j]; block 0 also stores count and
// threshold.  tot, bef: [G][b + 2] ints of LDS; the others [G].  Every thread of the block calls it.
template <int G, int W>
__device__ __forceinline__ void block_selection(const int32_t* __restrict__ blk_cum, int64_t bh0, int blocks_pitch,
                                                int n_blocks, int bx, int block_tokens, int n, int lo, int hi, int k,
                                                int* tot, int* bef, int* thr, int* posb, int* quotab, int* own_ge_s,
                                                int* own_gt_s, int32_t* __restrict__ count,
                                                uint8_t* __restrict__ threshold)
{
    constexpr int kBinsW = bins_of(W), kRow = kBinsW + 1;
    const int tid = threadIdx.x;
    if (tid < G) { thr[tid] = -1; own_ge_s[tid] = own_gt_s[tid] = 0; }
    // sums over the whole sequence (tot), over the blocks before this one (bef), and this block's own row
    // (kept in registers until the threshold says which two of its entries matter)
    constexpr int kIter = (G * kRow + kThreads - 1) / kThreads;
    int own_r[kIter];
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
        const int i = tid + it * kThreads;
        own_r[it] = 0;
        if (i < G * kRow) {
            const int j = i / kRow, col = i - j * kRow;
            const int32_t* p = blk_cum + (bh0 + j) * blocks_pitch * kRow + col;
            int v = 0, vb = 0;
            for (int blk0 = 0; blk0 < n_blocks; blk0 += 16) {           // sixteen independent loads per trip to memory
                int part[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) part[u] = blk0 + u < n_blocks ? p[(int64_t)(blk0 + u) * kRow] : 0;
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    v += part[u];
                    if (blk0 + u < bx) vb += part[u];
                    if (blk0 + u == bx) own_r[it] = part[u];
                }
            }
            tot[i] = v;
            bef[i] = vb;
        }
    }
    __syncthreads();
    if (k > 0) {                                                         // C(0) = number of scored tokens >= k
        for (int i = tid; i < G * kBinsW; i += kThreads) {
            const int j = i / kBinsW, sc = i - j * kBinsW;
            if (tot[j * kRow + sc] >= k) atomicMax(&thr[j], sc);
        }
    }
    __syncthreads();
    if (k > 0) {
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int i = tid + it * kThreads;
            if (i < G * kRow) {
                const int j = i / kRow, col = i - j * kRow;
                if (col == thr[j]) own_ge_s[j] = own_r[it];
                if (col == thr[j] + 1) own_gt_s[j] = own_r[it];
            }
        }
    }
    __syncthreads();
    if (tid < G) {
        const int j = tid;
        const int64_t bh = bh0 + j;
        const int T = k > 0 ? thr[j] : kBinsW;                           // k = 0: nothing reaches the threshold
        int r = 0, gt = 0, ge = 0, own_eq = 0;
        if (k > 0) {
            r = k - tot[j * kRow + T + 1];                               // slot b + 1 holds 0
            ge = bef[j * kRow + T];                                      // #{score >= T} before this block
            gt = bef[j * kRow + T + 1];
            own_eq = own_ge_s[j] - own_gt_s[j];                          // #{score == T} inside this block
        }
        const int eq_before = ge - gt, left = r - eq_before;
        const int bs = (int)min((int64_t)n, (int64_t)bx * block_tokens);   // always-kept tokens before this block
        thr[j] = T;
        posb[j] = gt + min(eq_before, r) + min(lo, bs) + max(0, bs - hi);
        quotab[j] = left >= own_eq ? kAllTies : max(left, 0);
        if (bx == 0) {
            count[bh] = lo + k + (n - hi);
            if (threshold) threshold[bh] = (uint8_t)(k > 0 ? min(T, 255) : 0);   // saturates for b >= 256
        }
    }
    __syncthreads();
}

template <int G, bool PAGED, int W>
__global__ __launch_bounds__(kThreads) void topk_select_wide_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                                    const int32_t* __restrict__ k_per_seq, int k_max,
                                                                    int n_sink, int n_local, int pitch, int n_q_heads,
                                                                    int n_cap, int unit_tokens, int blocks_pitch,
                                                                    const int32_t* __restrict__ blk_cum,
                                                                    int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                                    uint8_t* __restrict__ threshold)
{
    constexpr int kBinsW = bins_of(W), kRow = kBinsW + 1;
    __shared__ int tot[G * kRow], bef[G * kRow];
    __shared__ int thr[G], posb[G], quotab[G], own_ge_s[G], own_gt_s[G];
    __shared__ int wgt[kWpb][G], weq[kWpb][G];                     // per wave: tokens taken for sure / tied
    __shared__ uint64_t m_gt[kWpb][kMaxSteps][G], m_eq[kWpb][kMaxSteps][G];
    __shared__ uint32_t qs[G * W];
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);
    const int64_t bh0 = (int64_t)b * n_q_heads + kvh * G;
    const int n = min(c.seq_lens[b], n_cap);
    const int k_raw = k_per_seq ? k_per_seq[b] : k_max;
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);
    const int k = max(0, min(k_raw, min(k_max, hi - lo)));
    const bool nothing = k == 0 && lo == 0 && hi == n;
    const int block_tokens = kWpb * unit_tokens;
    if (bx > 0 && ((int64_t)bx * block_tokens >= n || nothing)) return;   // block 0 reports the counts
    const int n_blocks = (n + block_tokens - 1) / block_tokens;
    const int64_t t_begin = ((int64_t)bx * kWpb + wave) * unit_tokens;
    const bool active = t_begin < n && !nothing;
    const int t_end = (int)min((int64_t)n, t_begin + unit_tokens);

    // the first codes are requested before the tables are summed: they are not needed until the
    // threshold is known, and by then they have arrived
    const int n_steps = active ? (t_end - (int)t_begin + kWave - 1) / kWave : 0;
    auto fetch = [&](int t) {                                        // the code of token t (the unit's last one past its end)
        CodeWords<W> r;
#pragma unroll
        for (int i = 0; i < W; ++i) r.w[i] = 0u;
        if (active) r = load_code<PAGED, W>(c, b, kvh, min(t, t_end - 1));   // unconditional, see score_hist_wide_kernel
        return r;
    };
    constexpr int kDepth = depth_of(W);
    CodeWords<W> ring[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) ring[d] = fetch((int)t_begin + d * kWave + lane);

    if (tid < G * W) qs[tid] = q_codes[bh0 * W + tid];
    block_selection<G, W>(blk_cum, bh0, blocks_pitch, n_blocks, bx, block_tokens, n, lo, hi, k, tot, bef, thr, posb, quotab,
                          own_ge_s, own_gt_s, count, threshold);

    // ---- pass 1: score the unit once; masks per 64-token step and head, counts per wave
    // A head whose ties all fit the quota at this block (or whose quota is used up) needs one mask only:
    // "score >= T" (or "> T"); the tie mask is built for a head whose quota ends inside the block.
    // Steps past the unit's end (the step count is rounded up to the ring depth) leave empty masks.
    int T[G], take_from[G], cgt[G], ceq[G];
    bool partial[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        T[j] = uniform(thr[j]);
        const int quota = uniform(quotab[j]);
        take_from[j] = quota == kAllTies ? T[j] : T[j] + 1;
        partial[j] = quota != kAllTies && quota != 0;
        cgt[j] = ceq[j] = 0;
    }
    for (int s0 = 0; s0 < n_steps; s0 += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int s = s0 + d;                                    // < kMaxSteps: units are whole multiples of the depth
            const int t = (int)t_begin + s * kWave + lane;
            const CodeWords<W> kc = ring[d];
            ring[d] = load_code<PAGED, W>(c, b, kvh, min(t + kDepth * kWave, t_end - 1));   // refill: kDepth steps ahead
            const bool valid = t < t_end, scored = valid && t >= lo && t < hi;
#pragma unroll
            for (int j = 0; j < G; ++j) {
                const int sc = similarity<W>(kc, qs + j * W);
                const uint64_t g_mask = __builtin_amdgcn_ballot_w64((scored && sc >= take_from[j]) || (valid && !scored));   // kept tokens are always taken
                const uint64_t e_mask = partial[j] ? __builtin_amdgcn_ballot_w64(scored && sc == T[j]) : 0ull;
                if (lane == 0) { m_gt[wave][s][j] = g_mask; m_eq[wave][s][j] = e_mask; }
                cgt[j] += __popcll(g_mask);
                ceq[j] += __popcll(e_mask);
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < G; ++j) { wgt[wave][j] = cgt[j]; weq[wave][j] = ceq[j]; }
    }
    __syncthreads();
    if (!active) return;

    // ---- pass 2: every lane takes a run of unit_tokens / 64 consecutive tokens (4, 8 or 16), cuts its
    // bits out of the step masks and proceeds as the 32-bit select does: ties are taken in token order
    // while the wave's share of the quota lasts, a wave scan gives the lane's first slot, and the ids
    // go out a few rounds at a time
    const int tpl = unit_tokens >> 6;
    const int run0 = lane * tpl;                                     // first token of the run inside the unit
    const int rs = run0 >> 6, roff = run0 & 63;                      // its step and first bit there
    const unsigned run_bits = rs < n_steps ? (1u << tpl) - 1u : 0u;  // steps never scored hold stale masks
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int gt_before = wave_sum_i32(lane < wave ? wgt[lane][j] : 0);
        const int eq_before = wave_sum_i32(lane < wave ? weq[lane][j] : 0);
        const int quota_b = uniform(quotab[j]);
        const int quota_w = quota_b == kAllTies ? kAllTies : max(0, quota_b - eq_before);
        const int start = uniform(posb[j]) + gt_before + min(eq_before, quota_b);
        unsigned sel = (unsigned)(m_gt[wave][rs][j] >> roff) & run_bits;
        const unsigned tie = (unsigned)(m_eq[wave][rs][j] >> roff) & run_bits;
        if (quota_w == kAllTies) {
            sel |= tie;
        } else if (quota_w > 0) {
            const int mine = __popc(tie);
            const int incl = wave_incl_scan_i32(mine);
            sel |= lowest_bits(tie, max(0, min(mine, quota_w - (incl - mine))));
        }
        const int cnt = __popc(sel);
        const int incl = wave_incl_scan_i32(cnt);
        emit_ids(sel, start + incl - cnt, (int)t_begin + run0, pitch, idx + (bh0 + j) * pitch);
    }
}

// ---------------------------------------------------------------------------------------------
// 64- and 128-bit signatures (W = 2, 4) with units of up to 8 x 16 bytes per lane: the select of the
// 32-bit path carried over.  The wave loads its unit coalesced, transposes it through LDS so that a
// lane holds kTpl consecutive tokens (W words each), and builds a lane's take mask with 2 W + 1
// instructions per token and head (xor and a counting add per word, one funnel shift for the top bit
// of "distance + bias"): no wave ballots, no masks in LDS.  NIT: 16-byte loads per lane.
template <int TPL, int W>
__device__ __forceinline__ unsigned within_mask_words(const uint32_t (&w)[TPL * W], const uint32_t (&q)[W], int lim)
{
    const unsigned bias = 0x7fffffffu - (unsigned)lim;          // top bit of distance + bias: distance > lim
    unsigned m = 0;
#pragma unroll
    for (int p = TPL - 1; p >= 0; --p) {
        unsigned d = bias;
#pragma unroll
        for (int i = 0; i < W; ++i)                              // the count instruction adds its second operand
            asm("v_xor_b32 %0, %2, %1\n\tv_bcnt_u32_b32 %0, %0, %3" : "=&v"(d) : "v"(w[p * W + i]), "s"(q[i]), "v"(d));
        m = __builtin_amdgcn_alignbit(m, d, 31);                 // (m << 1) | top bit of d
    }
    return ~m;
}

template <int TPL, int W>
__device__ __forceinline__ unsigned equal_mask_words(const uint32_t (&w)[TPL * W], const uint32_t (&q)[W], int dist)
{
    unsigned m = 0;
#pragma unroll
    for (int p = TPL - 1; p >= 0; --p) {
        int d = 0;
#pragma unroll
        for (int i = 0; i < W; ++i) d += __popc(w[p * W + i] ^ q[i]);
        m = (m << 1) | (unsigned)(d == dist);
    }
    return m;
}

template <int G, bool PAGED, int W, int NIT>
__global__ __launch_bounds__(kThreads) void topk_select_runs_kernel(KvView c, const uint32_t* __restrict__ q_codes,
                                                                    const int32_t* __restrict__ k_per_seq, int k_max,
                                                                    int n_sink, int n_local, int pitch, int n_q_heads,
                                                                    int n_cap, int blocks_pitch,
                                                                    const int32_t* __restrict__ blk_cum,
                                                                    int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                                    uint8_t* __restrict__ threshold)
{
    constexpr int kBinsW = bins_of(W), kRow = kBinsW + 1, kBitsW = 32 * W;
    constexpr int kPieceTokens = 4 / W;                              // tokens in 16 bytes
    constexpr int kUnit = NIT * kWave * kPieceTokens;                // tokens per wave: 256 NIT / W
    constexpr int kTpl = kUnit / kWave;                              // tokens per lane after the transposition
    static_assert(kTpl >= 4 && kTpl <= 16, "a lane's take mask must fit the emit helpers");
    extern __shared__ uint4 stage_all[];                             // 64 NIT pieces per wave
    __shared__ int tot[G * kRow], bef[G * kRow];
    __shared__ int thr[G], posb[G], quotab[G], own_ge_s[G], own_gt_s[G];
    __shared__ int wgt[kWpb][G], weq[kWpb][G];
    __shared__ uint32_t qs[G * W];
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int bx = rotated_block(blockIdx.x, kvh + b, gridDim.x);
    const int64_t bh0 = (int64_t)b * n_q_heads + kvh * G;
    const int n = min(c.seq_lens[b], n_cap);
    const int k_raw = k_per_seq ? k_per_seq[b] : k_max;
    const int lo = min(n_sink, n), hi = max(lo, n - n_local);
    const int k = max(0, min(k_raw, min(k_max, hi - lo)));
    const bool nothing = k == 0 && lo == 0 && hi == n;
    constexpr int block_tokens = kWpb * kUnit;
    if (bx > 0 && ((int64_t)bx * block_tokens >= n || nothing)) return;   // block 0 reports the counts
    const int n_blocks = (n + block_tokens - 1) / block_tokens;
    const int64_t t_begin = ((int64_t)bx * kWpb + wave) * kUnit;
    const bool active = t_begin < n && !nothing;
    const int t_end = (int)min((int64_t)n, t_begin + kUnit);

    // the unit's codes, coalesced: piece it * 64 + lane holds tokens t_begin + piece * kPieceTokens ..; a
    // piece past the end repeats the last one (masked below), so the loads are unconditional
    uint4 cw[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) cw[it] = make_uint4(0u, 0u, 0u, 0u);
    if (active) {
        const int last = (t_end - 1) & ~(kPieceTokens - 1);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int t = min((int)t_begin + (it * kWave + lane) * kPieceTokens, last);
            cw[it] = *reinterpret_cast<const uint4*>(c.codes + row_of<PAGED>(c, b, kvh, t) * W);
        }
    }

    if (tid < G * W) qs[tid] = q_codes[bh0 * W + tid];
    block_selection<G, W>(blk_cum, bh0, blocks_pitch, n_blocks, bx, block_tokens, n, lo, hi, k, tot, bef, thr, posb, quotab,
                          own_ge_s, own_gt_s, count, threshold);

    // ---- lane runs and masks
    unsigned sel[G], tie[G];
    int quota[G];
#pragma unroll
    for (int j = 0; j < G; ++j) { sel[j] = tie[j] = 0u; quota[j] = uniform(quotab[j]); }
    if (active) {
        uint32_t w[kTpl * W];
        uint4* stage = stage_all + wave * (kWave * NIT);
#pragma unroll
        for (int it = 0; it < NIT; ++it) stage[it * kWave + lane] = cw[it];     // piece p belongs to lane p / NIT
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int i = 0; i < NIT; ++i) {
            const uint4 x = stage[lane * NIT + i];
            w[4 * i] = x.x; w[4 * i + 1] = x.y; w[4 * i + 2] = x.z; w[4 * i + 3] = x.w;
        }
        const int first = (int)t_begin + lane * kTpl;                              // first token of this lane's run
        auto below = [&](int t) { return (1u << max(0, min(t - first, kTpl))) - 1u; };   // bits of tokens < t
        const unsigned valid = below(t_end);
        const unsigned scored = below(hi) & ~below(lo) & valid;
        const unsigned kept = valid & ~scored;
#pragma unroll
        for (int j = 0; j < G; ++j) {
            uint32_t q[W];
#pragma unroll
            for (int i = 0; i < W; ++i) q[i] = (uint32_t)uniform((int)qs[j * W + i]);
            const int T = uniform(thr[j]);
            const int lim = quota[j] == kAllTies ? kBitsW - T : kBitsW - T - 1;   // bound on the Hamming distance
            sel[j] = (within_mask_words<kTpl, W>(w, q, lim) & scored) | kept;
            if (quota[j] != kAllTies && quota[j] != 0) tie[j] = equal_mask_words<kTpl, W>(w, q, kBitsW - T) & scored;
        }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int cs = wave_sum_i32(__popc(sel[j]));
        const int es = wave_sum_i32(__popc(tie[j]));
        if (lane == 0) { wgt[wave][j] = cs; weq[wave][j] = es; }
    }
    __syncthreads();
    if (!active) return;

    // ---- ranks and ids (ties in token order while the wave's share of the quota lasts)
    const int first = (int)t_begin + lane * kTpl;
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int gt_before = wave_sum_i32(lane < wave ? wgt[lane][j] : 0);
        const int eq_before = wave_sum_i32(lane < wave ? weq[lane][j] : 0);
        const int quota_w = quota[j] == kAllTies ? kAllTies : max(0, quota[j] - eq_before);
        const int start = uniform(posb[j]) + gt_before + min(eq_before, quota[j] == kAllTies ? 0 : quota[j]);
        unsigned take = sel[j];
        if (quota_w != kAllTies && quota_w > 0) {
            const int mine = __popc(tie[j]);
            const int incl = wave_incl_scan_i32(mine);
            take |= lowest_bits(tie[j], max(0, min(mine, quota_w - (incl - mine))));
        }
        const int cnt = __popc(take);
        const int incl = wave_incl_scan_i32(cnt);
        emit_ids(take, start + incl - cnt, first, pitch, idx + (bh0 + j) * pitch);
    }
}

// The lane-run select: launch (or, with setup_only, raise the dynamic LDS limit of) the variant
// with NIT 16-byte loads per lane.
template <int G, bool PAGED, int W, int NIT>
hipError_t select_runs(bool setup_only, const KvView& kv, const TopkCall& a, const TopkScratch& sc, dim3 grid,
                       hipStream_t stream)
{
    constexpr int lds = kWpb * kWave * NIT * (int)sizeof(uint4);
    if (setup_only)
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&topk_select_runs_kernel<G, PAGED, W, NIT>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    topk_select_runs_kernel<G, PAGED, W, NIT><<<grid, dim3(kThreads), lds, stream>>>(
        kv, a.q_codes, a.k_per_seq, a.k_max, a.n_sink, a.n_local, a.k_max + a.n_sink + a.n_local, a.n_q_heads,
        a.max_seq_len, sc.blocks_pitch, sc.blk_cum, a.idx, a.count, a.threshold);
    return hipSuccess;
}

// true if a lane-run variant serves (W, unit_tokens): up to eight 16-byte loads per lane, i.e. 64 bits in
// all unit sizes and 128 bits in units of up to 512 tokens.  (128 bits with two chunks per unit of 1024
// tokens measured much slower than the step-mask select: 107 against 70 us at 16 x 128K tokens.)
template <int G, bool PAGED, int W>
bool select_runs_by_unit(bool setup_only, int unit_tokens, const KvView& kv, const TopkCall& a, const TopkScratch& sc,
                         dim3 grid, hipStream_t stream, hipError_t* e)
{
    *e = hipSuccess;
    if constexpr (W == 2 || W == 4) {
        switch (unit_tokens * W / 256) {
        case 2: if constexpr (W == 2) { *e = select_runs<G, PAGED, W, 2>(setup_only, kv, a, sc, grid, stream); return true; } break;
        case 4: *e = select_runs<G, PAGED, W, 4>(setup_only, kv, a, sc, grid, stream); return true;
        case 8: *e = select_runs<G, PAGED, W, 8>(setup_only, kv, a, sc, grid, stream); return true;
        default: break;
        }
    }
    return false;
}

template <int G, bool PAGED, int W>
hipError_t launch_w(bool setup_only, const KvView& kv, const TopkCall& a, int unit_tokens, const TopkScratch& sc,
                    hipStream_t stream)
{
    if (setup_only) {
        hipError_t e = hipSuccess;
        for (int unit = 256; unit <= 1024; unit *= 2)
            if (select_runs_by_unit<G, PAGED, W>(true, unit, kv, a, sc, dim3(1), stream, &e) && e != hipSuccess) return e;
        return hipSuccess;
    }
    const int64_t block_tokens = (int64_t)kWpb * unit_tokens;
    int n_blocks = (int)((a.max_seq_len + block_tokens - 1) / block_tokens);
    if (n_blocks < 1) n_blocks = 1;
    const dim3 grid(n_blocks, kv.n_kv_heads, a.batch), block(kThreads);
    score_hist_wide_kernel<G, PAGED, W><<<grid, block, 0, stream>>>(kv, a.q_codes, a.n_q_heads, a.max_seq_len, unit_tokens,
                                                                   a.n_sink, a.n_local, sc.blocks_pitch, sc.blk_cum);
    hipError_t e = hipSuccess;
    if (select_runs_by_unit<G, PAGED, W>(false, unit_tokens, kv, a, sc, grid, stream, &e))
        return e != hipSuccess ? e : hipGetLastError();
    topk_select_wide_kernel<G, PAGED, W><<<grid, block, 0, stream>>>(
        kv, a.q_codes, a.k_per_seq, a.k_max, a.n_sink, a.n_local, a.k_max + a.n_sink + a.n_local, a.n_q_heads,
        a.max_seq_len, unit_tokens, sc.blocks_pitch, sc.blk_cum, a.idx, a.count, a.threshold);
    return hipGetLastError();
}

template <int G, bool PAGED>
hipError_t launch_words(bool setup_only, int words, const KvView& kv, const TopkCall& a, int unit_tokens,
                        const TopkScratch& sc, hipStream_t stream)
{
    switch (words) {
    case 2: return launch_w<G, PAGED, 2>(setup_only, kv, a, unit_tokens, sc, stream);
    case 4: return launch_w<G, PAGED, 4>(setup_only, kv, a, unit_tokens, sc, stream);
    case 8: return launch_w<G, PAGED, 8>(setup_only, kv, a, unit_tokens, sc, stream);
    case 16: return launch_w<G, PAGED, 16>(setup_only, kv, a, unit_tokens, sc, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int G>
hipError_t launch_group(bool setup_only, bool paged, int words, const KvView& kv, const TopkCall& a, int unit_tokens,
                        const TopkScratch& sc, hipStream_t stream)
{
    if (setup_only) {
        if (hipError_t e = launch_words<G, false>(true, words, kv, a, unit_tokens, sc, stream); e != hipSuccess) return e;
        return launch_words<G, true>(true, words, kv, a, unit_tokens, sc, stream);
    }
    return paged ? launch_words<G, true>(false, words, kv, a, unit_tokens, sc, stream)
                 : launch_words<G, false>(false, words, kv, a, unit_tokens, sc, stream);
}

hipError_t dispatch_wide(bool setup_only, bool paged, int group, int words, const KvView& kv, const TopkCall& call,
                         int unit_tokens, const TopkScratch& sc, hipStream_t stream)
{
    switch (group) {
    case 1: return launch_group<1>(setup_only, paged, words, kv, call, unit_tokens, sc, stream);
    case 2: return launch_group<2>(setup_only, paged, words, kv, call, unit_tokens, sc, stream);
    case 4: return launch_group<4>(setup_only, paged, words, kv, call, unit_tokens, sc, stream);
    case 8: return launch_group<8>(setup_only, paged, words, kv, call, unit_tokens, sc, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Raises the dynamic LDS limit of the lane-run select kernels of this group size and width (their staging
// area reaches 64 KiB); called once when a context is created, never on the launch path.
hipError_t setup_score_topk_wide(int group, int words)
{
    return dispatch_wide(true, false, group, words, KvView{}, TopkCall{}, 0, TopkScratch{}, nullptr);
}

// unit_tokens: 256, 512 or 1024
hipError_t launch_score_topk_wide(const KvView& kv, bool paged, int group, int words, const TopkCall& call,
                                  int unit_tokens, const TopkScratch& sc, hipStream_t stream)
{
    if (unit_tokens > kMaxSteps * kWave) return hipErrorInvalidValue;
    return dispatch_wide(false, paged, group, words, kv, call, unit_tokens, sc, stream);
}

}  // namespace ha
