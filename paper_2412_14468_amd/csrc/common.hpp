// Device-side helpers shared by the HashAttention kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ha {

constexpr int kHeadDim = 128;     // bf16 elements per K/V row (256 bytes)
constexpr int kBits = 32;         // signature width
constexpr int kBins = 33;         // Hamming similarity takes values 0..32
constexpr int kCumRow = 34;       // row of cumulative score counts: bins 0..32 and a zero slot
constexpr int kPage = 16;         // tokens per page in the paged layout
constexpr int kWave = 64;
constexpr int kTopkWavesPerBlock = 8;    // SCORE/TOPK: units (waves) per block
constexpr int kMaxTopkBlocks = 256;      // SCORE/TOPK: most blocks per sequence (every block sums the per-block tables)
constexpr int kPartStride = 132;  // floats per split partial: acc[128], m, l, pad

// Plain view of the caller's KV cache, passed to kernels by value.
struct KvView {
    const uint16_t* k;
    const uint16_t* v;
    uint32_t* codes;
    const int32_t* page_table;
    int32_t* seq_lens;
    int64_t n_max;
    int32_t max_pages_per_seq;
    int32_t n_kv_heads;
};

// Row index (in rows) of token t of sequence b, KV head h.
template <bool PAGED>
__device__ __forceinline__ int64_t row_of(const KvView& c, int b, int h, int t)
{
    if constexpr (PAGED) {
        const int64_t page = c.page_table[(int64_t)b * c.max_pages_per_seq + (t >> 4)];
        return (page * c.n_kv_heads + h) * kPage + (t & (kPage - 1));
    } else {
        return ((int64_t)b * c.n_kv_heads + h) * c.n_max + t;
    }
}

// The same in two steps, for callers that fetch the page-table entry ahead of time
// (0 when the cache is contiguous).
template <bool PAGED>
__device__ __forceinline__ int page_of(const KvView& c, int b, int t)
{
    if constexpr (PAGED) return c.page_table[(int64_t)b * c.max_pages_per_seq + (t >> 4)];
    else return 0;
}

template <bool PAGED>
__device__ __forceinline__ int64_t row_in_page(const KvView& c, int b, int h, int t, int page)
{
    if constexpr (PAGED) return ((int64_t)page * c.n_kv_heads + h) * kPage + (t & (kPage - 1));
    else return ((int64_t)b * c.n_kv_heads + h) * c.n_max + t;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float silu(float z) { return z / (1.f + expf(-z)); }

// fp32 -> bf16 bits, round to nearest even (inputs are finite here).
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Unpack 8 bf16 (one 16-byte load) to fp32.
__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[8])
{
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x);
    f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z);
    f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

// DPP rotate inside a 16-lane row (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_f<0x128>(x);   // row_ror:8
    x += dpp_f<0x124>(x);   // row_ror:4
    x += dpp_f<0x122>(x);   // row_ror:2
    x += dpp_f<0x121>(x);   // row_ror:1
    return x;
}

template <int CTRL>
__device__ __forceinline__ int dpp_i(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);    // lanes shifted in from outside read 0
}

// Sum over the 64 lanes; every lane gets the total.  DPP inside 16-lane rows, readlane across rows.
__device__ __forceinline__ int wave_sum_i32(int x)
{
    x += dpp_i<0x128>(x);   // row_ror:8
    x += dpp_i<0x124>(x);   // row_ror:4
    x += dpp_i<0x122>(x);   // row_ror:2
    x += dpp_i<0x121>(x);   // row_ror:1
    return (__builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16)) +
           (__builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48));
}

// Inclusive prefix sum over the 64 lanes (lane i gets x_0 + ... + x_i).
__device__ __forceinline__ int wave_incl_scan_i32(int x)
{
    x += dpp_i<0x111>(x);   // row_shr:1
    x += dpp_i<0x112>(x);   // row_shr:2
    x += dpp_i<0x114>(x);   // row_shr:4
    x += dpp_i<0x118>(x);   // row_shr:8
    const int r0 = __builtin_amdgcn_readlane(x, 15), r1 = __builtin_amdgcn_readlane(x, 31),
              r2 = __builtin_amdgcn_readlane(x, 47);
    const int row = (int)(threadIdx.x & 63) >> 4;
    return x + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// Number of set bits of a wave mask in lanes below the calling lane.
__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                          __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// The lowest `take` set bits of x.
__device__ __forceinline__ unsigned lowest_bits(unsigned x, int take)
{
    unsigned r = 0;
    for (int i = 0; i < take && x; ++i) {
        const unsigned low = x & (0u - x);
        r |= low;
        x ^= low;
    }
    return r;
}

// Token ids of the set bits of m (bit p = token t0 + p), written to out[rank], out[rank + 1], ...
// At 1/32 density a lane rarely holds more than three of its sixteen tokens: three rounds without a
// branch (a lane with nothing left just does not store), then a loop for the rest.  Ranks stay below
// the row's pitch when the counts that produced them match the codes; a mask that would pass it is cut
// to the room that is left, once, so that the rounds need no check of their own.  `out` is the same
// for the whole wave.
__device__ __forceinline__ void emit_ids(unsigned m, int rank, int t0, int pitch, int32_t* __restrict__ out)
{
    const int room = pitch - rank;
    if (__builtin_amdgcn_ballot_w64(__popc(m) > room) != 0ull) m = lowest_bits(m, max(room, 0));
    int32_t* p = out + (unsigned)max(rank, 0);          // the lane's ids go to p[0], p[1], ...: one address, constant offsets
    const unsigned m1 = m & (m - 1u), m2 = m1 & (m1 - 1u);        // m without its lowest one / two set bits; 0 stays 0
    if (m != 0u) p[0] = t0 + (__ffs((int)m) - 1);
    if (m1 != 0u) p[1] = t0 + (__ffs((int)m1) - 1);
    if (m2 != 0u) p[2] = t0 + (__ffs((int)m2) - 1);
    m = m2 & (m2 - 1u);
    p += 3;
    while (__builtin_amdgcn_ballot_w64(m != 0u) != 0ull) {
        if (m != 0u) *p++ = t0 + (__ffs((int)m) - 1);
        m &= m - 1u;
    }
}

// Workgroups go to the eight XCDs round-robin in launch order, x fastest.  With the piece index
// of a (sequence, head) in blockIdx.x and a piece count that divides (or is divided by) eight,
// piece p of every list would land on the same XCD, and in a batch of mixed lengths the high
// pieces exist for long sequences only.  Rotating by the list's index spreads them.
__device__ __forceinline__ int rotated_block(unsigned x, int list, int n)
{
    return (int)((x + (unsigned)list) % (unsigned)n);
}

}  // namespace ha
