// GATHER-ATT (section 4) and dense single-query SDPA (section 3.1) for gfx950.
//
// Both are split-K flash-decode kernels: the token list of one (sequence, head)
// is cut into splits; a block keeps an online-softmax state (running max m,
// running sum l, fp32 accumulator) per 16-lane row group, merges its 16 states
// through LDS and writes one partial (acc[128], m, l).  A second, small kernel
// merges the partials of a head and rounds to bf16.  Short lists with many heads
// skip the split: one 16-wave block per head writes the output itself (with few
// heads that is slower: one CU pulls only about 30 GB/s of scattered rows).
// Merging in the block that finishes last was measured and dropped: the
// device-scope release/acquire it needs writes back and invalidates the XCD's
// whole L2 in every block, which cost far more than the extra launch.
//
// A K or V row is 128 bf16 = 256 bytes = 16 lanes x 16 bytes, so one wave load
// instruction fetches four rows; the <q, k> reduction runs inside a 16-lane DPP
// row.  Each row group works on 4 rows at a time; list entry, page-table entry
// and row loads of successive iterations run as a pipeline (see the kernel), so
// a block keeps up to 64 KiB of rows in flight.  The piece of the list a block
// takes is rotated by the list's index, which spreads the pieces of lists of
// different lengths over the XCDs.  The work is HBM bound (about one flop per
// byte), so there is no MFMA here.  Logits are kept in log2 units (scale *
// log2(e) folded into q) so that exp2 is the only transcendental.
#include "kernels.hpp"

#include <math.h>
#include <mutex>

// Split partials of hashattn_gather_attend_noalloc, the entry point for callers that cannot allocate:
// 8 MiB of device memory that every GPU the library runs on holds until the process ends.  Host code
// never uses this name as an address: it asks the runtime for the array's address on the current
// device (static_partials below) and passes that pointer to the kernels.
constexpr int64_t kStaticPartFloats = 2 * 1024 * 1024;
static __device__ __align__(256) float scratch[kStaticPartFloats];

namespace ha {

namespace {

constexpr int kDirectRows = 1024;  // lists up to this long can be handled by one 16-wave block per head ...
constexpr int kDirectMinHeads = 128;   // ... when there are at least this many (sequence, head) pairs
constexpr int kMaxSplits = 256;
constexpr float kNegInf = -INFINITY;

// 16 bytes of a K or V row.  A row is read once per step and never again before the caches have turned
// over, so the load carries the non-temporal hint: measured 3-11 % faster GATHER-ATT than plain loads.
__device__ __forceinline__ uint4 load_row16(const uint16_t* base, int64_t row, int sub)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + row * kHeadDim + sub * 8));
    return make_uint4(x.x, x.y, x.z, x.w);
}

// Online-softmax update of one row group with 4 rows (logits x in log2 units, -inf = no row).
__device__ __forceinline__ void absorb4(const float (&x)[4], const uint4 (&vr)[4], float& m, float& l,
                                        float (&acc)[8])
{
    const float m_new = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), m);
    const float ref = (m_new == kNegInf) ? 0.f : m_new;      // a group may have seen no valid row yet
    const float alpha = exp2f(m - ref);
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = exp2f(x[i] - ref);
    l = l * alpha + (p[0] + p[1]) + (p[2] + p[3]);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float vf[8];
        unpack8(vr[i], vf);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(p[i], vf[e], acc[e]);
    }
    m = m_new;
}

__device__ __forceinline__ float dot8_row16(const float (&qf)[8], const uint4& kr)
{
    float kf[8];
    unpack8(kr, kf);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) d = fmaf(qf[e], kf[e], d);
    return row16_sum(d);
}

// Merge the SLOTS per-group states of a block (st: [SLOTS][kPartStride] floats in LDS, already
// filled and synchronised).  Threads 0..127 get their channel's weighted sum, thread 129 the weighted
// sum of l; M is the block's running max (all in the returned struct, valid for tid < 130).
struct BlockState { float sum, M; };

template <int SLOTS>
__device__ __forceinline__ BlockState merge_slots(const float* st)
{
    const int tid = threadIdx.x;
    BlockState r{0.f, kNegInf};
    if (tid < kHeadDim + 2) {
#pragma unroll 8
        for (int s = 0; s < SLOTS; ++s) r.M = fmaxf(r.M, st[s * kPartStride + kHeadDim]);
        const float Ms = (r.M == kNegInf) ? 0.f : r.M;
        const int col = tid < kHeadDim ? tid : kHeadDim + 1;      // channel, or the l column
#pragma unroll 8
        for (int s = 0; s < SLOTS; ++s)
            r.sum += st[s * kPartStride + col] * exp2f(st[s * kPartStride + kHeadDim] - Ms);
    }
    return r;
}

// Write the block's partial (acc[128], m, l).
template <int SLOTS>
__device__ __forceinline__ void write_partial(const float* st, float* part)
{
    const int tid = threadIdx.x;
    const BlockState r = merge_slots<SLOTS>(st);
    if (tid < kHeadDim) part[tid] = r.sum;
    else if (tid == kHeadDim) part[kHeadDim] = r.M;
    else if (tid == kHeadDim + 1) part[kHeadDim + 1] = r.sum;
}

// The block holds the whole token list of its head: normalise and round to bf16 directly.
// red: one float of LDS outside st.
template <int SLOTS>
__device__ __forceinline__ void write_output(const float* st, float* red, uint16_t* out)
{
    const int tid = threadIdx.x;
    const BlockState r = merge_slots<SLOTS>(st);
    if (tid == kHeadDim + 1) *red = r.sum;
    __syncthreads();
    if (tid < kHeadDim) {
        const float den = *red;
        out[tid] = (uint16_t)f32_to_bf16(den > 0.f ? r.sum / den : 0.f);
    }
}

// Whole block: out = sum_s acc_s 2^(m_s - M) / sum_s l_s 2^(m_s - M) over the first `used` of the
// n_slots partials, to bf16; used = min(n_slots, ceil(min(*len_ptr, len_cap) / chunk)).
// All n_slots slots are memory of the scratch buffer, so m, l and the first sixteen partials are
// requested before the length has arrived (one trip to memory instead of three); what lies past
// `used` may be stale and is masked, never multiplied.
// lds: at least 2 * kMaxSplits + 8 floats.  Every thread of the block must call it.
__device__ __forceinline__ void merge_partials_block(const float* __restrict__ p, int n_slots,
                                                     const int32_t* __restrict__ len_ptr, int len_cap, int chunk,
                                                     uint16_t* __restrict__ out, float* lds)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* w = lds;                       // [kMaxSplits] weights 2^(m_s - M)
    float* red = lds + kMaxSplits;        // [8]
    float* half = lds + kMaxSplits + 8;   // [128]
    const int ch = tid & (kHeadDim - 1), h = tid >> 7;       // two thread halves take alternate partials
    const int len_raw = *len_ptr;
    float my_m = kNegInf, my_l = 0.f;
    if (tid < n_slots) {
        my_m = p[tid * kPartStride + kHeadDim];
        my_l = p[tid * kPartStride + kHeadDim + 1];
    }
    float v0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int s = h + 2 * u;
        v0[u] = s < n_slots ? p[s * kPartStride + ch] : 0.f;
    }
    const int used = min(n_slots, (min(len_raw, len_cap) + chunk - 1) / chunk);
    if (tid >= used) { my_m = kNegInf; my_l = 0.f; }

    float M = my_m;
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, kWave));
    if (lane == 0) red[wave] = M;
    __syncthreads();
    M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float my_w = (tid < used && M != kNegInf) ? exp2f(my_m - M) : 0.f;
    if (tid < kMaxSplits) w[tid] = my_w;
    float den = my_l * my_w;
    for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o, kWave);
    if (lane == 0) red[4 + wave] = den;
    __syncthreads();
    den = (red[4] + red[5]) + (red[6] + red[7]);

    float num = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int s = h + 2 * u;
        if (s < used) num = fmaf(v0[u], w[s], num);
    }
    int s = h + 16;
#pragma unroll 1
    for (; s + 14 < used; s += 16) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(s + 2 * u) * kPartStride + ch];
#pragma unroll
        for (int u = 0; u < 8; ++u) num = fmaf(v[u], w[s + 2 * u], num);
    }
    for (; s < used; s += 2) num = fmaf(p[s * kPartStride + ch], w[s], num);
    if (h == 1) half[ch] = num;
    __syncthreads();
    if (h == 0) {
        num += half[ch];
        const float o = den > 0.f ? num / den : 0.f;
        out[ch] = (uint16_t)f32_to_bf16(o);
    }
}

// WAVES waves per block; every 16-lane group ("slot") owns rows slot, slot + SLOTS, ... of the block's
// share of the list.  DIRECT: one block per (sequence, head) takes the whole list and writes the bf16
// output itself (short lists: no partials, no second launch).
template <bool PAGED, int WAVES, bool DIRECT>
__global__ __launch_bounds__(WAVES * 64) void gather_attend_kernel(KvView c, const uint16_t* __restrict__ q,
                                                                   const int32_t* __restrict__ idx,
                                                                   const int32_t* __restrict__ count,
                                                                   int n_q_heads, int group, int k_max, int chunk,
                                                                   int n_splits, float scale_log2e,
                                                                   float* __restrict__ part,
                                                                   uint16_t* __restrict__ out)
{
    constexpr int kSlots = WAVES * 4, kRowsPerIter = kSlots * 4;
    __shared__ float st[kSlots * kPartStride];
    __shared__ float red;
    const int tid = threadIdx.x, lane = tid & 63, sub = lane & 15;
    const int slot = tid >> 4;                       // 0..kSlots-1
    const int hq = blockIdx.y, b = blockIdx.z, kvh = hq / group;
    const int split = rotated_block(blockIdx.x, hq + b, n_splits);
    const int64_t bh = (int64_t)b * n_q_heads + hq;
    const int32_t* my_idx = idx + bh * k_max;
    const int begin = split * chunk;

    // Three loads chain up for a row: its list entry, (paged) the page-table entry of that token,
    // the row itself.  They run as a pipeline over the iterations: while rows i are consumed, rows
    // i+1 are in flight, page entries i+2 have been asked for and list entries i+3 are requested,
    // so no iteration waits on a load it has issued itself.  Loads complete in issue order, which
    // is why every iteration issues the small loads before the rows.
    // The first list loads do not wait for the count: entries past it are valid memory, their
    // contents are only used once known to be below the count.
    auto list_at = [&](int r) { return my_idx[min(r, k_max - 1)]; };
    int tok0[4], tok1[4], tok2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = begin + i * kSlots + slot;
        tok0[i] = list_at(r);
        tok1[i] = list_at(r + kRowsPerIter);
        tok2[i] = list_at(r + 2 * kRowsPerIter);
    }
    const int cnt = min(count[bh], k_max);
    const uint4 qraw = *reinterpret_cast<const uint4*>(q + bh * kHeadDim + sub * 8);
    if (begin >= cnt) {
        if (DIRECT && tid < kHeadDim) out[bh * kHeadDim + tid] = 0;   // empty list: zero row
        return;                                      // split mode: the merge kernel skips unused splits
    }
    const int end = DIRECT ? cnt : min(begin + chunk, cnt);

    float qf[8];
    unpack8(qraw, qf);
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[i] *= scale_log2e;

    float m = kNegInf, l = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
    uint4 kr[4], vr[4];
    bool ok[4], ok1[4];
    int pg1[4];                                      // page entries of the rows one iteration ahead
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = begin + i * kSlots + slot;
        ok[i] = r < end;
        ok1[i] = r + kRowsPerIter < end;
        const int pg0 = ok[i] ? page_of<PAGED>(c, b, tok0[i]) : 0;
        pg1[i] = ok1[i] ? page_of<PAGED>(c, b, tok1[i]) : 0;
        kr[i] = zero4;
        vr[i] = zero4;
        if (ok[i]) {
            const int64_t row = row_in_page<PAGED>(c, b, kvh, tok0[i], pg0);
            kr[i] = load_row16(c.k, row, sub);
            vr[i] = load_row16(c.v, row, sub);
        }
    }
    for (int base = begin; base < end; base += kRowsPerIter) {
        int pg2[4], tok3[4];
        bool ok2[4];
        uint4 kn[4], vn[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = base + i * kSlots + slot;
            ok2[i] = r + 2 * kRowsPerIter < end;
            pg2[i] = ok2[i] ? page_of<PAGED>(c, b, tok2[i]) : 0;
            tok3[i] = r + 3 * kRowsPerIter < end ? my_idx[r + 3 * kRowsPerIter] : 0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kn[i] = zero4;
            vn[i] = zero4;
            if (ok1[i]) {
                const int64_t row = row_in_page<PAGED>(c, b, kvh, tok1[i], pg1[i]);
                kn[i] = load_row16(c.k, row, sub);
                vn[i] = load_row16(c.v, row, sub);
            }
        }
        float x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float d = dot8_row16(qf, kr[i]);
            x[i] = ok[i] ? d : kNegInf;
        }
        absorb4(x, vr, m, l, acc);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kr[i] = kn[i]; vr[i] = vn[i];
            ok[i] = ok1[i]; ok1[i] = ok2[i];
            tok1[i] = tok2[i]; tok2[i] = tok3[i];
            pg1[i] = pg2[i];
        }
    }

    // a group that saw no valid row keeps m = -inf, l = 0 (possible when end - begin < 16)
    float* mine = st + slot * kPartStride;
#pragma unroll
    for (int e = 0; e < 8; ++e) mine[sub * 8 + e] = acc[e];
    if (sub == 0) { mine[kHeadDim] = m; mine[kHeadDim + 1] = l; }
    __syncthreads();
    if constexpr (DIRECT) write_output<kSlots>(st, &red, out + bh * kHeadDim);
    else write_partial<kSlots>(st, part + (bh * n_splits + split) * kPartStride);
}

// Dense decode: the block walks a contiguous token range of one KV head and serves
// the G query heads of the group from one read of every K/V row.
template <int G, bool PAGED>
__global__ __launch_bounds__(256) void dense_attend_kernel(KvView c, const uint16_t* __restrict__ q,
                                                           int n_q_heads, int n_cap, int chunk, int n_splits,
                                                           float scale_log2e, float* __restrict__ part)
{
    constexpr int kSlots = 16, kRowsPerIter = 64;    // 4 waves x 4 row groups, 4 rows per group and iteration
    __shared__ float st[kSlots * kPartStride];
    const int tid = threadIdx.x, lane = tid & 63, sub = lane & 15;
    const int slot = tid >> 4;
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int split = rotated_block(blockIdx.x, kvh + b, n_splits);
    const int n = min(c.seq_lens[b], n_cap);
    const int begin = split * chunk;
    const int64_t bh0 = (int64_t)b * n_q_heads + kvh * G;
    if (begin >= n) return;
    const int end = min(begin + chunk, n);

    float qf[G][8], acc[G][8], m[G], l[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        unpack8(*reinterpret_cast<const uint4*>(q + (bh0 + j) * kHeadDim + sub * 8), qf[j]);
        m[j] = kNegInf;
        l[j] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { qf[j][e] *= scale_log2e; acc[j][e] = 0.f; }
    }

    // rows one iteration ahead, their page-table entries two ahead (see gather_attend_kernel)
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
    uint4 kr[4], vr[4];
    bool ok[4], ok1[4];
    int pg1[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = begin + i * kSlots + slot;
        ok[i] = t < end;
        ok1[i] = t + kRowsPerIter < end;
        const int pg0 = ok[i] ? page_of<PAGED>(c, b, t) : 0;
        pg1[i] = ok1[i] ? page_of<PAGED>(c, b, t + kRowsPerIter) : 0;
        kr[i] = zero4;
        vr[i] = zero4;
        if (ok[i]) {
            const int64_t row = row_in_page<PAGED>(c, b, kvh, t, pg0);
            kr[i] = load_row16(c.k, row, sub);
            vr[i] = load_row16(c.v, row, sub);
        }
    }
    for (int base = begin; base < end; base += kRowsPerIter) {
        uint4 kn[4], vn[4];
        bool ok2[4];
        int pg2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = base + 2 * kRowsPerIter + i * kSlots + slot;
            ok2[i] = t < end;
            pg2[i] = ok2[i] ? page_of<PAGED>(c, b, t) : 0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int t = base + kRowsPerIter + i * kSlots + slot;
            kn[i] = zero4;
            vn[i] = zero4;
            if (ok1[i]) {
                const int64_t row = row_in_page<PAGED>(c, b, kvh, t, pg1[i]);
                kn[i] = load_row16(c.k, row, sub);
                vn[i] = load_row16(c.v, row, sub);
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            float x[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float d = dot8_row16(qf[j], kr[i]);
                x[i] = ok[i] ? d : kNegInf;
            }
            absorb4(x, vr, m[j], l[j], acc[j]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kr[i] = kn[i]; vr[i] = vn[i];
            ok[i] = ok1[i]; ok1[i] = ok2[i];
            pg1[i] = pg2[i];
        }
    }

    float* mine = st + slot * kPartStride;
#pragma unroll
    for (int j = 0; j < G; ++j) {
        if (j > 0) __syncthreads();                  // st is reused head after head
#pragma unroll
        for (int e = 0; e < 8; ++e) mine[sub * 8 + e] = acc[j][e];
        if (sub == 0) { mine[kHeadDim] = m[j]; mine[kHeadDim + 1] = l[j]; }
        __syncthreads();
        write_partial<kSlots>(st, part + ((bh0 + j) * n_splits + split) * kPartStride);
    }
}

// Merge the split partials of one (sequence, query head).  lens: per head (count, PER_HEAD) or per
// sequence (seq_lens); splits beyond ceil(len / chunk) were not written.  len = 0 gives a zero row.
template <bool PER_HEAD>
__global__ __launch_bounds__(256) void merge_partials_kernel(const float* __restrict__ part,
                                                             const int32_t* __restrict__ lens, int len_cap,
                                                             int n_q_heads, int chunk, int n_splits,
                                                             uint16_t* __restrict__ out)
{
    __shared__ float lds[2 * kMaxSplits + 8];
    const int hq = blockIdx.x, b = blockIdx.y;
    const int64_t bh = (int64_t)b * n_q_heads + hq;
    merge_partials_block(part + bh * n_splits * kPartStride, n_splits, PER_HEAD ? lens + bh : lens + b, len_cap, chunk,
                         out + bh * kHeadDim, lds);
}

constexpr float kLog2e = 1.4426950408889634f;

}  // namespace

// Address and size (in floats) of the static partials array on the current device.  The address is
// looked up once per device (every GPU has its own copy of the array at its own address) and kept.
hipError_t static_partials(float** ptr, int64_t* n_floats)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static float* per_device[kMaxDevices] = {};
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        float* p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)); e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    *n_floats = kStaticPartFloats;
    return hipSuccess;
}

hipError_t launch_gather_attend(const KvView& kv, bool paged, int group, const uint16_t* q,
                                const int32_t* idx, const int32_t* count, int batch, int n_q_heads,
                                int k_max, int chunk, int n_splits, float scale, float* part,
                                uint16_t* out, hipStream_t stream)
{
    // short lists and enough heads to fill the chip: one block per head, no partials
    if (k_max <= kDirectRows && (int64_t)batch * n_q_heads >= kDirectMinHeads) {
        const dim3 grid(1, n_q_heads, batch), block(1024);
        if (paged)
            gather_attend_kernel<true, 16, true><<<grid, block, 0, stream>>>(kv, q, idx, count, n_q_heads, group, k_max,
                                                                             k_max, 1, scale * kLog2e, part, out);
        else
            gather_attend_kernel<false, 16, true><<<grid, block, 0, stream>>>(kv, q, idx, count, n_q_heads, group, k_max,
                                                                              k_max, 1, scale * kLog2e, part, out);
        return hipGetLastError();
    }
    const dim3 grid(n_splits, n_q_heads, batch), block(256);
    if (paged)
        gather_attend_kernel<true, 4, false><<<grid, block, 0, stream>>>(kv, q, idx, count, n_q_heads, group, k_max, chunk,
                                                                         n_splits, scale * kLog2e, part, out);
    else
        gather_attend_kernel<false, 4, false><<<grid, block, 0, stream>>>(kv, q, idx, count, n_q_heads, group, k_max, chunk,
                                                                          n_splits, scale * kLog2e, part, out);
    merge_partials_kernel<true><<<dim3(n_q_heads, batch), block, 0, stream>>>(part, count, k_max, n_q_heads, chunk,
                                                                              n_splits, out);
    return hipGetLastError();
}

template <int G>
static void launch_dense_g(const KvView& kv, bool paged, const uint16_t* q, int batch, int n_q_heads,
                           int max_seq_len, int chunk, int n_splits, float scale, float* part,
                           hipStream_t stream)
{
    const dim3 grid(n_splits, kv.n_kv_heads, batch), block(256);
    if (paged)
        dense_attend_kernel<G, true><<<grid, block, 0, stream>>>(kv, q, n_q_heads, max_seq_len, chunk, n_splits,
                                                                 scale * kLog2e, part);
    else
        dense_attend_kernel<G, false><<<grid, block, 0, stream>>>(kv, q, n_q_heads, max_seq_len, chunk, n_splits,
                                                                  scale * kLog2e, part);
}

hipError_t launch_dense_attend(const KvView& kv, bool paged, int group, const uint16_t* q,
                               int batch, int n_q_heads, int max_seq_len, int chunk, int n_splits,
                               float scale, float* part, uint16_t* out, hipStream_t stream)
{
    switch (group) {
    case 1: launch_dense_g<1>(kv, paged, q, batch, n_q_heads, max_seq_len, chunk, n_splits, scale, part, stream); break;
    case 2: launch_dense_g<2>(kv, paged, q, batch, n_q_heads, max_seq_len, chunk, n_splits, scale, part, stream); break;
    case 4: launch_dense_g<4>(kv, paged, q, batch, n_q_heads, max_seq_len, chunk, n_splits, scale, part, stream); break;
    case 8: launch_dense_g<8>(kv, paged, q, batch, n_q_heads, max_seq_len, chunk, n_splits, scale, part, stream); break;
    default: return hipErrorInvalidValue;
    }
    merge_partials_kernel<false><<<dim3(n_q_heads, batch), 256, 0, stream>>>(part, kv.seq_lens, max_seq_len, n_q_heads,
                                                                             chunk, n_splits, out);
    return hipGetLastError();
}

}  // namespace ha
