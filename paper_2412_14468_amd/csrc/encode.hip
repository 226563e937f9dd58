// Mapping functions phi_q and phi_kv (section 4.1, eq. 2) for gfx950:
//   code = pack_j [ F(x)_j > 0 ],  F = small MLP with SiLU between layers, fp32.
//
// Two kernels:
//   encode_vec   few vectors per head (the decode step: one query per head, one
//                appended key per KV head).  GEMV shaped: a block owns one head
//                and up to 8 vectors, each weight is read once per block and
//                applied to all of them.
//   encode_bulk  many tokens per head (building the key-code store after
//                prefill).  A block owns a tile of 64 tokens of one KV head; the
//                activations sit in LDS, every thread keeps an (R x 8) register
//                tile of outputs and streams the weights from L2.
// Weights are fp32 and the accumulation is fp32, so a bit can differ from an
// fp64 evaluation only where the pre-sign activation is within rounding of 0.
#include "kernels.hpp"

namespace ha {

namespace {

constexpr int kMaxWidth = 512;        // widest layer of the general vector kernel (the last one: up to 512 bits)
constexpr int kFixedWidth = 256;      // activation pitch of the kernels with compile-time shapes
constexpr int kVecPerBlock = 8;
constexpr int kTile = 64;


// ---------------------------------------------------------------- encode_vec
// act: [2][kVecPerBlock][kMaxWidth] floats; r: kVecPerBlock * 256 floats of partial sums, indexed
// [part][vec][j] with parts * cols = 256, cols = min(dout, 256) columns per pass (a 512-wide layer takes
// two passes).  On return act[cur] holds the pre-sign activations of the last layer; returns cur.
__device__ int mlp_gemv(const MlpView& phi, int head, float (*act)[kVecPerBlock][kMaxWidth], float* r)
{
    const int tid = threadIdx.x;
    int cur = 0;
    for (int l = 0; l < phi.n_layers; ++l) {
        const int di = phi.dims[l], dout = phi.dims[l + 1];
        const int cols = min(dout, 256), parts = 256 / cols;
        const int j = tid % cols, p = tid / cols;
        const int span = di / parts;
        const float* W = phi.W[l] + (int64_t)head * di * dout;
        const bool last = (l + 1 == phi.n_layers);
        for (int j0 = 0; j0 < dout; j0 += 256) {
            float acc[kVecPerBlock];
#pragma unroll
            for (int v = 0; v < kVecPerBlock; ++v) acc[v] = 0.f;
            for (int i = p * span; i < (p + 1) * span; ++i) {
                const float w = W[(int64_t)i * dout + j0 + j];
#pragma unroll
                for (int v = 0; v < kVecPerBlock; ++v) acc[v] = fmaf(act[cur][v][i], w, acc[v]);
            }
#pragma unroll
            for (int v = 0; v < kVecPerBlock; ++v) r[(p * kVecPerBlock + v) * cols + j] = acc[v];
            __syncthreads();
            for (int o = tid; o < kVecPerBlock * cols; o += 256) {
                const int v = o / cols, jj = o - v * cols;
                float z = 0.f;
                for (int pp = 0; pp < parts; ++pp) z += r[(pp * kVecPerBlock + v) * cols + jj];
                if (phi.bias[l]) z += phi.bias[l][(int64_t)head * dout + j0 + jj];
                act[cur ^ 1][v][j0 + jj] = last ? z : silu(z);
            }
            __syncthreads();
        }
        cur ^= 1;
    }
    return cur;
}

// MODE 0: queries.  x = q [B][H][128]; codes -> q_codes [B][H]; vector index = b.
// MODE 1: appended keys.  x = k_new [B][H][n_new][128]; vector index = b * n_new + j; the K and V rows
//         are copied to cache position seq_lens[b] + j and the code stored there.
template <int MODE, int WD, int VB>
__device__ __forceinline__ void load_vectors(float (*act0)[WD], int n_heads, int head, int v0,
                                             const uint16_t* __restrict__ x, int n_vec, int n_new)
{
    const int tid = threadIdx.x;
    for (int o = tid; o < VB * kHeadDim; o += 256) {
        const int v = o / kHeadDim, i = o - v * kHeadDim, vec = v0 + v;
        float val = 0.f;
        if (vec < n_vec) {
            const int b = MODE == 0 ? vec : vec / n_new, jn = MODE == 0 ? 0 : vec - b * n_new;
            const int64_t src = MODE == 0 ? ((int64_t)b * n_heads + head)
                                          : (((int64_t)b * n_heads + head) * n_new + jn);
            val = __uint_as_float((uint32_t)x[src * kHeadDim + i] << 16);
        }
        act0[v][i] = val;
    }
}

// Cache position of the row this thread will place (MODE 1; same thread-to-vector mapping as store_codes):
// the sequence's length plus the row's number among the appended ones.  Asked for when the kernel
// starts, so that the block can count itself in (finish_append) long before it has finished computing.
template <int VB>
__device__ __forceinline__ int append_position(const KvView& c, int v0, int n_vec, int n_new, int n_cap)
{
    const int slot = threadIdx.x >> 5, v = min(slot, VB - 1), vec = v0 + v;
    if (slot >= VB || vec >= n_vec) return 0;
    const int b = vec / n_new;
    return min(c.seq_lens[b], n_cap) + (vec - b * n_new);
}

// The 16 bytes of the new K row (threads 0..15 of a vector's 32) or V row (16..31) that this thread
// copies into the cache in store_codes, also requested when the kernel starts.
template <int VB>
__device__ __forceinline__ uint4 append_piece(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                                              int n_heads, int head, int v0, int n_vec, int n_new)
{
    const int slot = threadIdx.x >> 5, j = threadIdx.x & 31, v = min(slot, VB - 1), vec = v0 + v;
    if (slot >= VB || vec >= n_vec) return make_uint4(0u, 0u, 0u, 0u);
    const int b = vec / n_new, jn = vec - b * n_new;
    const int64_t src = ((int64_t)b * n_heads + head) * n_new + jn;
    return *(reinterpret_cast<const uint4*>((j < 16 ? k_new : v_new) + src * kHeadDim) + (j & 15));
}

// a: [VB][WD] pre-sign activations of the last layer of the block's VB vectors
template <int MODE, bool PAGED, int WD, int VB>
__device__ __forceinline__ void store_codes(const float (*a)[WD], int n_heads, int head, int v0,
                                            const uint16_t* __restrict__ x, const uint16_t* __restrict__ v_new,
                                            int n_vec, int n_new, uint32_t* __restrict__ q_codes,
                                            const KvView& c, int pos, const uint4& piece, int words = 1)
{
    // thread (v = tid / 32, j = tid % 32) owns bit j of every code word of vector v (unit 32 w + j of
    // word w); a wave ballot packs one word of two vectors
    const int tid = threadIdx.x;
    const int slot = tid >> 5, j = tid & 31, v = min(slot, VB - 1), vec = v0 + v;
    const bool live = slot < VB && vec < n_vec;
    const int b = MODE == 0 ? vec : vec / n_new;
    int64_t row = 0;
    if constexpr (MODE == 1) {
        if (live) row = row_of<PAGED>(c, b, head, pos);        // pos: this thread's value of append_position()
    }
    for (int w = 0; w < words; ++w) {
        const uint64_t mask = __ballot(a[v][32 * w + j] > 0.f);
        const uint32_t code = (uint32_t)((tid & 32) ? (mask >> 32) : mask);
        if (live && j == 0) {
            if constexpr (MODE == 0) q_codes[((int64_t)b * n_heads + head) * words + w] = code;
            else c.codes[row * words + w] = code;
        }
    }
    if (live) {
        if constexpr (MODE == 1) {
            // 32 threads copy the 256-byte K row and V row, 16 bytes each (16 + 16 threads; see append_piece)
            uint4* to = reinterpret_cast<uint4*>(const_cast<uint16_t*>(j < 16 ? c.k : c.v) + row * kHeadDim) + (j & 15);
            *to = piece;
        }
    }
}

// Append mode: the sequence lengths may only move once every block has read them, and a separate
// launch for that costs more than the encoding.  Every block reads the lengths it needs when it
// starts (append_position) and counts itself in right after; the block that completes the count adds
// n_new to every length, as a rule while the others are still computing.  Nothing a block wrote has
// to be visible to another one here, only the counter, an atomic at device scope.
// state[0] counts the blocks of all append launches of the context and is never reset; state[1] is
// its value when the current launch began, moved on by the block that completes the launch (the next
// launch, later in the stream, reads the new value).  So a block's number inside its launch is
// state[0] - state[1] (modulo 2^32), and a launch that starts while an earlier one has not counted all
// its blocks in (it did not run to its end) sees numbers beyond its grid: the block that does
// raises `fault`, a word of pinned host memory that the C ABI reads at the start of every call on the
// context, so the broken state is reported instead of lengths silently moving at the wrong time.
// state[1] only changes once every block of the launch has counted itself in, so a block may read it
// at any time before it does so itself: append_base() asks for it together with the lengths.
__device__ __forceinline__ uint32_t append_base(const uint32_t* __restrict__ state)
{
    return __hip_atomic_load(state + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void finish_append(uint32_t* __restrict__ state, uint32_t base, int32_t* __restrict__ fault,
                                              int32_t* __restrict__ seq_lens, int batch, int n_new, uint32_t total)
{
    __shared__ int last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's length (and the base) have arrived
    __syncthreads();                                   // all threads of the block have read seq_lens
    if (threadIdx.x == 0) {                            // total: blocks of this launch that append
        const uint32_t mine = atomicAdd(state, 1u) - base;
        last = mine == total - 1u;
        if (last) __hip_atomic_store(state + 1, base + total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (mine >= total) __hip_atomic_store(fault, (int32_t)min(mine, 0x7fffffffu), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    __syncthreads();
    if (last)
        for (int b = threadIdx.x; b < batch; b += blockDim.x) seq_lens[b] += n_new;
}

// Test hook: leaves the append counter as a launch that stopped after `value` of its blocks would.
__global__ void set_append_counter_kernel(uint32_t* state, uint32_t value) { state[0] = state[1] + value; }

// Any supported network shape; weights are fetched inside the layer loops.
template <int MODE, bool PAGED>
__global__ __launch_bounds__(256) void encode_vec_kernel(MlpView phi, int n_heads, const uint16_t* __restrict__ x,
                                                         const uint16_t* __restrict__ v_new, int n_vec, int n_new,
                                                         uint32_t* __restrict__ q_codes, KvView c, int n_cap,
                                                         uint32_t* __restrict__ done, int32_t* __restrict__ fault)
{
    __shared__ float act[2][kVecPerBlock][kMaxWidth];
    __shared__ float red[kVecPerBlock * 256];
    const int head = blockIdx.x, v0 = blockIdx.y * kVecPerBlock;
    int pos = 0;
    uint4 piece = make_uint4(0u, 0u, 0u, 0u);
    if constexpr (MODE == 1) {
        const uint32_t base = append_base(done);
        pos = append_position<kVecPerBlock>(c, v0, n_vec, n_new, n_cap);
        piece = append_piece<kVecPerBlock>(x, v_new, n_heads, head, v0, n_vec, n_new);
        finish_append(done, base, fault, c.seq_lens, n_vec / n_new, n_new, gridDim.x * gridDim.y);
    }
    load_vectors<MODE, kMaxWidth, kVecPerBlock>(act[0], n_heads, head, v0, x, n_vec, n_new);
    __syncthreads();
    const int cur = mlp_gemv(phi, head, act, red);
    store_codes<MODE, PAGED, kMaxWidth, kVecPerBlock>(act[cur], n_heads, head, v0, x, v_new, n_vec, n_new, q_codes, c, pos,
                             piece, phi.dims[phi.n_layers] / kBits);
}

// ---- shapes known at compile time: every thread fetches all its weights of all layers up front,
// so the kernel costs about one trip to HBM instead of one per input row (the weights of a layer
// are cold at every decode step: 80 KiB per head for 128-128-32).
template <int DI, int DOUT>
__device__ __forceinline__ void fetch_weights(const float* __restrict__ W, float (&w)[DI * DOUT / 256])
{
    constexpr int SPAN = DI * DOUT / 256;
    const int j = threadIdx.x % DOUT, p = threadIdx.x / DOUT;
#pragma unroll
    for (int i = 0; i < SPAN; ++i) w[i] = W[(int64_t)(p * SPAN + i) * DOUT + j];
}

// VT: vectors per block
template <int DI, int DOUT, int VT>
__device__ __forceinline__ void gemv_layer(const float (&w)[DI * DOUT / 256], const float* __restrict__ bias,
                                           const float (*in)[kFixedWidth], float (*out)[kFixedWidth], float* red,
                                           bool last)
{
    constexpr int SPAN = DI * DOUT / 256, PARTS = 256 / DOUT;
    const int tid = threadIdx.x, j = tid % DOUT, p = tid / DOUT;
    float acc[VT];
#pragma unroll
    for (int v = 0; v < VT; ++v) acc[v] = 0.f;
#pragma unroll
    for (int i = 0; i < SPAN; ++i)
#pragma unroll
        for (int v = 0; v < VT; ++v) acc[v] = fmaf(in[v][p * SPAN + i], w[i], acc[v]);
#pragma unroll
    for (int v = 0; v < VT; ++v) red[(p * VT + v) * DOUT + j] = acc[v];
    __syncthreads();
    for (int o = tid; o < VT * DOUT; o += 256) {
        const int v = o / DOUT, jj = o - v * DOUT;
        float z = 0.f;
#pragma unroll
        for (int pp = 0; pp < PARTS; ++pp) z += red[(pp * VT + v) * DOUT + jj];
        if (bias) z += bias[jj];
        out[v][jj] = last ? z : silu(z);
    }
    __syncthreads();
}

// One block's work: `head` and the vectors v0 .. v0 + VT - 1.  append_blocks: blocks of the launch that append
// (MODE 1; the count that moves the sequence lengths runs over them).
template <int MODE, bool PAGED, int NL, int D1, int D2, int VT>
__device__ __forceinline__ void encode_fixed_block(const MlpView& phi, int n_heads, int head, int v0,
                                                   const uint16_t* __restrict__ x, const uint16_t* __restrict__ v_new,
                                                   int n_vec, int n_new, uint32_t* __restrict__ q_codes, const KvView& c,
                                                   int n_cap, uint32_t* __restrict__ done, int32_t* __restrict__ fault,
                                                   uint32_t append_blocks, float (*act)[VT][kFixedWidth], float* red)
{
    constexpr int O0 = NL == 1 ? kBits : D1;            // outputs of layer 0
    constexpr int I1 = D1, O1 = NL == 2 ? kBits : D2;   // layer 1 (NL >= 2)
    constexpr int I2 = D2;                              // layer 2 (NL == 3), 32 outputs
    float w0[kHeadDim * O0 / 256];
    float w1[NL >= 2 ? I1 * O1 / 256 : 1];
    float w2[NL == 3 ? I2 * kBits / 256 : 1];
    fetch_weights<kHeadDim, O0>(phi.W[0] + (int64_t)head * kHeadDim * O0, w0);
    if constexpr (NL >= 2) fetch_weights<I1, O1>(phi.W[1] + (int64_t)head * I1 * O1, w1);
    if constexpr (NL == 3) fetch_weights<I2, kBits>(phi.W[2] + (int64_t)head * I2 * kBits, w2);
    load_vectors<MODE, kFixedWidth, VT>(act[0], n_heads, head, v0, x, n_vec, n_new);
    int pos = 0;
    uint4 piece = make_uint4(0u, 0u, 0u, 0u);
    if constexpr (MODE == 1) {               // the weights are on their way; the wait in finish_append covers them too
        const uint32_t base = append_base(done);
        pos = append_position<VT>(c, v0, n_vec, n_new, n_cap);
        piece = append_piece<VT>(x, v_new, n_heads, head, v0, n_vec, n_new);
        finish_append(done, base, fault, c.seq_lens, n_vec / n_new, n_new, append_blocks);
    }
    __syncthreads();
    gemv_layer<kHeadDim, O0, VT>(w0, phi.bias[0] ? phi.bias[0] + (int64_t)head * O0 : nullptr, act[0], act[1], red, NL == 1);
    if constexpr (NL >= 2)
        gemv_layer<I1, O1, VT>(w1, phi.bias[1] ? phi.bias[1] + (int64_t)head * O1 : nullptr, act[1], act[0], red, NL == 2);
    if constexpr (NL == 3)
        gemv_layer<I2, kBits, VT>(w2, phi.bias[2] ? phi.bias[2] + (int64_t)head * kBits : nullptr, act[0], act[1], red, true);
    store_codes<MODE, PAGED, kFixedWidth, VT>(act[NL & 1], n_heads, head, v0, x, v_new, n_vec, n_new, q_codes, c, pos, piece);
}

// NL layers: 128 -> D1 -> D2 -> 32 (NL = 3), 128 -> D1 -> 32 (NL = 2), 128 -> 32 (NL = 1).
// VT vectors per block: every vector costs a block its LDS reads and multiplies one after the other, so
// a launch with few vectors spreads them over more blocks (the weights are then read VT times less often
// than once per vector, from L2 after the first block of a head).
template <int MODE, bool PAGED, int NL, int D1, int D2, int VT>
__global__ __launch_bounds__(256) void encode_vec_fixed_kernel(MlpView phi, int n_heads,
                                                               const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ v_new, int n_vec,
                                                               int n_new, uint32_t* __restrict__ q_codes,
                                                               KvView c, int n_cap, uint32_t* __restrict__ done,
                                                               int32_t* __restrict__ fault)
{
    __shared__ float act[2][VT][kFixedWidth];
    __shared__ float red[VT * 256];
    encode_fixed_block<MODE, PAGED, NL, D1, D2, VT>(phi, n_heads, blockIdx.x, blockIdx.y * VT, x, v_new, n_vec, n_new, q_codes,
                                                    c, n_cap, done, fault, gridDim.x * gridDim.y, act, red);
}

// The decode step's two mappings in one launch: the first append_blocks blocks append one token per sequence
// (its K/V rows, its key code, the sequence lengths), the others encode the queries.  Both mappings have the
// same fixed shape.  Block i of a role takes head i % heads and the vectors (i / heads) VT ...
template <bool PAGED, int NL, int D1, int D2, int VT>
__global__ __launch_bounds__(256) void encode_step_kernel(MlpView phi_kv, MlpView phi_q, int n_kv_heads, int n_q_heads,
                                                          const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new,
                                                          const uint16_t* __restrict__ q, int batch,
                                                          uint32_t* __restrict__ q_codes, KvView c, int n_cap,
                                                          uint32_t* __restrict__ done, int32_t* __restrict__ fault,
                                                          int append_blocks)
{
    __shared__ float act[2][VT][kFixedWidth];
    __shared__ float red[VT * 256];
    const int i = blockIdx.x;
    if (i < append_blocks)
        encode_fixed_block<1, PAGED, NL, D1, D2, VT>(phi_kv, n_kv_heads, i % n_kv_heads, (i / n_kv_heads) * VT, k_new, v_new, batch,
                                                     1, nullptr, c, n_cap, done, fault, (uint32_t)append_blocks, act, red);
    else
        encode_fixed_block<0, PAGED, NL, D1, D2, VT>(phi_q, n_q_heads, (i - append_blocks) % n_q_heads,
                                                     ((i - append_blocks) / n_q_heads) * VT, q, nullptr, batch, 1, q_codes, c,
                                                     n_cap, nullptr, nullptr, 0u, act, red);
}

template <int MODE, bool PAGED, int NL, int D1, int D2>
void launch_fixed(int vt, const MlpView& phi, int n_heads, const uint16_t* x, const uint16_t* v_new, int n_vec,
                  int n_new, uint32_t* q_codes, const KvView& c, int n_cap, uint32_t* done, int32_t* fault,
                  hipStream_t stream)
{
    const dim3 grid(n_heads, (n_vec + vt - 1) / vt);
    switch (vt) {
    case 1: encode_vec_fixed_kernel<MODE, PAGED, NL, D1, D2, 1><<<grid, 256, 0, stream>>>(phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault); break;
    case 2: encode_vec_fixed_kernel<MODE, PAGED, NL, D1, D2, 2><<<grid, 256, 0, stream>>>(phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault); break;
    case 4: encode_vec_fixed_kernel<MODE, PAGED, NL, D1, D2, 4><<<grid, 256, 0, stream>>>(phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault); break;
    default: encode_vec_fixed_kernel<MODE, PAGED, NL, D1, D2, 8><<<grid, 256, 0, stream>>>(phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault); break;
    }
}

template <int MODE, bool PAGED>
void launch_encode_vec(const MlpView& phi, int n_heads, const uint16_t* x, const uint16_t* v_new,
                       int n_vec, int n_new, uint32_t* q_codes, const KvView& c, int n_cap, uint32_t* done,
                       int32_t* fault, hipStream_t stream)
{
    const int nl = phi.n_layers, d1 = phi.dims[1], d2 = phi.dims[2];
    // vectors per block: the fewest (of 2, 4, 8; 1 for a single vector) that keep the launch within 512
    // blocks (measured at 16 and 64 vectors for 32 heads and at 16 for 8)
    int vt = n_vec == 1 ? 1 : 2;
    while (vt < kVecPerBlock && (int64_t)n_heads * ((n_vec + vt - 1) / vt) > 512) vt *= 2;
    const bool narrow = phi.dims[nl] == kBits;          // wider signatures take the general kernel
    if (narrow && nl == 1)
        launch_fixed<MODE, PAGED, 1, 32, 32>(vt, phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault, stream);
    else if (narrow && nl == 2 && d1 == 128)
        launch_fixed<MODE, PAGED, 2, 128, 32>(vt, phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault, stream);
    else if (narrow && nl == 3 && d1 == 128 && d2 == 128)
        launch_fixed<MODE, PAGED, 3, 128, 128>(vt, phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault, stream);
    else {
        const dim3 grid(n_heads, (n_vec + kVecPerBlock - 1) / kVecPerBlock);
        encode_vec_kernel<MODE, PAGED><<<grid, 256, 0, stream>>>(phi, n_heads, x, v_new, n_vec, n_new, q_codes, c, n_cap, done, fault);
    }
}

__global__ void bump_seq_lens_kernel(int32_t* seq_lens, int batch, int n_new)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) seq_lens[b] += n_new;
}

// ---------------------------------------------------------------- encode_bulk
// One layer on a 64-token tile: out[t][o] = sum_i in[t][i] W[i][o] (+bias), then SiLU; the last layer
// keeps only the signs: byte tx of token t's code, at ((uint8_t*)out)[t * DOUT / 8 + tx], has bit e set
// when output tx*8 + e is positive (output 32 w + j is bit j of word w, least significant byte first).
// Thread (ty, tx): outputs tx*8 .. tx*8+7 of tokens ty + rows*r, r < R.
template <int DOUT>
__device__ __forceinline__ void bulk_layer(const float* __restrict__ W, const float* __restrict__ bias, int di,
                                           const float* in, int in_pitch, float* out, int out_pitch, bool last)
{
    constexpr int NOT = DOUT / 8, ROWS = 256 / NOT, R = kTile / ROWS;
    const int tx = threadIdx.x % NOT, ty = threadIdx.x / NOT;
    float acc[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    for (int i = 0; i < di; ++i) {
        const float4 w0 = *reinterpret_cast<const float4*>(W + (int64_t)i * DOUT + tx * 8);
        const float4 w1 = *reinterpret_cast<const float4*>(W + (int64_t)i * DOUT + tx * 8 + 4);
        const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float xv = in[(ty + ROWS * r) * in_pitch + i];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = fmaf(xv, w[e], acc[r][e]);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        uint32_t byte = 0u;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float z = acc[r][e];
            if (bias) z += bias[tx * 8 + e];
            if (last) byte |= (z > 0.f ? 1u : 0u) << e;
            else out[(ty + ROWS * r) * out_pitch + tx * 8 + e] = silu(z);
        }
        if (last) reinterpret_cast<uint8_t*>(out)[(ty + ROWS * r) * NOT + tx] = (uint8_t)byte;
    }
}

__device__ __forceinline__ void bulk_layer_any(int dout, const float* W, const float* bias, int di,
                                               const float* in, int in_pitch, float* out, int out_pitch, bool last)
{
    switch (dout) {
    case 32:  bulk_layer<32>(W, bias, di, in, in_pitch, out, out_pitch, last); break;
    case 64:  bulk_layer<64>(W, bias, di, in, in_pitch, out, out_pitch, last); break;
    case 128: bulk_layer<128>(W, bias, di, in, in_pitch, out, out_pitch, last); break;
    case 256: bulk_layer<256>(W, bias, di, in, in_pitch, out, out_pitch, last); break;
    default:  bulk_layer<512>(W, bias, di, in, in_pitch, out, out_pitch, last); break;   // last layer only
    }
}

// Encodes, for every sequence, the cached key rows of tokens [start_b, start_b + cnt_b):
//   from_end = 1: the last min(n_new, len) tokens (in-place rebuild)
//   from_end = 0: the n_new tokens starting at len (rows just appended, seq_lens not yet bumped)
template <bool PAGED>
__global__ __launch_bounds__(256) void encode_bulk_kernel(MlpView phi, KvView c, int n_cap, int64_t n_new, int from_end)
{
    extern __shared__ float lds[];                         // 2 x kTile x P floats
    int widest = phi.dims[0];                              // of the layers' inputs: the last layer leaves code bytes
    for (int l = 1; l < phi.n_layers; ++l) widest = max(widest, phi.dims[l]);
    const int P = widest + 1;                              // LDS pitch, odd to spread banks
    float* bufA = lds;
    float* bufB = lds + kTile * P;
    const int tid = threadIdx.x;
    const int head = blockIdx.y, b = blockIdx.z;
    const int len = min(c.seq_lens[b], n_cap);
    const int64_t start = from_end ? (len > n_new ? len - n_new : 0) : len;
    const int64_t cnt = from_end ? len - start : n_new;
    const int64_t t0 = (int64_t)blockIdx.x * kTile;
    if (t0 >= cnt) return;
    const int n_tok = (int)min((int64_t)kTile, cnt - t0);

    // load the key tile as fp32: 16 lanes x 16 bytes per row
    for (int o = tid; o < kTile * 16; o += 256) {
        const int t = o >> 4, sub = o & 15;
        float f[8];
        if (t < n_tok) {
            const int64_t row = row_of<PAGED>(c, b, head, (int)(start + t0 + t));
            unpack8(*reinterpret_cast<const uint4*>(c.k + row * kHeadDim + sub * 8), f);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) bufA[t * P + sub * 8 + e] = f[e];
    }
    __syncthreads();

    float* in = bufA;
    float* out = bufB;
    for (int l = 0; l < phi.n_layers; ++l) {
        const int di = phi.dims[l], dout = phi.dims[l + 1];
        const float* W = phi.W[l] + (int64_t)head * di * dout;
        const float* bias = phi.bias[l] ? phi.bias[l] + (int64_t)head * dout : nullptr;
        bulk_layer_any(dout, W, bias, di, in, P, out, P, l + 1 == phi.n_layers);
        __syncthreads();
        float* t = in; in = out; out = t;
    }
    const int words = phi.dims[phi.n_layers] / kBits;          // unit 32 w + j -> bit j of word w
    const uint32_t* packed = reinterpret_cast<const uint32_t*>(in);     // [kTile][words], written by the last layer
    for (int o = tid; o < n_tok * words; o += 256) {
        const int t = o / words, w = o - t * words;
        c.codes[row_of<PAGED>(c, b, head, (int)(start + t0 + t)) * words + w] = packed[o];
    }
}

// Copies appended rows k_new/v_new [B][H][n_new][128] into the cache at positions len_b + j.
template <bool PAGED>
__global__ __launch_bounds__(256) void append_rows_kernel(KvView c, const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new, int64_t n_new, int n_cap)
{
    const int head = blockIdx.y, b = blockIdx.z;
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;     // 16-byte piece index inside (b, head)
    const int64_t j = o >> 4;
    const int sub = (int)(o & 15);
    if (j >= n_new) return;
    const int64_t src = (((int64_t)b * c.n_kv_heads + head) * n_new + j) * kHeadDim + sub * 8;
    const int64_t row = row_of<PAGED>(c, b, head, (int)(min(c.seq_lens[b], n_cap) + j));
    *reinterpret_cast<uint4*>(const_cast<uint16_t*>(c.k) + row * kHeadDim + sub * 8) =
        *reinterpret_cast<const uint4*>(k_new + src);
    *reinterpret_cast<uint4*>(const_cast<uint16_t*>(c.v) + row * kHeadDim + sub * 8) =
        *reinterpret_cast<const uint4*>(v_new + src);
}

// LDS bytes of encode_bulk for this network (two tiles of the widest layer input, at most 256 wide).
size_t bulk_lds_bytes(const MlpView& phi)
{
    int widest = phi.dims[0];
    for (int l = 1; l < phi.n_layers; ++l) widest = widest > phi.dims[l] ? widest : phi.dims[l];
    return sizeof(float) * 2 * kTile * (size_t)(widest + 1);
}

}  // namespace

// Raises the dynamic LDS limit of the vector-unit bulk encoder to what its widest network (256-wide
// layers) needs; called once when a context is created, never on the launch path.
hipError_t setup_encode_bulk()
{
    const int bytes = (int)(sizeof(float) * 2 * kTile * (256 + 1));
    if (hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_bulk_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, bytes); e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_bulk_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t launch_set_append_counter(uint32_t* state, uint32_t value, hipStream_t stream)
{
    set_append_counter_kernel<<<1, 1, 0, stream>>>(state, value);
    return hipGetLastError();
}

namespace {

template <bool PAGED, int NL, int D1, int D2>
void launch_step_fixed(int vt, const MlpView& phi_kv, const MlpView& phi_q, const KvView& kv, int n_q_heads,
                       const uint16_t* k_new, const uint16_t* v_new, const uint16_t* q, int batch, uint32_t* q_codes,
                       int n_cap, const EncodeScratch& sc, hipStream_t stream)
{
    const int per_role = (batch + vt - 1) / vt;
    const int append_blocks = kv.n_kv_heads * per_role, blocks = append_blocks + n_q_heads * per_role;
#define HA_STEP(VT) encode_step_kernel<PAGED, NL, D1, D2, VT><<<blocks, 256, 0, stream>>>(phi_kv, phi_q, kv.n_kv_heads, n_q_heads, k_new, v_new, q, batch, q_codes, kv, n_cap, sc.append_done, sc.append_fault, append_blocks)
    switch (vt) {
    case 1: HA_STEP(1); break;
    case 2: HA_STEP(2); break;
    case 4: HA_STEP(4); break;
    default: HA_STEP(8); break;
    }
#undef HA_STEP
}

// 1, 2 or 3 when the mapping has one of the fixed shapes of the vector kernels (128 -> 32, 128 -> 128 -> 32,
// 128 -> 128 -> 128 -> 32), else 0
int fixed_shape(const MlpView& phi)
{
    if (phi.dims[0] != kHeadDim || phi.dims[phi.n_layers] != kBits) return 0;
    if (phi.n_layers == 1) return 1;
    if (phi.n_layers == 2 && phi.dims[1] == 128) return 2;
    if (phi.n_layers == 3 && phi.dims[1] == 128 && phi.dims[2] == 128) return 3;
    return 0;
}

}  // namespace

bool encode_step_supported(const MlpView& phi_kv, const MlpView& phi_q)
{
    const int a = fixed_shape(phi_kv);
    return a != 0 && a == fixed_shape(phi_q);
}

// One token per sequence appended (rows, key code, lengths) and the queries encoded, in one launch.
hipError_t launch_encode_step(const MlpView& phi_kv, const MlpView& phi_q, const KvView& kv, bool paged, int n_q_heads,
                              const uint16_t* k_new, const uint16_t* v_new, const uint16_t* q, int batch,
                              uint32_t* q_codes, int max_seq_len, const EncodeScratch& sc, hipStream_t stream)
{
    if (!encode_step_supported(phi_kv, phi_q)) return hipErrorInvalidValue;
    // vectors per block as for a query launch of its own (the role with more heads decides)
    int vt = batch == 1 ? 1 : 2;
    while (vt < kVecPerBlock && (int64_t)n_q_heads * ((batch + vt - 1) / vt) > 512) vt *= 2;
    const int nl = fixed_shape(phi_q);
#define HA_STEP_NL(P) \
    if (nl == 1) launch_step_fixed<P, 1, 32, 32>(vt, phi_kv, phi_q, kv, n_q_heads, k_new, v_new, q, batch, q_codes, max_seq_len, sc, stream); \
    else if (nl == 2) launch_step_fixed<P, 2, 128, 32>(vt, phi_kv, phi_q, kv, n_q_heads, k_new, v_new, q, batch, q_codes, max_seq_len, sc, stream); \
    else launch_step_fixed<P, 3, 128, 128>(vt, phi_kv, phi_q, kv, n_q_heads, k_new, v_new, q, batch, q_codes, max_seq_len, sc, stream)
    if (paged) { HA_STEP_NL(true); } else { HA_STEP_NL(false); }
#undef HA_STEP_NL
    return hipGetLastError();
}

hipError_t launch_encode_query(const MlpView& phi, const uint16_t* q, int batch, int n_heads,
                               uint32_t* q_codes, hipStream_t stream)
{
    KvView none{};
    launch_encode_vec<0, false>(phi, n_heads, q, nullptr, batch, 1, q_codes, none, 0, nullptr, nullptr, stream);
    return hipGetLastError();
}

hipError_t launch_encode_keys(const MlpView& phi, const KvView& kv, bool paged,
                              const uint16_t* k_new, const uint16_t* v_new,
                              int batch, int64_t n_new, int max_seq_len, const EncodeScratch* sc,
                              hipStream_t stream)
{
    const int H = kv.n_kv_heads;
    const size_t lds_bytes = bulk_lds_bytes(phi);
    const bool mfma = sc->frags && encode_mfma_supported(phi);          // bulk work goes to the matrix cores
    if (k_new) {
        if (n_new * batch <= 4 * kVecPerBlock) {
            // decode-time append: one GEMV-shaped launch writes rows and codes and moves the lengths
            const int n_vec = (int)(batch * n_new);
            if (paged)
                launch_encode_vec<1, true>(phi, H, k_new, v_new, n_vec, (int)n_new, nullptr, kv, max_seq_len, sc->append_done, sc->append_fault, stream);
            else
                launch_encode_vec<1, false>(phi, H, k_new, v_new, n_vec, (int)n_new, nullptr, kv, max_seq_len, sc->append_done, sc->append_fault, stream);
        } else {
            const dim3 cgrid((unsigned)((n_new * 16 + 255) / 256), H, batch);
            const dim3 egrid((unsigned)((n_new + kTile - 1) / kTile), H, batch);
            if (paged) append_rows_kernel<true><<<cgrid, 256, 0, stream>>>(kv, k_new, v_new, n_new, max_seq_len);
            else append_rows_kernel<false><<<cgrid, 256, 0, stream>>>(kv, k_new, v_new, n_new, max_seq_len);
            if (mfma) {
                if (hipError_t e = launch_encode_bulk_mfma(phi, kv, paged, batch, n_new, n_new, max_seq_len, 0, *sc, stream); e != hipSuccess) return e;
            } else {
                if (paged) encode_bulk_kernel<true><<<egrid, 256, lds_bytes, stream>>>(phi, kv, max_seq_len, n_new, 0);
                else encode_bulk_kernel<false><<<egrid, 256, lds_bytes, stream>>>(phi, kv, max_seq_len, n_new, 0);
            }
            bump_seq_lens_kernel<<<(batch + 255) / 256, 256, 0, stream>>>(kv.seq_lens, batch, (int)n_new);
        }
    } else {
        const int64_t span = n_new < max_seq_len ? n_new : max_seq_len;
        if (span > 0 && mfma) {
            if (hipError_t e = launch_encode_bulk_mfma(phi, kv, paged, batch, span, n_new, max_seq_len, 1, *sc, stream); e != hipSuccess) return e;
        } else if (span > 0) {
            const dim3 egrid((unsigned)((span + kTile - 1) / kTile), H, batch);
            if (paged)
                encode_bulk_kernel<true><<<egrid, 256, lds_bytes, stream>>>(phi, kv, max_seq_len, n_new, 1);
            else
                encode_bulk_kernel<false><<<egrid, 256, lds_bytes, stream>>>(phi, kv, max_seq_len, n_new, 1);
        }
    }
    return hipGetLastError();
}

}  // namespace ha
