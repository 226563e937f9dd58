// Bulk key encoding on the matrix cores (section 4.1, eq. 2; the mapping sizes of section 5.2) for gfx950.
//
// Building the key-code store of a whole context is a dense contraction, tokens x 128 inputs
// through F_kv = 128 -> 128 (-> 128) -> 32 per KV head: the one place of this library where MFMA
// belongs.  Codes must agree with an fp64 evaluation wherever the pre-sign activation is not tiny,
// so plain bf16 operands (8 significant bits) are not enough.  Every fp32 operand is split into two
// bf16 terms, w = w_hi + w_lo (16 significant bits, relative error 2^-18 with round to nearest), and
// the product is taken as w_hi x_hi + w_lo x_hi + w_hi x_lo with fp32 accumulation; keys are bf16
// already, so the first layer needs two terms only.  That is 2 to 3 bf16 MFMA passes per layer, still
// several times the fp32 vector rate.
//
// The contraction runs transposed, H^T = W^T X^T, with v_mfma_f32_32x32x16_bf16: the A operand is a
// 32-unit x 16-input slice of W^T, the B operand a 16-input x 32-token slice of X^T, so a lane owns
// one token (column) throughout.  Operand layout of that instruction (checked on the device):
// A[i][k] and B[k][j] sit in lane (i or j) + 32 (k / 8), element k % 8; D[i][j] sits in lane
// j + 32 g, register r with i = 8 (r / 4) + 4 g + r % 4.  The reduction index may be enumerated in
// any order as long as A and B agree, which is used twice:
//   - layer 1: in step s lane (token, g) loads bytes 32 s + 16 g .. + 15 of its key row, i.e. inputs
//     16 s + 8 g + j: the two lanes of a token read 32 adjacent bytes, so one load instruction of the wave
//     touches 32 cache lines rather than 64;
//   - later layers: the B operand of step s = 2 m + q is made, in registers, from the lane's own
//     accumulators 8 q .. 8 q + 7 of tile m of the previous layer (units 32 m + 16 q + 8 (j / 4) +
//     4 g + j % 4) after SiLU and the split: activations never leave the lane.
// A small kernel first rewrites the fp32 weights of every head into bf16 hi/lo fragments in exactly
// the order the lanes read them (one 16-byte LDS read per lane and MFMA, no bank conflicts); a block
// copies its head's fragments (80 to 145 KiB) into LDS once and its eight waves then walk 32-token
// tiles on their own, without further block synchronisation.
#include "kernels.hpp"

namespace ha {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTileTokens = 32;
// waves per block: three per SIMD where the registers allow it (up to two layers), else two
__host__ __device__ constexpr int mfma_threads(int n_layers) { return n_layers <= 2 ? 768 : 512; }
constexpr int kFragQuads = 64;          // a fragment: 64 lanes x 16 bytes
constexpr float kLog2eF = 1.4426950408889634f;

union Operand {
    uint4 q;
    bf16x8 v;
    uint32_t u[4];
};

// number of 32-unit tiles of layer l's output and fragments of that layer (hi and lo, all tiles, 8 steps)
__host__ __device__ constexpr int layer_tiles(int n_layers, int l) { return l + 1 == n_layers ? 1 : 4; }
__host__ __device__ constexpr int layer_frags(int n_layers, int l) { return 2 * layer_tiles(n_layers, l) * 8; }
__host__ __device__ constexpr int frags_before(int n_layers, int l)
{
    int f = 0;
    for (int i = 0; i < l; ++i) f += layer_frags(n_layers, i);
    return f;
}
__host__ __device__ constexpr int total_frags(int n_layers) { return frags_before(n_layers, n_layers); }
__host__ __device__ constexpr int total_units(int n_layers) { return 128 * (n_layers - 1) + 32; }
// bytes of one head's fragments plus biases
__host__ __device__ constexpr int head_bytes(int n_layers)
{
    return total_frags(n_layers) * kFragQuads * 16 + total_units(n_layers) * 4;
}

// Weights of one head, fp32 [in][out] per layer, to bf16 hi/lo fragments; biases (or zeros) behind them.
// grid (heads, slices): consecutive threads read consecutive output units of one input row (coalesced),
// one read gives the hi and the lo element.
__global__ __launch_bounds__(256) void mlp_fragments_kernel(MlpView phi, uint4* __restrict__ out, int64_t quads_per_head)
{
    const int head = blockIdx.x, NL = phi.n_layers;
    const int t0 = blockIdx.y * 256 + threadIdx.x, stride = gridDim.y * 256;
    uint16_t* dst = reinterpret_cast<uint16_t*>(out + head * quads_per_head);
    int frag0 = 0, unit0 = 0;
    for (int l = 0; l < NL; ++l) {
        const int din = phi.dims[l], dout = phi.dims[l + 1], M = dout / 32;
        const float* W = phi.W[l] + (int64_t)head * din * dout;
        const int n_elem = M * 8 * 16 * 32;                  // (tile m, step s, slot kk = 8 g + j, unit lane ol)
        for (int e = t0; e < n_elem; e += stride) {
            const int ol = e & 31, kk = (e >> 5) & 15, s = (e >> 9) & 7, m = e >> 12;
            const int g = kk >> 3, j = kk & 7, o = 32 * m + ol;
            const int k_in = l == 0 ? 16 * s + 8 * g + j
                                    : 32 * (s >> 1) + 16 * (s & 1) + 8 * (j >> 2) + 4 * g + (j & 3);
            const float w = W[(int64_t)k_in * dout + o];
            const uint32_t hi = f32_to_bf16(w);
            const uint32_t lo = f32_to_bf16(w - __uint_as_float(hi << 16));
            const int within = (32 * g + ol) * 8 + j;        // lane 32 g + ol, element j
            dst[(int64_t)(frag0 + (0 * M + m) * 8 + s) * 512 + within] = (uint16_t)hi;
            dst[(int64_t)(frag0 + (1 * M + m) * 8 + s) * 512 + within] = (uint16_t)lo;
        }
        float* bdst = reinterpret_cast<float*>(dst + (int64_t)total_frags(NL) * 512) + unit0;
        for (int u = t0; u < dout; u += stride) bdst[u] = phi.bias[l] ? phi.bias[l][(int64_t)head * dout + u] : 0.f;
        frag0 += 2 * M * 8;
        unit0 += dout;
    }
}

__device__ __forceinline__ f32x16 mfma(const uint4& a, const uint4& b, const f32x16& c)
{
    Operand x, y;
    x.q = a;
    y.q = b;
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, y.v, c, 0, 0, 0);
}

// One layer for one 32-token tile: acc[m] = bias + W^T slices x B operands (b_lo is not read unless SPLIT_B).
template <int M, bool SPLIT_B>
__device__ __forceinline__ void layer_tile(const uint4* __restrict__ frags, const float* __restrict__ bias, int lane,
                                           const uint4 (&b_hi)[8], const uint4 (&b_lo)[8], f32x16 (&acc)[M])
{
    const int g = lane >> 5;
#pragma unroll
    for (int m = 0; m < M; ++m)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const float4 bv = *reinterpret_cast<const float4*>(bias + 32 * m + 8 * r4 + 4 * g);
            acc[m][4 * r4] = bv.x; acc[m][4 * r4 + 1] = bv.y; acc[m][4 * r4 + 2] = bv.z; acc[m][4 * r4 + 3] = bv.w;
        }
    // fragments of step s + 1 are fetched while step s multiplies; the scheduling fence keeps the
    // compiler from pulling every LDS read of the layer to the front (hundreds of registers)
    uint4 a_hi[M], a_lo[M];
#pragma unroll
    for (int m = 0; m < M; ++m) {
        a_hi[m] = frags[((0 * M + m) * 8) * kFragQuads + lane];
        a_lo[m] = frags[((1 * M + m) * 8) * kFragQuads + lane];
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        uint4 n_hi[M], n_lo[M];
        if (s < 7) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                n_hi[m] = frags[((0 * M + m) * 8 + s + 1) * kFragQuads + lane];
                n_lo[m] = frags[((1 * M + m) * 8 + s + 1) * kFragQuads + lane];
            }
        }
#pragma unroll
        for (int m = 0; m < M; ++m) {
            acc[m] = mfma(a_hi[m], b_hi[s], acc[m]);
            acc[m] = mfma(a_lo[m], b_hi[s], acc[m]);
            if constexpr (SPLIT_B) acc[m] = mfma(a_hi[m], b_lo[s], acc[m]);
        }
        if (s < 7) {
#pragma unroll
            for (int m = 0; m < M; ++m) { a_hi[m] = n_hi[m]; a_lo[m] = n_lo[m]; }
        }
        // order inside the step: one LDS read of the next fragments after each multiply, so that the
        // reads are spread under the matrix pipe instead of bunched at the end of the step
        if (s < 7) {
#pragma unroll
            for (int i = 0; i < 2 * M; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one LDS read
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// SiLU of the lane's accumulators and the bf16 hi/lo split: B operands of the next layer.
__device__ __forceinline__ void activate_split(const f32x16 (&acc)[4], uint4 (&b_hi)[8], uint4 (&b_lo)[8])
{
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            Operand hi, lo;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float z0 = acc[m][8 * q + 2 * p], z1 = acc[m][8 * q + 2 * p + 1];
                const f32x2 h = {z0 * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-kLog2eF * z0)),
                                 z1 * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-kLog2eF * z1))};
                union { bf16x2 b; uint32_t u; } ph, pl;
                ph.b = __builtin_convertvector(h, bf16x2);                       // round to nearest even
                const f32x2 back = {__uint_as_float(ph.u << 16), __uint_as_float(ph.u & 0xffff0000u)};
                pl.b = __builtin_convertvector(h - back, bf16x2);
                hi.u[p] = ph.u;
                lo.u[p] = pl.u;
            }
            b_hi[2 * m + q] = hi.q;
            b_lo[2 * m + q] = lo.q;
        }
}

// Encodes, for every sequence, the cached key rows of tokens [start_b, start_b + cnt_b):
//   from_end = 1: the last min(n_new, len) tokens (in-place rebuild)
//   from_end = 0: the n_new tokens starting at len (rows just appended, seq_lens not yet bumped)
// A block takes block_tokens consecutive tokens of one (sequence, head).
template <bool PAGED, int NL>
__global__ __launch_bounds__(mfma_threads(NL)) void encode_bulk_mfma_kernel(KvView c, const uint4* __restrict__ frag_store,
                                                                        int64_t quads_per_head, int n_cap, int64_t n_new,
                                                                        int from_end, int block_tokens)
{
    extern __shared__ uint4 lds[];                         // this head's fragments, then its biases
    constexpr int kMfmaThreads = mfma_threads(NL);
    constexpr int kQuads = head_bytes(NL) / 16;
    const int tid = threadIdx.x, wave = uniform(tid >> 6), lane = tid & 63, g = lane >> 5, tl = lane & 31;
    const int head = blockIdx.y, b = blockIdx.z;
    const int len = min(c.seq_lens[b], n_cap);
    const int64_t start = from_end ? (len > n_new ? len - n_new : 0) : len;
    const int64_t cnt = from_end ? len - start : n_new;
    const int64_t t_blk = (int64_t)rotated_block(blockIdx.x, head + b, gridDim.x) * block_tokens;   // mixed lengths: spread over XCDs
    if (t_blk >= cnt) return;
    const int n_here = (int)min((int64_t)block_tokens, cnt - t_blk);
    const int n_tiles = (n_here + kTileTokens - 1) / kTileTokens;

    const uint4* src = frag_store + head * quads_per_head;
    for (int i = tid; i < kQuads; i += kMfmaThreads) lds[i] = src[i];
    const float* bias = reinterpret_cast<const float*>(lds + total_frags(NL) * kFragQuads);

    // key rows of a tile: lane (token, g) reads the 16-byte pieces g, g + 2, g + 4, ... of its row
    auto load_rows = [&](int tile, uint4 (&x)[8]) {
        const int t = min(tile * kTileTokens + tl, n_here - 1);          // past the end: repeat the last token
        const int64_t row = row_of<PAGED>(c, b, head, (int)(start + t_blk + t));
        const uint4* p = reinterpret_cast<const uint4*>(c.k + row * kHeadDim) + g;
#pragma unroll
        for (int s = 0; s < 8; ++s) x[s] = p[2 * s];
    };
    uint4 x[8];
    if (wave < n_tiles) load_rows(wave, x);
    __syncthreads();

    for (int tile = wave; tile < n_tiles; tile += kMfmaThreads / kWave) {
        const int next = min(tile + kMfmaThreads / kWave, n_tiles - 1);     // rows of the wave's next tile (or again the last)
        f32x16 out_acc[1];
        if constexpr (NL == 1) {
            layer_tile<1, false>(lds, bias, lane, x, x, out_acc);
            load_rows(next, x);
        } else {
            uint4 b_hi[8], b_lo[8];
            f32x16 acc[4];
            layer_tile<4, false>(lds, bias, lane, x, x, acc);
            load_rows(next, x);                          // x is free from here on: the fetch overlaps the other layers
            activate_split(acc, b_hi, b_lo);
            if constexpr (NL == 3) {
                layer_tile<4, true>(lds + frags_before(NL, 1) * kFragQuads, bias + 128, lane, b_hi, b_lo, acc);
                activate_split(acc, b_hi, b_lo);
            }
            layer_tile<1, true>(lds + frags_before(NL, NL - 1) * kFragQuads, bias + 128 * (NL - 1), lane, b_hi, b_lo, out_acc);
        }

        // sign bits: this lane holds 16 of its token's 32 units, lane ^ 32 the others
        uint32_t code = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) code |= (out_acc[0][r] > 0.f ? 1u : 0u) << (8 * (r / 4) + 4 * g + r % 4);
        code |= (uint32_t)__shfl_xor((int)code, 32, kWave);
        const int t = tile * kTileTokens + tl;
        if (g == 0 && t < n_here) c.codes[row_of<PAGED>(c, b, head, (int)(start + t_blk + t))] = code;
    }
}

template <bool PAGED, int NL>
hipError_t launch_nl(bool setup_only, const KvView& kv, const EncodeScratch& sc, int batch, int64_t span, int64_t n_new,
                     int max_seq_len, int from_end, hipStream_t stream)
{
    constexpr int lds = head_bytes(NL);
    if (setup_only)
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_bulk_mfma_kernel<PAGED, NL>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    // a block per 256..4096 tokens: about two blocks per CU when the job is large enough
    const int64_t lanes = (int64_t)batch * kv.n_kv_heads;
    int block_tokens = 256;
    while (block_tokens < 4096 && lanes * ((span + block_tokens - 1) / block_tokens) > 1024) block_tokens *= 2;
    const dim3 grid((unsigned)((span + block_tokens - 1) / block_tokens), kv.n_kv_heads, batch);
    encode_bulk_mfma_kernel<PAGED, NL><<<grid, mfma_threads(NL), lds, stream>>>(kv, sc.frags, sc.quads_per_head, max_seq_len,
                                                                           n_new, from_end, block_tokens);
    return hipSuccess;
}

template <bool PAGED>
hipError_t launch_paged(bool setup_only, int n_layers, const KvView& kv, const EncodeScratch& sc, int batch, int64_t span,
                        int64_t n_new, int max_seq_len, int from_end, hipStream_t stream)
{
    switch (n_layers) {
    case 1: return launch_nl<PAGED, 1>(setup_only, kv, sc, batch, span, n_new, max_seq_len, from_end, stream);
    case 2: return launch_nl<PAGED, 2>(setup_only, kv, sc, batch, span, n_new, max_seq_len, from_end, stream);
    case 3: return launch_nl<PAGED, 3>(setup_only, kv, sc, batch, span, n_new, max_seq_len, from_end, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

int64_t encode_mfma_scratch_bytes_per_head() { return (head_bytes(3) + 255) / 256 * 256; }

// The matrix-core path covers the mapping shapes of the paper: 128 -> 32, 128 -> 128 -> 32 and
// 128 -> 128 -> 128 -> 32; other widths take the vector kernel.
bool encode_mfma_supported(const MlpView& phi)
{
    if (phi.n_layers < 1 || phi.n_layers > 3 || phi.dims[0] != kHeadDim || phi.dims[phi.n_layers] != kBits) return false;
    for (int l = 1; l < phi.n_layers; ++l)
        if (phi.dims[l] != 128) return false;
    return true;
}

hipError_t setup_encode_mfma()
{
    for (int nl = 1; nl <= 3; ++nl) {
        if (hipError_t e = launch_paged<false>(true, nl, KvView{}, EncodeScratch{}, 0, 0, 0, 0, 0, nullptr); e != hipSuccess) return e;
        if (hipError_t e = launch_paged<true>(true, nl, KvView{}, EncodeScratch{}, 0, 0, 0, 0, 0, nullptr); e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_encode_bulk_mfma(const MlpView& phi, const KvView& kv, bool paged, int batch, int64_t span,
                                   int64_t n_new, int max_seq_len, int from_end, const EncodeScratch& sc,
                                   hipStream_t stream)
{
    mlp_fragments_kernel<<<dim3(kv.n_kv_heads, 16), 256, 0, stream>>>(phi, sc.frags, sc.quads_per_head);
    const hipError_t e = paged ? launch_paged<true>(false, phi.n_layers, kv, sc, batch, span, n_new, max_seq_len, from_end, stream)
                               : launch_paged<false>(false, phi.n_layers, kv, sc, batch, span, n_new, max_seq_len, from_end, stream);
    return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace ha
