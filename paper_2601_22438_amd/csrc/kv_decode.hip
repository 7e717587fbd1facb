// Paged decode attention for gfx950: one query token per sequence attends to that sequence's
// cached K/V, stored as fixed-size blocks reached through a block table (the block-represented
// KV cache of paper Sec. 3.2 item 3).
//
// The work is a scan of the KV cache (HBM-bound).  A workgroup of 4 wavefronts owns one
// (sequence, KV head, context partition); the G = Hq/Hkv query heads that share the KV head are
// the 16-wide N side of MFMA tiles, so every K/V byte is loaded once and used by all G heads:
//     S^T[token][head] = K[token][d] * Q^T[d][head]          (v_mfma_f32_16x16x32_bf16, 16 tokens)
//     O^T[d][head]    += V^T[d][token] * P^T[token][head]    (same instruction, 32 tokens)
// With this orientation each lane's softmax statistics belong to one head (lane % 16), the
// probabilities come out of the first product already in the register layout the second one
// wants, and the running rescale of O is lane-local.
//
// K rows go from HBM straight into the A-operand layout (lane = token row, 8 consecutive
// channels).  V rows are loaded fully coalesced, staged in a per-wave LDS tile and read back
// transposed (ds_read_b64_tr_b16) as the A operand of the second product.
// Each wavefront runs an online softmax over its tiles (every 4th 32-token tile of the
// partition) with the next tile's K/V loads in flight while the current tile is reduced; the
// 4 wavefronts are merged through LDS, and partitions of one sequence by a second small kernel
// in a fixed order, so the result depends only on logical token positions.

#include "kv_internal.h"

namespace kvflow {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

template <int D>
struct Shape {
    static constexpr int kSteps = D / 32;            // MFMA k-steps over the head dimension
    static constexpr int kDTiles = D / 16;           // 16-channel output tiles
    static constexpr int kLanesPerRow = D / 8;       // lanes covering one K/V row with 16-byte loads
    static constexpr int kRowsPerChunk = 64 / kLanesPerRow;
    static constexpr int kVChunks = kTileTokens / kRowsPerChunk;   // 1 KiB loads per 32-token V tile
    static constexpr int kPitch = D * 2 + 32;        // LDS row pitch in bytes (pad avoids bank conflicts)
    static constexpr int kVTileBytes = kTileTokens * kPitch;
    static constexpr int kMergeFloats = D + 2;       // workspace record per (head, partition): O[D], m, l
    static constexpr int kLdsRow = D + 4;            // same record in LDS, padded to keep 16-byte alignment
};

template <int D>
struct TileRegs {
    bf16x8 k[2][Shape<D>::kSteps];
    u32x4 v[Shape<D>::kVChunks];
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D>
__global__ __launch_bounds__(kThreads) void decode_partition_kernel(const DecodeParams p)
{
    using S = Shape<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;

    const int L = p.context_lens[b];
    const int start = split * p.partition_tokens;
    const int G = p.group;
    const int64_t out_row0 = (int64_t)b * p.num_q_heads + (int64_t)kvh * G;

    if (start >= L) {
        // Nothing cached in this partition.  An empty sequence still owes a row of zeros.
        if (L == 0 && split == 0 && p.splits == 1) {
            for (int e = threadIdx.x; e < G * D; e += kThreads) {
                if (p.out_f32) ((float*)p.out)[out_row0 * D + e] = 0.f;
                else ((uint16_t*)p.out)[out_row0 * D + e] = 0;
            }
        }
        return;
    }
    const int end = min(L, start + p.partition_tokens);
    const int n_tiles = (end - start + kTileTokens - 1) / kTileTokens;

    // ---- Q^T as the B operand: lane (g, j) holds head j, channels 32*ks + 8*g .. +7
    bf16x8 qreg[S::kSteps];
    {
        const uint16_t* qrow = p.q + (out_row0 + j) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < S::kSteps; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (j < G) t = *(const u32x4*)(qrow + 32 * ks);
            qreg[ks] = __builtin_bit_cast(bf16x8, t);
        }
    }

    const int32_t* table = p.block_table + (int64_t)b * p.max_blocks_per_seq;
    const int bs = p.block_size;
    const int64_t head_elems = (int64_t)bs * D;                       // one (block, K|V, head) tile
    const int64_t v_off = (int64_t)p.num_kv_heads * head_elems;       // K -> V within a block
    const int64_t blk_elems = 2 * v_off;
    const int koff = j * D + 8 * g;                                   // K operand: row j, channels 8g..
    const int vrow = lane / S::kLanesPerRow;                          // V natural: row within a chunk
    const int vcol = (lane % S::kLanesPerRow) * 8;

    unsigned char* vt = smem + wave * S::kVTileBytes;                 // this wave's V staging tile
    const int vw_off = vrow * S::kPitch + vcol * 2;                   // ds_write position (+ chunk rows)
    // transposed read: lanes 4e+c of a 16-lane group point at row 4g+e, channels 4c..4c+3 of a d-tile
    const int vr_off = (4 * g + (j >> 2)) * S::kPitch + (j & 3) * 8;

    // physical block of the 16-token subtile that starts at token t0 (t0 < end)
    auto subtile_base = [&](int t0) -> int64_t {
        const int blk = t0 >> p.block_shift;
        const int r0 = t0 & (bs - 1);
        const int64_t pb = table[blk];
        return pb * blk_elems + (int64_t)kvh * head_elems + (int64_t)r0 * D;
    };

    auto issue_loads = [&](TileRegs<D>& r, int tile) {
        const int t0 = start + tile * kTileTokens;
        const int64_t base0 = subtile_base(t0);
        // a subtile with no valid token reuses subtile 0's address: its data is masked out below
        const int64_t base1 = (t0 + 16 < end) ? subtile_base(t0 + 16) : base0;
        const uint16_t* k0 = p.pool + base0 + koff;
        const uint16_t* k1 = p.pool + base1 + koff;
#pragma unroll
        for (int ks = 0; ks < S::kSteps; ++ks) {
            r.k[0][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(k0 + 32 * ks));
            r.k[1][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(k1 + 32 * ks));
        }
        const uint16_t* v0 = p.pool + base0 + v_off + vrow * D + vcol;
        const uint16_t* v1 = p.pool + base1 + v_off + vrow * D + vcol;
#pragma unroll
        for (int c = 0; c < S::kVChunks; ++c) {
            const int row16 = (c * S::kRowsPerChunk) & 15;            // first row of the chunk in its subtile
            const uint16_t* src = (c * S::kRowsPerChunk < 16 ? v0 : v1) + row16 * D;
            r.v[c] = *(const u32x4*)src;
        }
    };

    float m_run = -INFINITY;      // running max of scaled scores (log2 domain) for head j
    float l_run = 0.f;            // this lane's share of the running denominator
    f32x4 oacc[S::kDTiles];
#pragma unroll
    for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto reduce_tile = [&](TileRegs<D>& r, int tile) {
        const int tok0 = start + tile * kTileTokens;                  // first token of the tile
        const bool ragged = tok0 + kTileTokens > end;                 // wave-uniform

        // ---- S^T = K Q^T for the two 16-token subtiles
        f32x4 s[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < S::kSteps; ++ks)
                s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.k[u][ks], qreg[ks], s[u], 0, 0, 0);
        }
        // lane (g, j): s[u][i] is head j, token tok0 + 16u + 4g + i
        float t[8];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) t[4 * u + i] = s[u][i] * p.scale_log2e;
        if (ragged) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tok0 + 16 * u + 4 * g + i >= end) t[4 * u + i] = -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);                         // finite: the tile has a valid token
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float pr[8];
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { pr[e] = fast_exp2(t[e] - m_new); psum += pr[e]; }
        l_run = l_run * alpha + psum;
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)pr[e];
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] *= alpha;

        // ---- V tile -> LDS (rows past the end are zeroed: 0 * NaN must not reach the sum)
#pragma unroll
        for (int c = 0; c < S::kVChunks; ++c) {
            u32x4 val = r.v[c];
            if (ragged && tok0 + c * S::kRowsPerChunk + vrow >= end) val = u32x4{0u, 0u, 0u, 0u};
            *(u32x4*)(vt + vw_off + c * S::kRowsPerChunk * S::kPitch) = val;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- O^T += V^T P^T over the tile's 32 tokens, one 16-channel tile at a time
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt) {
            typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt + vr_off + dt * 32));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt + vr_off + 16 * S::kPitch + dt * 32));
            typedef short s16x8 __attribute__((__vector_size__(16)));
            s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pb, oacc[dt], 0, 0, 0);
        }
        // the next tile's ds_write must not overtake these reads in program order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    // ---- this wave's tiles: wave, wave + 4, ... ; loads run one tile ahead of the arithmetic
    TileRegs<D> ra, rb;
    int tile = wave;
    if (tile < n_tiles) {
        issue_loads(ra, tile);
        while (true) {
            if (tile + kWaves < n_tiles) issue_loads(rb, tile + kWaves);
            reduce_tile(ra, tile);
            tile += kWaves;
            if (tile >= n_tiles) break;
            if (tile + kWaves < n_tiles) issue_loads(ra, tile + kWaves);
            reduce_tile(rb, tile);
            tile += kWaves;
            if (tile >= n_tiles) break;
        }
    }
    // lanes of the same head hold disjoint token subsets under one shared max
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // ---- merge the 4 waves through LDS: per wave and head, O[D], m, l
    __syncthreads();                                                  // V staging is dead from here on
    float* mg = (float*)smem;
    if (j < G) {
        float* row = mg + (wave * kMaxGroup + j) * S::kLdsRow;
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt)
            *(f32x4*)(row + 16 * dt + 4 * g) = oacc[dt];              // channels 16dt + 4g .. +3
        if (g == 0) { row[D] = m_run; row[D + 1] = l_run; }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < G * D; e += kThreads) {
        const int h = e / D, d = e % D;
        float mw[kWaves];
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            mw[w] = mg[(w * kMaxGroup + h) * S::kLdsRow + D];
            M = fmaxf(M, mw[w]);
        }
        float acc = 0.f, lsum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float* row = mg + (w * kMaxGroup + h) * S::kLdsRow;
            const float wgt = (mw[w] == -INFINITY) ? 0.f : fast_exp2(mw[w] - M);
            acc += wgt * row[d];
            lsum += wgt * row[D + 1];
        }
        if (p.splits == 1) {
            const float o = acc / lsum;
            if (p.out_f32) ((float*)p.out)[(out_row0 + h) * D + d] = o;
            else ((__bf16*)p.out)[(out_row0 + h) * D + d] = (__bf16)o;
        } else {
            float* ws = p.workspace + ((out_row0 + h) * p.splits + split) * S::kMergeFloats;
            ws[d] = acc;
            if (d == 0) { ws[D] = M; ws[D + 1] = lsum; }
        }
    }
}

// Combines the partitions of one (sequence, query head) in ascending partition order.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(const DecodeParams p)
{
    using S = Shape<D>;
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int64_t row = (int64_t)b * p.num_q_heads + h;
    const int L = p.context_lens[b];
    const int n = (L + p.partition_tokens - 1) / p.partition_tokens;
    const float* ws = p.workspace + row * p.splits * S::kMergeFloats;
    float o = 0.f;
    if (n > 0) {
        float M = -INFINITY;
        for (int s = 0; s < n; ++s) M = fmaxf(M, ws[s * S::kMergeFloats + D]);
        float acc = 0.f, lsum = 0.f;
        for (int s = 0; s < n; ++s) {
            const float wgt = fast_exp2(ws[s * S::kMergeFloats + D] - M);
            acc += wgt * ws[s * S::kMergeFloats + d];
            lsum += wgt * ws[s * S::kMergeFloats + D + 1];
        }
        o = acc / lsum;
    }
    if (p.out_f32) ((float*)p.out)[row * D + d] = o;
    else ((__bf16*)p.out)[row * D + d] = (__bf16)o;
}

int32_t choose_partition_tokens(int32_t batch, int32_t num_kv_heads, int32_t max_context_len)
{
    // Aim for a few workgroups per compute unit slot while keeping partitions long enough that
    // the partial results (written and re-read once) stay a small fraction of the KV bytes.
    const int64_t target_groups = 2048;
    const int64_t pairs = (int64_t)batch * num_kv_heads;
    int32_t part = 8192;
    while (part > 256 && pairs * ((max_context_len + part - 1) / part) < target_groups) part >>= 1;
    return part;
}

template <int D>
static hipError_t launch_decode_d(const DecodeParams& p, hipStream_t stream)
{
    using S = Shape<D>;
    const size_t stage = (size_t)kWaves * S::kVTileBytes;
    const size_t merge = (size_t)kWaves * kMaxGroup * S::kLdsRow * sizeof(float);
    const size_t lds = stage > merge ? stage : merge;
    dim3 grid((uint32_t)p.splits, (uint32_t)p.num_kv_heads, (uint32_t)p.batch);
    hipLaunchKernelGGL(decode_partition_kernel<D>, grid, dim3(kThreads), lds, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.splits > 1) {
        dim3 mgrid((uint32_t)p.num_q_heads, (uint32_t)p.batch, 1);
        hipLaunchKernelGGL(decode_merge_kernel<D>, mgrid, dim3(D), 0, stream, p);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_decode(const DecodeParams& p, int head_dim, hipStream_t stream)
{
    if (head_dim == 128) return launch_decode_d<128>(p, stream);
    if (head_dim == 64) return launch_decode_d<64>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvflow
