// Paged decode attention for gfx950: one query token per sequence attends to that sequence's
// cached K/V, stored as fixed-size blocks reached through a block table (the block-represented
// KV cache of paper Sec. 3.2 item 3).
//
// The work is one scan of the KV cache (HBM-bound), organised as a flat space of 32-token tiles:
// tile index = ((sequence, KV head), tile within the sequence), sequences in batch order.  The
// grid is persistent: every wavefront owns one contiguous, equally long run of that space, so the
// load is even for any mix of context lengths, and a wavefront streams tile after tile with the
// next tile's loads in flight.  Wavefronts never synchronise with each other after start-up.
//
// Per tile, the G = Hq/Hkv query heads that share the KV head form the 16-wide N side of MFMA
// tiles, so each K/V byte is loaded once and serves all G heads:
//     S^T[token][head] = K[token][d] * Q^T[d][head]          (v_mfma_f32_16x16x32_bf16, 16 tokens)
//     O^T[d][head]    += V^T[d][token] * P^T[token][head]    (same instruction, 32 tokens)
// In this orientation a lane's softmax statistics belong to one head (lane % 16), the
// probabilities leave the first product in the register layout the second one wants, and the
// running rescale of O is lane-local.  K rows go from HBM straight into the A-operand layout;
// V rows are loaded fully coalesced, staged in a per-wave LDS tile and read back transposed
// (ds_read_b64_tr_b16).  Registers that an MFMA or the LDS write has consumed are refilled at
// once with the next tile's loads.
//
// When a wavefront's run leaves a (sequence, KV head) row it writes one record (un-normalised
// O, running max, denominator) per query head; a second small kernel merges the records of a
// row in ascending run order.  Both the split and the merge order depend only on the context
// lengths, so the result depends only on logical token positions.

#include "kv_decode_common.h"

namespace kvflow {

template <int D>
struct Shape {
    static constexpr int kSteps = D / 32;            // MFMA k-steps over the head dimension
    static constexpr int kDTiles = D / 16;           // 16-channel output tiles
    static constexpr int kLanesPerRow = D / 8;       // lanes covering one K/V row with 16-byte loads
    static constexpr int kRowsPerChunk = 64 / kLanesPerRow;
    static constexpr int kVChunks = kTileTokens / kRowsPerChunk;   // 1 KiB loads per 32-token V tile
    static constexpr int kPitch = D * 2 + 32;        // LDS row pitch in bytes (pad avoids bank conflicts)
    static constexpr int kVTileBytes = kTileTokens * kPitch;
    static constexpr int kRecord = D + kRecordPad;   // floats per (run, row, head) record: O[D], m, l, pad
};

// One flat tile: which sequence / KV head / tile, plus the physical blocks of its two subtiles.
struct TileDesc {
    int b, kvh, tile, L, ntiles;
    int pb0, pb1;
};

// The pointers are separate __restrict__ kernel arguments (not members of the by-value struct) so
// that the compiler may read the block table and the context lengths with scalar loads, which
// do not share a counter with the K/V vector loads in flight.
// The register budget is capped at that of 3 waves per SIMD: the accumulators then stay in
// ordinary vector registers (no copies to and from the accumulation file around the rescale).
template <int D>
__global__ __launch_bounds__(kDecodeThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void decode_partition_kernel(
    const DecodeParams p, const uint16_t* __restrict__ q_ptr, const uint16_t* __restrict__ pool_ptr,
    const int32_t* __restrict__ table_ptr, const int32_t* __restrict__ lens_ptr,
    int32_t* __restrict__ ws_cum, float* __restrict__ ws_records)
{
    using S = Shape<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int B = p.batch, Hkv = p.num_kv_heads, G = p.group;

    // ---- start-up: tile counts of the sequences (scan in LDS), this wavefront's run, its first tile
    int* cum = (int*)smem;                                            // [B + 1]
    const RunSpan rs = split_into_runs<kTileTokens>(cum, ws_cum, lens_ptr, B, Hkv, lane, wave);
    const int t_begin = rs.t_begin, t_end = rs.t_end;
    TileDesc cur = {0, 0, 0, 0, 0, 0, 0};
    if (t_begin < t_end) {
        const TilePos pos = locate_tile(cum, lens_ptr, B, Hkv, t_begin);
        cur.b = pos.b; cur.kvh = pos.kvh; cur.tile = pos.tile; cur.L = pos.L; cur.ntiles = pos.ntiles;
    }
    __syncthreads();                                                  // cum[] is dead; LDS becomes V staging
    if (t_begin >= t_end) return;

    const int bs = p.block_size;
    const int64_t head_elems = (int64_t)bs * D;                       // one (block, K|V, head) tile
    const int64_t v_off = (int64_t)Hkv * head_elems;                  // K -> V within a block
    const int64_t blk_elems = 2 * v_off;
    const int koff = j * D + 8 * g;                                   // K operand: row j, channels 8g..
    const int vrow = lane / S::kLanesPerRow;                          // V natural: row within a chunk
    const int vcol = (lane % S::kLanesPerRow) * 8;
    unsigned char* vt = smem + wave * S::kVTileBytes;                 // this wave's V staging tile
    const int vw_off = vrow * S::kPitch + vcol * 2;
    // transposed read: lanes 4e+c of a 16-lane group point at row 4g+e, channels 4c..4c+3 of a d-tile
    const int vr_off = (4 * g + (j >> 2)) * S::kPitch + (j & 3) * 8;

    auto fetch_ids = [&](TileDesc& d) {
        const int32_t* row = table_ptr + (int64_t)d.b * p.max_blocks_per_seq;
        const int t0 = d.tile * kTileTokens;
        d.pb0 = row[t0 >> p.block_shift];
        // second subtile: if it has no valid token the index falls back to the block of the last
        // token, which is subtile 0's block; its data is masked out below.  Two independent loads.
        d.pb1 = row[min(t0 + 16, d.L - 1) >> p.block_shift];
    };
    // step to the next flat tile; the caller guarantees that one exists
    auto advance = [&](TileDesc& d) {
        if (++d.tile == d.ntiles) {
            d.tile = 0;
            if (++d.kvh == Hkv) {
                d.kvh = 0;
                do { d.L = lens_ptr[++d.b]; } while (d.L == 0);
                d.ntiles = (d.L + kTileTokens - 1) / kTileTokens;
            }
        }
    };
    auto subtile_base = [&](const TileDesc& d, int u) -> int64_t {
        const int t0 = d.tile * kTileTokens + 16 * u;
        const bool live = u == 0 || t0 < d.L;
        const int r0 = live ? (t0 & (bs - 1)) : ((t0 - 16) & (bs - 1));
        return (int64_t)(u == 0 ? d.pb0 : d.pb1) * blk_elems + (int64_t)d.kvh * head_elems + (int64_t)r0 * D;
    };

    bf16x8 qreg[S::kSteps];                                           // Q^T: head j, channels 32ks + 8g .. +7
    bf16x8 qnext[S::kSteps];                                          // same for the row that follows
    bf16x8 kreg[2][S::kSteps];
    u32x4 vreg[S::kVChunks];
    auto load_q = [&](bf16x8 (&dst)[S::kSteps], const TileDesc& d) {
        const uint16_t* qrow = q_ptr + ((int64_t)d.b * p.num_q_heads + (int64_t)d.kvh * G + j) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < S::kSteps; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (j < G) t = *(const u32x4*)(qrow + 32 * ks);
            dst[ks] = __builtin_bit_cast(bf16x8, t);
        }
    };
    auto issue_k = [&](int64_t base0, int64_t base1) {
        const uint16_t* k0 = pool_ptr + base0 + koff;
        const uint16_t* k1 = pool_ptr + base1 + koff;
#pragma unroll
        for (int ks = 0; ks < S::kSteps; ++ks) {
            kreg[0][ks] = __builtin_bit_cast(bf16x8, stream_load(k0 + 32 * ks));
            kreg[1][ks] = __builtin_bit_cast(bf16x8, stream_load(k1 + 32 * ks));
        }
    };
    auto issue_v = [&](int64_t base0, int64_t base1) {
        const uint16_t* v0 = pool_ptr + base0 + v_off + vrow * D + vcol;
        const uint16_t* v1 = pool_ptr + base1 + v_off + vrow * D + vcol;
#pragma unroll
        for (int c = 0; c < S::kVChunks; ++c) {
            const int row16 = (c * S::kRowsPerChunk) & 15;            // first row of the chunk in its subtile
            vreg[c] = stream_load((c * S::kRowsPerChunk < 16 ? v0 : v1) + row16 * D);
        }
    };

    float m_run = -INFINITY;      // running max of scaled scores (log2 domain) for head j
    float l_run = 0.f;            // this lane's share of the running denominator
    f32x4 oacc[S::kDTiles];
#pragma unroll
    for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    fetch_ids(cur);
    load_q(qreg, cur);
    issue_k(subtile_base(cur, 0), subtile_base(cur, 1));
    issue_v(subtile_base(cur, 0), subtile_base(cur, 1));
    TileDesc nxt = cur;
    if (t_begin + 1 < t_end) { advance(nxt); fetch_ids(nxt); }
#pragma unroll
    for (int ks = 0; ks < S::kSteps; ++ks) qnext[ks] = qreg[ks];
    if (t_begin + 1 < t_end && (nxt.b != cur.b || nxt.kvh != cur.kvh)) load_q(qnext, nxt);

    // One tile.  HAS_NXT is a compile-time flag: inside the steady-state loop the next tile's loads
    // are issued unconditionally, which lets the compiler count outstanding loads exactly and keep
    // them in flight across the whole iteration; the last tile of the run is a second instance.
    auto do_tile = [&](int t, auto has_nxt_tag) {
        constexpr bool has_nxt = decltype(has_nxt_tag)::value;
        // addresses of the next tile from block ids that were fetched a whole tile ago
        const int64_t nbase0 = has_nxt ? subtile_base(nxt, 0) : 0, nbase1 = has_nxt ? subtile_base(nxt, 1) : 0;
        const bool has_nn = t + 2 < t_end;
        const bool row_ends = !has_nxt || nxt.b != cur.b || nxt.kvh != cur.kvh;
        const int tok0 = cur.tile * kTileTokens;
        const bool ragged = tok0 + kTileTokens > cur.L;               // wave-uniform

        // ---- S^T = K Q^T for the two 16-token subtiles; then refill the K registers (and swap in
        //      the next row's Q, fetch the Q of the row after that)
        f32x4 s[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < S::kSteps; ++ks)
                s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[u][ks], qreg[ks], s[u], 0, 0, 0);
        }
        if (has_nxt) {
            issue_k(nbase0, nbase1);
            if (row_ends) {                                           // Q of the next row was fetched a tile ago
#pragma unroll
                for (int ks = 0; ks < S::kSteps; ++ks) qreg[ks] = qnext[ks];
            }
        }
        // block ids two tiles ahead (scalar loads, consumed at the top of the next tile): issued
        // here, after every address that depends on earlier scalar loads has been formed
        TileDesc nn = nxt;
        if (has_nn) { advance(nn); fetch_ids(nn); }
        if (has_nn && (nn.b != nxt.b || nn.kvh != nxt.kvh)) load_q(qnext, nn);

        // ---- V tile -> LDS (rows past the end are zeroed: 0 * NaN must not reach the sum)
#pragma unroll
        for (int c = 0; c < S::kVChunks; ++c) {
            u32x4 val = vreg[c];
            if (ragged && tok0 + c * S::kRowsPerChunk + vrow >= cur.L) val = u32x4{0u, 0u, 0u, 0u};
            *(u32x4*)(vt + vw_off + c * S::kRowsPerChunk * S::kPitch) = val;
        }
        if (has_nxt) issue_v(nbase0, nbase1);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- online softmax; lane (g, j): s[u][i] is head j, token tok0 + 16u + 4g + i
        float tt[8];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) tt[4 * u + i] = s[u][i] * p.scale_log2e;
        if (ragged) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tok0 + 16 * u + 4 * g + i >= cur.L) tt[4 * u + i] = -INFINITY;
        }
        float mx = fmaxf(fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3])),
                         fmaxf(fmaxf(tt[4], tt[5]), fmaxf(tt[6], tt[7])));
        // wave-uniform: does any lane see a score above its head's running max by more than the slack?
        if (__builtin_amdgcn_ballot_w64(mx > m_run + kMaxSlack) != 0) {
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);                     // finite: the tile has a valid token
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] *= alpha;
        }
        float psum = 0.f;
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float pe = fast_exp2(tt[e] - m_run);
            psum += pe;
            pb[e] = (__bf16)pe;
        }
        l_run += psum;

        // ---- O^T += V^T P^T over the tile's 32 tokens, one 16-channel tile at a time
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt) {
            typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt + vr_off + dt * 32));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s16x4_ptr)(vt + vr_off + 16 * S::kPitch + dt * 32));
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pb, oacc[dt], 0, 0, 0);
        }
        // the next tile's LDS writes must stay behind these reads in program order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- leaving the row: one record per query head, then start afresh
        if (row_ends) {
            leave_row<D>(ws_records, oacc, m_run, l_run, rs.w, cur.b, cur.kvh, Hkv, G, g, j);
            m_run = -INFINITY;
            l_run = 0.f;
#pragma unroll
            for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        cur = nxt;
        nxt = nn;
    };
    for (int t = t_begin; t + 1 < t_end; ++t) do_tile(t, std::true_type{});
    do_tile(t_end - 1, std::false_type{});
}

template <int D>
static hipError_t launch_decode_d(const DecodeParams& p, int workgroups, hipStream_t stream)
{
    using S = Shape<D>;
    const size_t stage = (size_t)kDecodeWaves * S::kVTileBytes;
    const size_t scan = (size_t)(p.batch + 1) * sizeof(int);
    const size_t lds = stage > scan ? stage : scan;
    hipLaunchKernelGGL(decode_partition_kernel<D>, dim3((uint32_t)workgroups), dim3(kDecodeThreads), lds,
                       stream, p, p.q, p.pool, p.block_table, p.context_lens, p.ws_cum, p.ws_records);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_merge<D>(p, workgroups, stream);
}

hipError_t launch_decode(const DecodeParams& p, int head_dim, int workgroups, hipStream_t stream)
{
    if (head_dim == 128) return launch_decode_d<128>(p, workgroups, stream);
    if (head_dim == 64) return launch_decode_d<64>(p, workgroups, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvflow
