// Paged decode attention over an FP8 (OCP E4M3) block pool for gfx950: the same persistent,
// flat-tile-space scan as the bf16 kernel, with half the bytes per cached token.
//
// What changes is the front end.  A tile is 64 tokens, so that a wavefront still has 16 KiB of
// loads in flight.  K rows are loaded as 16 consecutive channels per lane and converted in
// registers (v_cvt_scalef32_pk_bf16_fp8 with scale 1, exact) into two MFMA A operands; Q^T is
// loaded with the matching channel order.  V rows are loaded fully coalesced, converted, and
// staged in LDS as bf16, so the transposed read and the second product are those of the bf16
// kernel.  The per-tensor scales never touch the data: the K scale is folded into the softmax
// scale on the host, the V scale multiplies the output in the merge kernel.
// The tile is processed as two 32-token halves (QK^T for both, then per half: V staging,
// softmax, PV); K registers are refilled after the four QK^T products, V registers after the
// second half has been staged.

#include "kv_decode_common.h"

namespace kvflow {

constexpr int kTile8 = 64;                           // tokens per flat tile of the FP8 kernel

template <int D>
struct Shape8 {
    static constexpr int kSteps = D / 32;            // MFMA k-steps over the head dimension
    static constexpr int kDTiles = D / 16;           // 16-channel output tiles
    static constexpr int kKLoads = D / 64;           // 16-byte K loads per lane and 16-token subtile
    static constexpr int kVLanesPerRow = D / 16;     // lanes covering one V row with 16-byte loads
    static constexpr int kVRowsPerLoad = 64 / kVLanesPerRow;
    static constexpr int kVLoadsPerHalf = 32 / kVRowsPerLoad;
    // LDS row pitch of the bf16 staging tile.  A lane stages 32 bytes (16 converted channels) with two
    // 16-byte stores.  Measured on the LDS alone, 16-byte stores run at about 64 bytes per clock whatever
    // the pitch (the bank-conflict counter charges them the extra cycles), and the transposed 8-byte reads
    // run conflict-free at pitches of 272, 288 and 320 but at a third of that rate at 256 and half at 264.
    // Making a row's first stores contiguous (channels permuted within the row, reads following) took 15 %
    // off the LDS time in isolation and nothing measurable off the kernel: the LDS is busy for under a
    // tenth of a wave's cycles here.
    static constexpr int kPitch = D == 128 ? D * 2 + 16 : D * 2 + 32;
    static constexpr int kVTileBytes = 32 * kPitch;
    static constexpr int kRecord = D + kRecordPad;
};

// One flat tile: which sequence / KV head / tile, plus the physical blocks of its four subtiles.
struct TileDesc8 {
    int b, kvh, tile, L, ntiles;
    int pb[4];
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 16 FP8 E4M3 values -> 8 + 8 bf16 values, element order kept (byte i of the load is element i).
// v_cvt_scalef32_pk_bf16_fp8 turns two FP8 bytes (the low or the high half of a word) into a packed
// bf16 pair in one instruction; with scale 1 the conversion is exact (every E4M3 number is a bf16 number).
__device__ __forceinline__ void fp8x16_to_bf16(u32x4 raw, bf16x8& lo, bf16x8& hi)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, false);
        const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, true);
        bf16x8& dst = w < 2 ? lo : hi;
        const int o = (w & 1) * 4;
        dst[o + 0] = a.x;
        dst[o + 1] = a.y;
        dst[o + 2] = b.x;
        dst[o + 3] = b.y;
    }
}

__device__ __forceinline__ u32x4 stream_load8(const uint8_t* p)
{
    return __builtin_nontemporal_load((const u32x4*)p);
}

template <int D>
__global__ __launch_bounds__(kDecodeThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_partition_fp8_kernel(
    const DecodeParams p, const uint16_t* __restrict__ q_ptr, const uint8_t* __restrict__ pool_ptr,
    const int32_t* __restrict__ table_ptr, const int32_t* __restrict__ lens_ptr,
    int32_t* __restrict__ ws_cum, float* __restrict__ ws_records)
{
    using S = Shape8<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int B = p.batch, Hkv = p.num_kv_heads, G = p.group;

    // ---- start-up: 64-token tile counts of the sequences (scan in LDS), this wavefront's run, its first tile
    int* cum = (int*)smem;                                            // [B + 1]
    const RunSpan rs = split_into_runs<kTile8>(cum, ws_cum, lens_ptr, B, Hkv, lane, wave);
    const int t_begin = rs.t_begin, t_end = rs.t_end;
    TileDesc8 cur = {0, 0, 0, 0, 0, {0, 0, 0, 0}};
    if (t_begin < t_end) {
        const TilePos pos = locate_tile(cum, lens_ptr, B, Hkv, t_begin);
        cur.b = pos.b; cur.kvh = pos.kvh; cur.tile = pos.tile; cur.L = pos.L; cur.ntiles = pos.ntiles;
    }
    __syncthreads();                                                  // cum[] is dead; LDS becomes V staging
    if (t_begin >= t_end) return;

    const int bs = p.block_size;
    const int64_t head_bytes = (int64_t)bs * D;                       // one (block, K|V, head) tile, 1 byte per element
    const int64_t v_off = (int64_t)Hkv * head_bytes;                  // K -> V within a block
    const int64_t blk_bytes = 2 * v_off;
    const int koff = j * D + 16 * g;                                  // K: row j, channels 64m + 16g .. +15
    const int vrow = lane / S::kVLanesPerRow;                         // V natural: row within a load
    const int vcc = lane % S::kVLanesPerRow;                          // 16-channel group of the row
    unsigned char* vt = smem + wave * S::kVTileBytes;                 // this wave's bf16 V staging tile (32 tokens)
    const int vw_off = vrow * S::kPitch + vcc * 32;
    // transposed read: lanes 4e+c of a 16-lane group point at row 4g+e, channels 4c..4c+3 of a d-tile
    const int vr_off = (4 * g + (j >> 2)) * S::kPitch + (j & 3) * 8;

    auto fetch_ids = [&](TileDesc8& d) {
        const int32_t* row = table_ptr + (int64_t)d.b * p.max_blocks_per_seq;
        const int t0 = d.tile * kTile8;
        // a subtile with no valid token falls back to the block of the last token (valid memory; its
        // data is masked out below).  Four independent scalar loads.
#pragma unroll
        for (int u = 0; u < 4; ++u) d.pb[u] = row[min(t0 + 16 * u, d.L - 1) >> p.block_shift];
    };
    // step to the next flat tile; the caller guarantees that one exists
    auto advance = [&](TileDesc8& d) {
        if (++d.tile == d.ntiles) {
            d.tile = 0;
            if (++d.kvh == Hkv) {
                d.kvh = 0;
                do { d.L = lens_ptr[++d.b]; } while (d.L == 0);
                d.ntiles = (d.L + kTile8 - 1) / kTile8;
            }
        }
    };
    // byte offset of subtile u's K rows; a subtile past the end reads rows 0..15 of the fallback block
    auto subtile_base = [&](const TileDesc8& d, int u) -> int64_t {
        const int tu = d.tile * kTile8 + 16 * u;
        const int r0 = tu < d.L ? (tu & (bs - 1)) : 0;
        return (int64_t)d.pb[u] * blk_bytes + (int64_t)d.kvh * head_bytes + (int64_t)r0 * D;
    };

    bf16x8 qreg[S::kSteps];       // Q^T: head j; k-step s holds channels 64(s/2) + 16g + 8(s%2) .. +7
    bf16x8 qnext[S::kSteps];      // same for the row that follows
    u32x4 kraw[4][S::kKLoads];    // 16 FP8 channels per load
    u32x4 vraw[2 * S::kVLoadsPerHalf];
    auto load_q = [&](bf16x8 (&dst)[S::kSteps], const TileDesc8& d) {
        const uint16_t* qrow = q_ptr + ((int64_t)d.b * p.num_q_heads + (int64_t)d.kvh * G + j) * D + 16 * g;
#pragma unroll
        for (int s = 0; s < S::kSteps; ++s) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (j < G) t = *(const u32x4*)(qrow + 64 * (s / 2) + 8 * (s % 2));
            dst[s] = __builtin_bit_cast(bf16x8, t);
        }
    };
    auto issue_k = [&](const int64_t (&sb)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int m = 0; m < S::kKLoads; ++m) kraw[u][m] = stream_load8(pool_ptr + sb[u] + koff + 64 * m);
    };
    auto issue_v = [&](const int64_t (&sb)[4]) {
#pragma unroll
        for (int c = 0; c < 2 * S::kVLoadsPerHalf; ++c) {
            const int tt = c * S::kVRowsPerLoad;                      // first token of the load within the tile
            vraw[c] = stream_load8(pool_ptr + sb[tt / 16] + v_off + ((tt % 16) + vrow) * D + vcc * 16);
        }
    };

    float m_run = -INFINITY;      // running max of scaled scores (log2 domain) for head j
    float l_run = 0.f;            // this lane's share of the running denominator
    f32x4 oacc[S::kDTiles];
#pragma unroll
    for (int dt = 0; dt < S::kDTiles; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    fetch_ids(cur);
    load_q(qreg, cur);
    {
        const int64_t sb[4] = {subtile_base(cur, 0), subtile_base(cur, 1), subtile_base(cur, 2), subtile_base(cur, 3)};
        issue_k(sb);
        issue_v(sb);
    }
    TileDesc8 nxt = cur;
    if (t_begin + 1 < t_end) { advance(nxt); fetch_ids(nxt); }
#pragma unroll
    for (int s = 0; s < S::kSteps; ++s) qnext[s] = qreg[s];
    if (t_begin + 1 < t_end && (nxt.b != cur.b || nxt.kvh != cur.kvh)) load_q(qnext, nxt);

    // One 64-token tile.  HAS_NXT is a compile-time flag: inside the steady-state loop the next
    // tile's loads are unconditional, so the compiler counts outstanding loads exactly; the last
    // tile of the run is a second instance.
    auto do_tile = [&](int t, auto has_nxt_tag) {
        constexpr bool has_nxt = decltype(has_nxt_tag)::value;
        int64_t nsb[4] = {0, 0, 0, 0};                                // next tile's addresses, ids fetched a tile ago
        if (has_nxt) {
#pragma unroll
            for (int u = 0; u < 4; ++u) nsb[u] = subtile_base(nxt, u);
        }
        const bool has_nn = t + 2 < t_end;
        const bool row_ends = !has_nxt || nxt.b != cur.b || nxt.kvh != cur.kvh;
        const int tok0 = cur.tile * kTile8;
        const bool ragged = tok0 + kTile8 > cur.L;                    // wave-uniform

        // ---- S^T = K Q^T for the four 16-token subtiles; then refill the K registers
        f32x4 s[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < S::kKLoads; ++m) {
                bf16x8 klo, khi;
                fp8x16_to_bf16(kraw[u][m], klo, khi);
                s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(klo, qreg[2 * m], s[u], 0, 0, 0);
                s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khi, qreg[2 * m + 1], s[u], 0, 0, 0);
            }
        }
        if (has_nxt) {
            issue_k(nsb);
            if (row_ends) {                                           // Q of the next row was fetched a tile ago
#pragma unroll
                for (int ks = 0; ks < S::kSteps; ++ks) qreg[ks] = qnext[ks];
            }
        }
        // block ids two tiles ahead (scalar loads, consumed at the top of the next tile)
        TileDesc8 nn = nxt;
        if (has_nn) { advance(nn); fetch_ids(nn); }
        if (has_nn && (nn.b != nxt.b || nn.kvh != nxt.kvh)) load_q(qnext, nn);

#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int tokh = tok0 + 32 * h;
            // ---- V half -> bf16 -> LDS (rows past the end are zeroed: 0 * NaN must not reach the sum)
#pragma unroll
            for (int c = 0; c < S::kVLoadsPerHalf; ++c) {
                bf16x8 vlo, vhi;
                fp8x16_to_bf16(vraw[h * S::kVLoadsPerHalf + c], vlo, vhi);
                u32x4 a = __builtin_bit_cast(u32x4, vlo), b2 = __builtin_bit_cast(u32x4, vhi);
                if (ragged && tokh + c * S::kVRowsPerLoad + vrow >= cur.L) { a = u32x4{0u, 0u, 0u, 0u}; b2 = a; }
                unsigned char* dst = vt + vw_off + c * S::kVRowsPerLoad * S::kPitch;
                *(u32x4*)dst = a;
                *(u32x4*)(dst + 16) = b2;
            }
            if (h == 1 && has_nxt) issue_v(nsb);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

            // ---- online softmax; lane (g, j): s[2h + u][i] is head j, token tokh + 16u + 4g + i
            float tt[8];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) tt[4 * u + i] = s[2 * h + u][i] * p.scale_log2e;
            if (ragged) {
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (tokh + 16 * u + 4 * g + i >= cur.L) tt[4 * u + i] = -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3])),
                             fmaxf(fmaxf(tt[4], tt[5]), fmaxf(tt[6], tt[7])));
            // wave-uniform: does any lane see a score above its head's running max by more than the slack?
            if (__builtin_amdgcn_ballot_w64(mx > m_run + kMaxSlack) != 0) {
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run, mx);                 // finite: the first half always has a valid token
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

            // ---- O^T += V^T P^T over the half's 32 tokens, one 16-channel tile at a time
#pragma unroll
            for (int dt = 0; dt < S::kDTiles; ++dt) {
                typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt + vr_off + dt * 32));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_s16x4_ptr)(vt + vr_off + 16 * S::kPitch + dt * 32));
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pb, oacc[dt], 0, 0, 0);
            }
            // the next LDS writes must stay behind these reads in program order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }

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
static hipError_t launch_decode_fp8_d(const DecodeParams& p, int workgroups, hipStream_t stream)
{
    using S = Shape8<D>;
    const size_t stage = (size_t)kDecodeWaves * S::kVTileBytes;
    const size_t scan = (size_t)(p.batch + 1) * sizeof(int);
    const size_t lds = stage > scan ? stage : scan;
    hipLaunchKernelGGL(decode_partition_fp8_kernel<D>, dim3((uint32_t)workgroups), dim3(kDecodeThreads), lds, stream,
                       p, p.q, (const uint8_t*)p.pool, p.block_table, p.context_lens, p.ws_cum, p.ws_records);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_merge<D>(p, workgroups, stream);
}

hipError_t launch_decode_fp8(const DecodeParams& p, int head_dim, int workgroups, hipStream_t stream)
{
    if (head_dim == 128) return launch_decode_fp8_d<128>(p, workgroups, stream);
    if (head_dim == 64) return launch_decode_fp8_d<64>(p, workgroups, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvflow
