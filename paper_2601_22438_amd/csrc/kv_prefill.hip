// Causal attention of many query tokens per sequence over the block-paged KV cache: the
// recomputation that a node falls back to when it dropped replicas (paper Sec. 3.2 item 3).
// The query tokens are the newest q_len tokens of a sequence whose K/V rows are in the pool
// already; query j sits at position context_len - q_len + j and sees keys 0 .. its position.
//
// This is a dense contraction (4 * head_dim flops per (query, key) pair), bound by the matrix
// cores, not by HBM.  A workgroup of 8 wavefronts (two per SIMD) walks the keys of one
// (sequence, KV head) in 32-token tiles that it stages in LDS once (a ring of four stages, later
// tiles' global loads in flight) and that all wavefronts consume.  Each wavefront owns 16 * NQB
// query rows: query tokens of one query head, so the wavefronts are the query heads of a group
// over the same token range when the group allows it (same causal extent, K/V shared), else
// neighbouring token ranges.  Per tile and wavefront, in the same transposed orientation as the
// decode kernel:
//     S^T[key][query] = K[key][d] * Q^T[d][query]          (v_mfma_f32_16x16x32_bf16)
//     O^T[d][query]  += V^T[d][key] * P^T[key][query]
// so a lane's softmax statistics belong to one query (lane % 16), P leaves the first product in
// the layout the second one wants, Q stays in registers for the whole kernel and every K/V
// fragment read from LDS serves NQB MFMAs.  The loop is software-pipelined: while the vector ALU
// turns tile t's scores into probabilities the matrix core forms tile t + 1's scores, and the K
// fragments of tile t + 2 and the V fragments of tile t are read from LDS a phase before use.
//
// Grid: x = query-head group (fastest, so that with 8 or more groups the workgroups that read
// one KV head's tiles land on one XCD and share its L2), y = (token range, heaviest (latest)
// first) x (part of the key range), z = sequence.  With more than one part per key range every
// workgroup leaves a record per (query row, head) and prefill_merge_kernel combines them; this
// fills the chip when there are few query tokens over long contexts.

#include "kv_decode_common.h"

namespace kvflow {

// Floats per record of a part of the key range: O[head_dim], running max, denominator, pad to 16 bytes.
template <int D>
constexpr int kPrefillRecord = D + kRecordPad;
// "No key seen yet": a finite stand-in for minus infinity, so that differences of maxima stay finite.
constexpr float kPrefillNoMax = -1e30f;

template <int D>
struct PrefillShape {
    static constexpr int kSteps = D / 32;                 // MFMA k-steps over the head dimension
    static constexpr int kDTiles = D / 16;                // 16-channel output tiles
    static constexpr int kLanesPerRow = D / 8;            // lanes covering one K/V row with 16-byte loads
    static constexpr int kLoaders = kTileTokens * kLanesPerRow;   // threads that stage a tile, one row chunk each
    static_assert(kLoaders <= kPrefillThreads && kLoaders % 64 == 0, "whole wavefronts stage the tile");
    static constexpr int kKPitch = D * 2 + 16;            // LDS row pitches in bytes: 16 rows read by 16 lanes
    static constexpr int kVPitch = D * 2 + 32;            // (K) / transposed 4x16 reads (V) hit distinct banks
    static constexpr int kKBytes = kTileTokens * kKPitch;
    static constexpr int kVBytes = kTileTokens * kVPitch;
    static constexpr int kStage = kKBytes + kVBytes;
    static constexpr int kRing = 4;
    static constexpr int kLdsBytes = kRing * kStage;
};

// Register budget of 2 wavefronts per SIMD: the 8 wavefronts of a workgroup fill a compute unit.
// FP8: the pool holds OCP E4M3 bytes; a staged chunk of 8 elements is 8 bytes in the pool and is widened
// to bf16 (exactly) on its way into LDS, so everything after the staging is the bf16 path.  The K
// scale is folded into the score scale, the V scale into the final normalisation.
template <int D, int NQB, bool FP8>
__global__ __launch_bounds__(kPrefillThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_kernel(
    const PrefillParams p, const uint16_t* __restrict__ q_ptr, const void* __restrict__ pool_ptr,
    const int32_t* __restrict__ table_ptr, const int32_t* __restrict__ lens_ptr,
    const int32_t* __restrict__ qs_ptr, void* __restrict__ out_ptr)
{
    using S = PrefillShape<D>;
    constexpr int QW = 16 * NQB;                          // query rows per wavefront
    static_assert(kTileTokens == 32, "tile indices below are positions >> 5");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // S::kLdsBytes

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int b = blockIdx.z;
    const int L = lens_ptr[b];
    const int qs = qs_ptr[b];
    const int n = qs_ptr[b + 1] - qs;
    const int hpw = p.heads_per_wg, tbw = kPrefillWaves / hpw;
    const int ntb = (n + QW - 1) / QW;                    // token ranges of this sequence
    // blockIdx.y = (group of token ranges, heaviest first) x (part of the key range)
    const int ns = p.key_splits, split = (int)blockIdx.y % ns;
    const int tbg = (ntb + tbw - 1) / tbw - 1 - (int)blockIdx.y / ns;
    if (tbg < 0) return;

    const int head = blockIdx.x * hpw + wave % hpw;
    const int kvh = (blockIdx.x * hpw) / p.group;
    const int tb = tbg * tbw + wave / hpw;
    const bool active = tb < ntb;                         // wave-uniform
    const int j0 = tb * QW;
    const int p0 = L - n;                                 // position of query 0 (negative: more queries than context)
    const bool f32out = p.out_f32 != 0;

    // query rows of this lane: query block qb, column j
    int qidx[NQB], qpos[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        qidx[qb] = j0 + 16 * qb + j;
        qpos[qb] = p0 + min(qidx[qb], n - 1);
    }
    auto store_rows = [&](const f32x4 (&o)[NQB][S::kDTiles], const float (&inv)[NQB]) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            if (qidx[qb] >= n) continue;
            const float f = qpos[qb] < 0 ? 0.f : inv[qb] * p.out_scale;   // a query before position 0 sees nothing
            const int64_t row = ((int64_t)(qs + qidx[qb]) * p.num_q_heads + head) * D + 4 * g;
#pragma unroll
            for (int dt = 0; dt < S::kDTiles; ++dt) {
                const f32x4 v = qpos[qb] < 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : o[qb][dt] * f;
                if (f32out) {
                    *(f32x4*)((float*)out_ptr + row + 16 * dt) = v;
                } else {
                    typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
                    bf16x4 h;
#pragma unroll
                    for (int i = 0; i < 4; ++i) h[i] = (__bf16)v[i];
                    *(bf16x4*)((__bf16*)out_ptr + row + 16 * dt) = h;
                }
            }
        }
    };

    // With the key range cut into parts, a part leaves one record per (query row, head): O un-normalised,
    // running max, denominator; a second kernel combines the parts of a row in ascending order.
    auto store_records = [&](const f32x4 (&o)[NQB][S::kDTiles], const float (&m)[NQB], const float (&l)[NQB]) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            if (qidx[qb] >= n) continue;
            const bool none = qpos[qb] < 0;                          // a query before position 0 sees nothing
            float* rec = p.ws + (((int64_t)split * p.total_q + qs + qidx[qb]) * p.num_q_heads + head) * kPrefillRecord<D>;
#pragma unroll
            for (int dt = 0; dt < S::kDTiles; ++dt)
                *(f32x4*)(rec + 16 * dt + 4 * g) = none ? f32x4{0.f, 0.f, 0.f, 0.f} : o[qb][dt];
            if (g == 0) {
                rec[D] = none ? kPrefillNoMax : m[qb];
                rec[D + 1] = none ? 0.f : l[qb];
            }
        }
    };

    f32x4 oacc[NQB][S::kDTiles];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt) oacc[qb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (L <= 0) {                                         // no cached token at all: rows of zeros
        if (active) {
            const float z[NQB] = {};
            if (ns == 1) {
                store_rows(oacc, z);
            } else {
                float none[NQB];
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) none[qb] = kPrefillNoMax;
                store_records(oacc, none, z);
            }
        }
        return;
    }

    // keys this workgroup walks: up to the position of its last query
    const int jl = min((tbg * tbw + tbw) * QW, n) - 1;
    const int nt_all = (max(p0 + jl, 0) >> 5) + 1;
    // this workgroup's part of them: tiles [t0, nt)
    const int t0 = (int)((int64_t)split * nt_all / ns), nt = (int)((int64_t)(split + 1) * nt_all / ns);
    // this wavefront: first query position (tiles that reach past it need the mask), last tile (in this part)
    const int pa = p0 + j0;
    const int tl = active ? min(max(p0 + min(j0 + QW, n) - 1, 0) >> 5, nt - 1) : t0 - 1;

    // ---- global -> LDS staging of K/V tiles
    const int bs = p.block_size;
    constexpr int kElt = FP8 ? 1 : 2;                     // bytes per pool element
    const uint32_t head_bytes = (uint32_t)bs * D * kElt;
    const uint32_t v_bytes = (uint32_t)p.num_kv_heads * head_bytes;   // K -> V within a block
    const uint32_t blk_bytes = 2 * v_bytes;
    const int r = tid / S::kLanesPerRow, c = tid % S::kLanesPerRow;
    const bool loader = tid < S::kLoaders;                // wave-uniform: stages row r, 8-element chunk c
    const int32_t* trow = table_ptr + (int64_t)b * p.max_blocks_per_seq;
    const char* lane_base = (const char*)pool_ptr + (uint64_t)kvh * head_bytes + c * (8 * kElt);
    // rows past the last cached token are read from the last token's row (always mapped) and masked
    auto load_id = [&](int t) -> int {
        int id = 0;
        if (loader) id = trow[min(kTileTokens * t + r, L - 1) >> p.block_shift];
        return id;
    };
    u32x4 kg = {0u, 0u, 0u, 0u}, vg = {0u, 0u, 0u, 0u};   // FP8: only the first two words are used
    auto gload = [&](int t, int id) {
        if (loader) {
            const int kp = min(kTileTokens * t + r, L - 1);
            const uint32_t row_off = (uint32_t)(kp & (bs - 1)) * (D * kElt);
            const char* src = lane_base + ((uint64_t)(uint32_t)id * blk_bytes + row_off);
            if (FP8) {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 k2 = *(const u32x2*)src, v2 = *(const u32x2*)(src + v_bytes);
                kg[0] = k2.x; kg[1] = k2.y;
                vg[0] = v2.x; vg[1] = v2.y;
            } else {
                kg = *(const u32x4*)src;
                vg = *(const u32x4*)(src + v_bytes);
            }
        }
    };
    // 8 E4M3 bytes (two words) -> 8 bf16, element order kept (v_cvt_scalef32_pk_bf16_fp8 with scale 1: exact)
    auto widen = [](u32x4 raw) -> u32x4 {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x8 o;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, false);
            const bf16x2 b2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, true);
            o[4 * w + 0] = a.x;
            o[4 * w + 1] = a.y;
            o[4 * w + 2] = b2.x;
            o[4 * w + 3] = b2.y;
        }
        return __builtin_bit_cast(u32x4, o);
    };
    const int lds_k_off = r * S::kKPitch + c * 16, lds_v_off = S::kKBytes + r * S::kVPitch + c * 16;
    auto lstore = [&](int t, unsigned char* buf) {
        if (loader) {
            // V rows past the end are zeroed: 0 * NaN must not reach the sum
            u32x4 k = kg, v = vg;
            if (FP8) { k = widen(k); v = widen(v); }
            if (kTileTokens * t + r >= L) v = u32x4{0u, 0u, 0u, 0u};
            *(u32x4*)(buf + lds_k_off) = k;
            *(u32x4*)(buf + lds_v_off) = v;
        }
    };

    // ---- Q^T fragments: query column j of block qb, channels 32ks + 8g .. +7.  Columns past the last
    //      query re-read the last query's row (in bounds); their results are never stored.  The
    //      fragments are written by loads and read by MFMAs only, so they may live in either
    //      register file.
    bf16x8 qreg[NQB][S::kSteps];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const uint16_t* qrow = q_ptr + ((int64_t)(qs + min(qidx[qb], n - 1)) * p.num_q_heads + head) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < S::kSteps; ++ks) qreg[qb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + 32 * ks));
    }
    const float sc = p.scale_log2e;                       // > 0
    int qvis[NQB];                                        // last visible key position of the lane's queries
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) qvis[qb] = max(qpos[qb], 0);

    // Running max (scaled, log2 domain) and denominator.  The denominator is one more row block of
    // the second product (a block of ones in place of V^T): it sums the same bf16-rounded
    // probabilities as the numerator (a single visible key gives exactly its V row) and every entry
    // of l_acc[qb] is the full sum for the lane's query, with no cross-lane reduction.
    float m_run[NQB];
    f32x4 l_acc[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) { m_run[qb] = kPrefillNoMax; l_acc[qb] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});

    const int k_off = j * S::kKPitch + 16 * g;            // K operand: row j, channels 8g ..
    // transposed V read: lanes 4e+c of a 16-lane group point at row 4g+e, channels 4c..4c+3 of a d-tile
    const int v_off_lds = S::kKBytes + (4 * g + (j >> 2)) * S::kVPitch + (j & 3) * 8;

    // K fragments of one tile (two 16-key subtiles): row j of the subtile, channels 32ks + 8g ..
    bf16x8 kf[2][S::kSteps];
    auto read_k = [&](const unsigned char* buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int ks = 0; ks < S::kSteps; ++ks)
                kf[u][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(buf + k_off + u * 16 * S::kKPitch + ks * 64));
    };
    // S^T = K Q^T from the fragments; lane (g, j): s[qb][u][i] is query column j of block qb,
    // key 32t + 16u + 4g + i
    auto qk = [&](f32x4 (&s)[NQB][2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) s[qb][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < S::kSteps; ++ks)
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
                    s[qb][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[u][ks], qreg[qb][ks], s[qb][u], 0, 0, 0);
        }
    };
    // Fresh scores of tile t: mask what the queries must not see (diagonal tiles only), then make sure
    // the running max covers them up to the slack; raising it rescales O and the denominator.
    auto settle = [&](int t, f32x4 (&s)[NQB][2]) {
        if (kTileTokens * t + kTileTokens - 1 > pa) {                 // wave-uniform
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (kTileTokens * t + 16 * u + 4 * g + i > qvis[qb]) s[qb][u][i] = -INFINITY;
        }
        float mx[NQB];
        bool raise = false;
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            mx[qb] = sc * fmaxf(fmaxf(fmaxf(s[qb][0][0], s[qb][0][1]), fmaxf(s[qb][0][2], s[qb][0][3])),
                               fmaxf(fmaxf(s[qb][1][0], s[qb][1][1]), fmaxf(s[qb][1][2], s[qb][1][3])));
            raise |= mx[qb] > m_run[qb] + kMaxSlack;
        }
        // wave-uniform: does any lane see a score above its query's running max by more than the slack?
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                float v = fmaxf(mx[qb], __shfl_xor(mx[qb], 16));
                v = fmaxf(v, __shfl_xor(v, 32));
                const float m_new = fmaxf(m_run[qb], v);
                // m_run starts at a huge negative finite number, so nothing here is inf - inf
                const float alpha = fast_exp2(m_run[qb] - m_new);
                m_run[qb] = m_new;
                l_acc[qb] *= alpha;
#pragma unroll
                for (int dt = 0; dt < S::kDTiles; ++dt) oacc[qb][dt] *= alpha;
            }
        }
    };
    // probabilities of a settled tile, in the B-operand layout of the second product
    auto probs = [&](const f32x4 (&s)[NQB][2], bf16x8 (&pb)[NQB]) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                pb[qb][e] = (__bf16)fast_exp2(__builtin_fmaf(s[qb][e >> 2][e & 3], sc, -m_run[qb]));
    };
    // V^T fragments of one tile, one per 16-channel tile: channel row j, keys {4g.., 16 + 4g..}
    bf16x8 vf[S::kDTiles];
    auto read_v = [&](const unsigned char* buf) {
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt) {
            typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(buf + v_off_lds + dt * 32));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s16x4_ptr)(buf + v_off_lds + 16 * S::kVPitch + dt * 32));
            vf[dt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    // O^T += V^T P^T over the tile's 32 keys
    auto pv = [&](const bf16x8 (&pb)[NQB]) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
            l_acc[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[qb], l_acc[qb], 0, 0, 0);
#pragma unroll
        for (int dt = 0; dt < S::kDTiles; ++dt)
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
                oacc[qb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pb[qb], oacc[qb][dt], 0, 0, 0);
    };

    // ---- pipeline over a ring of four LDS stages.  Step t: V fragments of tile t are read; tile t's
    //      probabilities (vector ALU) overlap tile t + 1's scores (matrix core, K fragments read during
    //      the step before); then the K fragments of tile t + 2 are read, the second product of tile t
    //      runs, tile t + 3 goes registers -> LDS, tile t + 4 global -> registers (block id one more
    //      tile ahead), and tile t + 1's scores are settled.  One barrier per tile.  Tiles past the
    //      end re-read the last rows (in bounds) and are never consumed.
    unsigned char* ring[S::kRing];                        // ring[i] holds tile t + i
#pragma unroll
    for (int i = 0; i < S::kRing; ++i) ring[i] = smem + i * S::kStage;
    int id = load_id(t0);
    gload(t0, id);
    id = load_id(t0 + 1);
    lstore(t0, ring[0]);
    gload(t0 + 1, id);
    id = load_id(t0 + 2);
    lstore(t0 + 1, ring[1]);
    gload(t0 + 2, id);
    id = load_id(t0 + 3);
    lstore(t0 + 2, ring[2]);
    gload(t0 + 3, id);
    id = load_id(t0 + 4);
    __syncthreads();
    auto stage = [&](int t) {                             // part of step t
        lstore(t + 3, ring[3]);
        gload(t + 4, id);
        id = load_id(t + 5);
    };
    auto rotate = [&]() {
        unsigned char* const old = ring[0];
#pragma unroll
        for (int i = 0; i + 1 < S::kRing; ++i) ring[i] = ring[i + 1];
        ring[S::kRing - 1] = old;
    };
    f32x4 sa[NQB][2], sb[NQB][2];
    if (tl >= t0) {
        read_k(ring[0]);
        qk(sa);
        settle(t0, sa);
        read_k(ring[1]);
    }
    // a step whose tile has a successor for this wavefront
    auto step = [&](int t, f32x4 (&s_cur)[NQB][2], f32x4 (&s_next)[NQB][2]) {
        bf16x8 pb[NQB];
        read_v(ring[0]);
        probs(s_cur, pb);
        qk(s_next);
        read_k(ring[2]);
        pv(pb);
        stage(t);
        settle(t + 1, s_next);
        rotate();
        __syncthreads();
    };
    int t = t0;
    for (; t + 1 < tl; t += 2) {
        step(t, sa, sb);
        step(t + 1, sb, sa);
    }
    if (t < tl) {
        step(t, sa, sb);
        ++t;
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) { sa[qb][0] = sb[qb][0]; sa[qb][1] = sb[qb][1]; }
    }
    if (t == tl) {                                        // the wavefront's last tile
        bf16x8 pb[NQB];
        read_v(ring[0]);
        probs(sa, pb);
        pv(pb);
        stage(t);
        rotate();
        __syncthreads();
        ++t;
    }
    for (; t < nt; ++t) {                                 // other wavefronts of the workgroup go on
        stage(t);
        rotate();
        __syncthreads();
    }

    if (active) {
        float inv[NQB], l[NQB];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) { l[qb] = l_acc[qb][0]; inv[qb] = 1.f / l[qb]; }
        if (ns == 1) store_rows(oacc, inv);
        else store_records(oacc, m_run, l);
    }
}

// Combines the records that the parts of the key range left for one (query row, head), in ascending
// order of the parts, and normalises.  A lane owns 4 channels of a row.
template <int D>
__global__ __launch_bounds__(256) void prefill_merge_kernel(const PrefillParams p)
{
    constexpr int kLanes = D / 4, kRows = 256 / kLanes, kRec = kPrefillRecord<D>;
    const int64_t rows = p.total_q * p.num_q_heads;
    const int64_t row = (int64_t)blockIdx.x * kRows + threadIdx.x / kLanes;
    const int c = threadIdx.x % kLanes;
    if (row >= rows) return;
    const int ns = p.key_splits;
    const int64_t stride = rows * kRec;                   // part s -> part s + 1, same row
    const float* rec = p.ws + row * kRec;
    // every load is issued before the first use: the kernel is a handful of cold reads per row
    float m[kPrefillMaxKeySplits], l_part[kPrefillMaxKeySplits];
    f32x4 o[kPrefillMaxKeySplits];
#pragma unroll
    for (int s = 0; s < kPrefillMaxKeySplits; ++s) {
        m[s] = kPrefillNoMax;
        l_part[s] = 0.f;
        o[s] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (s < ns) {
            m[s] = rec[s * stride + D];
            l_part[s] = rec[s * stride + D + 1];
            o[s] = *(const f32x4*)(rec + s * stride + 4 * c);
        }
    }
    float M = kPrefillNoMax;
#pragma unroll
    for (int s = 0; s < kPrefillMaxKeySplits; ++s) M = fmaxf(M, m[s]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int s = 0; s < kPrefillMaxKeySplits; ++s) {       // absent parts: weight of a zero record
        const float w = fast_exp2(m[s] - M);
        acc += w * o[s];
        l += w * l_part[s];
    }
    // no visible key in any part (a query before position 0, an empty context): a row of zeros
    const float f = l > 0.f ? p.out_scale / l : 0.f;
    acc *= f;
    if (p.out_f32) {
        *(f32x4*)((float*)p.out + row * D + 4 * c) = acc;
    } else {
        typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
        bf16x4 h;
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = (__bf16)acc[i];
        *(bf16x4*)((__bf16*)p.out + row * D + 4 * c) = h;
    }
}

template <int D, bool FP8>
static hipError_t launch_prefill_d(const PrefillParams& p, int max_q_len, hipStream_t stream)
{
    constexpr int NQB = kPrefillQueryBlocks;
    const int tbw = kPrefillWaves / p.heads_per_wg;
    const int ranges = (max_q_len + 16 * NQB - 1) / (16 * NQB);
    const int64_t gy = (int64_t)((ranges + tbw - 1) / tbw) * p.key_splits;
    if (gy > 65535 || p.batch > 65535) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)(p.num_q_heads / p.heads_per_wg), (uint32_t)gy, (uint32_t)p.batch);
    using S = PrefillShape<D>;
    // the ring is larger than the 64 KiB a kernel gets without asking
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<D, NQB, FP8>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((prefill_kernel<D, NQB, FP8>), grid, dim3(kPrefillThreads), S::kLdsBytes, stream, p, p.q,
                       p.pool, p.block_table, p.context_lens, p.q_starts, p.out);
    e = hipGetLastError();
    if (e != hipSuccess || p.key_splits == 1) return e;
    constexpr int kRows = 256 / (D / 4);
    const int64_t rows = p.total_q * p.num_q_heads;
    if ((rows + kRows - 1) / kRows > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prefill_merge_kernel<D>, dim3((uint32_t)((rows + kRows - 1) / kRows)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillParams& p, int head_dim, int max_q_len, hipStream_t stream)
{
    if (head_dim == 128) return p.kv_fp8 ? launch_prefill_d<128, true>(p, max_q_len, stream)
                                         : launch_prefill_d<128, false>(p, max_q_len, stream);
    if (head_dim == 64) return p.kv_fp8 ? launch_prefill_d<64, true>(p, max_q_len, stream)
                                        : launch_prefill_d<64, false>(p, max_q_len, stream);
    return hipErrorInvalidValue;
}

}  // namespace kvflow
