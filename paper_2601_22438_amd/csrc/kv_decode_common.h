// Pieces shared by the decode kernels (bf16 pool and FP8 pool): vector types, the split of the
// flat tile space into runs, the record a run leaves when it leaves a (sequence, KV head) row,
// and the kernel that merges the records of a row.
#pragma once

#include "kv_internal.h"

#include <type_traits>

namespace kvflow {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// K/V bytes are used once per decode step: load them with the non-temporal hint so that they
// stream through the caches instead of displacing each other.
__device__ __forceinline__ u32x4 stream_load(const uint16_t* p)
{
    return __builtin_nontemporal_load((const u32x4*)p);
}

// The running max of a head only has to be an upper bound of the scores up to a bounded slack
// (softmax is invariant under the reference point): it is raised, with the cross-lane reduction
// and the rescale of O that go with it, only when some score of the tile exceeds it by more than
// this many binary orders of magnitude.  Probabilities then stay below 2^kMaxSlack.
constexpr float kMaxSlack = 8.f;

// First flat tile of run w when T tiles are dealt to W runs as evenly as possible.
__device__ __forceinline__ int run_start(int w, int base, int rem) { return w * base + min(w, rem); }

__device__ __forceinline__ int run_of_tile(int t, int base, int rem)
{
    const int big = rem * (base + 1);                // tiles held by the runs that got one extra
    return t < big ? t / (base + 1) : rem + (t - big) / base;
}

// The run of one wavefront: flat tiles [t_begin, t_end) of the T tiles dealt to W runs.
struct RunSpan {
    int w, W, base, rem, t_begin, t_end;
};

// Where a flat tile lies: sequence, KV head, tile within the sequence, and the sequence's size.
struct TilePos {
    int b, kvh, tile, ntiles, L;
};

// Start-up of a decode workgroup (all kDecodeThreads threads call it): cum[b] = number of
// kTile-token tiles of the sequences before b (exclusive scan of the context lengths in LDS,
// cum has batch + 1 entries; workgroup 0 also copies it to ws_cum for the merge kernel), then
// this wavefront's run.  cum[] is complete on return.
template <int kTile>
__device__ __forceinline__ RunSpan split_into_runs(int* cum, int32_t* __restrict__ ws_cum,
                                                   const int32_t* __restrict__ lens_ptr, int B, int Hkv, int lane,
                                                   int wave)
{
    __shared__ int wave_tot[kDecodeWaves];
    const int per = (B + kDecodeThreads - 1) / kDecodeThreads;
    const int lo = min(B, (int)threadIdx.x * per), hi = min(B, lo + per);
    int mine = 0;
    for (int b = lo; b < hi; ++b) mine += (lens_ptr[b] + kTile - 1) / kTile;
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = incl - mine;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    for (int b = lo; b < hi; ++b) {
        cum[b] = before;
        before += (lens_ptr[b] + kTile - 1) / kTile;
    }
    if (threadIdx.x == kDecodeThreads - 1) cum[B] = before;           // its range ends at B
    __syncthreads();
    if (blockIdx.x == 0)                                              // the merge kernel reads this copy
        for (int b = threadIdx.x; b <= B; b += kDecodeThreads) ws_cum[b] = cum[b];
    RunSpan rs;
    const int T = Hkv * cum[B];
    rs.W = gridDim.x * kDecodeWaves;
    rs.base = T / rs.W;
    rs.rem = T % rs.W;
    rs.w = blockIdx.x * kDecodeWaves + wave;
    rs.t_begin = run_start(rs.w, rs.base, rs.rem);
    rs.t_end = run_start(rs.w + 1, rs.base, rs.rem);
    return rs;
}

// Position of flat tile t (which must exist): the last b with Hkv * cum[b] <= t.
__device__ __forceinline__ TilePos locate_tile(const int* cum, const int32_t* __restrict__ lens_ptr, int B, int Hkv, int t)
{
    int lo = 0, hi = B;                                               // Hkv*cum[lo] <= t < Hkv*cum[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (Hkv * cum[mid] <= t) lo = mid; else hi = mid;
    }
    TilePos pos;
    pos.b = lo;
    pos.ntiles = cum[lo + 1] - cum[lo];
    const int r = t - Hkv * cum[lo];
    pos.kvh = r / pos.ntiles;
    pos.tile = r % pos.ntiles;
    pos.L = lens_ptr[lo];
    return pos;
}

// The run leaves row (b, kvh).  Lane (g, j) holds, for query head j of the group (j < G), the
// un-normalised output channels 16dt + 4g .. +3 in oacc[dt], the head's reference maximum m_run
// and its share l_run of the denominator.  One record per query head (O, m, l) goes to slot
// run + row index, unique because both grow along the flat space.
template <int D>
__device__ __forceinline__ void leave_row(float* __restrict__ ws_records, const f32x4 (&oacc)[D / 16], float m_run,
                                          float l_run, int run, int b, int kvh, int Hkv, int G, int g, int j)
{
    constexpr int kRecord = D + kRecordPad;
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (j < G) {
        const int64_t slot = (int64_t)run + (int64_t)b * Hkv + kvh;
        float* rec = ws_records + (slot * G + j) * kRecord;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) *(f32x4*)(rec + 16 * dt + 4 * g) = oacc[dt];  // channels 16dt + 4g .. +3
        if (g == 0) { rec[D] = m_run; rec[D + 1] = l_tot; }
    }
}

// Combines the records of one (sequence, query head) in a fixed order and normalises.
// The kernel is latency-bound (cold reads of a few KB per workgroup), so every load of a pass is
// issued before the first use: the threads are kSlices groups of D/4 lanes, a lane owns 4
// channels, group s takes runs s, s + kSlices, ... of the pass, and the running max and
// denominators of the pass go through LDS.  Partial sums of the groups are added in group order.
// For batches with thousands of pairs and a handful of records each, see decode_merge_rows_kernel.
constexpr int kMergePer = 8;                         // records per thread and pass

template <int D, int kMergeThreads>
__global__ __launch_bounds__(kMergeThreads) void decode_merge_kernel(const DecodeParams p, int W)
{
    constexpr int kRecord = D + kRecordPad;
    constexpr int kLanes = D / 4;
    constexpr int kSlices = kMergeThreads / kLanes;
    constexpr int kChunk = kSlices * kMergePer;                       // runs per pass (<= 128)
    __shared__ float sm[kChunk], sl[kChunk];
    __shared__ __attribute__((aligned(16))) float red[kSlices * D];
    __shared__ float redl[kSlices];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int Hkv = p.num_kv_heads, G = p.group;
    const int kvh = h / G, hg = h % G;
    const int slice = tid / kLanes, c = tid % kLanes;
    const int64_t out0 = ((int64_t)b * p.num_q_heads + h) * D;
    const int n = p.ws_cum[b + 1] - p.ws_cum[b];
    if (n == 0) {                                                     // empty sequence: a row of zeros
        for (int d = tid; d < D; d += kMergeThreads) {
            if (p.out_f32) ((float*)p.out)[out0 + d] = 0.f;
            else ((uint16_t*)p.out)[out0 + d] = 0;
        }
        return;
    }
    const int T = Hkv * p.ws_cum[p.batch];
    const int base = T / W, rem = T % W;
    const int first = Hkv * p.ws_cum[b] + kvh * n;                    // flat range of this row
    const int w0 = run_of_tile(first, base, rem), w1 = run_of_tile(first + n - 1, base, rem);
    const int nr = w1 - w0 + 1;
    const int64_t rec_stride = (int64_t)G * kRecord;               // run w -> run w + 1, same row and head
    const float* recs = p.ws_records + ((w0 + (int64_t)b * Hkv + kvh) * G + hg) * kRecord;

    float M = -INFINITY, lsum = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < nr; c0 += kChunk) {
        const int cn = min(kChunk, nr - c0);
        f32x4 vals[kMergePer];
#pragma unroll
        for (int k = 0; k < kMergePer; ++k) {
            const int i = k * kSlices + slice;
            vals[k] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (i < cn) vals[k] = *(const f32x4*)(recs + (c0 + i) * rec_stride + 4 * c);
        }
        if (tid < cn) {
            sm[tid] = recs[(c0 + tid) * rec_stride + D];
            sl[tid] = recs[(c0 + tid) * rec_stride + D + 1];
        }
        __syncthreads();
        float cm = -INFINITY;
        for (int i = 0; i < cn; ++i) cm = fmaxf(cm, sm[i]);
        const float Mn = fmaxf(M, cm);
        const float a = fast_exp2(M - Mn);
        M = Mn;
        acc *= a;
        lsum *= a;
#pragma unroll
        for (int k = 0; k < kMergePer; ++k) {
            const int i = k * kSlices + slice;
            if (i < cn) {
                const float wgt = fast_exp2(sm[i] - Mn);
                acc += wgt * vals[k];
                lsum += wgt * sl[i];
            }
        }
        __syncthreads();
    }
    *(f32x4*)(red + slice * D + 4 * c) = acc;
    if (c == 0) redl[slice] = lsum;
    __syncthreads();
    for (int d = tid; d < D; d += kMergeThreads) {
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int sidx = 0; sidx < kSlices; ++sidx) { o += red[sidx * D + d]; l += redl[sidx]; }
        o = o / l * p.out_scale;
        if (p.out_f32) ((float*)p.out)[out0 + d] = o;
        else ((__bf16*)p.out)[out0 + d] = (__bf16)o;
    }
}

// The same merge for batches with thousands of (sequence, head) pairs and a handful of records per
// pair: one 256-lane workgroup per (sequence, KV head) row takes all query heads of the row, a lane
// owns 4 channels of one head and walks that head's records in run order (all loads of up to
// kMergePer records in flight).  An eighth of the workgroups of the per-pair kernel, which at these
// shapes is bound by their dispatch.
template <int D>
__global__ __launch_bounds__(256) void decode_merge_rows_kernel(const DecodeParams p, int W)
{
    constexpr int kRecord = D + kRecordPad;
    constexpr int kLanes = D / 4;
    constexpr int kHeads = 256 / kLanes;                              // query heads per pass
    const int kvh = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int Hkv = p.num_kv_heads, G = p.group;
    const int n = p.ws_cum[b + 1] - p.ws_cum[b];
    const int c = tid % kLanes;
    int w0 = 0, nr = 0;
    if (n > 0) {
        const int T = Hkv * p.ws_cum[p.batch];
        const int base = T / W, rem = T % W;
        const int first = Hkv * p.ws_cum[b] + kvh * n;                // flat range of this row
        w0 = run_of_tile(first, base, rem);
        nr = run_of_tile(first + n - 1, base, rem) - w0 + 1;
    }
    for (int hg = tid / kLanes; hg < G; hg += kHeads) {
        const int64_t out0 = ((int64_t)b * p.num_q_heads + (int64_t)kvh * G + hg) * D + 4 * c;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};                               // empty sequence: a row of zeros
        if (n > 0) {
            const int64_t rec_stride = (int64_t)G * kRecord;          // run w -> run w + 1, same row and head
            const float* recs = p.ws_records + ((w0 + (int64_t)b * Hkv + kvh) * G + hg) * kRecord;
            float M = -INFINITY, lsum = 0.f;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int r0 = 0; r0 < nr; r0 += kMergePer) {
                f32x4 v[kMergePer];
                float m[kMergePer], l[kMergePer];
#pragma unroll
                for (int k = 0; k < kMergePer; ++k) {
                    const int r = min(r0 + k, nr - 1);               // past the end: the last record again, not used
                    v[k] = *(const f32x4*)(recs + r * rec_stride + 4 * c);
                    m[k] = recs[r * rec_stride + D];
                    l[k] = recs[r * rec_stride + D + 1];
                }
                float Mn = M;
#pragma unroll
                for (int k = 0; k < kMergePer; ++k) if (r0 + k < nr) Mn = fmaxf(Mn, m[k]);
                const float a = fast_exp2(M - Mn);                    // 0 on the first pass (M = -inf, Mn finite)
                M = Mn;
                acc *= a;
                lsum *= a;
#pragma unroll
                for (int k = 0; k < kMergePer; ++k) {
                    if (r0 + k < nr) {
                        const float wgt = fast_exp2(m[k] - Mn);
                        acc += wgt * v[k];
                        lsum += wgt * l[k];
                    }
                }
            }
            o = acc / lsum * p.out_scale;
        }
        if (p.out_f32) {
            *(f32x4*)((float*)p.out + out0) = o;
        } else {
            typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
            bf16x4 h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = (__bf16)o[i];
            *(bf16x4*)((__bf16*)p.out + out0) = h;
        }
    }
}

// Launches the merge kernel that fits the number of (sequence, head) pairs.
template <int D>
static hipError_t launch_merge(const DecodeParams& p, int workgroups, hipStream_t stream)
{
    const dim3 mgrid((uint32_t)p.num_q_heads, (uint32_t)p.batch, 1);
    if ((int64_t)p.batch * p.num_q_heads >= 2048)
        hipLaunchKernelGGL(decode_merge_rows_kernel<D>, dim3((uint32_t)p.num_kv_heads, (uint32_t)p.batch, 1), dim3(256), 0,
                           stream, p, workgroups * kDecodeWaves);
    else
        hipLaunchKernelGGL((decode_merge_kernel<D, 256>), mgrid, dim3(256), 0, stream, p, workgroups * kDecodeWaves);
    return hipGetLastError();
}

}  // namespace kvflow
