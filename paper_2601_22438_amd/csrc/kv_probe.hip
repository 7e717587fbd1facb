// Yardsticks for the roofline tables: what plain streaming kernels (read only, write only, contiguous
// copy) reach on the device at hand, with the same access style as the product kernels (16-byte
// accesses, non-temporal policy).  Diagnostics only; nothing else in the library uses them.
// Two designs of each, so that a ceiling does not rest on one kernel: modes 0-2 deal the buffer to
// the XCDs in contiguous eighths, one 16 KiB workgroup per piece, stores written through at device
// scope (the design of the block-copy kernels); modes 3-5 walk the buffer in workgroup order with
// plain non-temporal accesses (a persistent grid for the read).
// A third yardstick, for the recomputation kernel's roofline: what the matrix cores reach on registers
// alone (which depends on the operand data: the device lowers its clock under the switching activity
// of random operands), what the vector work of a softmax step costs, and how much of the one hides
// under the other when the two run on the wavefronts that share a SIMD.

#include "kv_internal.h"

namespace kvflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;
constexpr int kReadUnroll = 8;                        // 16-byte loads in flight per lane
constexpr int kReadGroups = 256 * 8;                  // persistent grid for the read: 8 workgroups per compute unit
constexpr int kMoveUnroll = 4;                        // write / copy: one workgroup per 16 KiB, as the pack kernel

// Reads n 16-byte vectors.  The reduction decides a store that needs one particular 128-bit value, so
// the loads cannot be removed and the sink is, for every practical purpose, never written.
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u32x4* __restrict__ src, size_t n,
                                                                   u32x4* __restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * kProbeThreads * kReadUnroll;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t base = (size_t)blockIdx.x * kProbeThreads * kReadUnroll + threadIdx.x; base < n; base += stride) {
        u32x4 r[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) {
            const size_t v = base + (size_t)u * kProbeThreads;
            r[u] = v < n ? __builtin_nontemporal_load(src + v) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc ^= r[u];
    }
    if (acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u && acc.z == 0xF39CC060u && acc.w == 0x5CEDC834u) sink[0] = acc;
}

__global__ __launch_bounds__(kProbeThreads) void probe_write_kernel(u32x4* __restrict__ dst, size_t n)
{
    const size_t base = (size_t)blockIdx.x * kProbeThreads * kMoveUnroll + threadIdx.x;
    const u32x4 val = {blockIdx.x, threadIdx.x, 0u, 0u};
#pragma unroll
    for (int u = 0; u < kMoveUnroll; ++u) {
        const size_t v = base + (size_t)u * kProbeThreads;
        if (v < n) __builtin_nontemporal_store(val, dst + v);
    }
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(u32x4* __restrict__ dst,
                                                                   const u32x4* __restrict__ src, size_t n)
{
    const size_t base = (size_t)blockIdx.x * kProbeThreads * kMoveUnroll + threadIdx.x;
    u32x4 r[kMoveUnroll];
#pragma unroll
    for (int u = 0; u < kMoveUnroll; ++u) {
        const size_t v = base + (size_t)u * kProbeThreads;
        r[u] = v < n ? __builtin_nontemporal_load(src + v) : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < kMoveUnroll; ++u) {
        const size_t v = base + (size_t)u * kProbeThreads;
        if (v < n) __builtin_nontemporal_store(r[u], dst + v);
    }
}

// ---- modes 0-2: XCD x = blockIdx % 8 owns chunks [x * per, (x + 1) * per) of 16 KiB
constexpr int kXThreads = 1024;
constexpr int kXcds = 8;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t span_rsrc(const void* base, size_t first_vec, size_t n)
{
    // the 16 KiB chunk starting at vector first_vec, cut off at the end of the buffer
    const size_t left = (n - first_vec) * 16;
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + first_vec * 16), 0,
                                             (int)(left < (size_t)kXThreads * 16 ? left : (size_t)kXThreads * 16), 0x00020000);
}

template <int MODE>
__global__ __launch_bounds__(kXThreads) void probe_xcd_kernel(u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                               size_t n, size_t per)
{
    const size_t x = blockIdx.x % kXcds, k = blockIdx.x / kXcds;
    const size_t first = (x * per + k) * kXThreads;
    if (k >= per || first >= n) return;
    const uint32_t off = threadIdx.x * 16;
    if (MODE == 0) {
        const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(span_rsrc(b, first, n), off, 0, 2);   // out of range reads 0
        if (r.x == 0x9E3779B9u && r.y == 0x7F4A7C15u && r.z == 0xF39CC060u && r.w == 0x5CEDC834u) a[0] = r;
    } else if (MODE == 1) {
        const u32x4 val = {blockIdx.x, threadIdx.x, 0u, 0u};
        __builtin_amdgcn_raw_buffer_store_b128(val, span_rsrc(a, first, n), off, 0, 2 | 16);
    } else {
        const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(span_rsrc(b, first, n), off, 0, 2);
        __builtin_amdgcn_raw_buffer_store_b128(r, span_rsrc(a, first, n), off, 0, 2 | 16);
    }
}

hipError_t launch_probe(int mode, void* a, const void* b, size_t bytes, hipStream_t stream)
{
    const size_t n = bytes / 16;
    const size_t per_group = (size_t)kProbeThreads * kMoveUnroll;
    const size_t groups = (n + per_group - 1) / per_group;
    if (groups > 0x7FFFFFFFu) return hipErrorInvalidValue;
    const dim3 block(kProbeThreads);
    if (mode <= 2) {
        const size_t chunks = (n + kXThreads - 1) / kXThreads, per = (chunks + kXcds - 1) / kXcds;
        if (per * kXcds > (1u << 21)) return hipErrorInvalidValue;         // gridDim.x * blockDim.x stays below 2^32
        const dim3 grid((uint32_t)(per * kXcds)), blk(kXThreads);
        if (mode == 0) hipLaunchKernelGGL(probe_xcd_kernel<0>, grid, blk, 0, stream, (u32x4*)a, (const u32x4*)b, n, per);
        else if (mode == 1) hipLaunchKernelGGL(probe_xcd_kernel<1>, grid, blk, 0, stream, (u32x4*)a, (const u32x4*)b, n, per);
        else hipLaunchKernelGGL(probe_xcd_kernel<2>, grid, blk, 0, stream, (u32x4*)a, (const u32x4*)b, n, per);
        return hipGetLastError();
    }
    mode -= 3;
    if (mode == 0)
        hipLaunchKernelGGL(probe_read_kernel, dim3(kReadGroups), block, 0, stream, (const u32x4*)b, n, (u32x4*)a);
    else if (mode == 1)
        hipLaunchKernelGGL(probe_write_kernel, dim3((uint32_t)groups), block, 0, stream, (u32x4*)a, n);
    else
        hipLaunchKernelGGL(probe_copy_kernel, dim3((uint32_t)groups), block, 0, stream, (u32x4*)a, (const u32x4*)b, n);
    return hipGetLastError();
}

// ---- matrix-core / vector-ALU yardstick.  One workgroup of 8 wavefronts per compute unit; wavefronts
//      w and w + 4 share a SIMD.  A matrix block is 32 v_mfma_f32_16x16x32_bf16 over 8 distinct A
//      fragments, 4 distinct B fragments and 16 accumulators (no instruction waits for another); a
//      vector block is 80 fused multiply-adds and 16 exp2 on 16 values (the vector work of one
//      32-key x 32-query softmax step is about that).
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float probe_f32x4;
constexpr int kMatrixThreads = 512;
constexpr int kMatrixGroups = 256;

__device__ __forceinline__ uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <bool RANDOM, bool MATRIX_FIRST, bool MATRIX_LAST, bool VECTOR_FIRST, bool VECTOR_LAST>
__global__ __launch_bounds__(kMatrixThreads) void probe_matrix_kernel(float* __restrict__ sink, int iters, float fa, float fb)
{
    const bool last = threadIdx.x >= kMatrixThreads / 2;              // wave-uniform: the SIMD partners
    const bool do_matrix = last ? MATRIX_LAST : MATRIX_FIRST;
    const bool do_vector = last ? VECTOR_LAST : VECTOR_FIRST;
    float result = 0.f;
    if (do_matrix) {
        probe_bf16x8 a[8], b[4];
        for (int r = 0; r < 12; ++r) {
            probe_bf16x8 v;
            for (int i = 0; i < 8; ++i) {
                const uint32_t h = probe_hash((blockIdx.x * (uint32_t)kMatrixThreads + threadIdx.x) * 131u + r * 17u + i);
                v[i] = (__bf16)(RANDOM ? (float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f : 0.f);   // uniform in [-1, 1)
            }
            if (r < 8) a[r] = v; else b[r - 8] = v;
        }
        probe_f32x4 acc[16];
        for (int c = 0; c < 16; ++c) acc[c] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int c = 0; c < 32; ++c)
                acc[c % 16] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[c % 8], b[c % 4], acc[c % 16], 0, 0, 0);
            if ((it & 1023) == 1023)                                  // keep the sums finite
                for (int c = 0; c < 16; ++c) acc[c] *= 1e-3f;
        }
        for (int c = 0; c < 16; ++c) result += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    }
    if (do_vector) {
        float x[16];
        for (int i = 0; i < 16; ++i) x[i] = -(float)((threadIdx.x + i) & 7);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 80; ++r) x[r % 16] = __builtin_fmaf(x[r % 16], fa, fb);
#pragma unroll
            for (int e = 0; e < 16; ++e) x[e] = __builtin_amdgcn_exp2f(x[e]) - 1.5f;
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int i = 0; i < 16; ++i) result += x[i];
    }
    sink[blockIdx.x * kMatrixThreads + threadIdx.x] = result;
}

hipError_t launch_probe_matrix(int mode, int iters, float* sink, hipStream_t stream)
{
    const dim3 grid(kMatrixGroups), block(kMatrixThreads);
    const float fa = 0.999f, fb = -0.001f;
    switch (mode) {
        case 0: hipLaunchKernelGGL((probe_matrix_kernel<false, true, true, false, false>), grid, block, 0, stream, sink, iters, fa, fb); break;
        case 1: hipLaunchKernelGGL((probe_matrix_kernel<true, true, true, false, false>), grid, block, 0, stream, sink, iters, fa, fb); break;
        case 2: hipLaunchKernelGGL((probe_matrix_kernel<true, false, false, true, true>), grid, block, 0, stream, sink, iters, fa, fb); break;
        case 3: hipLaunchKernelGGL((probe_matrix_kernel<true, true, false, false, true>), grid, block, 0, stream, sink, iters, fa, fb); break;
        case 4: hipLaunchKernelGGL((probe_matrix_kernel<true, true, false, false, false>), grid, block, 0, stream, sink, iters, fa, fb); break;
        case 5: hipLaunchKernelGGL((probe_matrix_kernel<true, false, false, false, true>), grid, block, 0, stream, sink, iters, fa, fb); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace kvflow
