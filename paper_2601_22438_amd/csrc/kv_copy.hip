// Block-granular gather/scatter between the KV block pool and a contiguous replica buffer
// (block-by-block replication and its inverse, paper Sec. 3.2 item 3).
//
// Pure HBM streaming: every byte is read once and written once, with the non-temporal cache
// policy on both sides.  A 1024-lane workgroup moves one segment of one block, every lane
// issuing all of its 128-bit loads before its first store.  Measured on MI355X, the gather
// direction (scattered reads, sequential writes) is fastest with many small segments (16 KiB,
// one load per lane), the scatter direction (sequential reads, scattered writes) with one
// workgroup writing a whole 64 KiB stretch of the destination block.
//
// Loads and stores go through buffer descriptors that span exactly one block (the buffer form
// carries the cache-policy bits); lanes of a ragged last segment past the block's end are
// predicated off.

#include "kv_internal.h"

namespace kvflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 1024;
constexpr int kPackUnroll = 1;        // 16 KiB per workgroup
constexpr int kRestoreUnroll = 4;     // 64 KiB per workgroup
// Workgroups along grid.x per launch row; keeps grid.x * blockDim.x below 2^32.
constexpr uint32_t kMaxGridX = 1u << 21;
// Cache-policy bits of the gfx950 buffer instructions: bit 1 = non-temporal.
constexpr int kAuxNonTemporal = 2;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t block_rsrc(const char* base, uint32_t bytes)
{
    // raw buffer (stride 0), num_records in bytes, 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

template <int U, bool TO_REPLICA>
__global__ __launch_bounds__(kCopyThreads) void copy_blocks_kernel(
    char* __restrict__ replica, char* __restrict__ pool, const int32_t* __restrict__ block_ids,
    uint32_t block_bytes, uint32_t segs_per_block, int64_t first, const int32_t* __restrict__ count)
{
    const uint32_t seg = blockIdx.x % segs_per_block;
    const int64_t i = blockIdx.x / segs_per_block + (int64_t)blockIdx.y * (kMaxGridX / segs_per_block);
    // a device-side count (list produced on the GPU) cuts the list short; first = entries before this launch
    if (count && first + i >= *count) return;
    const int64_t id = block_ids[i];
    const char* src = TO_REPLICA ? pool + id * block_bytes : replica + i * block_bytes;
    char* dst = TO_REPLICA ? replica + i * block_bytes : pool + id * block_bytes;
    const __amdgpu_buffer_rsrc_t rs = block_rsrc(src, block_bytes);
    const __amdgpu_buffer_rsrc_t rd = block_rsrc(dst, block_bytes);
    const uint32_t off0 = (seg * (kCopyThreads * U) + threadIdx.x) * 16;
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t off = off0 + u * kCopyThreads * 16;
        if (off < block_bytes) r[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kAuxNonTemporal);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t off = off0 + u * kCopyThreads * 16;
        if (off < block_bytes) __builtin_amdgcn_raw_buffer_store_b128(r[u], rd, off, 0, kAuxNonTemporal);
    }
}

template <int U, bool TO_REPLICA>
static hipError_t launch_dir(char* replica, char* pool, size_t block_bytes, const int32_t* block_ids,
                             int64_t n, const int32_t* count, hipStream_t stream)
{
    const uint32_t seg_bytes = kCopyThreads * 16 * U;
    const uint32_t segs = (uint32_t)((block_bytes + seg_bytes - 1) / seg_bytes);
    // blockIdx.x carries (block, segment); blocks beyond one row of kMaxGridX workgroups go to blockIdx.y.
    const int64_t blocks_per_row = kMaxGridX / segs;
    int64_t done = 0;
    while (done < n) {
        // full rows first, then one launch for the ragged last row: every index stays in range
        const int64_t left = n - done;
        const int64_t rows = left / blocks_per_row;
        dim3 grid;
        int64_t take;
        if (rows >= 1) {
            const int64_t r = rows > 65535 ? 65535 : rows;
            grid = dim3((uint32_t)(blocks_per_row * segs), (uint32_t)r, 1);
            take = r * blocks_per_row;
        } else {
            grid = dim3((uint32_t)(left * segs), 1, 1);
            take = left;
        }
        hipLaunchKernelGGL((copy_blocks_kernel<U, TO_REPLICA>), grid, dim3(kCopyThreads), 0, stream,
                           replica + done * block_bytes, pool, block_ids + done, (uint32_t)block_bytes, segs,
                           done, count);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += take;
    }
    return hipSuccess;
}

hipError_t launch_copy_blocks(void* replica, void* pool, size_t block_bytes, const int32_t* block_ids,
                              int64_t n, const int32_t* count, bool to_replica, hipStream_t stream)
{
    if (block_bytes == 0 || block_bytes > 0x7FFFFFF0u) return hipErrorInvalidValue;
    if (block_bytes / (kCopyThreads * 16) + 1 > kMaxGridX) return hipErrorInvalidValue;
    if (to_replica)
        return launch_dir<kPackUnroll, true>((char*)replica, (char*)pool, block_bytes, block_ids, n, count, stream);
    return launch_dir<kRestoreUnroll, false>((char*)replica, (char*)pool, block_bytes, block_ids, n, count, stream);
}

}  // namespace kvflow
