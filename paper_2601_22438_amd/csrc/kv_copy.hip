// Block-granular gather/scatter between the KV block pool and a contiguous replica buffer
// (block-by-block replication and its inverse, paper Sec. 3.2 item 3).
//
// Pure HBM streaming: every byte is read once and written once.  A 1024-lane workgroup moves one
// 16 KiB segment of one block with one 128-bit load and one 128-bit store per lane; the grid is
// one-shot (a workgroup per segment).  Two things decide the rate on MI355X (measured, in order
// of weight):
//   - which XCD touches what.  Workgroups are dealt to the eight XCDs round-robin by their index.
//     Here XCD x = blockIdx % 8 owns a contiguous eighth of the list, and its consecutive
//     workgroups take consecutive segments: every XCD streams through its own stretch of the
//     replica and handles whole blocks of the pool, instead of all eight interleaving 16 KiB
//     pieces of everything (+5 to +10 points of peak for both directions);
//   - the store policy: non-temporal and write-through at device scope (nt sc1), so that the
//     written lines are not kept dirty in the L2 (+3 to +4 points on top).  Loads are
//     non-temporal.
// Larger segments per workgroup and persistent grids with read-ahead are slower.
//
// Loads and stores go through buffer descriptors that span exactly one block (the buffer form
// carries the cache-policy bits); lanes of a ragged last segment past the block's end are
// predicated off.

#include "kv_internal.h"

namespace kvflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 1024;
constexpr uint32_t kSegBytes = kCopyThreads * 16;      // 16 KiB per workgroup
constexpr int kXcds = 8;                                // workgroup i runs on XCD i % 8
// Workgroups per launch; keeps gridDim.x * blockDim.x below 2^32.
constexpr uint32_t kMaxGridX = 1u << 21;
// Cache-policy bits of the gfx950 buffer instructions: bit 1 = non-temporal, bit 4 = sc1 (device scope).
constexpr int kAuxLoad = 2;
constexpr int kAuxStore = 2 | 16;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t block_rsrc(const char* base, uint32_t bytes)
{
    // raw buffer (stride 0), num_records in bytes, 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

// One launch covers list entries [0, n) of the arrays it is given (the host passes them already offset
// by `first`); count (device, may be NULL) cuts the whole list short at *count entries.
template <bool TO_REPLICA>
__global__ __launch_bounds__(kCopyThreads) void copy_blocks_kernel(
    char* __restrict__ replica, char* __restrict__ pool, const int32_t* __restrict__ block_ids,
    uint32_t block_bytes, uint32_t segs_per_block, int64_t n, int64_t first, const int32_t* __restrict__ count)
{
    if (count) {                                       // list produced on the GPU: its length is read here
        const int64_t left = (int64_t)*count - first;
        n = left < n ? left : n;
        if (n <= 0) return;
    }
    const int64_t per = (n + kXcds - 1) / kXcds;       // entries per XCD
    const int64_t x = blockIdx.x % kXcds, k = blockIdx.x / kXcds;
    const int64_t i = x * per + k / segs_per_block;
    const uint32_t seg = (uint32_t)(k % segs_per_block);
    if (k / segs_per_block >= per || i >= n) return;
    const int64_t id = block_ids[i];
    const char* src = TO_REPLICA ? pool + id * block_bytes : replica + i * block_bytes;
    char* dst = TO_REPLICA ? replica + i * block_bytes : pool + id * block_bytes;
    const __amdgpu_buffer_rsrc_t rs = block_rsrc(src, block_bytes);
    const __amdgpu_buffer_rsrc_t rd = block_rsrc(dst, block_bytes);
    const uint32_t off = seg * kSegBytes + threadIdx.x * 16;
    if (off < block_bytes) {
        const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kAuxLoad);
        __builtin_amdgcn_raw_buffer_store_b128(r, rd, off, 0, kAuxStore);
    }
}

template <bool TO_REPLICA>
static hipError_t launch_dir(char* replica, char* pool, size_t block_bytes, const int32_t* block_ids,
                             int64_t n, const int32_t* count, hipStream_t stream)
{
    const uint32_t segs = (uint32_t)((block_bytes + kSegBytes - 1) / kSegBytes);
    // entries per launch: eight equal parts of `take` entries, each rounded up, must fit the grid
    const int64_t max_take = ((int64_t)kMaxGridX / segs / kXcds) * kXcds;
    int64_t done = 0;
    while (done < n) {
        const int64_t take = n - done < max_take ? n - done : max_take;
        const int64_t per = (take + kXcds - 1) / kXcds;
        const dim3 grid((uint32_t)(per * kXcds * segs), 1, 1);
        hipLaunchKernelGGL((copy_blocks_kernel<TO_REPLICA>), grid, dim3(kCopyThreads), 0, stream,
                           replica + done * block_bytes, pool, block_ids + done, (uint32_t)block_bytes, segs,
                           take, done, count);
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
    if ((block_bytes / kSegBytes + 1) * kXcds > kMaxGridX) return hipErrorInvalidValue;
    if (to_replica)
        return launch_dir<true>((char*)replica, (char*)pool, block_bytes, block_ids, n, count, stream);
    return launch_dir<false>((char*)replica, (char*)pool, block_bytes, block_ids, n, count, stream);
}

}  // namespace kvflow
