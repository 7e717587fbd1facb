// Block-granular gather/scatter between the KV block pool and a contiguous replica buffer
// (block-by-block replication and its inverse, paper Sec. 3.2 item 3).
//
// Pure HBM streaming: every byte is read once and written once.  A workgroup moves one
// kSegBytes-long segment of one block; each lane issues kUnroll independent 128-bit loads
// before the first store so that many requests per lane are in flight.

#include "kv_internal.h"

namespace kvflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
constexpr int kUnroll = 4;
constexpr int kSegBytes = kCopyThreads * 16 * kUnroll;   // 16 KiB
// Workgroups along grid.x per launch row; keeps grid.x * blockDim.x below 2^32.
constexpr uint32_t kMaxGridX = 1u << 23;

template <bool TO_REPLICA>
__global__ __launch_bounds__(kCopyThreads) void copy_blocks_kernel(
    u32x4* __restrict__ replica, u32x4* __restrict__ pool, const int32_t* __restrict__ block_ids,
    uint32_t vec_per_block, uint32_t segs_per_block)
{
    const uint32_t seg = blockIdx.x % segs_per_block;
    const int64_t i = blockIdx.x / segs_per_block + (int64_t)blockIdx.y * (kMaxGridX / segs_per_block);
    const int64_t id = block_ids[i];
    const u32x4* src;
    u32x4* dst;
    if (TO_REPLICA) {
        src = pool + id * vec_per_block;
        dst = replica + i * vec_per_block;
    } else {
        src = replica + i * vec_per_block;
        dst = pool + id * vec_per_block;
    }
    const uint32_t v0 = seg * (kSegBytes / 16) + threadIdx.x;
    u32x4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t v = v0 + u * kCopyThreads;
        if (v < vec_per_block) r[u] = __builtin_nontemporal_load(src + v);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t v = v0 + u * kCopyThreads;
        if (v < vec_per_block) __builtin_nontemporal_store(r[u], dst + v);
    }
}

hipError_t launch_copy_blocks(void* replica, void* pool, size_t block_bytes, const int32_t* block_ids,
                              int64_t n, bool to_replica, hipStream_t stream)
{
    const uint32_t vec_per_block = (uint32_t)(block_bytes / 16);
    const uint32_t segs = (uint32_t)((block_bytes + kSegBytes - 1) / kSegBytes);
    // blockIdx.x carries (block, segment); blocks beyond one row of kMaxGridX workgroups go to blockIdx.y.
    const int64_t blocks_per_row = kMaxGridX / segs;
    int64_t done = 0;
    while (done < n) {
        // one launch per run of full rows plus one for the ragged last row keeps every index in range
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
        u32x4* rep = (u32x4*)replica + done * vec_per_block;
        const int32_t* ids = block_ids + done;
        if (to_replica)
            hipLaunchKernelGGL(copy_blocks_kernel<true>, grid, dim3(kCopyThreads), 0, stream, rep,
                               (u32x4*)pool, ids, vec_per_block, segs);
        else
            hipLaunchKernelGGL(copy_blocks_kernel<false>, grid, dim3(kCopyThreads), 0, stream, rep,
                               (u32x4*)pool, ids, vec_per_block, segs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += take;
    }
    return hipSuccess;
}

}  // namespace kvflow
