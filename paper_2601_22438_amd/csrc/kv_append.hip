// Writing a decode step's new K/V rows into the block pool, and keeping track of the blocks that
// became dirty so that background replication (paper Sec. 3.2 item 3) can ship exactly those,
// without the host ever seeing the list.
//
//   append_tokens_kernel   one 16-byte chunk per lane: new row -> its slot in the pool; one lane per
//                          sequence ORs the block's bit into the dirty bitmap (atomic, commutative:
//                          the bitmap does not depend on execution order).
//   collect_dirty_kernel   bitmap -> ascending id list + count, optional clear.  One workgroup:
//                          lanes own contiguous word ranges, a block-wide exclusive scan of their
//                          popcounts gives every lane its output offset, so the list is sorted.
// Both are latency-bound (a few KB to a few MB); the HBM-bound work stays in decode and pack.

#include "kv_internal.h"

namespace kvflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kAppendThreads = 256;
constexpr int kCollectThreads = 1024;

__global__ __launch_bounds__(kAppendThreads) void append_tokens_kernel(
    char* __restrict__ pool, const char* __restrict__ k_new, const char* __restrict__ v_new,
    const int32_t* __restrict__ block_table, int max_blocks_per_seq, const int32_t* __restrict__ positions,
    int batch, int num_kv_heads, int block_size, int block_shift, int row_bytes, uint32_t* __restrict__ dirty_bitmap)
{
    const int chunks_per_row = row_bytes / 16;                        // 16-byte chunks in one head's row
    const int chunks_per_seq = 2 * num_kv_heads * chunks_per_row;
    const int64_t idx = (int64_t)blockIdx.x * kAppendThreads + threadIdx.x;
    if (idx >= (int64_t)batch * chunks_per_seq) return;
    const int b = (int)(idx / chunks_per_seq), c = (int)(idx % chunks_per_seq);
    const int t = positions[b];
    if (t < 0) return;                                                // this sequence takes no token
    const int which = c / (num_kv_heads * chunks_per_row);            // 0 = K, 1 = V
    const int kvh = (c / chunks_per_row) % num_kv_heads;
    const int ch = c % chunks_per_row;
    const int64_t p = block_table[(int64_t)b * max_blocks_per_seq + (t >> block_shift)];
    const int r = t & (block_size - 1);
    const char* src = (which ? v_new : k_new) + ((int64_t)b * num_kv_heads + kvh) * row_bytes + ch * 16;
    char* dst = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)row_bytes) + ch * 16;
    *(u32x4*)dst = *(const u32x4*)src;
    if (c == 0) atomicOr(dirty_bitmap + (p >> 5), 1u << (p & 31));
}

// Many new tokens per sequence (recomputation / prefill): packed row t belongs to the sequence b with
// q_starts[b] <= t < q_starts[b + 1] and goes to position context_lens[b] - q_len_b + (t - q_starts[b]).
__global__ __launch_bounds__(kAppendThreads) void append_packed_kernel(
    char* __restrict__ pool, const char* __restrict__ k_new, const char* __restrict__ v_new,
    const int32_t* __restrict__ block_table, int max_blocks_per_seq, const int32_t* __restrict__ context_lens,
    const int32_t* __restrict__ q_starts, int batch, int64_t total_q, int num_kv_heads, int block_size,
    int block_shift, int row_bytes, uint32_t* __restrict__ dirty_bitmap)
{
    const int chunks_per_row = row_bytes / 16;
    const int chunks_per_tok = 2 * num_kv_heads * chunks_per_row;
    const int64_t idx = (int64_t)blockIdx.x * kAppendThreads + threadIdx.x;
    if (idx >= total_q * chunks_per_tok) return;
    const int64_t row = idx / chunks_per_tok;
    const int c = (int)(idx % chunks_per_tok);
    int lo = 0, hi = batch;                                           // q_starts[lo] <= row < q_starts[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (q_starts[mid] <= row) lo = mid; else hi = mid;
    }
    // sequences without query tokens share their start with the next one: step over them
    while (q_starts[lo + 1] <= row && lo + 1 < batch) ++lo;
    const int b = lo;
    const int first = q_starts[b], n = q_starts[b + 1] - first;
    if (row >= (int64_t)first + n) return;                            // q_starts[batch] < total_q: no owner
    const int t = context_lens[b] - n + (int)(row - first);
    if (t < 0) return;                                                // more new tokens than the context holds
    const int which = c / (num_kv_heads * chunks_per_row);            // 0 = K, 1 = V
    const int kvh = (c / chunks_per_row) % num_kv_heads;
    const int ch = c % chunks_per_row;
    const int64_t p = block_table[(int64_t)b * max_blocks_per_seq + (t >> block_shift)];
    const int r = t & (block_size - 1);
    const char* src = (which ? v_new : k_new) + (row * num_kv_heads + kvh) * row_bytes + ch * 16;
    char* dst = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)row_bytes) + ch * 16;
    *(u32x4*)dst = *(const u32x4*)src;
    if (c == 0) atomicOr(dirty_bitmap + (p >> 5), 1u << (p & 31));
}

// The inverse direction for token-granular replication: the rows at positions[b] leave the pool
// for contiguous arrays (what travels is the new token, not the block around it).
__global__ __launch_bounds__(kAppendThreads) void gather_tokens_kernel(
    const char* __restrict__ pool, char* __restrict__ k_out, char* __restrict__ v_out,
    const int32_t* __restrict__ block_table, int max_blocks_per_seq, const int32_t* __restrict__ positions,
    int batch, int num_kv_heads, int block_size, int block_shift, int row_bytes)
{
    const int chunks_per_row = row_bytes / 16;
    const int chunks_per_seq = 2 * num_kv_heads * chunks_per_row;
    const int64_t idx = (int64_t)blockIdx.x * kAppendThreads + threadIdx.x;
    if (idx >= (int64_t)batch * chunks_per_seq) return;
    const int b = (int)(idx / chunks_per_seq), c = (int)(idx % chunks_per_seq);
    const int t = positions[b];
    if (t < 0) return;
    const int which = c / (num_kv_heads * chunks_per_row);
    const int kvh = (c / chunks_per_row) % num_kv_heads;
    const int ch = c % chunks_per_row;
    const int64_t p = block_table[(int64_t)b * max_blocks_per_seq + (t >> block_shift)];
    const int r = t & (block_size - 1);
    const char* src = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)row_bytes) + ch * 16;
    char* dst = (which ? v_out : k_out) + ((int64_t)b * num_kv_heads + kvh) * row_bytes + ch * 16;
    *(u32x4*)dst = *(const u32x4*)src;
}

__global__ __launch_bounds__(kCollectThreads) void collect_dirty_kernel(
    uint32_t* __restrict__ dirty_bitmap, int64_t num_blocks, int32_t* __restrict__ ids_out, int64_t capacity,
    int32_t* __restrict__ count_out, int clear)
{
    __shared__ int64_t wave_tot[kCollectThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t num_words = (num_blocks + 31) / 32;
    const int64_t per = (num_words + kCollectThreads - 1) / kCollectThreads;
    const int64_t lo = min(num_words, (int64_t)tid * per), hi = min(num_words, lo + per);
    // bits past num_blocks in the last word are not blocks
    const uint32_t last_mask = (num_blocks & 31) ? ((1u << (num_blocks & 31)) - 1u) : 0xFFFFFFFFu;
    int64_t mine = 0;
    for (int64_t w = lo; w < hi; ++w) {
        uint32_t bits = dirty_bitmap[w];
        if (w == num_words - 1) bits &= last_mask;
        mine += __popc(bits);
    }
    int64_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int64_t out = incl - mine;
    for (int w = 0; w < wave; ++w) out += wave_tot[w];
    if (tid == kCollectThreads - 1) *count_out = (int32_t)(out + mine);  // total number of dirty blocks
    for (int64_t w = lo; w < hi; ++w) {
        uint32_t bits = dirty_bitmap[w];
        if (w == num_words - 1) bits &= last_mask;
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            if (out < capacity) ids_out[out] = (int32_t)(w * 32 + bit);
            ++out;
        }
        if (clear) dirty_bitmap[w] = 0u;
    }
}

hipError_t launch_append_tokens(void* pool, const void* k_new, const void* v_new,
                                const int32_t* block_table, int max_blocks_per_seq, const int32_t* positions,
                                int batch, int num_kv_heads, int block_size, int row_bytes,
                                uint32_t* dirty_bitmap, hipStream_t stream)
{
    const int64_t threads = (int64_t)batch * 2 * num_kv_heads * (row_bytes / 16);
    const int64_t groups = (threads + kAppendThreads - 1) / kAppendThreads;
    if (groups > 0x7FFFFFFF / kAppendThreads) return hipErrorInvalidValue;
    hipLaunchKernelGGL(append_tokens_kernel, dim3((uint32_t)groups), dim3(kAppendThreads), 0, stream, (char*)pool,
                       (const char*)k_new, (const char*)v_new, block_table, max_blocks_per_seq, positions, batch,
                       num_kv_heads, block_size, block_size == 16 ? 4 : 5, row_bytes, dirty_bitmap);
    return hipGetLastError();
}

hipError_t launch_append_packed(void* pool, const void* k_new, const void* v_new, const int32_t* block_table,
                                int max_blocks_per_seq, const int32_t* context_lens, const int32_t* q_starts,
                                int batch, int64_t total_q, int num_kv_heads, int block_size, int row_bytes,
                                uint32_t* dirty_bitmap, hipStream_t stream)
{
    const int64_t threads = total_q * 2 * num_kv_heads * (row_bytes / 16);
    const int64_t groups = (threads + kAppendThreads - 1) / kAppendThreads;
    if (groups > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(append_packed_kernel, dim3((uint32_t)groups), dim3(kAppendThreads), 0, stream, (char*)pool,
                       (const char*)k_new, (const char*)v_new, block_table, max_blocks_per_seq, context_lens,
                       q_starts, batch, total_q, num_kv_heads, block_size, block_size == 16 ? 4 : 5, row_bytes,
                       dirty_bitmap);
    return hipGetLastError();
}

hipError_t launch_gather_tokens(const void* pool, void* k_out, void* v_out, const int32_t* block_table,
                                int max_blocks_per_seq, const int32_t* positions, int batch, int num_kv_heads,
                                int block_size, int row_bytes, hipStream_t stream)
{
    const int64_t threads = (int64_t)batch * 2 * num_kv_heads * (row_bytes / 16);
    const int64_t groups = (threads + kAppendThreads - 1) / kAppendThreads;
    if (groups > 0x7FFFFFFF / kAppendThreads) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gather_tokens_kernel, dim3((uint32_t)groups), dim3(kAppendThreads), 0, stream,
                       (const char*)pool, (char*)k_out, (char*)v_out, block_table, max_blocks_per_seq, positions,
                       batch, num_kv_heads, block_size, block_size == 16 ? 4 : 5, row_bytes);
    return hipGetLastError();
}

hipError_t launch_collect_dirty(uint32_t* dirty_bitmap, int64_t num_blocks, int32_t* ids_out, int64_t capacity,
                                int32_t* count_out, int clear, hipStream_t stream)
{
    hipLaunchKernelGGL(collect_dirty_kernel, dim3(1), dim3(kCollectThreads), 0, stream, dirty_bitmap, num_blocks,
                       ids_out, capacity, count_out, clear);
    return hipGetLastError();
}

}  // namespace kvflow
