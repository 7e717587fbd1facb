// C ABI of libkvflow: host-side argument validation, then kernel launches on the caller's stream.
// Nothing here allocates device memory or synchronises, except the kv_validate_* debug helpers.

#include "../../include/kvflow.h"
#include "kv_internal.h"

#include <cmath>
#include <vector>

using namespace kvflow;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_pool(const kv_pool_desc* pool)
{
    if (!pool || !pool->base) return KV_ERR_NULL;
    if (pool->num_blocks <= 0 || pool->num_kv_heads <= 0 || pool->block_size <= 0 || pool->head_dim <= 0)
        return KV_ERR_SHAPE;
    if (pool->dtype != KV_DTYPE_BF16) return KV_ERR_UNSUPPORTED;
    if (pool->head_dim != 64 && pool->head_dim != 128) return KV_ERR_UNSUPPORTED;
    if (pool->block_size != 16 && pool->block_size != 32) return KV_ERR_UNSUPPORTED;
    if (pool->num_kv_heads > 65535) return KV_ERR_UNSUPPORTED;
    if (!aligned16(pool->base)) return KV_ERR_ALIGN;
    return KV_OK;
}

size_t block_bytes_of(const kv_pool_desc* pool)
{
    return (size_t)2 * pool->num_kv_heads * pool->block_size * pool->head_dim * 2;
}

int32_t resolve_partition(int32_t batch, int32_t num_kv_heads, int32_t max_context_len, int32_t requested)
{
    if (batch <= 0 || num_kv_heads <= 0 || max_context_len < 0 || requested < 0) return 0;
    if (requested == 0) return choose_partition_tokens(batch, num_kv_heads, max_context_len);
    if (requested % kTileTokens) return 0;
    return requested;
}

int copy_blocks(void* replica, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n,
                bool to_replica, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (n < 0) return KV_ERR_SHAPE;
    if (n == 0) return KV_OK;
    if (!replica || !block_ids) return KV_ERR_NULL;
    if (!aligned16(replica)) return KV_ERR_ALIGN;
    hipError_t e = launch_copy_blocks(replica, pool->base, block_bytes_of(pool), block_ids, n,
                                      to_replica, (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

}  // namespace

extern "C" {

size_t kv_block_bytes(const kv_pool_desc* pool)
{
    if (!pool || pool->num_kv_heads <= 0 || pool->block_size <= 0 || pool->head_dim <= 0) return 0;
    return block_bytes_of(pool);
}

int32_t kv_decode_partition_tokens(int32_t batch, int32_t num_kv_heads, int32_t max_context_len,
                                   int32_t partition_tokens)
{
    return resolve_partition(batch, num_kv_heads, max_context_len, partition_tokens);
}

size_t kv_decode_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                 int32_t head_dim, int32_t max_context_len, int32_t partition_tokens)
{
    const int32_t part = resolve_partition(batch, num_kv_heads, max_context_len, partition_tokens);
    if (part == 0 || num_q_heads <= 0 || head_dim <= 0) return 0;
    const int64_t splits = ((int64_t)max_context_len + part - 1) / part;
    if (splits <= 1) return 0;
    return (size_t)batch * num_q_heads * splits * (head_dim + 2) * sizeof(float);
}

int kv_decode_attn(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                   const int32_t* block_table, int32_t max_blocks_per_seq,
                   const int32_t* context_lens, int32_t batch, int32_t num_q_heads,
                   int32_t max_context_len, float scale, int32_t partition_tokens,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || num_q_heads <= 0 || max_blocks_per_seq <= 0 || max_context_len < 0) return KV_ERR_SHAPE;
    if (num_q_heads % pool->num_kv_heads) return KV_ERR_SHAPE;
    const int32_t group = num_q_heads / pool->num_kv_heads;
    if (group > kMaxGroup) return KV_ERR_SHAPE;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * pool->block_size) return KV_ERR_SHAPE;
    if (partition_tokens < 0 || partition_tokens % kTileTokens) return KV_ERR_SHAPE;
    if (out_dtype != KV_DTYPE_BF16 && out_dtype != KV_DTYPE_F32) return KV_ERR_UNSUPPORTED;
    if (batch > 65535) return KV_ERR_UNSUPPORTED;
    if (batch == 0) return KV_OK;
    if (!out || !q || !block_table || !context_lens) return KV_ERR_NULL;
    if (!aligned16(out) || !aligned16(q)) return KV_ERR_ALIGN;

    const int32_t part = resolve_partition(batch, pool->num_kv_heads, max_context_len, partition_tokens);
    int64_t splits = ((int64_t)max_context_len + part - 1) / part;
    if (splits < 1) splits = 1;
    if (splits > 0x7FFFFFFF / kTileTokens) return KV_ERR_SHAPE;
    const size_t need = kv_decode_workspace_bytes(batch, num_q_heads, pool->num_kv_heads, pool->head_dim,
                                                  max_context_len, part);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return KV_ERR_WORKSPACE;
        if (!aligned16(workspace)) return KV_ERR_ALIGN;
    }

    DecodeParams p;
    p.out = out;
    p.q = (const uint16_t*)q;
    p.pool = (const uint16_t*)pool->base;
    p.block_table = block_table;
    p.context_lens = context_lens;
    p.workspace = (float*)workspace;
    p.max_blocks_per_seq = max_blocks_per_seq;
    p.batch = batch;
    p.num_q_heads = num_q_heads;
    p.num_kv_heads = pool->num_kv_heads;
    p.group = group;
    p.block_size = pool->block_size;
    p.block_shift = pool->block_size == 16 ? 4 : 5;
    p.partition_tokens = part;
    p.splits = (int32_t)splits;
    p.out_f32 = out_dtype == KV_DTYPE_F32;
    p.scale_log2e = (float)((double)scale * 1.4426950408889634074);
    hipError_t e = launch_decode(p, pool->head_dim, (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_pack_blocks(void* replica, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n, void* stream)
{
    return copy_blocks(replica, pool, block_ids, n, true, stream);
}

int kv_restore_blocks(const kv_pool_desc* pool, const void* replica, const int32_t* block_ids, int64_t n,
                      void* stream)
{
    return copy_blocks(const_cast<void*>(replica), pool, block_ids, n, false, stream);
}

int kv_validate_decode(const kv_pool_desc* pool, const int32_t* block_table, int32_t max_blocks_per_seq,
                       const int32_t* context_lens, int32_t batch, int32_t max_context_len, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || max_blocks_per_seq <= 0 || max_context_len < 0) return KV_ERR_SHAPE;
    if (batch == 0) return KV_OK;
    if (!block_table || !context_lens) return KV_ERR_NULL;
    std::vector<int32_t> lens((size_t)batch), table((size_t)batch * max_blocks_per_seq);
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(lens.data(), context_lens, lens.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(table.data(), block_table, table.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return KV_ERR_LAUNCH;
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t L = lens[b];
        if (L < 0 || L > max_context_len || L > (int64_t)max_blocks_per_seq * pool->block_size)
            return KV_ERR_CONTENT;
        const int64_t nb = (L + pool->block_size - 1) / pool->block_size;
        for (int64_t jb = 0; jb < nb; ++jb) {
            const int32_t id = table[(size_t)b * max_blocks_per_seq + jb];
            if (id < 0 || id >= pool->num_blocks) return KV_ERR_CONTENT;
        }
    }
    return KV_OK;
}

int kv_validate_block_ids(const kv_pool_desc* pool, const int32_t* block_ids, int64_t n,
                          int32_t require_distinct, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (n < 0) return KV_ERR_SHAPE;
    if (n == 0) return KV_OK;
    if (!block_ids) return KV_ERR_NULL;
    std::vector<int32_t> ids((size_t)n);
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(ids.data(), block_ids, ids.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return KV_ERR_LAUNCH;
    std::vector<uint8_t> seen(require_distinct ? (size_t)pool->num_blocks : 0);
    for (int64_t i = 0; i < n; ++i) {
        const int32_t id = ids[(size_t)i];
        if (id < 0 || id >= pool->num_blocks) return KV_ERR_CONTENT;
        if (require_distinct) {
            if (seen[(size_t)id]) return KV_ERR_CONTENT;
            seen[(size_t)id] = 1;
        }
    }
    return KV_OK;
}

const char* kv_status_string(int status)
{
    switch (status) {
        case KV_OK: return "ok";
        case KV_ERR_NULL: return "a required pointer is NULL";
        case KV_ERR_SHAPE: return "non-positive or inconsistent dimension";
        case KV_ERR_UNSUPPORTED: return "dimension or dtype not supported by the kernels";
        case KV_ERR_ALIGN: return "buffer not 16-byte aligned";
        case KV_ERR_WORKSPACE: return "workspace missing or too small";
        case KV_ERR_LAUNCH: return "HIP runtime refused the launch";
        case KV_ERR_CONTENT: return "device array violates a documented precondition";
        default: return "unknown status";
    }
}

}  // extern "C"
