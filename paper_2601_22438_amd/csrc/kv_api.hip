// C ABI of libkvflow: host-side argument validation, then kernel launches on the caller's stream.
// Nothing here allocates device memory or synchronises, except the kv_validate_* debug helpers.

#include "../../include/kvflow.h"
#include "kv_internal.h"

#include <atomic>
#include <cmath>
#include <vector>

using namespace kvflow;

// Decode workspace of kv_decode_attn_static: lives in every device's copy of the loaded code
// object until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the per-device address it yields is what kernels and copies are given.
// No kernel names the array, and it needs no `used` attribute: the host-side reference below is
// what makes the compiler give the device symbol external linkage, which the runtime's lookup by
// name requires (with the attribute the symbol stays internal and the lookup aborts).
constexpr size_t kStaticScratchBytes = (size_t)KV_DECODE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` per device ordinal, looked up once per device with that device
// current.  Racing first calls look the same address up twice, which is harmless.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KV_ERR_LAUNCH;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KV_ERR_LAUNCH;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return KV_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_pool(const kv_pool_desc* pool)
{
    if (!pool || !pool->base) return KV_ERR_NULL;
    if (pool->num_blocks <= 0 || pool->num_kv_heads <= 0 || pool->block_size <= 0 || pool->head_dim <= 0)
        return KV_ERR_SHAPE;
    if (pool->dtype != KV_DTYPE_BF16 && pool->dtype != KV_DTYPE_FP8_E4M3) return KV_ERR_UNSUPPORTED;
    if (pool->dtype == KV_DTYPE_FP8_E4M3 &&
        !(pool->k_scale > 0.f && pool->v_scale > 0.f && std::isfinite(pool->k_scale) && std::isfinite(pool->v_scale)))
        return KV_ERR_SHAPE;
    if (pool->head_dim != 64 && pool->head_dim != 128) return KV_ERR_UNSUPPORTED;
    if (pool->block_size != 16 && pool->block_size != 32) return KV_ERR_UNSUPPORTED;
    if (pool->num_kv_heads > 65535) return KV_ERR_UNSUPPORTED;
    if (!aligned16(pool->base)) return KV_ERR_ALIGN;
    return KV_OK;
}

size_t elt_bytes_of(const kv_pool_desc* pool) { return pool->dtype == KV_DTYPE_FP8_E4M3 ? 1 : 2; }

size_t block_bytes_of(const kv_pool_desc* pool)
{
    return (size_t)2 * pool->num_kv_heads * pool->block_size * pool->head_dim * elt_bytes_of(pool);
}

// Sequences per launch: bounded by the LDS scan and by 32-bit flat tile indices.
int64_t slice_batch(int32_t num_kv_heads, int32_t max_context_len)
{
    const int64_t tiles_per_seq = ((int64_t)max_context_len + kTileTokens - 1) / kTileTokens;
    const int64_t per_seq = (tiles_per_seq > 0 ? tiles_per_seq : 1) * num_kv_heads;
    const int64_t fit = 0x7FFFFFFF / per_seq;
    return fit < kDecodeMaxBatchPerLaunch ? fit : kDecodeMaxBatchPerLaunch;
}

// Persistent workgroups for one launch; 0 on invalid arguments.
int32_t resolve_workgroups(int32_t batch, int32_t num_kv_heads, int32_t max_context_len, int32_t requested,
                           int tile_tokens = kTileTokens)
{
    if (batch <= 0 || num_kv_heads <= 0 || max_context_len < 0 || requested < 0) return 0;
    if (requested > 0) return requested > 65535 ? 0 : requested;
    int64_t bs = slice_batch(num_kv_heads, max_context_len);
    if (bs < 1) return 0;
    if (bs > batch) bs = batch;
    const int64_t tiles = bs * num_kv_heads * (((int64_t)max_context_len + tile_tokens - 1) / tile_tokens);
    int64_t wg = (tiles + kDecodeWaves * kDecodeMinTilesPerRun - 1) / (kDecodeWaves * kDecodeMinTilesPerRun);
    if (wg < 1) wg = 1;
    if (wg > kDecodeMaxWorkgroups) wg = kDecodeMaxWorkgroups;
    return (int32_t)wg;
}

size_t cum_bytes(int64_t batch_slice) { return (size_t)(((batch_slice + 1) * 4 + 15) / 16 * 16); }

int copy_blocks(void* replica, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n,
                const int32_t* count, bool to_replica, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (n < 0) return KV_ERR_SHAPE;
    if (n == 0) return KV_OK;
    if (!replica || !block_ids) return KV_ERR_NULL;
    if (!aligned16(replica)) return KV_ERR_ALIGN;
    hipError_t e = launch_copy_blocks(replica, pool->base, block_bytes_of(pool), block_ids, n, count,
                                      to_replica, (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

}  // namespace

namespace kvflow {
// defined beside the other yardstick kernels
hipError_t launch_probe_matrix(int mode, int iters, float* sink, hipStream_t stream);
}  // namespace kvflow

extern "C" {

size_t kv_block_bytes(const kv_pool_desc* pool)
{
    if (!pool || pool->num_kv_heads <= 0 || pool->block_size <= 0 || pool->head_dim <= 0) return 0;
    if (pool->dtype != KV_DTYPE_BF16 && pool->dtype != KV_DTYPE_FP8_E4M3) return 0;
    return block_bytes_of(pool);
}

int32_t kv_decode_workgroups(int32_t batch, int32_t num_kv_heads, int32_t max_context_len,
                             int32_t num_workgroups)
{
    return resolve_workgroups(batch, num_kv_heads, max_context_len, num_workgroups);
}

size_t kv_decode_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                 int32_t head_dim, int32_t max_context_len, int32_t num_workgroups)
{
    const int32_t wg = resolve_workgroups(batch, num_kv_heads, max_context_len, num_workgroups);
    if (wg == 0 || num_q_heads <= 0 || head_dim <= 0 || num_q_heads % num_kv_heads) return 0;
    int64_t bs = slice_batch(num_kv_heads, max_context_len);
    if (bs < 1) return 0;
    if (bs > batch) bs = batch;
    const int64_t slots = (int64_t)wg * kDecodeWaves + bs * num_kv_heads;
    const int64_t group = num_q_heads / num_kv_heads;
    return cum_bytes(bs) + (size_t)(slots * group * (head_dim + kRecordPad)) * sizeof(float);
}

int kv_decode_attn(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                   const int32_t* block_table, int32_t max_blocks_per_seq,
                   const int32_t* context_lens, int32_t batch, int32_t num_q_heads,
                   int32_t max_context_len, float scale, int32_t num_workgroups,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || num_q_heads <= 0 || max_blocks_per_seq <= 0 || max_context_len < 0) return KV_ERR_SHAPE;
    if (num_q_heads % pool->num_kv_heads) return KV_ERR_SHAPE;
    const int32_t group = num_q_heads / pool->num_kv_heads;
    if (group > kMaxGroup) return KV_ERR_SHAPE;
    if ((int64_t)max_context_len > (int64_t)max_blocks_per_seq * pool->block_size) return KV_ERR_SHAPE;
    if (num_workgroups < 0 || num_workgroups > 65535) return KV_ERR_SHAPE;
    if (num_q_heads > 65535) return KV_ERR_UNSUPPORTED;
    if (out_dtype != KV_DTYPE_BF16 && out_dtype != KV_DTYPE_F32) return KV_ERR_UNSUPPORTED;
    if (batch == 0) return KV_OK;
    if (!out || !q || !block_table || !context_lens) return KV_ERR_NULL;
    if (!aligned16(out) || !aligned16(q)) return KV_ERR_ALIGN;
    const int64_t slice = slice_batch(pool->num_kv_heads, max_context_len);
    if (slice < 1) return KV_ERR_SHAPE;
    const bool fp8 = pool->dtype == KV_DTYPE_FP8_E4M3;
    // an FP8 pool is scanned in tiles twice as long: never more workgroups than the size query assumed
    const int32_t wg = resolve_workgroups(batch, pool->num_kv_heads, max_context_len, num_workgroups,
                                          fp8 ? kFp8TileTokens : kTileTokens);
    const size_t need = kv_decode_workspace_bytes(batch, num_q_heads, pool->num_kv_heads, pool->head_dim,
                                                  max_context_len, num_workgroups);
    if (!workspace || workspace_bytes < need) return KV_ERR_WORKSPACE;
    if (!aligned16(workspace)) return KV_ERR_ALIGN;

    const int D = pool->head_dim;
    const size_t out_elt = out_dtype == KV_DTYPE_F32 ? 4 : 2;
    DecodeParams p;
    p.pool = (const uint16_t*)pool->base;
    p.max_blocks_per_seq = max_blocks_per_seq;
    p.num_q_heads = num_q_heads;
    p.num_kv_heads = pool->num_kv_heads;
    p.group = group;
    p.block_size = pool->block_size;
    p.block_shift = pool->block_size == 16 ? 4 : 5;
    p.out_f32 = out_dtype == KV_DTYPE_F32;
    p.scale_log2e = (float)((double)scale * (fp8 ? (double)pool->k_scale : 1.0) * 1.4426950408889634074);
    p.out_scale = fp8 ? pool->v_scale : 1.f;
    // Slices of the batch run back to back on the stream and reuse the workspace.
    for (int64_t b0 = 0; b0 < batch; b0 += slice) {
        const int64_t nb = batch - b0 < slice ? batch - b0 : slice;
        p.out = (char*)out + (size_t)b0 * num_q_heads * D * out_elt;
        p.q = (const uint16_t*)q + (size_t)b0 * num_q_heads * D;
        p.block_table = block_table + (size_t)b0 * max_blocks_per_seq;
        p.context_lens = context_lens + b0;
        p.batch = (int32_t)nb;
        p.ws_cum = (int32_t*)workspace;
        p.ws_records = (float*)((char*)workspace + cum_bytes(slice < batch ? slice : batch));
        hipError_t e = fp8 ? launch_decode_fp8(p, D, wg, (hipStream_t)stream)
                           : launch_decode(p, D, wg, (hipStream_t)stream);
        if (e != hipSuccess) return KV_ERR_LAUNCH;
    }
    return KV_OK;
}

int kv_decode_attn_static(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                          const int32_t* block_table, int32_t max_blocks_per_seq,
                          const int32_t* context_lens, int32_t batch, int32_t num_q_heads,
                          int32_t max_context_len, float scale, int32_t num_workgroups, void* stream)
{
    // sizes beyond the fixed array are refused before anything else is looked at on the device
    if (pool && batch > 0 && num_q_heads > 0) {
        const size_t need = kv_decode_workspace_bytes(batch, num_q_heads, pool->num_kv_heads, pool->head_dim,
                                                      max_context_len, num_workgroups);
        if (need > kStaticScratchBytes) return KV_ERR_WORKSPACE;
    }
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != KV_OK) return rc;
    return kv_decode_attn(out, out_dtype, q, pool, block_table, max_blocks_per_seq, context_lens, batch,
                          num_q_heads, max_context_len, scale, num_workgroups, ws, kStaticScratchBytes, stream);
}

int32_t kv_prefill_key_splits(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t max_q_len,
                              int32_t max_context_len)
{
    if (batch <= 0 || num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads || max_q_len <= 0 ||
        max_context_len <= 0)
        return 0;
    const int32_t group = num_q_heads / num_kv_heads;
    int32_t hpw = kPrefillWaves;
    while (group % hpw) hpw /= 2;
    const int64_t ranges = ((int64_t)max_q_len + 16 * kPrefillQueryBlocks - 1) / (16 * kPrefillQueryBlocks);
    const int64_t tbw = kPrefillWaves / hpw;
    const int64_t wgs = (int64_t)(num_q_heads / hpw) * ((ranges + tbw - 1) / tbw) * batch;
    // one workgroup per compute unit and causal ranges of unequal length: below four rounds of
    // workgroups, cut the key range, but keep parts of >= 16 tiles
    const int64_t want = (4 * 256 + wgs - 1) / wgs;
    const int64_t tiles = ((int64_t)max_context_len + kTileTokens - 1) / kTileTokens;
    int64_t ns = want < tiles / 16 ? want : tiles / 16;
    if (ns > kPrefillMaxKeySplits) ns = kPrefillMaxKeySplits;
    return ns < 1 ? 1 : (int32_t)ns;
}

size_t kv_prefill_workspace_bytes(int64_t total_q, int32_t num_q_heads, int32_t head_dim, int32_t key_splits)
{
    if (total_q <= 0 || num_q_heads <= 0 || head_dim <= 0 || key_splits <= 1 || key_splits > kPrefillMaxKeySplits)
        return 0;
    return (size_t)key_splits * (size_t)total_q * num_q_heads * (head_dim + kRecordPad) * sizeof(float);
}

int kv_prefill_attn(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                    const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* context_lens,
                    const int32_t* q_starts, int32_t batch, int32_t num_q_heads, int32_t max_q_len,
                    int64_t total_q, float scale, int32_t key_splits, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || num_q_heads <= 0 || max_blocks_per_seq <= 0 || max_q_len < 0) return KV_ERR_SHAPE;
    if (num_q_heads % pool->num_kv_heads) return KV_ERR_SHAPE;
    // the kernel takes the max of raw scores before scaling them
    if (!(scale > 0.f) || !std::isfinite(scale)) return KV_ERR_SHAPE;
    if (out_dtype != KV_DTYPE_BF16 && out_dtype != KV_DTYPE_F32) return KV_ERR_UNSUPPORTED;
    if (batch > 65535 || num_q_heads > 65535) return KV_ERR_UNSUPPORTED;
    if ((int64_t)max_q_len > (int64_t)65535 * 16 * kPrefillQueryBlocks) return KV_ERR_UNSUPPORTED;
    if (total_q < 0 || key_splits < 0 || key_splits > kPrefillMaxKeySplits) return KV_ERR_SHAPE;
    if (batch == 0 || max_q_len == 0 || total_q == 0) return KV_OK;
    if (!out || !q || !block_table || !context_lens || !q_starts) return KV_ERR_NULL;
    if (!aligned16(out) || !aligned16(q)) return KV_ERR_ALIGN;
    if (key_splits == 0) key_splits = 1;
    if (key_splits > 1) {
        if (!workspace || workspace_bytes < kv_prefill_workspace_bytes(total_q, num_q_heads, pool->head_dim, key_splits))
            return KV_ERR_WORKSPACE;
        if (!aligned16(workspace)) return KV_ERR_ALIGN;
    }
    const int32_t group = num_q_heads / pool->num_kv_heads;
    PrefillParams p;
    p.key_splits = key_splits;
    p.total_q = total_q;
    p.ws = (float*)workspace;
    p.out = out;
    p.q = (const uint16_t*)q;
    p.pool = pool->base;
    p.block_table = block_table;
    p.context_lens = context_lens;
    p.q_starts = q_starts;
    p.max_blocks_per_seq = max_blocks_per_seq;
    p.batch = batch;
    p.num_q_heads = num_q_heads;
    p.num_kv_heads = pool->num_kv_heads;
    p.group = group;
    p.heads_per_wg = kPrefillWaves;
    while (group % p.heads_per_wg) p.heads_per_wg /= 2;
    p.block_size = pool->block_size;
    p.block_shift = pool->block_size == 16 ? 4 : 5;
    p.out_f32 = out_dtype == KV_DTYPE_F32;
    const bool fp8 = pool->dtype == KV_DTYPE_FP8_E4M3;
    p.kv_fp8 = fp8;
    p.scale_log2e = (float)((double)scale * (fp8 ? (double)pool->k_scale : 1.0) * 1.4426950408889634074);
    p.out_scale = fp8 ? pool->v_scale : 1.f;
    hipError_t e = launch_prefill(p, pool->head_dim, max_q_len, (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_pack_blocks(void* replica, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n, void* stream)
{
    return copy_blocks(replica, pool, block_ids, n, nullptr, true, stream);
}

int kv_restore_blocks(const kv_pool_desc* pool, const void* replica, const int32_t* block_ids, int64_t n,
                      void* stream)
{
    return copy_blocks(const_cast<void*>(replica), pool, block_ids, n, nullptr, false, stream);
}

int kv_pack_blocks_counted(void* replica, const kv_pool_desc* pool, const int32_t* block_ids,
                           const int32_t* count, int64_t max_n, void* stream)
{
    if (max_n > 0 && !count) return KV_ERR_NULL;
    return copy_blocks(replica, pool, block_ids, max_n, count, true, stream);
}

int kv_pack_blocks_staged(void* dst, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n, void* staging,
                          int64_t chunk_blocks, void* pack_stream, void* copy_stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (n < 0 || chunk_blocks <= 0) return KV_ERR_SHAPE;
    if (n == 0) return KV_OK;
    if (!dst || !block_ids || !staging) return KV_ERR_NULL;
    if (!aligned16(dst) || !aligned16(staging)) return KV_ERR_ALIGN;
    const size_t bb = block_bytes_of(pool);
    const size_t chunk_bytes = (size_t)chunk_blocks * bb;
    hipStream_t ps = (hipStream_t)pack_stream, cs = (hipStream_t)copy_stream;
    // packed[k]: staging half k holds a packed chunk; copied[k]: its copy has left the half
    hipEvent_t packed[2] = {nullptr, nullptr}, copied[2] = {nullptr, nullptr};
    for (int k = 0; k < 2; ++k)
        if (hipEventCreateWithFlags(&packed[k], hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&copied[k], hipEventDisableTiming) != hipSuccess)
            rc = KV_ERR_LAUNCH;
    int64_t chunk = 0;
    for (int64_t first = 0; rc == KV_OK && first < n; first += chunk_blocks, ++chunk) {
        const int k = (int)(chunk & 1);
        const int64_t nb = n - first < chunk_blocks ? n - first : chunk_blocks;
        char* half = (char*)staging + (size_t)k * chunk_bytes;
        if (chunk >= 2 && hipStreamWaitEvent(ps, copied[k], 0) != hipSuccess) { rc = KV_ERR_LAUNCH; break; }
        rc = copy_blocks(half, pool, block_ids + first, nb, nullptr, true, ps);
        if (rc != KV_OK) break;
        if (hipEventRecord(packed[k], ps) != hipSuccess || hipStreamWaitEvent(cs, packed[k], 0) != hipSuccess ||
            hipMemcpyAsync((char*)dst + (size_t)first * bb, half, (size_t)nb * bb, hipMemcpyDefault, cs) != hipSuccess ||
            hipEventRecord(copied[k], cs) != hipSuccess)
            rc = KV_ERR_LAUNCH;
    }
    // an event may be destroyed while work that uses it is still in flight: the runtime keeps it until then
    for (int k = 0; k < 2; ++k) {
        if (packed[k]) (void)hipEventDestroy(packed[k]);
        if (copied[k]) (void)hipEventDestroy(copied[k]);
    }
    return rc;
}

int kv_append_tokens(const kv_pool_desc* pool, const void* k_new, const void* v_new,
                     const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* positions,
                     int32_t batch, uint32_t* dirty_bitmap, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || max_blocks_per_seq <= 0) return KV_ERR_SHAPE;
    if (batch == 0) return KV_OK;
    if (!k_new || !v_new || !block_table || !positions || !dirty_bitmap) return KV_ERR_NULL;
    if (!aligned16(k_new) || !aligned16(v_new)) return KV_ERR_ALIGN;
    hipError_t e = launch_append_tokens(pool->base, k_new, v_new, block_table, max_blocks_per_seq, positions, batch,
                                        pool->num_kv_heads, pool->block_size,
                                        (int)(pool->head_dim * elt_bytes_of(pool)), dirty_bitmap,
                                        (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_append_packed(const kv_pool_desc* pool, const void* k_new, const void* v_new,
                     const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* context_lens,
                     const int32_t* q_starts, int32_t batch, int64_t total_q, uint32_t* dirty_bitmap, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || max_blocks_per_seq <= 0 || total_q < 0) return KV_ERR_SHAPE;
    if (batch == 0 || total_q == 0) return KV_OK;
    if (!k_new || !v_new || !block_table || !context_lens || !q_starts || !dirty_bitmap) return KV_ERR_NULL;
    if (!aligned16(k_new) || !aligned16(v_new)) return KV_ERR_ALIGN;
    hipError_t e = launch_append_packed(pool->base, k_new, v_new, block_table, max_blocks_per_seq, context_lens,
                                        q_starts, batch, total_q, pool->num_kv_heads, pool->block_size,
                                        (int)(pool->head_dim * elt_bytes_of(pool)), dirty_bitmap,
                                        (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_gather_tokens(void* k_out, void* v_out, const kv_pool_desc* pool, const int32_t* block_table,
                     int32_t max_blocks_per_seq, const int32_t* positions, int32_t batch, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || max_blocks_per_seq <= 0) return KV_ERR_SHAPE;
    if (batch == 0) return KV_OK;
    if (!k_out || !v_out || !block_table || !positions) return KV_ERR_NULL;
    if (!aligned16(k_out) || !aligned16(v_out)) return KV_ERR_ALIGN;
    hipError_t e = launch_gather_tokens(pool->base, k_out, v_out, block_table, max_blocks_per_seq, positions, batch,
                                        pool->num_kv_heads, pool->block_size,
                                        (int)(pool->head_dim * elt_bytes_of(pool)), (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_collect_dirty(uint32_t* dirty_bitmap, int64_t num_blocks, int32_t* dirty_ids, int64_t capacity,
                     int32_t* dirty_count, int32_t clear, void* stream)
{
    if (num_blocks <= 0 || capacity < 0 || num_blocks > 0x7FFFFFFF) return KV_ERR_SHAPE;
    if (!dirty_bitmap || !dirty_count || (capacity > 0 && !dirty_ids)) return KV_ERR_NULL;
    hipError_t e = launch_collect_dirty(dirty_bitmap, num_blocks, dirty_ids, capacity, dirty_count, clear != 0,
                                        (hipStream_t)stream);
    return e == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
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

int kv_validate_prefill(const kv_pool_desc* pool, const int32_t* block_table, int32_t max_blocks_per_seq,
                        const int32_t* context_lens, const int32_t* q_starts, int32_t batch, int32_t max_q_len,
                        int64_t total_q, void* stream)
{
    int rc = check_pool(pool);
    if (rc != KV_OK) return rc;
    if (batch < 0 || max_blocks_per_seq <= 0 || max_q_len < 0 || total_q < 0) return KV_ERR_SHAPE;
    if (batch == 0) return total_q == 0 ? KV_OK : KV_ERR_SHAPE;
    if (!block_table || !context_lens || !q_starts) return KV_ERR_NULL;
    std::vector<int32_t> lens((size_t)batch), starts((size_t)batch + 1);
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(lens.data(), context_lens, lens.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(starts.data(), q_starts, starts.size() * 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return KV_ERR_LAUNCH;
    if (starts[0] != 0 || starts[(size_t)batch] != total_q) return KV_ERR_CONTENT;
    int32_t max_len = 0;
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t n = (int64_t)starts[(size_t)b + 1] - starts[(size_t)b];
        // more query tokens than cached tokens is outside the contract of a recomputation
        if (n < 0 || n > max_q_len || lens[(size_t)b] < 0 || n > lens[(size_t)b]) return KV_ERR_CONTENT;
        if (lens[(size_t)b] > max_len) max_len = lens[(size_t)b];
    }
    // table entries and lengths against the table row: the decode check, with the largest length as bound
    return kv_validate_decode(pool, block_table, max_blocks_per_seq, context_lens, batch, max_len, stream);
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

int kv_probe_stream(int32_t mode, void* a, const void* b, size_t bytes, void* stream)
{
    if (mode < 0 || mode > 5 || bytes % 16) return KV_ERR_SHAPE;
    if (bytes == 0) return KV_OK;
    const int kind = mode % 3;
    if (!a || (kind != 1 && !b)) return KV_ERR_NULL;
    if (!aligned16(a) || (kind != 1 && !aligned16(b))) return KV_ERR_ALIGN;
    if (mode <= 2 && bytes > ((size_t)32 << 30)) return KV_ERR_SHAPE;
    return launch_probe(mode, a, b, bytes, (hipStream_t)stream) == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
}

int kv_probe_matrix(int32_t mode, int32_t iters, void* sink, size_t sink_bytes, void* stream)
{
    if (mode < 0 || mode > 5 || iters < 0) return KV_ERR_SHAPE;
    if (!sink) return KV_ERR_NULL;
    if (!aligned16(sink)) return KV_ERR_ALIGN;
    if (sink_bytes < KV_PROBE_MATRIX_SINK_BYTES) return KV_ERR_WORKSPACE;
    return launch_probe_matrix(mode, iters, (float*)sink, (hipStream_t)stream) == hipSuccess ? KV_OK : KV_ERR_LAUNCH;
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
