// Internal declarations shared by the translation units of libkvflow (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace kvflow {

// Tokens one wavefront reduces per loop iteration.
constexpr int kTileTokens = 32;
// Decode workgroup: 4 independent wavefronts.
constexpr int kDecodeWaves = 4;
constexpr int kDecodeThreads = kDecodeWaves * 64;
// Persistent decode grid that fills the chip: one workgroup per compute unit (256).  Measured: 4
// wavefronts per compute unit with 16 KiB in flight each already saturate HBM, and a second resident
// workgroup only adds records and contention (2-5 points slower on every case).
constexpr int kDecodeMaxWorkgroups = 256;
// A run shorter than this many tiles is not worth its record traffic: small problems get fewer runs.
constexpr int kDecodeMinTilesPerRun = 4;
// Sequences handled by one launch (their tile counts are scanned in LDS); larger batches are sliced.
constexpr int kDecodeMaxBatchPerLaunch = 4096;
// A record is O[head_dim], running max, denominator, padded to a multiple of 16 bytes.
constexpr int kRecordPad = 4;
// Largest query-head group (num_q_heads / num_kv_heads) the decode kernel handles: one MFMA tile.
constexpr int kMaxGroup = 16;

struct DecodeParams {
    void* out;                 // [B][Hq][D] bf16 or fp32
    const uint16_t* q;         // [B][Hq][D] bf16
    const uint16_t* pool;      // [NB][2][Hkv][bs][D] bf16
    const int32_t* block_table;
    const int32_t* context_lens;
    int32_t* ws_cum;           // [batch + 1] tiles of the sequences before b (written by the kernel)
    float* ws_records;         // [runs + batch*Hkv][group][D + kRecordPad] fp32
    int32_t max_blocks_per_seq;
    int32_t batch, num_q_heads, num_kv_heads, group;
    int32_t block_size, block_shift;
    int32_t out_f32;
    float scale_log2e;         // scale * log2(e), times the K scale of an FP8 pool
    float out_scale;           // 1, or the V scale of an FP8 pool (applied by the merge kernel)
};

hipError_t launch_decode(const DecodeParams& p, int head_dim, int workgroups, hipStream_t stream);
// FP8 (E4M3) pool: p.pool points at bytes; tiles are kFp8TileTokens tokens.
hipError_t launch_decode_fp8(const DecodeParams& p, int head_dim, int workgroups, hipStream_t stream);
constexpr int kFp8TileTokens = 64;

// Prefill (recomputation): a workgroup is 8 wavefronts, each owning 16 * kPrefillQueryBlocks query rows.
constexpr int kPrefillWaves = 8;
constexpr int kPrefillThreads = kPrefillWaves * 64;
constexpr int kPrefillQueryBlocks = 2;

struct PrefillParams {
    void* out;                 // [total_q][Hq][D] bf16 or fp32
    const uint16_t* q;         // [total_q][Hq][D] bf16
    const void* pool;          // [NB][2][Hkv][bs][D] bf16, or FP8 E4M3 bytes
    const int32_t* block_table;
    const int32_t* context_lens;
    const int32_t* q_starts;   // [batch + 1]
    int32_t max_blocks_per_seq;
    int32_t batch, num_q_heads, num_kv_heads, group;
    int32_t heads_per_wg;      // 8, 4, 2 or 1 query heads of one group per workgroup (divides group)
    int32_t block_size, block_shift;
    int32_t out_f32;
    int32_t kv_fp8;
    float scale_log2e;         // scale * log2(e), times the K scale of an FP8 pool; > 0
    float out_scale;           // 1, or the V scale of an FP8 pool
    int32_t key_splits;        // >= 1 parts of the key range, each handled by its own workgroups
    int64_t total_q;           // packed query rows (only used when key_splits > 1)
    float* ws;                 // [key_splits][total_q][Hq][D + kRecordPad] fp32 (only when key_splits > 1)
};
constexpr int kPrefillMaxKeySplits = 16;

hipError_t launch_prefill(const PrefillParams& p, int head_dim, int max_q_len, hipStream_t stream);

// dst/src are the replica and the pool; to_replica selects the direction.  count (device, may be
// NULL) limits the list to its first *count entries; n then is the launch bound.
hipError_t launch_copy_blocks(void* replica, void* pool, size_t block_bytes, const int32_t* block_ids,
                              int64_t n, const int32_t* count, bool to_replica, hipStream_t stream);

// row_bytes = head_dim * element size (a multiple of 16).
hipError_t launch_append_tokens(void* pool, const void* k_new, const void* v_new,
                                const int32_t* block_table, int max_blocks_per_seq, const int32_t* positions,
                                int batch, int num_kv_heads, int block_size, int row_bytes,
                                uint32_t* dirty_bitmap, hipStream_t stream);

hipError_t launch_append_packed(void* pool, const void* k_new, const void* v_new, const int32_t* block_table,
                                int max_blocks_per_seq, const int32_t* context_lens, const int32_t* q_starts,
                                int batch, int64_t total_q, int num_kv_heads, int block_size, int row_bytes,
                                uint32_t* dirty_bitmap, hipStream_t stream);

hipError_t launch_gather_tokens(const void* pool, void* k_out, void* v_out, const int32_t* block_table,
                                int max_blocks_per_seq, const int32_t* positions, int batch, int num_kv_heads,
                                int block_size, int row_bytes, hipStream_t stream);

hipError_t launch_collect_dirty(uint32_t* dirty_bitmap, int64_t num_blocks, int32_t* ids_out, int64_t capacity,
                                int32_t* count_out, int clear, hipStream_t stream);

// mode 0 / 3: read b (a = 16 writable bytes), 1 / 4: fill a, 2 / 5: a <- b; bytes is a multiple of 16
hipError_t launch_probe(int mode, void* a, const void* b, size_t bytes, hipStream_t stream);

}  // namespace kvflow
