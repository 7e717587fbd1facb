// Internal declarations shared by the translation units of libkvflow (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace kvflow {

// Tokens one wavefront reduces per loop iteration; partitions are multiples of it.
constexpr int kTileTokens = 32;
// Largest query-head group (num_q_heads / num_kv_heads) the decode kernel handles: one MFMA tile.
constexpr int kMaxGroup = 16;

struct DecodeParams {
    void* out;                 // [B][Hq][D] bf16 or fp32
    const uint16_t* q;         // [B][Hq][D] bf16
    const uint16_t* pool;      // [NB][2][Hkv][bs][D] bf16
    const int32_t* block_table;
    const int32_t* context_lens;
    float* workspace;          // [B][Hq][splits][D+2] fp32, used when splits > 1
    int32_t max_blocks_per_seq;
    int32_t batch, num_q_heads, num_kv_heads, group;
    int32_t block_size, block_shift;
    int32_t partition_tokens, splits;
    int32_t out_f32;
    float scale_log2e;         // scale * log2(e)
};

// Library's choice of partition size (tokens) for a problem; multiple of kTileTokens.
int32_t choose_partition_tokens(int32_t batch, int32_t num_kv_heads, int32_t max_context_len);

hipError_t launch_decode(const DecodeParams& p, int head_dim, hipStream_t stream);

// dst/src are the replica and the pool; to_replica selects the direction.
hipError_t launch_copy_blocks(void* replica, void* pool, size_t block_bytes, const int32_t* block_ids,
                              int64_t n, bool to_replica, hipStream_t stream);

}  // namespace kvflow
