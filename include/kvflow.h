/*
 * kvflow.h - C ABI of the paged KV-cache data path for one MI355X (gfx950).
 *
 * The library serves the two uses the paper makes of a block-paged KV cache
 * (Sec. 3.2 item 3, background replication of the KV cache; overhead in Sec. 4.4):
 *   1. the decode step itself: one query token per in-flight request attends to
 *      that request's cached keys/values, stored as fixed-size blocks that a
 *      per-request block table maps from logical to physical position;
 *   2. block-by-block replication: the blocks a step has written are gathered
 *      into a contiguous replica buffer on a separate stream (pack), and a
 *      replication target scatters a replica into its own pool so that requests
 *      go on from the replica (restore).
 * The method's contract is three calls: kv_decode_attn, kv_pack_blocks, kv_restore_blocks.  The
 * calls that widen it (append, dirty list, counted and staged pack, token gather, recomputation)
 * say so where they are declared.  kv_probe_stream, kv_probe_matrix, kv_decode_workgroups and kv_validate_* are
 * diagnostics for benchmarks and debugging, outside the method's contract.
 *
 * General rules
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer.  The library allocates no device memory, keeps no
 *     state between calls (but the address of kv_decode_attn_static's fixed array, looked
 *     up once per GPU) and never synchronises: a call validates its host
 *     arguments, enqueues kernels on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns.  Buffers must stay alive and
 *     unmodified until the stream has passed the enqueued work.
 *   - Return value: KV_OK (0) or a negative kv_status.  Host-checkable mistakes
 *     are reported before anything is launched; nothing is written in that case.
 *   - Contents of device arrays (block ids, context lengths) cannot be checked
 *     without a device-to-host copy and are PRECONDITIONS, listed per call.
 *     kv_validate_* checks them with a synchronising copy, for debugging.
 *   - pack || decode on two streams is legal (both only read the pool);
 *     restore -> decode needs stream order or an event.
 *
 * Pool layout: [num_blocks][2][num_kv_heads][block_size][head_dim], elements bf16 or
 * FP8 E4M3 (half the bytes for every call below; one fp32 scale for K and one for V),
 * second axis 0 = K, 1 = V.  One block is one contiguous chunk of
 * kv_block_bytes() bytes; layers are stacked as separate blocks of one flat pool.
 */
#ifndef KVFLOW_H
#define KVFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KV_OK = 0,
    KV_ERR_NULL = -1,        /* a required pointer is NULL */
    KV_ERR_SHAPE = -2,       /* non-positive or inconsistent dimension */
    KV_ERR_UNSUPPORTED = -3, /* dimension or dtype outside what the kernels are built for */
    KV_ERR_ALIGN = -4,       /* a buffer is not 16-byte aligned */
    KV_ERR_WORKSPACE = -5,   /* workspace missing or too small */
    KV_ERR_LAUNCH = -6,      /* the HIP runtime refused the launch */
    KV_ERR_CONTENT = -7      /* kv_validate_*: a device array violates a precondition */
} kv_status;

enum { KV_DTYPE_BF16 = 0, KV_DTYPE_F32 = 1, KV_DTYPE_FP8_E4M3 = 2 };

/* Host struct describing the block pool; read during the call only. */
typedef struct {
    void*   base;          /* device, 16-byte aligned, layout above */
    int64_t num_blocks;    /* > 0 */
    int32_t num_kv_heads;  /* > 0 */
    int32_t block_size;    /* tokens per block: 16 or 32 */
    int32_t head_dim;      /* 64 or 128 */
    int32_t dtype;         /* KV_DTYPE_BF16, or KV_DTYPE_FP8_E4M3 (OCP 8-bit float, 1-4-3, bias 7) */
    float   k_scale;       /* FP8 pool only: key value = stored number * k_scale; > 0, finite */
    float   v_scale;       /* FP8 pool only: value value = stored number * v_scale; > 0, finite */
} kv_pool_desc;

/* Bytes of one block = 2 * num_kv_heads * block_size * head_dim * element bytes (2 for bf16, 1 for
 * FP8); 0 if pool is NULL/invalid. */
size_t kv_block_bytes(const kv_pool_desc* pool);

/*
 * Decode runs on a persistent grid: the cached tokens of the whole batch are cut into
 * equally long runs, one per wavefront (4 wavefronts per workgroup), whatever the mix of context
 * lengths.  num_workgroups == 0 asks for the library's choice (enough to fill the chip, fewer for
 * small problems); a caller may pass a smaller positive number to leave compute units to other
 * streams.  Returns the number of workgroups a call with these arguments launches, 0 on invalid
 * arguments (non-positive sizes, num_workgroups < 0 or > 65535).
 */
int32_t kv_decode_workgroups(int32_t batch, int32_t num_kv_heads, int32_t max_context_len,
                             int32_t num_workgroups);

/*
 * Bytes of workspace kv_decode_attn needs for these arguments (always > 0 for valid arguments):
 * the per-sequence tile counts plus one partial-result record per (run, KV-head row it touches,
 * query head).  0 on invalid arguments.
 */
size_t kv_decode_workspace_bytes(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                 int32_t head_dim, int32_t max_context_len, int32_t num_workgroups);

/*
 * Paged decode attention (Sec. 3.2 item 3: attention state kept in a
 * block-represented KV cache).  For every sequence b and query head h, with
 * kvh = h / (num_q_heads / num_kv_heads) and L = context_lens[b]:
 *     s[t]   = scale * sum_d q[b,h,d] * K[table[b][t / bs], kvh, t % bs, d]     0 <= t < L
 *     out[b,h,:] = sum_t softmax(s)[t] * V[table[b][t / bs], kvh, t % bs, :]
 * bf16 inputs, fp32 accumulation; L == 0 gives a row of zeros.  With an FP8 pool K and V are
 * the stored numbers times k_scale / v_scale (decoded exactly, products in bf16 x bf16 -> fp32);
 * q stays bf16.
 *
 *   out            [batch][num_q_heads][head_dim], out_dtype KV_DTYPE_BF16 or KV_DTYPE_F32, written
 *   q              [batch][num_q_heads][head_dim] bf16, read
 *   pool           host struct; the pool is read
 *   block_table    int32 [batch][max_blocks_per_seq], read; only the first
 *                  ceil(L/bs) entries of a row are dereferenced
 *   context_lens   int32 [batch], read
 *   max_context_len host-side upper bound of context_lens[]; sizes the grid and the workspace
 *   num_workgroups 0 = library's choice, else the persistent grid size (see above)
 *   workspace      >= kv_decode_workspace_bytes(...) bytes (same arguments), 16-byte aligned,
 *                  scratch: contents on entry are ignored, contents on return are unspecified
 * Preconditions on device contents: 0 <= context_lens[b] <= max_context_len;
 * 0 <= block_table[b][j] < num_blocks for j < ceil(context_lens[b] / bs).
 * Slots past L in the last block, unreferenced table entries and unreferenced
 * blocks are never used and may hold anything, including NaN patterns.
 * The result depends only on logical token positions: for the same batch, context
 * lengths and num_workgroups, two pools that hold the same blocks under different
 * physical ids give bitwise equal outputs.
 * Errors: NULL, SHAPE (dims <= 0, num_q_heads % num_kv_heads, num_q_heads /
 * num_kv_heads > 16, max_context_len > max_blocks_per_seq * bs, num_workgroups out of
 * range), UNSUPPORTED (head_dim, block_size, dtypes), ALIGN, WORKSPACE, LAUNCH.
 * batch == 0 returns KV_OK without a launch.
 */
int kv_decode_attn(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                   const int32_t* block_table, int32_t max_blocks_per_seq,
                   const int32_t* context_lens, int32_t batch, int32_t num_q_heads,
                   int32_t max_context_len, float scale, int32_t num_workgroups,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * kv_decode_attn for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, preconditions and results (bit for bit) as kv_decode_attn; the
 * workspace is a fixed array of KV_DECODE_STATIC_SCRATCH_BYTES inside the library's device code,
 * one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 *   - Arguments whose kv_decode_workspace_bytes() exceeds KV_DECODE_STATIC_SCRATCH_BYTES are
 *     refused with KV_ERR_WORKSPACE before any launch (at 8 query heads per KV head and head_dim
 *     128 the array covers 256 workgroups and batch * num_kv_heads up to about 2900).
 *   - The device that `stream` belongs to must be the current device of the calling thread.
 *   - All calls on one GPU share that GPU's array: two calls that may overlap on the same GPU
 *     (different streams without an ordering between them) race on it and give undefined
 *     results.  Calls ordered by a stream or by events are fine; nothing has to be cleared
 *     between them (the kernels never read what an earlier call left there).
 *   - The first call on a device looks the array's address up (no allocation); make that call
 *     outside graph capture.
 * Errors: those of kv_decode_attn; WORKSPACE as above; LAUNCH also when the current device or
 * the array's address cannot be obtained.
 */
#define KV_DECODE_STATIC_SCRATCH_BYTES (16u << 20)
int kv_decode_attn_static(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                          const int32_t* block_table, int32_t max_blocks_per_seq,
                          const int32_t* context_lens, int32_t batch, int32_t num_q_heads,
                          int32_t max_context_len, float scale, int32_t num_workgroups, void* stream);

/*
 * Recomputation of attention state over the paged cache (Sec. 3.2 item 3: a node that dropped
 * replicas under memory pressure recomputes them): causal attention of many query tokens per
 * sequence.  Sequence b has L = context_lens[b] tokens in the pool, the newest
 * n = q_starts[b+1] - q_starts[b] of which are this call's query tokens (their K/V rows are in
 * the pool already, e.g. written by kv_append_tokens or restored from a replica).  Query token i
 * of sequence b (packed row t = q_starts[b] + i) sits at position pos = L - n + i and, with
 * kvh = h / (num_q_heads / num_kv_heads):
 *     s[u]       = scale * sum_d q[t,h,d] * K[table[b][u / bs], kvh, u % bs, d]     0 <= u <= pos
 *     out[t,h,:] = sum_u softmax(s)[u] * V[table[b][u / bs], kvh, u % bs, :]
 * bf16 inputs, fp32 accumulation.  n == 1 is kv_decode_attn's operation.  A query with pos < 0
 * (n > L) sees no key and gives a row of zeros.  With an FP8 pool K and V are the stored numbers
 * times k_scale / v_scale, as for kv_decode_attn.
 *
 *   out            [total_q][num_q_heads][head_dim], out_dtype KV_DTYPE_BF16 or KV_DTYPE_F32, written;
 *                  total_q = q_starts[batch]
 *   q              [total_q][num_q_heads][head_dim] bf16, read; sequences packed in batch order
 *   pool           host struct; bf16 or FP8 pool, read
 *   block_table    int32 [batch][max_blocks_per_seq], read; only the first ceil(L/bs) entries of a row
 *   context_lens   int32 [batch], read; counts the query tokens too
 *   q_starts       int32 [batch + 1], read; non-decreasing, q_starts[0] == 0
 *   max_q_len      host-side upper bound of the n above; sizes the grid
 *   total_q        number of packed query rows (the host's copy of q_starts[batch])
 *   key_splits     0 or 1: every (sequence, KV head, token range) is walked by one workgroup.  2..16: the key
 *                  range is cut into that many parts handled by separate workgroups, which fills the chip
 *                  when there are few query tokens over long contexts; the parts are combined in a fixed
 *                  order by a second kernel.  kv_prefill_key_splits() suggests a value.
 *   workspace      only for key_splits > 1: >= kv_prefill_workspace_bytes(...) bytes, 16-byte aligned,
 *                  scratch (contents on entry ignored, on return unspecified); else may be NULL
 * Preconditions on device contents: 0 <= context_lens[b] <= max_blocks_per_seq * bs; table entries as
 * for kv_decode_attn; 0 <= n <= max_q_len; q_starts[batch] == total_q.
 * The result depends only on logical token positions (and on key_splits).
 * scale must be positive and finite (the kernel takes the max of raw scores before scaling them).
 * Errors: NULL, SHAPE (also a scale that is not positive and finite), UNSUPPORTED (head_dim, block_size,
 * dtypes, batch or num_q_heads > 65535, max_q_len > 65535 * 32), ALIGN, WORKSPACE, LAUNCH (also a grid
 * of more than 65535 token-range groups x parts).  batch == 0, max_q_len == 0 or total_q == 0 returns
 * KV_OK without a launch.
 */
int kv_prefill_attn(void* out, int32_t out_dtype, const void* q, const kv_pool_desc* pool,
                    const int32_t* block_table, int32_t max_blocks_per_seq,
                    const int32_t* context_lens, const int32_t* q_starts, int32_t batch,
                    int32_t num_q_heads, int32_t max_q_len, int64_t total_q, float scale,
                    int32_t key_splits, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Parts of the key range that fill the chip for these host-side bounds: 1 when the token ranges alone
 * give enough workgroups, up to 16 otherwise (never parts shorter than 512 keys).  0 on invalid arguments.
 */
int32_t kv_prefill_key_splits(int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t max_q_len,
                              int32_t max_context_len);

/* Bytes of workspace kv_prefill_attn needs: key_splits records of (head_dim + 4) floats per (query row,
 * head); 0 for key_splits <= 1 or invalid arguments. */
size_t kv_prefill_workspace_bytes(int64_t total_q, int32_t num_q_heads, int32_t head_dim, int32_t key_splits);

/*
 * Gather side of block-by-block replication (Sec. 3.2 item 3; meant to run on a
 * stream of its own beside decode, Sec. 4.4):
 *     replica[i] <- pool[block_ids[i]]   for i in [0, n), whole blocks, list order.
 *   replica    [n][kv_block_bytes] bytes, 16-byte aligned, written
 *   block_ids  int32 [n], read; ids may repeat
 * Precondition: 0 <= block_ids[i] < num_blocks.  n == 0 returns KV_OK without a launch.
 */
int kv_pack_blocks(void* replica, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n,
                   void* stream);

/*
 * Scatter side, used on the replication target at recovery (Sec. 3.2 item 3:
 * requests continue from the replicated state):
 *     pool[block_ids[i]] <- replica[i]   for i in [0, n).
 * Blocks not listed are left untouched.
 * Preconditions: 0 <= block_ids[i] < num_blocks and the ids are pairwise
 * distinct (a repeated id is a write race; the result for that block is undefined).
 */
int kv_restore_blocks(const kv_pool_desc* pool, const void* replica, const int32_t* block_ids,
                      int64_t n, void* stream);

/*
 * Appending a decode step's new tokens and tracking dirty blocks: the step that produces "the
 * blocks a step has written" which background replication then ships (Sec. 3.2 item 3).
 *
 * kv_append_tokens: one new token per sequence.  For every b with positions[b] >= 0 the rows
 * k_new[b], v_new[b] (all KV heads) are written to position t = positions[b] of sequence b, i.e.
 * row t % bs of block block_table[b][t / bs], and that block's bit is OR-ed into dirty_bitmap.
 *   k_new, v_new   [batch][num_kv_heads][head_dim] in the pool's element type (for an FP8 pool:
 *                  already divided by the scales and rounded), 16-byte aligned, read
 *   positions      int32 [batch], read; < 0 = the sequence takes no token
 *   dirty_bitmap   uint32 [ceil(num_blocks / 32)], bit p % 32 of word p / 32 stands for block p;
 *                  read-modify-written (atomic OR), so it accumulates over steps until collected.
 *                  The caller zeroes it once after allocation.
 * Preconditions: positions[b] < max_blocks_per_seq * bs; the table entry it selects is a valid
 * block id; no two sequences map to the same (block, row).
 */
int kv_append_tokens(const kv_pool_desc* pool, const void* k_new, const void* v_new,
                     const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* positions,
                     int32_t batch, uint32_t* dirty_bitmap, void* stream);

/*
 * The same for many new tokens per sequence (the K/V rows of recomputed or prefilled tokens), with
 * kv_prefill_attn's conventions: packed row t = q_starts[b] + i of k_new / v_new
 * ([total_q][num_kv_heads][head_dim], pool element type) goes to position context_lens[b] - n + i of
 * sequence b, n = q_starts[b+1] - q_starts[b], and its block is marked dirty.  Rows whose position
 * would be negative are skipped.  Call it before kv_prefill_attn on the same stream.
 * Preconditions on device contents as for kv_prefill_attn; q_starts[batch] == total_q.
 * Errors: NULL, SHAPE, UNSUPPORTED, ALIGN, LAUNCH.  batch == 0 or total_q == 0 returns KV_OK without a launch.
 */
int kv_append_packed(const kv_pool_desc* pool, const void* k_new, const void* v_new,
                     const int32_t* block_table, int32_t max_blocks_per_seq, const int32_t* context_lens,
                     const int32_t* q_starts, int32_t batch, int64_t total_q, uint32_t* dirty_bitmap,
                     void* stream);

/*
 * kv_gather_tokens: the inverse of kv_append_tokens, for replication at token granularity (what
 * a step has written is one row per sequence, not the block around it; over a slow link the
 * difference is a factor of block_size).  For every b with positions[b] >= 0 the K and V rows at
 * position positions[b] of sequence b are copied to k_out[b], v_out[b]; other rows of k_out, v_out
 * are left untouched.  The replication target applies the received rows with kv_append_tokens.
 *   k_out, v_out   [batch][num_kv_heads][head_dim] in the pool's element type, 16-byte aligned, written
 * Preconditions as for kv_append_tokens.
 */
int kv_gather_tokens(void* k_out, void* v_out, const kv_pool_desc* pool, const int32_t* block_table,
                     int32_t max_blocks_per_seq, const int32_t* positions, int32_t batch, void* stream);

/*
 * kv_collect_dirty: dirty bitmap -> ascending list of block ids, on the device.
 *   dirty_ids    int32 [capacity], written: the first min(count, capacity) dirty ids, ascending
 *   dirty_count  int32 [1], written: the number of dirty blocks (may exceed capacity: the caller
 *                sized the list too small and sees it here)
 *   clear        non-zero: the bitmap is zeroed for the next round of steps
 * One workgroup; meant for pools of up to a few million blocks.
 */
int kv_collect_dirty(uint32_t* dirty_bitmap, int64_t num_blocks, int32_t* dirty_ids, int64_t capacity,
                     int32_t* dirty_count, int32_t clear, void* stream);

/*
 * kv_pack_blocks into a destination on the far side of a slow link (pinned host memory standing in
 * for a peer's buffer; Sec. 3.2 item 3: replication proceeds block by block in the background,
 * Sec. 3.3: over the network), through a small double-buffered device staging area:
 *     dst[i] <- pool[block_ids[i]]   for i in [0, n), list order, as kv_pack_blocks.
 * The list is cut into chunks of chunk_blocks blocks.  Chunk c is packed at HBM speed into half
 * c % 2 of `staging` on pack_stream and then copied to dst by the copy engine on copy_stream, so
 * that the pack of chunk c + 1 runs beside the copy of chunk c and the compute units are busy with
 * replication only for the short pack kernels.  The ordering between the two streams (half
 * packed -> copy may start; copy done -> half may be packed again) is enqueued with events that
 * the call creates and releases itself; the call does not wait for anything.
 *   dst           n * kv_block_bytes() bytes, 16-byte aligned: pinned host memory, or device
 *                 memory the copy engine can reach; written
 *   staging       device, 2 * chunk_blocks * kv_block_bytes() bytes, 16-byte aligned; scratch
 *   chunk_blocks  > 0; blocks per chunk (e.g. 32 MiB worth)
 *   pack_stream, copy_stream   two streams of the caller (they may be the same stream, which
 *                 serialises packs and copies); the transfer is complete when copy_stream has passed
 *                 the enqueued work, and staging may be reused when both streams have
 * Preconditions as for kv_pack_blocks.  Errors: NULL, SHAPE, UNSUPPORTED, ALIGN, LAUNCH (also when
 * an event cannot be created or a copy cannot be enqueued).  n == 0 returns KV_OK with nothing enqueued.
 */
int kv_pack_blocks_staged(void* dst, const kv_pool_desc* pool, const int32_t* block_ids, int64_t n, void* staging,
                          int64_t chunk_blocks, void* pack_stream, void* copy_stream);

/*
 * kv_pack_blocks with the list length taken from device memory, so that the loop
 * append -> collect -> pack runs without the host seeing the list:
 *     replica[i] <- pool[block_ids[i]]   for i in [0, min(*count, max_n)).
 *   count   int32 [1], device, read when the kernel runs
 *   max_n   host bound of the list length; sizes the launch and the replica buffer
 */
int kv_pack_blocks_counted(void* replica, const kv_pool_desc* pool, const int32_t* block_ids,
                           const int32_t* count, int64_t max_n, void* stream);

/*
 * Debug helpers: copy the device arrays to the host (synchronising `stream`)
 * and check the preconditions above.  Return KV_OK, KV_ERR_CONTENT, or an
 * argument error.  Not for the hot path.
 */
int kv_validate_decode(const kv_pool_desc* pool, const int32_t* block_table,
                       int32_t max_blocks_per_seq, const int32_t* context_lens, int32_t batch,
                       int32_t max_context_len, void* stream);
int kv_validate_block_ids(const kv_pool_desc* pool, const int32_t* block_ids, int64_t n,
                          int32_t require_distinct, void* stream);
/* Preconditions of kv_prefill_attn: q_starts starts at 0, does not decrease, ends at total_q; every
 * sequence has 0 <= n <= max_q_len query tokens and at least n cached ones; lengths and table entries
 * as for kv_validate_decode. */
int kv_validate_prefill(const kv_pool_desc* pool, const int32_t* block_table, int32_t max_blocks_per_seq,
                        const int32_t* context_lens, const int32_t* q_starts, int32_t batch,
                        int32_t max_q_len, int64_t total_q, void* stream);

/*
 * HBM yardsticks for roofline tables (for callers that measure: benchmarks, bring-up): one plain
 * streaming kernel over `bytes` bytes (a multiple of 16) with 16-byte non-temporal accesses.
 *   mode 0  read b once; a points at >= 16 writable bytes that are left untouched
 *   mode 1  write a once (contents unspecified)
 *   mode 2  a <- b, contiguous copy
 *   mode 3, 4, 5  the same three with a second kernel design, so that a ceiling read off these
 *           numbers does not rest on one kernel
 * Modes 0-2 give every XCD a contiguous eighth of the buffer and write through at device scope
 * (the design of the block-copy kernels; at most 32 GiB per call); modes 3-5 walk the buffer in
 * workgroup order (a persistent grid for the read).
 * a, b: device pointers, 16-byte aligned, must not overlap.  Errors: SHAPE, NULL, ALIGN, LAUNCH.
 */
int kv_probe_stream(int32_t mode, void* a, const void* b, size_t bytes, void* stream);

/*
 * Matrix-core yardstick for the recomputation kernel's roofline (for callers that measure): 256
 * workgroups of 8 wavefronts (one per compute unit; wavefronts w and w + 4 share a SIMD) repeat,
 * `iters` times, a matrix block (32 MFMAs 16x16x32 bf16 on registers: 8 A fragments, 4 B fragments,
 * 16 accumulators; 32 * 16384 flop per wavefront) and/or a vector block (80 fused multiply-adds and
 * 16 exp2 on 16 values: about the vector work of one 32-key x 32-query softmax step).
 *   mode 0  all wavefronts: matrix blocks, operands all zero
 *   mode 1  all wavefronts: matrix blocks, operands uniform in [-1, 1) (the device lowers its clock
 *           under the switching activity of such data; compare with mode 0)
 *   mode 2  all wavefronts: vector blocks
 *   mode 3  wavefronts 0-3 matrix blocks (operands as in mode 1), their SIMD partners vector blocks
 *   mode 4  wavefronts 0-3 matrix blocks, the partners idle
 *   mode 5  wavefronts 4-7 vector blocks, the partners idle
 * sink: device pointer, 16-byte aligned, at least KV_PROBE_MATRIX_SINK_BYTES bytes, overwritten
 * with values of no meaning.  Errors: SHAPE (mode, negative iters), NULL, ALIGN, WORKSPACE (sink
 * too small), LAUNCH.
 */
#define KV_PROBE_MATRIX_SINK_BYTES (256u * 512u * 4u)
int kv_probe_matrix(int32_t mode, int32_t iters, void* sink, size_t sink_bytes, void* stream);

/* Static, human-readable text for a kv_status value. */
const char* kv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* KVFLOW_H */
