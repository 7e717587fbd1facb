/*
 * CPU oracle for the paged KV-cache data path.  TEST INFRASTRUCTURE ONLY: it is
 * the slow, plain definition that the GPU library is checked against; nothing
 * in the product path may call it.
 *
 * What it defines
 *   - decode attention of one query token per sequence over that sequence's
 *     cached keys/values, where the cache is stored as fixed-size blocks that a
 *     per-sequence block table maps from logical to physical position.  This is
 *     the block-structured cache that Sec. 3.2 item 3 (background replication
 *     of the KV cache) of the paper builds on; the attention formula is
 *     the textbook scaled dot-product attention with grouped query heads
 *     (consecutive query heads share one KV head).
 *   - block-by-block replication (Sec. 3.2 item 3, Sec. 4.4): gather listed
 *     pool blocks into a contiguous replica, and the inverse used when a
 *     replication target takes over requests and continues them from its copy.
 *
 * All floating point is IEEE double.  Inputs are bf16 bit patterns (uint16)
 * widened exactly: bf16 -> fp32 by a 16-bit left shift -> double.  The pool may
 * instead hold FP8 E4M3 bit patterns (uint8) with one fp32 scale for K and one
 * for V; they are decoded exactly and multiplied by the scale in double.
 *
 * Pool layout: [num_blocks][2][num_kv_heads][block_size][head_dim] bf16,
 * index 0 of the second axis is K, index 1 is V.  Only the accessor kv_at()
 * knows this.
 *
 * No blocking, fusion or reordering: scores in ascending token order, then the
 * max, then the weights, then their sum, then the weighted sum of V rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    const void* base;
    int64_t num_blocks;
    int num_kv_heads, block_size, head_dim;
    int fp8;                /* 0: bf16 elements; 1: OCP FP8 E4M3 elements */
    double k_scale, v_scale; /* FP8 pools store value / scale; 1 for bf16 */
} pool_view;

static double bf16_to_double(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/*
 * OCP 8-bit floating point, E4M3 variant: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
 * exponent field 0 is subnormal (m/8 * 2^-6), there are no infinities, and exponent 15 with
 * mantissa 7 is NaN, so the largest magnitude is 1.75 * 2^8 = 448.
 */
static double fp8_e4m3_to_double(uint8_t bits)
{
    int e = (bits >> 3) & 15, m = bits & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (bits & 0x80) ? -v : v;
}

/* which: 0 = key, 1 = value; p physical block; kvh KV head; r row in block; d channel.
 * For an FP8 pool the stored number times the pool's K or V scale is the value. */
static double kv_at(const pool_view* pv, int which, int64_t p, int kvh, int r, int d)
{
    int64_t idx = (((p * 2 + which) * pv->num_kv_heads + kvh) * pv->block_size + r) * (int64_t)pv->head_dim + d;
    if (pv->fp8)
        return fp8_e4m3_to_double(((const uint8_t*)pv->base)[idx]) * (which ? pv->v_scale : pv->k_scale);
    return bf16_to_double(((const uint16_t*)pv->base)[idx]);
}

/* One (sequence, query head) output row.  s and w are caller scratch of >= L doubles. */
static void decode_row(double* out_row, const uint16_t* q_row, const pool_view* pv,
                       const int32_t* table_row, int L, int kvh, double scale,
                       double* s, double* w)
{
    const int D = pv->head_dim, bs = pv->block_size;
    if (L == 0) {
        for (int d = 0; d < D; ++d) out_row[d] = 0.0;
        return;
    }
    for (int t = 0; t < L; ++t) {
        int64_t p = table_row[t / bs];
        int r = t % bs;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += bf16_to_double(q_row[d]) * kv_at(pv, 0, p, kvh, r, d);
        s[t] = scale * dot;
    }
    double m = s[0];
    for (int t = 1; t < L; ++t) if (s[t] > m) m = s[t];
    double l = 0.0;
    for (int t = 0; t < L; ++t) { w[t] = exp(s[t] - m); l += w[t]; }
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int t = 0; t < L; ++t) {
            int64_t p = table_row[t / bs];
            acc += w[t] * kv_at(pv, 1, p, kvh, t % bs, d);
        }
        out_row[d] = acc / l;
    }
}

static int check_decode_args(int64_t num_blocks, int num_kv_heads, int block_size, int head_dim,
                             const int32_t* block_table, int max_blocks_per_seq,
                             const int32_t* context_lens, int batch, int num_q_heads)
{
    if (num_blocks <= 0 || num_kv_heads <= 0 || block_size <= 0 || head_dim <= 0) return -2;
    if (batch < 0 || num_q_heads <= 0 || num_q_heads % num_kv_heads != 0) return -2;
    for (int b = 0; b < batch; ++b) {
        int L = context_lens[b];
        if (L < 0 || (int64_t)L > (int64_t)max_blocks_per_seq * block_size) return -3;
        int nb = (L + block_size - 1) / block_size;
        for (int j = 0; j < nb; ++j) {
            int32_t p = block_table[(int64_t)b * max_blocks_per_seq + j];
            if (p < 0 || p >= num_blocks) return -4;
        }
    }
    return 0;
}

/*
 * rows: optional list of n_rows (b, h) pairs (int32[2*n_rows]); when NULL every
 * (b, h) is computed and out is [batch][num_q_heads][head_dim]; otherwise out
 * is [n_rows][head_dim].  Returns the number of threads used (>= 1) or a
 * negative error.
 */
int kvo_decode_attn(double* out, const uint16_t* q, const void* pool, int kv_fp8, float k_scale, float v_scale,
                    int64_t num_blocks, int num_kv_heads, int block_size, int head_dim,
                    const int32_t* block_table, int max_blocks_per_seq,
                    const int32_t* context_lens, int batch, int num_q_heads, float scale,
                    const int32_t* rows, int64_t n_rows, int num_threads)
{
    int rc = check_decode_args(num_blocks, num_kv_heads, block_size, head_dim, block_table,
                               max_blocks_per_seq, context_lens, batch, num_q_heads);
    if (rc) return rc;
    pool_view pv = { pool, num_blocks, num_kv_heads, block_size, head_dim, kv_fp8 != 0,
                     kv_fp8 ? (double)k_scale : 1.0, kv_fp8 ? (double)v_scale : 1.0 };
    const int G = num_q_heads / num_kv_heads;
    const int64_t total = rows ? n_rows : (int64_t)batch * num_q_heads;
    int maxL = 1;
    for (int b = 0; b < batch; ++b) if (context_lens[b] > maxL) maxL = context_lens[b];
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#pragma omp parallel
#endif
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)maxL);
        double* w = (double*)malloc(sizeof(double) * (size_t)maxL);
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t i = 0; i < total; ++i) {
            int b = rows ? rows[2 * i] : (int)(i / num_q_heads);
            int h = rows ? rows[2 * i + 1] : (int)(i % num_q_heads);
            decode_row(out + i * head_dim, q + ((int64_t)b * num_q_heads + h) * head_dim, &pv,
                       block_table + (int64_t)b * max_blocks_per_seq, context_lens[b], h / G,
                       (double)scale, s, w);
        }
        free(s);
        free(w);
    }
    return used;
}

/* replica[i] <- pool[ids[i]], whole blocks, list order; ids may repeat. */
int kvo_pack_blocks(uint8_t* replica, const uint8_t* pool, int64_t block_bytes, int64_t num_blocks,
                    const int32_t* ids, int64_t n, int num_threads)
{
    for (int64_t i = 0; i < n; ++i) if (ids[i] < 0 || ids[i] >= num_blocks) return -4;
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i)
            memcpy(replica + i * block_bytes, pool + (int64_t)ids[i] * block_bytes, (size_t)block_bytes);
    }
#else
    for (int64_t i = 0; i < n; ++i)
        memcpy(replica + i * block_bytes, pool + (int64_t)ids[i] * block_bytes, (size_t)block_bytes);
#endif
    return used;
}

/* pool[ids[i]] <- replica[i]; ids must be pairwise distinct (else -5, nothing written). */
int kvo_restore_blocks(uint8_t* pool, const uint8_t* replica, int64_t block_bytes, int64_t num_blocks,
                       const int32_t* ids, int64_t n, int num_threads)
{
    uint8_t* seen = (uint8_t*)calloc((size_t)num_blocks, 1);
    if (!seen) return -6;
    for (int64_t i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= num_blocks) { free(seen); return -4; }
        if (seen[ids[i]]) { free(seen); return -5; }
        seen[ids[i]] = 1;
    }
    free(seen);
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(static)
        for (int64_t i = 0; i < n; ++i)
            memcpy(pool + (int64_t)ids[i] * block_bytes, replica + i * block_bytes, (size_t)block_bytes);
    }
#else
    for (int64_t i = 0; i < n; ++i)
        memcpy(pool + (int64_t)ids[i] * block_bytes, replica + i * block_bytes, (size_t)block_bytes);
#endif
    return used;
}

/*
 * Writing a step's new tokens into the pool and tracking the blocks that became dirty (the
 * blocks that hold new tokens, which background replication then ships block by block;
 * Sec. 3.2 item 3).  One new token per sequence: sequence b's K/V rows (all KV heads) go to
 * position positions[b] of its context, i.e. to row positions[b] % bs of physical block
 * block_table[b][positions[b] / bs]; positions[b] < 0 means the sequence takes no token.
 * The dirty bitmap has one bit per pool block (bit p % 32 of word p / 32) and is OR-ed into,
 * so it accumulates over steps until it is collected.
 * k_new, v_new: bf16 [batch][num_kv_heads][head_dim].
 */
int kvo_append_tokens(uint16_t* pool, int64_t num_blocks, int num_kv_heads, int block_size, int head_dim,
                      const uint16_t* k_new, const uint16_t* v_new, const int32_t* block_table,
                      int max_blocks_per_seq, const int32_t* positions, int batch, uint32_t* dirty_bitmap)
{
    if (num_blocks <= 0 || num_kv_heads <= 0 || block_size <= 0 || head_dim <= 0 || batch < 0) return -2;
    for (int b = 0; b < batch; ++b) {
        int t = positions[b];
        if (t < 0) continue;
        if ((int64_t)t >= (int64_t)max_blocks_per_seq * block_size) return -3;
        int32_t p = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
        if (p < 0 || p >= num_blocks) return -4;
    }
    for (int b = 0; b < batch; ++b) {
        int t = positions[b];
        if (t < 0) continue;
        int64_t p = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
        int r = t % block_size;
        for (int kvh = 0; kvh < num_kv_heads; ++kvh) {
            for (int which = 0; which < 2; ++which) {
                const uint16_t* src = (which ? v_new : k_new) + ((int64_t)b * num_kv_heads + kvh) * head_dim;
                uint16_t* dst = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)head_dim);
                for (int d = 0; d < head_dim; ++d) dst[d] = src[d];
            }
        }
        dirty_bitmap[p / 32] |= (uint32_t)1 << (p % 32);
    }
    return 0;
}

/* Dirty bitmap -> ascending list of block ids; returns their number.  clear != 0 zeroes the bitmap. */
int64_t kvo_collect_dirty(uint32_t* dirty_bitmap, int64_t num_blocks, int32_t* ids_out, int clear)
{
    int64_t n = 0;
    for (int64_t p = 0; p < num_blocks; ++p)
        if (dirty_bitmap[p / 32] >> (p % 32) & 1u) ids_out[n++] = (int32_t)p;
    if (clear) for (int64_t w = 0; w < (num_blocks + 31) / 32; ++w) dirty_bitmap[w] = 0;
    return n;
}

/*
 * Token-granular replication, gather side: the rows of the tokens at positions[b] (the ones a
 * step has just written) are copied out of the pool into contiguous arrays
 * k_out, v_out [batch][num_kv_heads][row_elems]; the inverse of kvo_append_tokens, which is what
 * the replication target runs on the received rows.  Rows of sequences with positions[b] < 0
 * are left untouched.  Elements are 16-bit; an FP8 row is passed as head_dim / 2 of them.
 */
int kvo_gather_tokens(const uint16_t* pool, int64_t num_blocks, int num_kv_heads, int block_size, int row_elems,
                      uint16_t* k_out, uint16_t* v_out, const int32_t* block_table, int max_blocks_per_seq,
                      const int32_t* positions, int batch)
{
    if (num_blocks <= 0 || num_kv_heads <= 0 || block_size <= 0 || row_elems <= 0 || batch < 0) return -2;
    for (int b = 0; b < batch; ++b) {
        int t = positions[b];
        if (t < 0) continue;
        if ((int64_t)t >= (int64_t)max_blocks_per_seq * block_size) return -3;
        int32_t p = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
        if (p < 0 || p >= num_blocks) return -4;
    }
    for (int b = 0; b < batch; ++b) {
        int t = positions[b];
        if (t < 0) continue;
        int64_t p = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
        int r = t % block_size;
        for (int kvh = 0; kvh < num_kv_heads; ++kvh)
            for (int which = 0; which < 2; ++which) {
                const uint16_t* src = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)row_elems);
                uint16_t* dst = (which ? v_out : k_out) + ((int64_t)b * num_kv_heads + kvh) * row_elems;
                for (int d = 0; d < row_elems; ++d) dst[d] = src[d];
            }
    }
    return 0;
}

/*
 * Prefill / recomputation over the paged cache (the fallback of Sec. 3.2 item 3: a node that
 * dropped replicas under memory pressure recomputes them).  Sequence b has context_lens[b]
 * tokens in the pool, the last q_len_b = q_starts[b + 1] - q_starts[b] of which are the query
 * tokens of this call (their K/V rows are already in the pool).  Query token j of sequence b
 * sits at position pos = context_lens[b] - q_len_b + j and attends causally: to the keys at
 * positions 0 .. pos and to nothing later.  That is the decode definition above with the
 * context cut off after pos, which is how it is written here.  A query whose position would be
 * negative (q_len_b > context_lens[b]) has no key and gives a row of zeros.
 *
 * q: bf16 [total_q][num_q_heads][head_dim], sequences packed in batch order (total_q =
 * q_starts[batch]).  rows: optional list of n_rows (t, h) pairs, t a packed query-token index;
 * when NULL every (t, h) is computed and out is [total_q][num_q_heads][head_dim], otherwise
 * out is [n_rows][head_dim].  Returns the number of threads used or a negative error.
 */
int kvo_prefill_attn(double* out, const uint16_t* q, const void* pool, int kv_fp8, float k_scale, float v_scale,
                     int64_t num_blocks, int num_kv_heads, int block_size, int head_dim,
                     const int32_t* block_table, int max_blocks_per_seq,
                     const int32_t* context_lens, const int32_t* q_starts, int batch, int num_q_heads,
                     float scale, const int32_t* rows, int64_t n_rows, int num_threads)
{
    int rc = check_decode_args(num_blocks, num_kv_heads, block_size, head_dim, block_table,
                               max_blocks_per_seq, context_lens, batch, num_q_heads);
    if (rc) return rc;
    if (q_starts[0] != 0) return -2;
    for (int b = 0; b < batch; ++b) if (q_starts[b + 1] < q_starts[b]) return -2;
    pool_view pv = { pool, num_blocks, num_kv_heads, block_size, head_dim, kv_fp8 != 0,
                     kv_fp8 ? (double)k_scale : 1.0, kv_fp8 ? (double)v_scale : 1.0 };
    const int G = num_q_heads / num_kv_heads;
    const int64_t total_q = q_starts[batch];
    const int64_t total = rows ? n_rows : total_q * num_q_heads;
    int maxL = 1;
    for (int b = 0; b < batch; ++b) if (context_lens[b] > maxL) maxL = context_lens[b];
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#pragma omp parallel
#endif
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)maxL);
        double* w = (double*)malloc(sizeof(double) * (size_t)maxL);
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t i = 0; i < total; ++i) {
            int64_t t = rows ? rows[2 * i] : i / num_q_heads;
            int h = rows ? rows[2 * i + 1] : (int)(i % num_q_heads);
            int b = 0;
            while (b + 1 < batch && q_starts[b + 1] <= t) ++b;      /* the sequence that owns packed token t */
            int q_len = q_starts[b + 1] - q_starts[b];
            int pos = context_lens[b] - q_len + (int)(t - q_starts[b]);
            decode_row(out + i * head_dim, q + (t * num_q_heads + h) * head_dim, &pv,
                       block_table + (int64_t)b * max_blocks_per_seq, pos < 0 ? 0 : pos + 1, h / G,
                       (double)scale, s, w);
        }
        free(s);
        free(w);
    }
    return used;
}

/*
 * Writing the K/V rows of recomputed (or prefilled) tokens into the pool: the step before
 * kvo_prefill_attn, with the same conventions.  k_new, v_new: [total_q][num_kv_heads][head_dim]
 * 16-bit elements, sequences packed in batch order; token i of sequence b (packed row
 * q_starts[b] + i) goes to position context_lens[b] - q_len_b + i of that sequence, and the block
 * that holds it is marked dirty.  Rows whose position would be negative are skipped.
 */
int kvo_append_packed(uint16_t* pool, int64_t num_blocks, int num_kv_heads, int block_size, int head_dim,
                      const uint16_t* k_new, const uint16_t* v_new, const int32_t* block_table,
                      int max_blocks_per_seq, const int32_t* context_lens, const int32_t* q_starts, int batch,
                      uint32_t* dirty_bitmap)
{
    int rc = check_decode_args(num_blocks, num_kv_heads, block_size, head_dim, block_table,
                               max_blocks_per_seq, context_lens, batch, num_kv_heads);
    if (rc) return rc;
    if (q_starts[0] != 0) return -2;
    for (int b = 0; b < batch; ++b) if (q_starts[b + 1] < q_starts[b]) return -2;
    for (int b = 0; b < batch; ++b) {
        int n = q_starts[b + 1] - q_starts[b];
        for (int i = 0; i < n; ++i) {
            int t = context_lens[b] - n + i;
            if (t < 0) continue;
            int64_t row = (int64_t)q_starts[b] + i;
            int64_t p = block_table[(int64_t)b * max_blocks_per_seq + t / block_size];
            int r = t % block_size;
            for (int kvh = 0; kvh < num_kv_heads; ++kvh)
                for (int which = 0; which < 2; ++which) {
                    const uint16_t* src = (which ? v_new : k_new) + (row * num_kv_heads + kvh) * head_dim;
                    uint16_t* dst = pool + ((((p * 2 + which) * num_kv_heads + kvh) * block_size + r) * (int64_t)head_dim);
                    for (int d = 0; d < head_dim; ++d) dst[d] = src[d];
                }
            dirty_bitmap[p / 32] |= (uint32_t)1 << (p % 32);
        }
    }
    return 0;
}
