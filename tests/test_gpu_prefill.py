"""GPU parity of kv_prefill_attn (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import gpu_util as U
from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu


class DevicePrefill:
    def __init__(self, case: W.PrefillCase, pool=None, k_scale=1.0, v_scale=1.0):
        self.case = case
        kv = case.kv
        if pool is None and kv.pool.dtype == np.uint8:
            pool = U.pool_tensor(kv.pool, k_scale, v_scale)
        self.q = U.bf16_tensor(case.q) if case.total_q else torch.empty((0,) + case.q.shape[1:],
                                                                        dtype=torch.bfloat16, device="cuda")
        self.pool = U.bf16_tensor(kv.pool) if pool is None else pool
        self.block_table = torch.from_numpy(kv.block_table).cuda()
        self.context_lens = torch.from_numpy(kv.context_lens).cuda()
        self.q_starts = torch.from_numpy(case.q_starts).cuda()

    def run(self, out_dtype=torch.float32, canary_rows=3, max_q_len=None, block_table=None, pool=None,
            key_splits=1):
        c, g = self.case, self.case.geom
        # rows after the last packed query token must stay untouched
        out = torch.full((c.total_q + canary_rows, g.num_q_heads, g.head_dim), float("nan"),
                         dtype=out_dtype, device="cuda")
        ws = None
        if key_splits > 1:                                  # workspace contents on entry must not matter
            nbytes = kvflow.kv_prefill_workspace_bytes(c.total_q, g.num_q_heads, g.head_dim, key_splits)
            ws = torch.full((max(nbytes, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda")
        kvflow.kv_prefill_attn(out[:c.total_q], self.q, self.pool if pool is None else pool,
                               self.block_table if block_table is None else block_table, self.context_lens,
                               self.q_starts, c.max_q_len if max_q_len is None else max_q_len, float(g.scale),
                               key_splits, ws)
        torch.cuda.synchronize()
        assert torch.isnan(out[c.total_q:].float()).all(), "wrote past the last query row"
        return out[:c.total_q]


def oracle_out(oracle, case, rows=None):
    kv = case.kv
    return oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, case.geom.scale,
                               rows=rows)


def test_prefill_tiny_matches_oracle(oracle):
    case = W.prefill_tiny()
    want = oracle_out(oracle, case)
    dev = DevicePrefill(case)
    U.assert_close_to_oracle(dev.run(torch.float32), want, "fp32 out")
    # bf16 output: the fp32 result rounded once more (half an ulp of |x| < 4 is 2^-7), same gates
    U.assert_close_to_oracle(dev.run(torch.bfloat16), want, "bf16 out")


# (Hq, Hkv, D, bs): groups of 1, 2, 3, 4, 8 and 16 query heads per KV head, both head sizes and block sizes
@pytest.mark.parametrize("geom", [(4, 4, 128, 16), (4, 2, 64, 32), (6, 2, 64, 16), (8, 2, 128, 32),
                                  (16, 2, 128, 16), (16, 1, 64, 16)])
def test_geometries_and_ragged_lengths(oracle, geom):
    Hq, Hkv, D, bs = geom
    g = W.Geometry(Hq, Hkv, D, bs)
    lens = np.array([1, 31, 32, 33, 97, 300, 200, 129], np.int32)
    q_lens = np.array([1, 31, 5, 33, 64, 300, 65, 128], np.int32)
    case = W.make_prefill_case("geom", 40 + Hq, g, lens, q_lens, max_blocks_per_seq=-(-300 // bs), dirty="last")
    U.assert_close_to_oracle(DevicePrefill(case).run(), oracle_out(oracle, case), str(geom))


def test_first_token_returns_its_own_value_row_exactly(oracle):
    """Position 0 sees one key; numerator and denominator use the same rounded probability."""
    g = W.Geometry(8, 2, 64, 16)
    case = W.make_prefill_case("first", 50, g, np.array([40, 7], np.int32), np.array([40, 7], np.int32),
                               max_blocks_per_seq=4, dirty="last")
    got = DevicePrefill(case).run().cpu().numpy()
    v = W.bf16_bits_to_f32(case.kv.pool)
    for b in range(case.batch):
        blk = case.kv.block_table[b, 0]
        for h in range(g.num_q_heads):
            assert np.array_equal(got[case.q_starts[b], h], v[blk, 1, h // g.group, 0])


def test_single_query_per_sequence_is_the_decode_result(oracle):
    g = W.Geometry(32, 8, 128, 16)
    lens = np.array([700, 33, 1, 256], np.int32)
    case = W.make_prefill_case("as_decode", 51, g, lens, np.ones(4, np.int32), max_blocks_per_seq=64, dirty="last")
    got = DevicePrefill(case).run()
    want = oracle.decode_attn(case.q, case.kv.pool, case.kv.block_table, case.kv.context_lens, g.scale)
    U.assert_close_to_oracle(got, want, "q_len 1")


def test_sequences_without_queries_and_empty_batch(oracle):
    g = W.Geometry(8, 2, 64, 16)
    lens = np.array([40, 0, 77], np.int32)
    case = W.make_prefill_case("gaps", 52, g, lens, np.array([0, 0, 50], np.int32), max_blocks_per_seq=8,
                               dirty="last")
    U.assert_close_to_oracle(DevicePrefill(case).run(), oracle_out(oracle, case), "gaps")
    none = W.make_prefill_case("none", 53, g, lens, np.zeros(3, np.int32), max_blocks_per_seq=8, dirty="last")
    assert DevicePrefill(none).run().shape[0] == 0


def test_more_queries_than_cached_tokens_gives_zero_rows(oracle):
    """Outside the normal contract (q_len <= context length) the excess queries see no key."""
    g = W.Geometry(8, 2, 64, 16)
    case = W.make_prefill_case("excess", 54, g, np.array([70, 20], np.int32), np.array([70, 20], np.int32),
                               max_blocks_per_seq=8, dirty="last")
    kv = case.kv
    # sequence 1 now claims only 12 cached tokens for its 20 queries; sequence 0 none at all
    kv.context_lens[:] = [0, 12]
    want = oracle_out(oracle, case)
    assert np.array_equal(want[:70 + 8], np.zeros_like(want[:78]))
    U.assert_close_to_oracle(DevicePrefill(case).run(), want, "excess")


def test_result_depends_only_on_logical_positions(oracle):
    """Same blocks under other physical ids, garbage in every unreferenced slot: bitwise equal output."""
    case = W.prefill_tiny(seed=55)
    kv, g = case.kv, case.geom
    base = DevicePrefill(case).run()
    rng = np.random.default_rng(56)
    perm = rng.permutation(kv.num_blocks).astype(np.int32)
    pool2 = np.full_like(kv.pool, 0x7FC0)                             # NaN patterns everywhere
    pool2[perm] = kv.pool
    table2 = np.where(kv.block_table >= 0, perm[np.maximum(kv.block_table, 0)], -1).astype(np.int32)
    for b, L in enumerate(kv.context_lens):                            # slots past the end of the last block: NaN
        if L % g.block_size:
            pool2[table2[b, L // g.block_size], :, :, L % g.block_size:, :] = 0x7FC0
    used = np.zeros(kv.num_blocks, bool)
    for b, L in enumerate(kv.context_lens):
        used[table2[b, :-(-int(L) // g.block_size)]] = True
    pool2[~used] = 0x7FC0
    got = DevicePrefill(case, pool=U.bf16_tensor(pool2)).run(block_table=torch.from_numpy(table2).cuda())
    assert torch.equal(base, got)


def test_grid_bound_larger_than_needed_changes_nothing(oracle):
    case = W.prefill_tiny(seed=57)
    dev = DevicePrefill(case)
    assert torch.equal(dev.run(), dev.run(max_q_len=case.max_q_len + 1000))


def test_recompute_shrunk_matches_oracle_on_every_row(oracle):
    case = W.recompute(shrink=16)
    U.assert_close_to_oracle(DevicePrefill(case).run(), oracle_out(oracle, case), "recompute/16")


def sample_rows(case, n_rows, seed):
    """First and last query of every sequence for a few heads, plus uniformly drawn (token, head) pairs."""
    rng = np.random.default_rng(seed)
    Hq = case.geom.num_q_heads
    rows = []
    for b in range(case.batch):
        if case.q_lens[b]:
            rows += [(int(case.q_starts[b]), 0), (int(case.q_starts[b + 1]) - 1, Hq - 1)]
    t = rng.integers(0, case.total_q, n_rows)
    h = rng.integers(0, Hq, n_rows)
    rows += list(zip(t.tolist(), h.tolist()))
    return np.array(rows, np.int32)


# The oracle needs ~1e12 fp64 multiply-adds for every row of `recompute` and ~5e12 for
# `chunked_recompute` (minutes to tens of minutes on 16 host cores), so these two cases are checked
# on sampled rows: the first and last query of every sequence plus 2000 / 1000 uniformly drawn rows.
@pytest.mark.parametrize("maker,n_rows", [(W.recompute, 2000), (W.chunked_recompute, 1000)])
def test_full_size_cases_on_sampled_rows(oracle, maker, n_rows):
    case = maker()
    rows = sample_rows(case, n_rows, 58)
    want = oracle_out(oracle, case, rows=rows)
    got = DevicePrefill(case).run(torch.float32, canary_rows=1)
    pick = got[torch.from_numpy(rows[:, 0].astype(np.int64)).cuda(), torch.from_numpy(rows[:, 1].astype(np.int64)).cuda()]
    U.assert_close_to_oracle(pick, want, case.name)


# ---- FP8 (E4M3) pool: the oracle consumes the same bit patterns and scales
@pytest.mark.parametrize("geom", [(8, 2, 128, 16), (16, 2, 64, 32), (4, 4, 128, 32)])
@pytest.mark.parametrize("scales", [(0.25, 0.25), (0.5, 0.125)])
def test_fp8_pool_geometries_and_scales(oracle, geom, scales):
    Hq, Hkv, D, bs = geom
    ks, vs = scales
    g = W.Geometry(Hq, Hkv, D, bs, kv_elt_bytes=1)
    lens = np.array([1, 33, 97, 300, 200], np.int32)
    q_lens = np.array([1, 33, 64, 300, 65], np.int32)
    case = W.make_prefill_case("fp8geom", 60 + Hq, g, lens, q_lens, max_blocks_per_seq=-(-300 // bs), dirty="last")
    kv = case.kv
    want = oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, g.scale,
                               k_scale=ks, v_scale=vs)
    U.assert_close_to_oracle(DevicePrefill(case, k_scale=ks, v_scale=vs).run(), want, f"fp8 {geom} {scales}")


def test_fp8_first_token_returns_decoded_v_times_scale_exactly(oracle):
    g = W.Geometry(8, 2, 128, 16, kv_elt_bytes=1)
    case = W.make_prefill_case("fp8first", 61, g, np.array([20, 5], np.int32), np.array([20, 5], np.int32),
                               max_blocks_per_seq=2, dirty="last")
    kv = case.kv
    got = DevicePrefill(case, k_scale=0.25, v_scale=0.5).run().cpu().numpy()
    v = W.fp8_e4m3_bits_to_f32(kv.pool) * np.float32(0.5)
    for b in range(case.batch):
        blk = kv.block_table[b, 0]
        for h in range(g.num_q_heads):
            assert np.array_equal(got[case.q_starts[b], h], v[blk, 1, h // g.group, 0])


def test_fp8_recompute_shrunk_sampled_rows(oracle):
    base = W.recompute(shrink=4)
    g = W.Geometry(32, 8, 128, 16, kv_elt_bytes=1)
    case = W.make_prefill_case("fp8recompute", 62, g, base.kv.context_lens, base.q_lens, max_blocks_per_seq=128,
                               dirty="last")
    kv = case.kv
    rows = sample_rows(case, 300, 63)
    want = oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, g.scale, rows=rows,
                               k_scale=W.FP8_KV_SCALE, v_scale=W.FP8_KV_SCALE)
    got = DevicePrefill(case, k_scale=W.FP8_KV_SCALE, v_scale=W.FP8_KV_SCALE).run(canary_rows=1)
    pick = got[torch.from_numpy(rows[:, 0].astype(np.int64)).cuda(), torch.from_numpy(rows[:, 1].astype(np.int64)).cuda()]
    U.assert_close_to_oracle(pick, want, "fp8 recompute/4")


# ---- key range cut into parts (few query tokens over long contexts)
@pytest.mark.parametrize("key_splits", [2, 3, 16])
def test_key_splits_match_oracle_on_ragged_cases(oracle, key_splits):
    """More parts than tiles, parts that end on the diagonal, sequences without queries or without context."""
    case = W.prefill_tiny(seed=70)
    want = oracle_out(oracle, case)
    dev = DevicePrefill(case)
    U.assert_close_to_oracle(dev.run(key_splits=key_splits), want, f"tiny, {key_splits} parts")
    U.assert_close_to_oracle(dev.run(torch.bfloat16, key_splits=key_splits), want, f"tiny bf16, {key_splits} parts")


@pytest.mark.parametrize("geom", [(4, 4, 128, 16), (6, 2, 64, 16), (16, 2, 128, 32)])
def test_key_splits_geometries(oracle, geom):
    Hq, Hkv, D, bs = geom
    g = W.Geometry(Hq, Hkv, D, bs)
    lens = np.array([1, 33, 700, 300, 1000], np.int32)
    q_lens = np.array([1, 33, 40, 300, 7], np.int32)
    case = W.make_prefill_case("splitgeom", 71 + Hq, g, lens, q_lens, max_blocks_per_seq=-(-1000 // bs), dirty="last")
    U.assert_close_to_oracle(DevicePrefill(case).run(key_splits=5), oracle_out(oracle, case), str(geom))


def test_key_splits_excess_queries_and_empty_context(oracle):
    g = W.Geometry(8, 2, 64, 16)
    case = W.make_prefill_case("excess_split", 72, g, np.array([70, 20], np.int32), np.array([70, 20], np.int32),
                               max_blocks_per_seq=8, dirty="last")
    case.kv.context_lens[:] = [0, 12]
    U.assert_close_to_oracle(DevicePrefill(case).run(key_splits=4), oracle_out(oracle, case), "excess, 4 parts")


def test_key_splits_fp8_pool(oracle):
    g = W.Geometry(8, 2, 128, 16, kv_elt_bytes=1)
    case = W.make_prefill_case("fp8split", 73, g, np.array([900, 260], np.int32), np.array([33, 260], np.int32),
                               max_blocks_per_seq=64, dirty="last")
    kv = case.kv
    want = oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, g.scale,
                               k_scale=0.25, v_scale=0.5)
    U.assert_close_to_oracle(DevicePrefill(case, k_scale=0.25, v_scale=0.5).run(key_splits=6), want, "fp8, 6 parts")


def test_short_chunk_over_long_context_with_suggested_splits(oracle):
    """One sequence, 256 newest tokens over 40k cached ones: the library suggests cutting the key range."""
    g = W.Geometry(32, 8, 128, 16)
    lens = np.array([40_000], np.int32)
    case = W.make_prefill_case("short_chunk", 74, g, lens, np.array([256], np.int32), max_blocks_per_seq=2500,
                               dirty="last")
    ks = kvflow.kv_prefill_key_splits(1, 32, 8, 256, 40_000)
    assert ks == 16
    rows = sample_rows(case, 150, 75)
    want = oracle_out(oracle, case, rows=rows)
    dev = DevicePrefill(case)
    idx = (torch.from_numpy(rows[:, 0].astype(np.int64)).cuda(), torch.from_numpy(rows[:, 1].astype(np.int64)).cuda())
    U.assert_close_to_oracle(dev.run(key_splits=ks)[idx], want, "16 parts")
    U.assert_close_to_oracle(dev.run(key_splits=1)[idx], want, "1 part")


def test_validate_prefill_catches_bad_device_contents():
    case = W.prefill_tiny(seed=90)
    dev = DevicePrefill(case)
    args = lambda **kw: (kw.get("pool", dev.pool), kw.get("table", dev.block_table), kw.get("lens", dev.context_lens),
                         kw.get("starts", dev.q_starts), kw.get("max_q", case.max_q_len), kw.get("total", case.total_q))
    assert kvflow.kv_validate_prefill(*args()) == 0
    assert kvflow.kv_validate_prefill(*args(max_q=case.max_q_len - 1)) == -7
    assert kvflow.kv_validate_prefill(*args(total=case.total_q + 1)) == -7
    short = dev.context_lens.clone()
    short[0] = int(case.q_lens[0]) - 1                               # more queries than cached tokens
    assert kvflow.kv_validate_prefill(*args(lens=short)) == -7
    bad = dev.block_table.clone()
    bad[1, 0] = case.kv.num_blocks
    assert kvflow.kv_validate_prefill(*args(table=bad)) == -7
    dec = dev.q_starts.clone()
    dec[2] = dec[1] - 1
    assert kvflow.kv_validate_prefill(*args(starts=dec)) == -7


# ---- writing the recomputed tokens' K/V rows (the step before the attention call)
def packed_rows(case, seed, fp8=False):
    g = case.geom
    ss = np.random.SeedSequence(seed).spawn(2)
    shape = (case.total_q, g.num_kv_heads, g.head_dim)
    gen = (lambda s: W.normal_fp8(s, shape, W.FP8_KV_SCALE)) if fp8 else (lambda s: W.normal_bf16(s, shape))
    return gen(ss[0]), gen(ss[1])


@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (32, 8, 128, 16), (16, 2, 128, 32)])
def test_append_packed_is_bit_exact_and_marks_the_blocks(oracle, geom):
    Hq, Hkv, D, bs = geom
    g = W.Geometry(Hq, Hkv, D, bs)
    lens = np.array([1, 33, 97, 300, 200, 64], np.int32)
    q_lens = np.array([1, 33, 64, 300, 0, 17], np.int32)
    case = W.make_prefill_case("append_packed", 95 + Hq, g, lens, q_lens, max_blocks_per_seq=-(-300 // bs), dirty="last")
    kv = case.kv
    k_new, v_new = packed_rows(case, 96)
    want_pool = kv.pool.copy()
    want_bm = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    want_bm[0] = 0x5                                                  # bits that are already set must survive
    oracle.append_packed(want_pool, k_new, v_new, kv.block_table, kv.context_lens, case.q_starts, want_bm)
    dev = DevicePrefill(case)
    bm = torch.zeros(len(want_bm), dtype=torch.int32, device="cuda")
    bm[0] = 0x5
    kvflow.kv_append_packed(dev.pool, U.bf16_tensor(k_new), U.bf16_tensor(v_new), dev.block_table, dev.context_lens,
                            dev.q_starts, bm)
    torch.cuda.synchronize()
    assert np.array_equal(U.bits_of(dev.pool), want_pool)
    assert np.array_equal(bm.cpu().numpy().view(np.uint32), want_bm)


def test_append_packed_then_recompute_matches_the_oracle_flow(oracle):
    """FP8 pool: rows are moved as bytes; then the attention call reads what was just written (same stream)."""
    g = W.Geometry(8, 2, 128, 16, kv_elt_bytes=1)
    case = W.make_prefill_case("flow", 97, g, np.array([500, 130], np.int32), np.array([260, 130], np.int32),
                               max_blocks_per_seq=32, dirty="last")
    kv = case.kv
    k_new, v_new = packed_rows(case, 98, fp8=True)
    # the oracle's append moves 16-bit elements; an FP8 row is moved as head_dim/2 of them
    pool16 = kv.pool.view(np.uint16).copy()
    bm_want = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    oracle.append_packed(pool16, k_new.view(np.uint16), v_new.view(np.uint16), kv.block_table, kv.context_lens,
                         case.q_starts, bm_want)
    want_pool = pool16.view(np.uint8)
    want = oracle.prefill_attn(case.q, want_pool, kv.block_table, kv.context_lens, case.q_starts, g.scale,
                               k_scale=0.25, v_scale=0.25)
    dev = DevicePrefill(case, k_scale=0.25, v_scale=0.25)
    bm = torch.zeros(len(bm_want), dtype=torch.int32, device="cuda")
    kvflow.kv_append_packed(dev.pool, torch.from_numpy(k_new).cuda(), torch.from_numpy(v_new).cuda(), dev.block_table,
                            dev.context_lens, dev.q_starts, bm)
    got = dev.run()
    assert np.array_equal(dev.pool.data.cpu().numpy(), want_pool)
    assert np.array_equal(bm.cpu().numpy().view(np.uint32), bm_want)
    U.assert_close_to_oracle(got, want, "append + recompute, fp8")


@pytest.mark.parametrize("key_splits", [1, 4])
def test_large_scores_rising_and_falling_maximum(oracle, key_splits):
    """Keys that grow along the context force repeated raises of the running maximum; keys that shrink
    leave it far above the later scores.  Also a future key with a huge score that no query may see."""
    g = W.Geometry(8, 2, 64, 16)
    case = W.make_prefill_case("rising", 99, g, np.array([300, 150, 200], np.int32), np.array([300, 40, 200], np.int32),
                               max_blocks_per_seq=20, dirty="last")
    kv = case.kv
    kf = W.bf16_bits_to_f32(kv.pool[:, 0]).copy()
    for b, L in enumerate(kv.context_lens):
        for t in range(int(L)):
            pid = kv.block_table[b, t // g.block_size]
            gain = (0.2 + 0.05 * t) if b < 2 else (12.0 / (1.0 + 0.1 * t))
            kf[pid, :, t % g.block_size, :] *= gain
    kv.pool[:, 0] = W.f32_to_bf16_bits(kf)
    # the last key of sequence 1 is enormous: only the last query sees it, every other query must not feel it
    pid = kv.block_table[1, 149 // g.block_size]
    kv.pool[pid, 0, :, 149 % g.block_size, :] = W.f32_to_bf16_bits(
        W.bf16_bits_to_f32(kv.pool[pid, 0, :, 149 % g.block_size, :]) * np.float32(40.0))
    want = oracle_out(oracle, case)
    U.assert_close_to_oracle(DevicePrefill(case).run(key_splits=key_splits), want, f"rising/falling, {key_splits} parts")
