"""Pins of the prefill (recomputation) oracle against things other than itself (no GPU).

The paper states only that dropped replicas are recomputed (Sec. 3.2 item 3); what is recomputed is
ordinary causal attention over the tokens of a sequence.  The oracle is therefore held by a library
routine (torch SDPA in fp64, with its own causal mask), an independently written dense numpy
attention, closed forms and invariants, each chosen so that one plausible mistake (mask off by one,
queries aligned to the start instead of the end of the context, wrong packed-row offset, wrong head
mapping) fails it.
"""
import numpy as np
import pytest

from paper_2601_22438_amd import workloads as W
from test_oracle_pins import gather_contiguous


def small_prefill(seed=21, Hq=8, Hkv=2, D=64, bs=16, lens=(40, 70, 5, 33), q_lens=(40, 17, 1, 0), NB=48):
    g = W.Geometry(Hq, Hkv, D, bs)
    return W.make_prefill_case("small_prefill", seed, g, np.array(lens, np.int32), np.array(q_lens, np.int32),
                               num_blocks=NB, max_blocks_per_seq=8, dirty="any", n_dirty=4)


def run(oracle, case, **kw):
    kv = case.kv
    return oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts,
                               case.geom.scale, **kw)


def dense_causal(case):
    """Independent numpy version on contiguous K/V: explicit position mask, softmax over the last axis."""
    g = case.geom
    scale = float(np.float32(g.scale))
    q = W.bf16_bits_to_f32(case.q).astype(np.float64)
    ks, vs = gather_contiguous(case.kv)
    out = np.zeros(q.shape)
    for b in range(case.batch):
        n, L = int(case.q_lens[b]), int(case.kv.context_lens[b])
        if n == 0:
            continue
        qb = q[case.q_starts[b]:case.q_starts[b + 1]]                # [n][Hq][D]
        k = np.repeat(ks[b], g.group, axis=1)                        # [L][Hq][D]
        v = np.repeat(vs[b], g.group, axis=1)
        s = np.einsum("nhd,lhd->hnl", qb, k) * scale
        q_pos = L - n + np.arange(n)
        visible = np.arange(L)[None, :] <= q_pos[:, None]            # [n][L]
        s = np.where(visible[None], s, -np.inf)
        p = np.exp(s - s.max(axis=2, keepdims=True))
        p /= p.sum(axis=2, keepdims=True)
        out[case.q_starts[b]:case.q_starts[b + 1]] = np.einsum("hnl,lhd->nhd", p, v)
    return out


@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (4, 4, 128, 16), (16, 2, 128, 32), (6, 3, 64, 16)])
def test_matches_dense_numpy_attention(oracle, geom):
    Hq, Hkv, D, bs = geom
    case = small_prefill(seed=22, Hq=Hq, Hkv=Hkv, D=D, bs=bs)
    np.testing.assert_allclose(run(oracle, case), dense_causal(case), rtol=0, atol=1e-12)


def test_prefill_tiny_matches_dense_numpy_attention(oracle):
    case = W.prefill_tiny()
    np.testing.assert_allclose(run(oracle, case), dense_causal(case), rtol=0, atol=1e-12)


def test_full_recompute_matches_torch_causal_sdpa(oracle):
    """q_len = context length: the library's own is_causal mask (top-left aligned = bottom-right here)."""
    import torch
    case = small_prefill(seed=23, lens=(40, 19, 64), q_lens=(40, 19, 64))
    g = case.geom
    got = run(oracle, case)
    ks, vs = gather_contiguous(case.kv)
    q = torch.from_numpy(W.bf16_bits_to_f32(case.q).astype(np.float64))
    for b in range(case.batch):
        qb = q[case.q_starts[b]:case.q_starts[b + 1]].permute(1, 0, 2)                    # [Hq][n][D]
        k = torch.from_numpy(ks[b]).permute(1, 0, 2).repeat_interleave(g.group, dim=0)    # [Hq][L][D]
        v = torch.from_numpy(vs[b]).permute(1, 0, 2).repeat_interleave(g.group, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(qb, k, v, is_causal=True,
                                                               scale=float(np.float32(g.scale)))
        np.testing.assert_allclose(got[case.q_starts[b]:case.q_starts[b + 1]], ref.permute(1, 0, 2).numpy(),
                                   rtol=0, atol=1e-12)


def test_chunk_over_a_prefix_matches_the_tail_of_a_full_recompute(oracle):
    """The last n query rows of a full causal pass (library routine) are what a chunk of n queries gives."""
    import torch
    case = small_prefill(seed=24, lens=(50, 70), q_lens=(13, 33))
    g = case.geom
    got = run(oracle, case)
    ks, vs = gather_contiguous(case.kv)
    q = W.bf16_bits_to_f32(case.q).astype(np.float64)
    for b in range(case.batch):
        n, L = int(case.q_lens[b]), int(case.kv.context_lens[b])
        full_q = np.zeros((L, g.num_q_heads, g.head_dim))
        full_q[L - n:] = q[case.q_starts[b]:case.q_starts[b + 1]]
        k = torch.from_numpy(ks[b]).permute(1, 0, 2).repeat_interleave(g.group, dim=0)
        v = torch.from_numpy(vs[b]).permute(1, 0, 2).repeat_interleave(g.group, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(full_q).permute(1, 0, 2), k, v, is_causal=True, scale=float(np.float32(g.scale)))
        np.testing.assert_allclose(got[case.q_starts[b]:case.q_starts[b + 1]],
                                   ref.permute(1, 0, 2).numpy()[L - n:], rtol=0, atol=1e-12)


def test_single_query_is_decode(oracle):
    """One query token per sequence, at the end of its context: the decode operation, which has its own pins."""
    case = small_prefill(seed=25, lens=(40, 70, 5, 33), q_lens=(1, 1, 1, 1))
    kv = case.kv
    got = run(oracle, case)
    dec = oracle.decode_attn(case.q.reshape(case.batch, *case.q.shape[1:]), kv.pool, kv.block_table,
                             kv.context_lens, case.geom.scale)
    assert np.array_equal(got, dec)


def test_first_token_returns_its_own_value_row(oracle):
    """Position 0 sees one key: the output is V[0] exactly, whatever q and K are."""
    case = small_prefill(seed=26, lens=(20, 33), q_lens=(20, 33))
    g = case.geom
    got = run(oracle, case)
    v = W.bf16_bits_to_f32(case.kv.pool).astype(np.float64)
    for b in range(case.batch):
        p = case.kv.block_table[b, 0]
        for h in range(g.num_q_heads):
            assert np.array_equal(got[case.q_starts[b], h], v[p, 1, h // g.group, 0])


def test_zero_queries_give_running_means_of_v(oracle):
    """All scores equal: query at position p returns the mean of V[0..p]."""
    case = small_prefill(seed=27, lens=(37, 50), q_lens=(37, 21))
    case.q[:] = 0
    got = run(oracle, case)
    _, vs = gather_contiguous(case.kv)
    for b in range(case.batch):
        n, L = int(case.q_lens[b]), int(case.kv.context_lens[b])
        run_mean = np.cumsum(vs[b], axis=0) / np.arange(1, L + 1)[:, None, None]          # [L][Hkv][D]
        want = np.repeat(run_mean[L - n:], case.geom.group, axis=1)
        np.testing.assert_allclose(got[case.q_starts[b]:case.q_starts[b + 1]], want, rtol=1e-13, atol=1e-14)


def test_later_tokens_do_not_influence_earlier_queries(oracle):
    """Changing K/V at position p changes exactly the queries at positions >= p."""
    case = small_prefill(seed=28, lens=(48,), q_lens=(48,), NB=8)
    g = case.geom
    before = run(oracle, case)
    p = 29
    blk, row = case.kv.block_table[0, p // g.block_size], p % g.block_size
    case.kv.pool[blk, :, :, row, :] ^= 0x0040                        # flip a mantissa bit of K and V rows
    after = run(oracle, case)
    assert np.array_equal(before[:p], after[:p])
    assert (np.abs(before[p:] - after[p:]).max(axis=(1, 2)) > 0).all()


def test_queries_are_aligned_to_the_end_of_the_context(oracle):
    """Two sequences share one pool prefix; the longer chunk's last rows equal the shorter chunk's rows."""
    a = small_prefill(seed=29, lens=(60,), q_lens=(25,), NB=8)
    b = small_prefill(seed=29, lens=(60,), q_lens=(9,), NB=8)
    b.q[:] = a.q[25 - 9:]
    ga, gb = run(oracle, a), run(oracle, b)
    assert np.array_equal(ga[25 - 9:], gb)


def test_packed_rows_follow_q_starts(oracle):
    """Batched call = the sequences run one at a time and concatenated."""
    case = small_prefill(seed=30)
    kv = case.kv
    got = run(oracle, case)
    for b in range(case.batch):
        lo, hi = int(case.q_starts[b]), int(case.q_starts[b + 1])
        one = oracle.prefill_attn(case.q[lo:hi], kv.pool, kv.block_table[b:b + 1], kv.context_lens[b:b + 1],
                                  np.array([0, hi - lo], np.int32), case.geom.scale)
        assert np.array_equal(got[lo:hi], one)


def test_rows_subset_matches_full(oracle):
    case = small_prefill(seed=31)
    full = run(oracle, case)
    rows = np.array([[0, 0], [39, 7], [40, 3], [56, 1], [57, 6]], np.int32)
    sub = run(oracle, case, rows=rows)
    for i, (t, h) in enumerate(rows):
        assert np.array_equal(sub[i], full[t, h])


def test_more_queries_than_context_gives_zero_rows_for_the_excess(oracle):
    case = small_prefill(seed=32, lens=(10,), q_lens=(10,), NB=4)
    kv = case.kv
    q = np.concatenate([case.q[:3], case.q])                         # 13 queries over 10 cached tokens
    got = oracle.prefill_attn(q, kv.pool, kv.block_table, kv.context_lens, np.array([0, 13], np.int32),
                              case.geom.scale)
    assert np.array_equal(got[:3], np.zeros_like(got[:3]))
    assert np.array_equal(got[3:], run(oracle, case))


def test_fp8_pool_equals_bf16_pool_holding_the_decoded_values(oracle):
    """E4M3 values times a power-of-two scale are bf16 numbers: both pools must give identical rows."""
    g = W.Geometry(8, 2, 64, 16, kv_elt_bytes=1)
    case = W.make_prefill_case("fp8", 33, g, np.array([40, 70], np.int32), np.array([40, 17], np.int32),
                               num_blocks=16, max_blocks_per_seq=8, dirty="last")
    kv = case.kv
    assert kv.pool.dtype == np.uint8
    ks, vs = 0.25, 0.5
    dec = W.fp8_e4m3_bits_to_f32(kv.pool)
    dec[:, 0] *= np.float32(ks)
    dec[:, 1] *= np.float32(vs)
    as_bf16 = W.f32_to_bf16_bits(dec)
    assert np.array_equal(W.bf16_bits_to_f32(as_bf16), dec)          # exactly representable
    a = oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, g.scale,
                            k_scale=ks, v_scale=vs)
    b = oracle.prefill_attn(case.q, as_bf16, kv.block_table, kv.context_lens, case.q_starts, g.scale)
    np.testing.assert_allclose(a, b, rtol=1e-15, atol=0)


def new_rows(case, seed):
    g = case.geom
    ss = np.random.SeedSequence(seed).spawn(2)
    shape = (case.total_q, g.num_kv_heads, g.head_dim)
    return W.normal_bf16(ss[0], shape), W.normal_bf16(ss[1], shape)


def test_append_packed_matches_numpy_indexing_and_touches_nothing_else(oracle):
    case = small_prefill(seed=34, lens=(40, 70, 5, 33), q_lens=(40, 17, 1, 0))
    g, kv = case.geom, case.kv
    k_new, v_new = new_rows(case, 35)
    pool = kv.pool.copy()
    bitmap = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    oracle.append_packed(pool, k_new, v_new, kv.block_table, kv.context_lens, case.q_starts, bitmap)
    expect = kv.pool.copy()
    dirty = set()
    for b in range(case.batch):
        n, L = int(case.q_lens[b]), int(kv.context_lens[b])
        for i in range(n):
            t = L - n + i
            pid, r = kv.block_table[b, t // g.block_size], t % g.block_size
            expect[pid, 0, :, r, :] = k_new[case.q_starts[b] + i]
            expect[pid, 1, :, r, :] = v_new[case.q_starts[b] + i]
            dirty.add(int(pid))
    assert np.array_equal(pool, expect)
    bits = np.unpackbits(bitmap.view(np.uint8), bitorder="little")[:kv.num_blocks]
    assert set(np.flatnonzero(bits).tolist()) == dirty


def test_append_packed_equals_token_by_token_append(oracle):
    """The packed call is the single-token append applied once per query position."""
    case = small_prefill(seed=36, lens=(23, 50), q_lens=(9, 17))
    kv = case.kv
    k_new, v_new = new_rows(case, 37)
    a, b_ = kv.pool.copy(), kv.pool.copy()
    bm_a = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    bm_b = bm_a.copy()
    oracle.append_packed(a, k_new, v_new, kv.block_table, kv.context_lens, case.q_starts, bm_a)
    for i in range(int(case.q_lens.max())):
        positions = np.where(i < case.q_lens, kv.context_lens - case.q_lens + i, -1).astype(np.int32)
        rows = np.minimum(case.q_starts[:-1] + i, case.total_q - 1)
        oracle.append_tokens(b_, k_new[rows], v_new[rows], kv.block_table, positions, bm_b)
    assert np.array_equal(a, b_) and np.array_equal(bm_a, bm_b)


def test_append_packed_then_prefill_equals_dense_attention_over_the_new_rows(oracle):
    case = small_prefill(seed=38, lens=(40, 70), q_lens=(40, 17))
    kv = case.kv
    k_new, v_new = new_rows(case, 39)
    bitmap = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    oracle.append_packed(kv.pool, k_new, v_new, kv.block_table, kv.context_lens, case.q_starts, bitmap)
    ks, vs = gather_contiguous(kv)
    for b in range(case.batch):                                       # the tail of each sequence is the new rows
        n = int(case.q_lens[b])
        lo, hi = int(case.q_starts[b]), int(case.q_starts[b + 1])
        assert np.array_equal(ks[b][-n:], W.bf16_bits_to_f32(k_new[lo:hi]).astype(np.float64))
        assert np.array_equal(vs[b][-n:], W.bf16_bits_to_f32(v_new[lo:hi]).astype(np.float64))
    np.testing.assert_allclose(run(oracle, case), dense_causal(case), rtol=0, atol=1e-12)


def test_append_packed_skips_rows_before_position_zero_and_rejects_bad_input(oracle):
    case = small_prefill(seed=40, lens=(10,), q_lens=(10,), NB=4)
    kv = case.kv
    k_new, v_new = new_rows(case, 41)
    k13, v13 = np.concatenate([k_new[:3], k_new]), np.concatenate([v_new[:3], v_new])
    a, b_ = kv.pool.copy(), kv.pool.copy()
    bm = np.zeros(oracle.bitmap_words(kv.num_blocks), np.uint32)
    oracle.append_packed(a, k13, v13, kv.block_table, kv.context_lens, np.array([0, 13], np.int32), bm)
    oracle.append_packed(b_, k_new, v_new, kv.block_table, kv.context_lens, case.q_starts, bm.copy())
    assert np.array_equal(a, b_)
    bad = kv.block_table.copy()
    bad[0, 0] = kv.num_blocks
    with pytest.raises(oracle.OracleError):
        oracle.append_packed(a, k_new, v_new, bad, kv.context_lens, case.q_starts, bm)
    with pytest.raises(oracle.OracleError):
        oracle.append_packed(a, k_new, v_new, kv.block_table, kv.context_lens, np.array([1, 10], np.int32), bm)
