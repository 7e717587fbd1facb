"""GPU parity: the HIP path, called through the C ABI binding, against the CPU fp64 oracle.

Pack/restore must be bit-exact.  Decode must be within max-abs 2e-2 and mean-abs 2e-3 of the
oracle (bf16 inputs, fp32 accumulation); where the mathematics fixes the result exactly
(single-token contexts, permuted physical blocks) the comparison is bit-exact.
"""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle, bf16_tensor, bits_of  # noqa: E402


def oracle_decode(oracle, case, pool=None, table=None, rows=None):
    return oracle.decode_attn(case.q, case.pool if pool is None else pool,
                              case.block_table if table is None else table,
                              case.context_lens, case.geom.scale, rows=rows)


def make(seed, Hq, Hkv, D, bs, lens, NB=None, MB=None, dirty="last", n_dirty=None):
    g = W.Geometry(Hq, Hkv, D, bs)
    return W.make_decode_case("t", seed, g, np.asarray(lens, np.int32), num_blocks=NB,
                              max_blocks_per_seq=MB, dirty=dirty, n_dirty=n_dirty)


# ------------------------------------------------------------------ pack / restore, bit-exact
@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 32), (6, 3, 64, 32)])
def test_pack_matches_oracle_bitwise(oracle, geom):
    Hq, Hkv, D, bs = geom
    case = make(101, Hq, Hkv, D, bs, [40, 100, 7], NB=96, dirty="any", n_dirty=37)
    ids = np.concatenate([case.dirty_ids, case.dirty_ids[:5]]).astype(np.int32)       # repeats are legal
    want = oracle.pack_blocks(case.pool, ids)
    pool = bf16_tensor(case.pool)
    replica = torch.zeros((len(ids),) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, pool, torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(replica), want)
    assert np.array_equal(bits_of(pool), case.pool)                                  # source untouched


@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 32)])
def test_restore_matches_oracle_bitwise_and_leaves_other_blocks(oracle, geom):
    Hq, Hkv, D, bs = geom
    case = make(103, Hq, Hkv, D, bs, [40, 100, 7], NB=80, dirty="any", n_dirty=33)
    ids = case.dirty_ids
    replica_bits = W.normal_bf16(np.random.SeedSequence(5), (len(ids),) + case.pool.shape[1:])
    want = case.pool.copy()
    oracle.restore_blocks(want, replica_bits, ids)
    pool = bf16_tensor(case.pool)
    kvflow.kv_restore_blocks(pool, bf16_tensor(replica_bits), torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(pool), want)


def test_pack_restore_empty_list_and_prefix(oracle):
    case = make(105, 8, 2, 64, 16, [33], NB=20, dirty="any", n_dirty=9)
    pool = bf16_tensor(case.pool)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.zeros((9,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, pool, ids, n=0)
    kvflow.kv_pack_blocks(replica, pool, ids, n=4)                                   # only the first 4
    torch.cuda.synchronize()
    got = bits_of(replica)
    assert np.array_equal(got[:4], case.pool[case.dirty_ids[:4]]) and not got[4:].any()


@pytest.mark.parametrize("n", [1, 7, 8, 9, 63, 1000])
def test_pack_restore_list_lengths_around_the_xcd_split(oracle, n):
    """The list is dealt to the eight XCDs in contiguous parts: lengths below, at and above eight entries."""
    case = make(107, 8, 2, 64, 16, [16 * 1000], NB=1200, dirty="any", n_dirty=1000)
    pool = bf16_tensor(case.pool)
    ids_h = case.dirty_ids[:n].copy()
    ids = torch.from_numpy(ids_h).cuda()
    replica = torch.zeros((n + 1,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, pool, ids)
    torch.cuda.synchronize()
    got = bits_of(replica)
    assert np.array_equal(got[:n], oracle.pack_blocks(case.pool, ids_h)) and not got[n:].any()
    target = torch.zeros_like(pool)
    kvflow.kv_restore_blocks(target, replica, ids)
    torch.cuda.synchronize()
    want = np.zeros_like(case.pool)
    oracle.restore_blocks(want, got[:n], ids_h)
    assert np.array_equal(bits_of(target), want)


def test_pack_list_longer_than_one_launch(oracle):
    """More list entries than one launch covers (2^21 workgroups): the second launch continues the list and
    the replica where the first one stopped.  Blocks of 2 KiB (FP8, one KV head, head_dim 64), ids with repeats."""
    g = W.Geometry(1, 1, 64, 16, kv_elt_bytes=1)
    case = W.make_decode_case("t", 109, g, np.array([16 * 500], np.int32), num_blocks=512, dirty="any", n_dirty=8)
    assert g.block_bytes == 2048
    n = (1 << 21) + 1000
    ids_h = np.random.default_rng(5).integers(0, case.num_blocks, size=n, dtype=np.int32)
    pool = kvflow.Fp8Pool(torch.from_numpy(case.pool).cuda(), 1.0, 1.0)
    replica = torch.zeros((n + 1,) + case.pool.shape[1:], dtype=torch.uint8, device="cuda")
    kvflow.kv_pack_blocks(replica, pool, torch.from_numpy(ids_h).cuda())
    torch.cuda.synchronize()
    got = replica.cpu().numpy()
    assert np.array_equal(got[:n], oracle.pack_blocks(case.pool, ids_h)) and not got[n:].any()


def test_tiny_config_pack_restore_round_trip(oracle):
    case = W.tiny()
    pool = bf16_tensor(case.pool)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.empty((len(case.dirty_ids),) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, pool, ids)
    assert np.array_equal(bits_of(replica), oracle.pack_blocks(case.pool, case.dirty_ids))
    fresh_ids = np.random.default_rng(0).permutation(case.num_blocks)[:len(case.dirty_ids)].astype(np.int32)
    target = torch.full_like(pool, float("nan"))
    want = bits_of(target)
    kvflow.kv_restore_blocks(target, replica, torch.from_numpy(fresh_ids).cuda())
    torch.cuda.synchronize()
    oracle.restore_blocks(want, oracle.pack_blocks(case.pool, case.dirty_ids), fresh_ids)
    assert np.array_equal(bits_of(target), want)


# ------------------------------------------------------------------ decode vs oracle, small shapes
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_tiny_config_decode(oracle, out_dtype):
    case = W.tiny()
    dc = DeviceCase(case)
    assert_close_to_oracle(dc.decode(out_dtype), oracle_decode(oracle, case), "tiny")


GEOMS = [(8, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 32), (4, 4, 128, 16), (16, 1, 64, 32),
         (6, 3, 64, 16), (2, 1, 128, 32)]
RAGGED = [1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 127, 128, 129, 200, 257, 300]


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("wgs", [0, 1, 3, 64])
def test_decode_ragged_lengths_and_grid_sizes(oracle, geom, wgs):
    Hq, Hkv, D, bs = geom
    case = make(107, Hq, Hkv, D, bs, RAGGED, MB=-(-300 // bs))
    want = oracle_decode(oracle, case)
    dc = DeviceCase(case)
    for dt in (torch.float32, torch.bfloat16):
        assert_close_to_oracle(dc.decode(dt, workgroups=wgs), want, f"{geom} workgroups={wgs} {dt}")


def test_decode_zero_length_sequences(oracle):
    case = make(109, 8, 2, 64, 16, [0, 50, 0, 17], MB=8)
    want = oracle_decode(oracle, case)
    dc = DeviceCase(case)
    for wgs in (0, 2):
        got = dc.decode(torch.float32, workgroups=wgs)
        assert_close_to_oracle(got, want, f"zero-length workgroups={wgs}")
        assert torch.count_nonzero(got[0]) == 0 and torch.count_nonzero(got[2]) == 0


def test_decode_single_token_returns_v_exactly(oracle):
    case = make(111, 32, 8, 128, 16, [1] * 6, MB=4)
    want = oracle_decode(oracle, case)                       # equals V exactly (pinned on the CPU)
    dc = DeviceCase(case)
    for dt in (torch.float32, torch.bfloat16):
        got = dc.decode(dt).to(torch.float64).cpu().numpy()
        assert np.array_equal(got, want)


def test_decode_equal_scores_give_mean_of_v(oracle):
    case = make(113, 8, 2, 64, 16, [33, 64, 100], MB=8)
    case.q[:] = 0
    want = oracle_decode(oracle, case)
    got = DeviceCase(case).decode(torch.float32).to(torch.float64).cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-3)    # only bf16 rounding of the weights is left


def test_decode_ignores_poisoned_tail_slots_unused_blocks_and_table_entries(oracle):
    case = make(115, 32, 8, 128, 16, [5, 37, 81, 130], MB=12)
    g = case.geom
    want = oracle_decode(oracle, case)
    pool = np.full_like(case.pool, 0x7FC0)
    for b, L in enumerate(case.context_lens):
        for jb in range(-(-int(L) // g.block_size)):
            valid = min(g.block_size, int(L) - jb * g.block_size)
            pid = case.block_table[b, jb]
            pool[pid, :, :, :valid] = case.pool[pid, :, :, :valid]
    dc = DeviceCase(case, pool_bits=pool)
    for wgs in (0, 5):
        got = dc.decode(torch.float32, workgroups=wgs)
        assert_close_to_oracle(got, want, "poisoned")
    # a looser host bound on the context length must not change anything either
    got2 = dc.decode(torch.float32, max_len=12 * 16)
    assert_close_to_oracle(got2, want, "poisoned, loose bound")


def test_decode_bitwise_invariant_under_block_permutation(oracle):
    case = make(117, 32, 8, 128, 16, [100, 513, 700], MB=64)
    dc = DeviceCase(case)
    perm = np.random.default_rng(3).permutation(case.num_blocks)
    pool2 = np.empty_like(case.pool)
    pool2[perm] = case.pool
    table2 = np.where(case.block_table >= 0, perm[np.maximum(case.block_table, 0)], -1).astype(np.int32)
    for wgs in (0, 7):
        a = dc.decode(torch.float32, workgroups=wgs)
        b = dc.decode(torch.float32, workgroups=wgs, pool=bf16_tensor(pool2),
                      block_table=torch.from_numpy(table2).cuda())
        assert torch.equal(a, b)


def test_recovery_round_trip_on_gpu(oracle):
    """pack on the 'failed' pool, restore into a NaN-filled target under fresh ids, decode there."""
    case = make(119, 64, 8, 128, 16, [300, 1000, 77, 512], MB=64)
    dc = DeviceCase(case)
    before = dc.decode(torch.bfloat16)
    ids = case.in_use_ids
    replica = torch.empty((len(ids),) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, dc.pool, torch.from_numpy(ids).cuda())
    new_ids = np.random.default_rng(4).permutation(case.num_blocks)[:len(ids)].astype(np.int32)
    target = torch.full_like(dc.pool, float("nan"))
    kvflow.kv_restore_blocks(target, replica, torch.from_numpy(new_ids).cuda())
    remap = np.full(case.num_blocks, -1, np.int32)
    remap[ids] = new_ids
    table2 = np.where(case.block_table >= 0, remap[np.maximum(case.block_table, 0)], -1).astype(np.int32)
    dc.pool.fill_(float("nan"))                               # the source node is gone
    after = dc.decode(torch.bfloat16, pool=target, block_table=torch.from_numpy(table2).cuda())
    assert torch.equal(before, after)
    assert_close_to_oracle(after, oracle_decode(oracle, case), "recovered")


def test_validate_helpers_catch_bad_device_contents():
    case = make(121, 8, 2, 64, 16, [40, 20], NB=16, MB=4)
    dc = DeviceCase(case)
    assert kvflow.kv_validate_decode(dc.pool, dc.block_table, dc.context_lens, dc.max_len) == 0
    bad = dc.block_table.clone()
    bad[0, 1] = 16
    assert kvflow.kv_validate_decode(dc.pool, bad, dc.context_lens, dc.max_len) == -7
    assert kvflow.kv_validate_decode(dc.pool, dc.block_table, dc.context_lens, 39) == -7
    ids = torch.tensor([1, 2, 2], dtype=torch.int32, device="cuda")
    assert kvflow.kv_validate_block_ids(dc.pool, ids, require_distinct=False) == 0
    assert kvflow.kv_validate_block_ids(dc.pool, ids, require_distinct=True) == -7


def test_binding_rejects_wrong_dtype_layout_and_shape():
    """Index arrays of torch's default int64, strided views and mismatched shapes are refused on the host
    (the kernels would read them as raw int32 / bf16 memory)."""
    case = W.tiny()
    dc = DeviceCase(case)
    g = case.geom
    out = torch.empty((case.batch, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim,
                                                      dc.max_len) // 4, dtype=torch.float32, device="cuda")

    def call(**kw):
        a = dict(out=out, q=dc.q, pool=dc.pool, block_table=dc.block_table, context_lens=dc.context_lens)
        a.update(kw)
        kvflow.kv_decode_attn(a["out"], a["q"], a["pool"], a["block_table"], a["context_lens"], dc.max_len,
                              dc.scale, 0, ws)

    call()                                                             # the well-formed call goes through
    for bad in (dict(block_table=dc.block_table.long()), dict(context_lens=dc.context_lens.long()),
                dict(q=dc.q.float()), dict(q=dc.q.transpose(0, 1)), dict(out=out[:, :, :32]),
                dict(q=dc.q[:, :, :32].contiguous()), dict(block_table=dc.block_table[:2]),
                dict(context_lens=dc.context_lens.cpu()), dict(out=out.to(torch.float16))):
        with pytest.raises(ValueError):
            call(**bad)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.empty((len(case.dirty_ids),) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, dc.pool, ids)
    with pytest.raises(ValueError):
        kvflow.kv_pack_blocks(replica, dc.pool, ids.long())
    with pytest.raises(ValueError):
        kvflow.kv_pack_blocks(replica[:4], dc.pool, ids)                 # replica too small for the list
    with pytest.raises(ValueError):
        kvflow.kv_restore_blocks(dc.pool, replica, ids[::2])             # strided id list
    torch.cuda.synchronize()


def test_decode_batch_larger_than_one_launch_slice(oracle):
    """More sequences than one launch scans (4096): the call slices the batch; tiny contexts."""
    rng = np.random.default_rng(11)
    lens = rng.integers(0, 40, size=4500).astype(np.int32)
    case = make(123, 4, 2, 64, 16, lens, MB=3)
    want = oracle_decode(oracle, case)
    dc = DeviceCase(case)
    for dt in (torch.float32, torch.bfloat16):
        assert_close_to_oracle(dc.decode(dt), want, f"sliced batch {dt}")


def test_decode_group_of_16_and_single_kv_head(oracle):
    case = make(125, 16, 1, 128, 32, [1, 31, 32, 33, 500, 1000], MB=32)
    want = oracle_decode(oracle, case)
    dc = DeviceCase(case)
    for wgs in (0, 2, 9):
        assert_close_to_oracle(dc.decode(torch.float32, workgroups=wgs), want, f"G=16 workgroups={wgs}")


def test_decode_stays_inside_its_workspace_and_output(oracle):
    """Guard words after the workspace and around the output must survive the call."""
    case = make(127, 32, 8, 128, 16, [700, 33, 1500, 64], MB=100)
    g = case.geom
    dc = DeviceCase(case)
    nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len)
    guard = 4096
    ws = torch.full((nbytes // 4 + guard,), -123.0, dtype=torch.float32, device="cuda")
    n_out = case.batch * g.num_q_heads * g.head_dim
    out = torch.full((n_out + 2 * guard,), -77.0, dtype=torch.float32, device="cuda")
    view = out[guard:guard + n_out].view(case.batch, g.num_q_heads, g.head_dim)
    kvflow.kv_decode_attn(view, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0,
                          ws[:nbytes // 4])
    torch.cuda.synchronize()
    assert torch.all(ws[nbytes // 4:] == -123.0)
    assert torch.all(out[:guard] == -77.0) and torch.all(out[guard + n_out:] == -77.0)
    assert_close_to_oracle(view, oracle_decode(oracle, case), "guarded")
    # one byte less of workspace is refused
    with pytest.raises(kvflow.KvflowError) as err:
        kvflow.kv_decode_attn(view, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0,
                              ws[:nbytes // 4 - 1])
    assert err.value.status == -5


def test_decode_large_scores_and_rising_maximum(oracle):
    """Scores that keep growing along the context force repeated updates of the running maximum."""
    case = make(129, 8, 2, 64, 16, [300, 77], MB=20)
    g = case.geom
    kf = W.bf16_bits_to_f32(case.pool[:, 0]).copy()
    for b, L in enumerate(case.context_lens):
        for t in range(int(L)):
            pid = case.block_table[b, t // g.block_size]
            kf[pid, :, t % g.block_size, :] *= 0.2 + 0.05 * t          # later keys are much larger
    case.pool[:, 0] = W.f32_to_bf16_bits(kf)
    want = oracle_decode(oracle, case)
    dc = DeviceCase(case)
    for wgs in (0, 1):
        assert_close_to_oracle(dc.decode(torch.float32, workgroups=wgs), want, f"rising max workgroups={wgs}")


@pytest.mark.parametrize("design", [0, 3])
def test_streaming_probes_copy_exactly_and_leave_the_sink_alone(design):
    n = (1 << 22) + 16 * 37                                         # not a multiple of the kernels' stride
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
    kvflow.kv_probe_stream(design + 2, dst, src, n)
    sink = torch.full((16,), 7, dtype=torch.uint8, device="cuda")
    kvflow.kv_probe_stream(design, sink, src, n)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and torch.all(dst[n:] == 0)
    assert torch.all(sink == 7)
    kvflow.kv_probe_stream(design + 1, dst, None, n)                # contents unspecified, bounds are not
    torch.cuda.synchronize()
    assert torch.all(dst[n:] == 0)
    # a buffer shorter than one XCD's share, and one of a single vector
    for m in (16, 16 * 5, 16 * 1024 * 3 + 16):
        small = torch.zeros(m + 32, dtype=torch.uint8, device="cuda")
        kvflow.kv_probe_stream(design + 2, small, src, m)
        torch.cuda.synchronize()
        assert torch.equal(small[:m], src[:m]) and torch.all(small[m:] == 0)


def test_matrix_probe_runs_every_mode_and_leaves_zeros_for_zero_operands():
    """The matrix-core yardstick: every mode returns, writes only its sink, and with all-zero operands (mode 0)
    every accumulator, hence every sink entry, is zero."""
    n = kvflow.KV_PROBE_MATRIX_SINK_BYTES // 4
    buf = torch.full((n + 64,), 7.0, dtype=torch.float32, device="cuda")
    for mode in range(6):
        kvflow.kv_probe_matrix(mode, 50, buf[:n])
        torch.cuda.synchronize()
        assert torch.isfinite(buf).all(), f"mode {mode}"
        assert (buf[n:] == 7.0).all(), f"mode {mode}: wrote past the sink"
        if mode == 0:
            assert (buf[:n] == 0).all()
    with pytest.raises(kvflow.KvflowError):
        kvflow.kv_probe_matrix(1, 10, buf[: n - 4])

