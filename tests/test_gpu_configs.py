"""GPU parity at the full sizes of the five serving-shaped cases, in the launch configuration the
bench times (library's choice of grid).  Every output element of every case is compared with the
fp64 oracle (its pass over the largest case takes about a second on the host); copies are compared
byte for byte, the 200 000-block restore chunk by chunk over all chunks."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle, bf16_tensor, bits_of  # noqa: E402


def oracle_all_rows(oracle, case, pool=None, table=None):
    """The oracle over every (sequence, query head) row of the case: fp64 [B][Hq][D]."""
    return oracle.decode_attn(case.q, case.pool if pool is None else pool,
                              case.block_table if table is None else table,
                              case.context_lens, case.geom.scale)


def pack_restore_check(oracle, case, dc):
    """pack the case's dirty list, compare with the oracle, restore into a second pool under fresh ids."""
    ids = case.dirty_ids
    replica = torch.empty((len(ids),) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    kvflow.kv_pack_blocks(replica, dc.pool, torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    want = oracle.pack_blocks(case.pool, ids)
    assert np.array_equal(bits_of(replica), want)
    fresh = np.random.default_rng(99).permutation(case.num_blocks)[:len(ids)].astype(np.int32)
    target_bits = W.normal_bf16(np.random.SeedSequence(77), case.pool.shape)
    target = bf16_tensor(target_bits)
    kvflow.kv_restore_blocks(target, replica, torch.from_numpy(fresh).cuda())
    torch.cuda.synchronize()
    oracle.restore_blocks(target_bits, want, fresh)
    assert np.array_equal(bits_of(target), target_bits)


def test_llama8b_layer_full(oracle):
    case = W.llama8b_layer()
    dc = DeviceCase(case)
    want = oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens, case.geom.scale)
    for dt in (torch.bfloat16, torch.float32):
        assert_close_to_oracle(dc.decode(dt), want, f"llama8b_layer {dt}")
    pack_restore_check(oracle, case, dc)


def test_long_context_every_row_and_pack(oracle):
    case = W.long_context()
    g = case.geom
    dc = DeviceCase(case)
    assert kvflow.kv_decode_workgroups(case.batch, g.num_kv_heads, case.max_context_len) == 256
    want = oracle_all_rows(oracle, case)
    for dt in (torch.bfloat16, torch.float32):
        assert_close_to_oracle(dc.decode(dt), want, f"long_context {dt}")
    assert len(case.dirty_ids) == round(0.10 * len(case.in_use_ids))
    pack_restore_check(oracle, case, dc)


def test_replication_mix_with_pack_on_side_stream(oracle):
    case = W.replication_mix()
    dc = DeviceCase(case)
    want = oracle_all_rows(oracle, case)
    alone = dc.decode(torch.bfloat16)
    assert_close_to_oracle(alone, want, "replication_mix alone")
    # pack of every sequence's newest block on a side stream while decode runs on the main stream
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.zeros((len(case.dirty_ids),) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    side, main = torch.cuda.Stream(), torch.cuda.current_stream()
    g = case.geom
    out = torch.empty_like(alone)
    nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(3):
        fork = torch.cuda.Event()
        fork.record(main)
        side.wait_event(fork)
        kvflow.kv_pack_blocks(replica, dc.pool, ids, stream=side)
        kvflow.kv_decode_attn(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0, ws)
        join = torch.cuda.Event()
        join.record(side)
        main.wait_event(join)
    torch.cuda.synchronize()
    assert torch.equal(out, alone)                              # overlap changes nothing, bit for bit
    assert np.array_equal(bits_of(replica), oracle.pack_blocks(case.pool, case.dirty_ids))
    assert_close_to_oracle(dc.decode(torch.float32), want, "replication_mix fp32")


def test_recovery_restore_200k_blocks_then_decode(oracle):
    rc = W.recovery()
    g, n = rc.geom, rc.num_blocks
    dec = rc.decode
    shape = (n, 2, g.num_kv_heads, g.block_size, g.head_dim)
    replica = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    # host copy, under compact ids, of just the blocks the verifying decode will read
    inv = np.empty(n, np.int64)
    inv[rc.restore_ids] = np.arange(n)                          # pool id -> replica index
    need_rep = inv[dec.in_use_ids]                              # replica indices of the in-use blocks
    compact_of_rep = {int(r): k for k, r in enumerate(need_rep)}
    compact_pool = np.empty((len(need_rep),) + shape[1:], np.uint16)
    step = 16 * W.REPLICA_CHUNK_BLOCKS
    chunks = {}                                                 # every chunk, kept on the host for the byte compare
    for first in range(0, n, step):
        nb = min(step, n - first)
        chunk = rc.replica_chunk(first, nb)
        replica[first:first + nb] = bf16_tensor(chunk)
        hit = np.nonzero((need_rep >= first) & (need_rep < first + nb))[0]
        compact_pool[hit] = chunk[need_rep[hit] - first]
        chunks[first] = chunk
    assert len(compact_of_rep) == len(need_rep)
    pool = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ids = torch.from_numpy(rc.restore_ids).cuda()
    kvflow.kv_restore_blocks(pool, replica, ids)
    torch.cuda.synchronize()
    # (i) bit-exact against the oracle's scatter, over all chunks, each on a pool relabelled to the chunk
    for first, chunk in chunks.items():
        dst = rc.restore_ids[first:first + len(chunk)]
        order = np.argsort(dst)
        rank = np.empty(len(dst), np.int32)
        rank[order] = np.arange(len(dst), dtype=np.int32)       # destination id -> rank among the chunk's ids
        mini = np.zeros_like(chunk)
        oracle.restore_blocks(mini, chunk, rank)
        got = bits_of(pool[torch.from_numpy(dst[order].astype(np.int64)).cuda()])
        assert np.array_equal(got, mini), f"restore mismatch in chunk at {first}"
    del chunks
    # every block was written exactly once: pack it all back and compare on the device
    back = torch.empty_like(replica)
    kvflow.kv_pack_blocks(back, pool, ids)
    torch.cuda.synchronize()
    assert torch.equal(back.view(torch.int16), replica.view(torch.int16))
    del back
    # (ii) decode on the restored pool matches the oracle on every row
    compact_id = np.full(n, -1, np.int32)
    compact_id[dec.in_use_ids] = np.arange(len(need_rep), dtype=np.int32)
    table_c = np.where(dec.block_table >= 0, compact_id[np.maximum(dec.block_table, 0)], -1).astype(np.int32)
    dc = DeviceCase(dec, pool_bits=pool)
    got = dc.decode(torch.bfloat16)
    assert_close_to_oracle(got, oracle_all_rows(oracle, dec, pool=compact_pool, table=table_c), "recovery decode")
    # (iii) and equals, bit for bit, the decode on the pre-failure layout (the replica read as a
    # pool under identity ids, tables mapped back through the permutation)
    table_src = np.where(dec.block_table >= 0, inv[np.maximum(dec.block_table, 0)], -1).astype(np.int32)
    before = dc.decode(torch.bfloat16, pool=replica, block_table=torch.from_numpy(table_src).cuda())
    assert torch.equal(before, got)
