"""Pack straight into pinned host memory (the stand-in for a transport buffer on a peer) and restore
from it: the same entry points, with the replica living on the other side of the PCIe link."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, bf16_tensor, bits_of  # noqa: E402


def host_bits(t):
    return t.view(torch.int16).numpy().view(np.uint16)


def test_pack_to_pinned_host_and_restore_from_it(oracle):
    g = W.Geometry(32, 8, 128, 16)
    case = W.make_decode_case("t", 301, g, np.array([300, 1000, 50], np.int32), dirty="fraction", n_dirty=40)
    pool = bf16_tensor(case.pool)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.zeros((len(case.dirty_ids),) + pool.shape[1:], dtype=torch.bfloat16).pin_memory()
    kvflow.kv_pack_blocks(replica, pool, ids)
    torch.cuda.synchronize()
    want = oracle.pack_blocks(case.pool, case.dirty_ids)
    assert np.array_equal(host_bits(replica), want)
    # the target reads the replica straight from host memory
    fresh = np.random.default_rng(1).permutation(case.num_blocks)[:len(case.dirty_ids)].astype(np.int32)
    target = torch.zeros_like(pool)
    kvflow.kv_restore_blocks(target, replica, torch.from_numpy(fresh).cuda())
    torch.cuda.synchronize()
    expect = np.zeros_like(case.pool)
    oracle.restore_blocks(expect, want, fresh)
    assert np.array_equal(bits_of(target), expect)


def test_staged_transfer_pack_to_device_then_dma_to_host(oracle):
    """The transfer path that leaves decode alone: pack at HBM speed into a device staging replica,
    then a DMA copy to the pinned host buffer on the same side stream."""
    g = W.Geometry(64, 8, 128, 32)
    case = W.make_decode_case("t", 305, g, np.array([700, 90, 2000], np.int32), dirty="fraction", n_dirty=25)
    pool = bf16_tensor(case.pool)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    staging = torch.empty((len(case.dirty_ids),) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    host = torch.zeros(staging.shape, dtype=torch.bfloat16).pin_memory()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    kvflow.kv_pack_blocks(staging, pool, ids, stream=side)
    with torch.cuda.stream(side):
        host.copy_(staging, non_blocking=True)
    side.synchronize()
    assert np.array_equal(host_bits(host), oracle.pack_blocks(case.pool, case.dirty_ids))


def test_decode_is_unchanged_while_packing_to_host_on_a_side_stream(oracle):
    case = W.llama8b_layer(shrink=2)
    dc = DeviceCase(case)
    alone = dc.decode(torch.bfloat16)
    ids = torch.from_numpy(case.in_use_ids[:512].copy()).cuda()         # 32 MiB over the link: slow on purpose
    replica = torch.zeros((512,) + dc.pool.shape[1:], dtype=torch.bfloat16).pin_memory()
    side, main = torch.cuda.Stream(), torch.cuda.current_stream()
    g = case.geom
    nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
    out = torch.empty_like(alone)
    fork = torch.cuda.Event()
    fork.record(main)
    side.wait_event(fork)
    kvflow.kv_pack_blocks(replica, dc.pool, ids, stream=side)
    for _ in range(5):                                               # several decode steps pass meanwhile
        kvflow.kv_decode_attn(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, alone)
    assert np.array_equal(host_bits(replica), oracle.pack_blocks(case.pool, case.in_use_ids[:512]))


@pytest.mark.parametrize("n_list,chunk", [(4096, 512), (1000, 300), (7, 16), (5, 1), (0, 8)])
def test_double_buffered_staged_transfer_matches_oracle(oracle, n_list, chunk):
    """kv_pack_blocks_staged: the list goes to pinned host memory through two staging halves of `chunk`
    blocks each (4096 blocks of 64 KiB = 268 MB through 2 x 32 MiB in the first case; ragged last
    chunks, a list shorter than one chunk, one block per chunk and the empty list in the others)."""
    g = W.Geometry(32, 8, 128, 16)
    lens = np.full(8, 8192, np.int32)                                   # 4096 in-use blocks of 64 KiB
    case = W.make_decode_case("t", 307, g, lens, dirty="last")
    pool = bf16_tensor(case.pool)
    rng = np.random.default_rng(11)
    ids_h = rng.permutation(case.in_use_ids)[:n_list].astype(np.int32) if n_list else np.zeros(0, np.int32)
    assert len(ids_h) == n_list
    ids = torch.from_numpy(np.concatenate([ids_h, np.zeros(1, np.int32)])).cuda()[:n_list]   # never an empty allocation
    staging = torch.full((2 * chunk,) + pool.shape[1:], float("nan"), dtype=torch.bfloat16, device="cuda")
    host = torch.zeros((max(n_list, 1) + 1,) + pool.shape[1:], dtype=torch.bfloat16).pin_memory()
    pack_s, copy_s = torch.cuda.Stream(), torch.cuda.Stream()
    pack_s.wait_stream(torch.cuda.current_stream())
    for rnd in range(2):                                                # twice: the halves and events are reused
        host.zero_()
        kvflow.kv_pack_blocks_staged(host, pool, ids, staging, chunk, pack_s, copy_s, n=n_list)
        copy_s.synchronize()
        pack_s.synchronize()
        got = host_bits(host)
        if n_list:
            assert np.array_equal(got[:n_list], oracle.pack_blocks(case.pool, ids_h)), f"round {rnd}"
        assert not got[n_list:].any(), "wrote past the end of the list"


def test_staged_transfer_on_one_stream_and_bad_arguments(oracle):
    g = W.Geometry(8, 2, 64, 16)
    case = W.make_decode_case("t", 309, g, np.array([300, 77], np.int32), dirty="fraction", n_dirty=20)
    pool = bf16_tensor(case.pool)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    n = len(case.dirty_ids)
    staging = torch.empty((2 * 3,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    host = torch.zeros((n,) + pool.shape[1:], dtype=torch.bfloat16).pin_memory()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    kvflow.kv_pack_blocks_staged(host, pool, ids, staging, 3, s, s)     # same stream: packs and copies alternate
    s.synchronize()
    assert np.array_equal(host_bits(host), oracle.pack_blocks(case.pool, case.dirty_ids))
    with pytest.raises(ValueError):
        kvflow.kv_pack_blocks_staged(host, pool, ids, staging[:5], 3, s, s)          # staging smaller than two halves
    with pytest.raises(ValueError):
        kvflow.kv_pack_blocks_staged(host[:n - 1], pool, ids, staging, 3, s, s)      # destination too small
    with pytest.raises(kvflow.KvflowError) as e:
        kvflow.kv_pack_blocks_staged(host, pool, ids, staging, 0, s, s)
    assert e.value.status == -2
