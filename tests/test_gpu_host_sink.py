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
