"""The calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset
nodes), so a serving step can be captured into a HIP graph.  Every replay must equal the eager result."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle, bf16_tensor, bits_of  # noqa: E402


def test_step_captured_in_a_graph_replays_like_eager(oracle):
    case = W.llama8b_layer(shrink=4)
    g = case.geom
    dc = DeviceCase(case)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    n = len(case.dirty_ids)
    replica = torch.zeros((n,) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    target = torch.zeros_like(dc.pool)
    out = torch.zeros((case.batch, g.num_q_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
    nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")

    def step():
        kvflow.kv_decode_attn(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0, ws)
        kvflow.kv_pack_blocks(replica, dc.pool, ids)
        kvflow.kv_restore_blocks(target, replica, ids)

    step()
    torch.cuda.synchronize()
    eager_out, eager_rep = out.clone(), replica.clone()
    assert_close_to_oracle(eager_out, oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens,
                                                         g.scale), "eager")
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for i in range(4):
        out.zero_(); replica.zero_(); target.zero_(); ws.fill_(float("nan"))     # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out), f"replay {i}: decode differs"
        assert torch.equal(replica.view(torch.int16), eager_rep.view(torch.int16)), f"replay {i}: pack differs"
        got = bits_of(target)
        assert np.array_equal(got[case.dirty_ids], case.pool[case.dirty_ids])
        # new inputs in the same buffers are picked up by the next replay
        if i == 1:
            q2 = W.normal_bf16(np.random.SeedSequence(900), case.q.shape)
            dc.q.copy_(bf16_tensor(q2))
            case.q = q2
            torch.cuda.synchronize()
            eager_out = None
            graph.replay()
            torch.cuda.synchronize()
            eager_out = out.clone()
            assert_close_to_oracle(eager_out, oracle.decode_attn(q2, case.pool, case.block_table, case.context_lens,
                                                                 g.scale), "replay with new q")


@pytest.mark.parametrize("key_splits", [1, 3])
def test_recompute_call_captured_in_a_graph(oracle, key_splits):
    """kv_prefill_attn (with and without a cut key range) replays like eager, also when the first call of
    the process for this kernel happens during capture."""
    g = W.Geometry(8, 2, 64 if key_splits == 1 else 128, 16)
    case = W.make_prefill_case("graph_prefill", 910 + key_splits, g, np.array([300, 77], np.int32),
                               np.array([120, 77], np.int32), max_blocks_per_seq=32, dirty="last")
    kv = case.kv
    q, pool = bf16_tensor(case.q), bf16_tensor(kv.pool)
    table, lens = torch.from_numpy(kv.block_table).cuda(), torch.from_numpy(kv.context_lens).cuda()
    starts = torch.from_numpy(case.q_starts).cuda()
    out = torch.zeros((case.total_q, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda")
    nbytes = kvflow.kv_prefill_workspace_bytes(case.total_q, g.num_q_heads, g.head_dim, key_splits)
    ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda")
    want = oracle.prefill_attn(case.q, kv.pool, kv.block_table, kv.context_lens, case.q_starts, g.scale)

    def call():
        kvflow.kv_prefill_attn(out, q, pool, table, lens, starts, case.max_q_len, float(g.scale), key_splits, ws)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    for i in range(3):
        out.zero_(); ws.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_close_to_oracle(out, want, f"replay {i}")
    replayed = out.clone()
    out.zero_()
    call()
    torch.cuda.synchronize()
    assert torch.equal(out, replayed)


def test_two_stream_step_captured_in_a_graph(oracle):
    """The replication step as a graph: fork -> {decode on the capture stream, pack on a second stream} ->
    join, three steps per graph.  The cross-stream edges are graph dependencies (no host-side event calls at
    replay); every replay gives the decode output of decode alone, bit for bit, and the oracle's replica."""
    case = W.replication_mix(shrink=8, batch=32)
    g = case.geom
    dc = DeviceCase(case)
    alone = dc.decode(torch.bfloat16)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replica = torch.zeros((len(case.dirty_ids),) + dc.pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(alone)
    nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
    want_replica = oracle.pack_blocks(case.pool, case.dirty_ids)
    # warm both kernels outside the capture
    kvflow.kv_decode_attn(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 0, ws)
    kvflow.kv_pack_blocks(replica, dc.pool, ids)
    torch.cuda.synchronize()
    cap, side = torch.cuda.Stream(), torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            for _ in range(3):
                side.wait_stream(cap)                                   # fork
                kvflow.kv_pack_blocks(replica, dc.pool, ids, stream=side)
                kvflow.kv_decode_attn(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale,
                                      0, ws, stream=cap)
                cap.wait_stream(side)                                   # join
    torch.cuda.synchronize()
    for i in range(4):
        out.zero_(); replica.zero_(); ws.fill_(float("nan"))           # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, alone), f"replay {i}: decode beside pack differs from decode alone"
        assert np.array_equal(bits_of(replica), want_replica), f"replay {i}: replica differs from the oracle's"
    assert_close_to_oracle(out, oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens, g.scale),
                           "two-stream graph")
