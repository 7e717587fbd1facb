"""The allocation-free decode entry point (kv_decode_attn_static: the workspace is a fixed array in
the library's device code) against kv_decode_attn with a caller-owned workspace, bit for bit, on
two calls in a row that share the array, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle  # noqa: E402


def static_decode(dc, out_dtype, workgroups=0):
    c, g = dc.case, dc.case.geom
    out = torch.full((c.batch, g.num_q_heads, g.head_dim), float("nan"), dtype=out_dtype, device="cuda")
    kvflow.kv_decode_attn_static(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale,
                                 workgroups)
    torch.cuda.synchronize()
    return out


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row(oracle):
    big = W.llama8b_layer(shrink=4)                      # 32 sequences, several runs per row
    small = W.tiny()
    cases = [(big, DeviceCase(big)), (small, DeviceCase(small))]
    before = torch.cuda.memory_allocated()
    got = []
    for case, dc in cases:                               # back to back: the second call finds the first one's records
        for dt in (torch.float32, torch.bfloat16):
            got.append(static_decode(dc, dt))
    # the call itself took no memory from torch's allocator beyond the output tensors kept here
    assert torch.cuda.memory_allocated() - before <= sum(t.numel() * t.element_size() for t in got) + 4096
    k = 0
    for case, dc in cases:
        want64 = oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens, case.geom.scale)
        for dt in (torch.float32, torch.bfloat16):
            want = dc.decode(dt)                         # caller-owned workspace, filled with NaN on entry
            assert torch.equal(got[k], want), f"{case.name} {dt}: static scratch differs from workspace"
            assert_close_to_oracle(got[k], want64, f"{case.name} {dt} static scratch")
            k += 1
    # and once more in the other order, with an explicit grid size
    for case, dc in reversed(cases):
        assert torch.equal(static_decode(dc, torch.float32, workgroups=7), dc.decode(torch.float32, workgroups=7))


def test_static_scratch_decode_rejects_sizes_beyond_the_array():
    case = W.tiny()
    dc = DeviceCase(case)
    g = case.geom
    out = torch.empty((case.batch, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda")
    # the same tensors, but a grid whose records cannot fit: 65535 workgroups x 4 runs
    need = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim, dc.max_len, 65535)
    assert need > kvflow.KV_DECODE_STATIC_SCRATCH_BYTES
    with pytest.raises(kvflow.KvflowError) as e:
        kvflow.kv_decode_attn_static(out, dc.q, dc.pool, dc.block_table, dc.context_lens, dc.max_len, dc.scale, 65535)
    assert e.value.status == -5
    torch.cuda.synchronize()
