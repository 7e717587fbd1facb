"""Seeded random geometries through every kernel family against the oracle: head counts with groups of 1 to 16
(3 included), head dimensions 64 and 128, block sizes 16 and 32, bf16 and FP8 pools, batches with empty
sequences, chosen and automatic workgroup counts, cut and uncut key ranges.  The fixed cases elsewhere pin
known edges; this sweep looks for the combinations nobody listed."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle, bf16_tensor, bits_of, pool_tensor  # noqa: E402

CASES_PER_SEED = 8


def draw_geometry(rng):
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 3, 4, 8, 16]))
    fp8 = bool(rng.integers(0, 3) == 0)
    g = W.Geometry(hkv * group, hkv, int(rng.choice([64, 128])), int(rng.choice([16, 32])), 1 if fp8 else 2)
    batch = int(rng.integers(1, 24))
    lens = rng.integers(0, int(rng.choice([40, 300, 1500])) + 1, size=batch).astype(np.int32)
    if rng.integers(0, 4) == 0:
        lens[rng.integers(0, batch)] = 0
    if lens.max() == 0:
        lens[0] = 5
    return g, fp8, lens, int(rng.choice([0, 0, 1, 3, 7, 64, 300]))


@pytest.mark.parametrize("seed", range(4))
def test_random_shapes_match_the_oracle(oracle, seed):
    rng = np.random.default_rng(5000 + seed)
    for it in range(CASES_PER_SEED):
        g, fp8, lens, wgs = draw_geometry(rng)
        what = (f"seed {seed} case {it}: Hq {g.num_q_heads} Hkv {g.num_kv_heads} D {g.head_dim} bs {g.block_size} "
                f"fp8 {fp8} lens {lens.tolist()} workgroups {wgs}")
        print(what, flush=True)
        scales = {"k_scale": W.FP8_KV_SCALE, "v_scale": W.FP8_KV_SCALE} if fp8 else {}
        n_dirty = max(1, int(W.blocks_needed(lens, g.block_size).sum()) // 3)
        case = W.make_decode_case("random", 6000 + 100 * seed + it, g, lens, dirty="fraction", n_dirty=n_dirty)
        dc = DeviceCase(case, **scales)
        want = oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens, g.scale, **scales)
        for dtype in (torch.float32, torch.bfloat16):
            assert_close_to_oracle(dc.decode(dtype, workgroups=wgs), want, f"{what}, decode {dtype}")

        ids = torch.from_numpy(case.dirty_ids).cuda()
        data = dc.pool.data if fp8 else dc.pool
        host_bits = (lambda t: t.cpu().numpy()) if fp8 else bits_of
        replica = torch.zeros((len(case.dirty_ids),) + tuple(data.shape[1:]), dtype=data.dtype, device="cuda")
        kvflow.kv_pack_blocks(replica, dc.pool, ids)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(replica), oracle.pack_blocks(case.pool, case.dirty_ids)), f"{what}, pack"
        target = torch.zeros_like(data)
        kvflow.kv_restore_blocks(kvflow.Fp8Pool(target, 1.0, 1.0) if fp8 else target, replica, ids)
        torch.cuda.synchronize()
        want_pool = np.zeros_like(case.pool)
        oracle.restore_blocks(want_pool, host_bits(replica), case.dirty_ids)
        assert np.array_equal(host_bits(target), want_pool), f"{what}, restore"

        q_lens = np.array([int(rng.integers(0, min(int(n), 200) + 1)) for n in lens], np.int32)
        if q_lens.sum() == 0:
            continue
        pc = W.make_prefill_case("random_prefill", 7000 + 100 * seed + it, g, lens, q_lens)
        kv = pc.kv
        q, pool = bf16_tensor(pc.q), pool_tensor(kv.pool, *(scales.values() if fp8 else ()))
        table, lens_t = torch.from_numpy(kv.block_table).cuda(), torch.from_numpy(kv.context_lens).cuda()
        starts = torch.from_numpy(pc.q_starts).cuda()
        want_rows = oracle.prefill_attn(pc.q, kv.pool, kv.block_table, kv.context_lens, pc.q_starts, g.scale, **scales)
        for splits in (1, int(rng.choice([2, 3, 5]))):
            out = torch.full((pc.total_q, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            nbytes = kvflow.kv_prefill_workspace_bytes(pc.total_q, g.num_q_heads, g.head_dim, splits)
            ws = torch.full((max(nbytes, 4) // 4,), float("nan"), dtype=torch.float32, device="cuda")
            kvflow.kv_prefill_attn(out, q, pool, table, lens_t, starts, pc.max_q_len, float(g.scale), splits, ws)
            torch.cuda.synchronize()
            assert_close_to_oracle(out, want_rows, f"{what}, recomputation with {splits} key parts")
