"""GPU parity of the append / dirty-tracking / counted-pack entry points against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

from paper_2601_22438_amd import kvflow
from paper_2601_22438_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import DeviceCase, assert_close_to_oracle, bf16_tensor, bits_of  # noqa: E402


def case_with_room(seed, Hq, Hkv, D, bs, lens, steps):
    """A decode case whose block tables already hold the blocks that `steps` more tokens will need."""
    g = W.Geometry(Hq, Hkv, D, bs)
    lens = np.asarray(lens, np.int32)
    grown = W.make_decode_case("t", seed, g, lens + steps, max_blocks_per_seq=int(-(-(lens.max() + steps) // bs)) + 1)
    grown.context_lens = lens.copy()
    return grown


def new_tokens(case, seed):
    g = case.geom
    ss = np.random.SeedSequence(seed).spawn(2)
    shape = (case.batch, g.num_kv_heads, g.head_dim)
    return W.normal_bf16(ss[0], shape), W.normal_bf16(ss[1], shape)


@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 32), (6, 3, 64, 32)])
def test_append_steps_match_oracle_bitwise(oracle, geom):
    Hq, Hkv, D, bs = geom
    steps = 5
    case = case_with_room(201, Hq, Hkv, D, bs, [0, 1, 15, 16, 31, 32, 100, 255], steps)
    pool_h = case.pool.copy()
    bitmap_h = np.zeros(oracle.bitmap_words(case.num_blocks), np.uint32)
    pool_d = bf16_tensor(case.pool)
    bitmap_d = torch.zeros(len(bitmap_h), dtype=torch.int32, device="cuda")
    table_d = torch.from_numpy(case.block_table).cuda()
    lens = case.context_lens.copy()
    for s in range(steps):
        k_new, v_new = new_tokens(case, 300 + s)
        pos = lens.copy()
        if s == 2:
            pos[[1, 4]] = -1                                        # two sequences sit this step out
        oracle.append_tokens(pool_h, k_new, v_new, case.block_table, pos, bitmap_h)
        kvflow.kv_append_tokens(pool_d, bf16_tensor(k_new), bf16_tensor(v_new), table_d,
                                torch.from_numpy(pos).cuda(), bitmap_d)
        lens[pos >= 0] += 1
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(pool_d), pool_h)
    assert np.array_equal(bitmap_d.cpu().numpy().view(np.uint32), bitmap_h)
    # collect: ascending ids, count, clear
    want = oracle.collect_dirty(bitmap_h, case.num_blocks, clear=True)
    ids_d = torch.full((case.num_blocks,), -1, dtype=torch.int32, device="cuda")
    cnt_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvflow.kv_collect_dirty(bitmap_d, case.num_blocks, ids_d, cnt_d, clear=True)
    torch.cuda.synchronize()
    n = int(cnt_d.item())
    assert n == len(want) and np.array_equal(ids_d[:n].cpu().numpy(), want)
    assert torch.all(ids_d[n:] == -1) and not bitmap_d.any()
    # the pool after the steps decodes like the oracle's
    case.pool, case.context_lens = pool_h, lens
    dc = DeviceCase(case, pool_bits=pool_d)
    got = dc.decode(torch.float32)
    assert_close_to_oracle(got, oracle.decode_attn(case.q, pool_h, case.block_table, lens, case.geom.scale), "after append")


def test_collect_capacity_partial_last_word_and_no_clear(oracle):
    nb = 1000                                                       # 31 full words + 8 bits
    rng = np.random.default_rng(5)
    bitmap_h = rng.integers(0, 2 ** 32, size=oracle.bitmap_words(nb), dtype=np.uint64).astype(np.uint32)
    bitmap_h[-1] |= np.uint32(0xFFFFFF00)                           # garbage beyond block 999 must be ignored
    want = oracle.collect_dirty(bitmap_h.copy(), nb, clear=False)
    assert want.max() < nb
    bitmap_d = torch.from_numpy(bitmap_h.view(np.int32)).cuda()
    ids_d = torch.full((100,), -1, dtype=torch.int32, device="cuda")     # too small on purpose
    cnt_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvflow.kv_collect_dirty(bitmap_d, nb, ids_d, cnt_d, clear=False)
    torch.cuda.synchronize()
    assert int(cnt_d.item()) == len(want) > 100
    assert np.array_equal(ids_d.cpu().numpy(), want[:100])
    assert np.array_equal(bitmap_d.cpu().numpy().view(np.uint32), bitmap_h)   # not cleared
    # large sparse bitmap (200k blocks)
    nb = 200_000
    bm = np.zeros(oracle.bitmap_words(nb), np.uint32)
    some = np.sort(rng.choice(nb, size=777, replace=False))
    for p in some:
        bm[p // 32] |= np.uint32(1 << (p % 32))
    bm_d = torch.from_numpy(bm.view(np.int32)).cuda()
    ids_d = torch.empty(1024, dtype=torch.int32, device="cuda")
    kvflow.kv_collect_dirty(bm_d, nb, ids_d, cnt_d, clear=True)
    torch.cuda.synchronize()
    assert int(cnt_d.item()) == 777 and np.array_equal(ids_d[:777].cpu().numpy(), some)
    assert np.array_equal(oracle.collect_dirty(bm, nb), some)


def test_replication_loop_on_device(oracle):
    """append -> collect -> counted pack on the source, restore on a target, decode there: no host list."""
    case = case_with_room(203, 64, 8, 128, 32, [40, 500, 31, 1000, 63, 64], 2)
    g = case.geom
    src = bf16_tensor(case.pool)
    table_d = torch.from_numpy(case.block_table).cuda()
    bitmap_d = torch.zeros(oracle.bitmap_words(case.num_blocks), dtype=torch.int32, device="cuda")
    ids_d = torch.empty(case.batch * 2, dtype=torch.int32, device="cuda")
    cnt_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    replica = torch.full((case.batch * 2,) + src.shape[1:], float("nan"), dtype=torch.bfloat16, device="cuda")
    # the target holds the pre-step state under the same ids (a second pool)
    target = src.clone()
    pool_h = case.pool.copy()
    bitmap_h = np.zeros(oracle.bitmap_words(case.num_blocks), np.uint32)
    lens = case.context_lens.copy()
    for s in range(2):
        k_new, v_new = new_tokens(case, 400 + s)
        oracle.append_tokens(pool_h, k_new, v_new, case.block_table, lens, bitmap_h)
        kvflow.kv_append_tokens(src, bf16_tensor(k_new), bf16_tensor(v_new), table_d,
                                torch.from_numpy(lens).cuda(), bitmap_d)
        lens += 1
    kvflow.kv_collect_dirty(bitmap_d, case.num_blocks, ids_d, cnt_d, clear=True)
    kvflow.kv_pack_blocks_counted(replica, src, ids_d, cnt_d)
    torch.cuda.synchronize()
    want_ids = oracle.collect_dirty(bitmap_h, case.num_blocks)
    n = int(cnt_d.item())
    assert n == len(want_ids) and np.array_equal(ids_d[:n].cpu().numpy(), want_ids)
    assert np.array_equal(bits_of(replica[:n]), oracle.pack_blocks(pool_h, want_ids))
    assert torch.isnan(replica[n:].float()).all()                   # entries past the device count stay untouched
    kvflow.kv_restore_blocks(target, replica, ids_d, n=n)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(target), pool_h)
    case.context_lens = lens
    a = DeviceCase(case, pool_bits=src).decode(torch.bfloat16)
    b = DeviceCase(case, pool_bits=target).decode(torch.bfloat16)
    assert torch.equal(a, b)
    assert_close_to_oracle(b, oracle.decode_attn(case.q, pool_h, case.block_table, lens, g.scale), "target decode")


@pytest.mark.parametrize("geom", [(8, 2, 64, 16), (64, 8, 128, 32)])
def test_gather_tokens_and_token_granular_replication(oracle, geom):
    Hq, Hkv, D, bs = geom
    case = case_with_room(205, Hq, Hkv, D, bs, [3, 16, 31, 100, 255, 64], 1)
    g = case.geom
    table_d = torch.from_numpy(case.block_table).cuda()
    src = bf16_tensor(case.pool)
    target = src.clone()                                            # the target holds the state before the step
    k_new, v_new = new_tokens(case, 500)
    pos = case.context_lens.copy()
    pos[2] = -1
    pos_d = torch.from_numpy(pos).cuda()
    bm = torch.zeros(oracle.bitmap_words(case.num_blocks), dtype=torch.int32, device="cuda")
    kvflow.kv_append_tokens(src, bf16_tensor(k_new), bf16_tensor(v_new), table_d, pos_d, bm)
    # what travels: the new rows only
    k_out = torch.full((case.batch, g.num_kv_heads, g.head_dim), 7.0, dtype=torch.bfloat16, device="cuda")
    v_out = torch.full_like(k_out, 7.0)
    kvflow.kv_gather_tokens(k_out, v_out, src, table_d, pos_d)
    torch.cuda.synchronize()
    pool_h = case.pool.copy()
    oracle.append_tokens(pool_h, k_new, v_new, case.block_table, pos, np.zeros(len(bm), np.uint32))
    seven = bits_of(torch.full((1,), 7.0, dtype=torch.bfloat16))[0]
    want_k, want_v = oracle.gather_tokens(pool_h, case.block_table, pos,
                                          np.full(k_new.shape, seven, np.uint16), np.full(k_new.shape, seven, np.uint16))
    assert np.array_equal(bits_of(k_out), want_k) and np.array_equal(bits_of(v_out), want_v)
    kvflow.kv_append_tokens(target, k_out, v_out, table_d, pos_d, bm)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(target), pool_h) and np.array_equal(bits_of(src), pool_h)
