"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before any launch (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvflow.h")
LIB = os.path.join(ROOT, "paper_2601_22438_amd", "libkvflow.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2601_22438_amd.build import build_library
        build_library()
    from paper_2601_22438_amd import kvflow
    return kvflow.load()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(kv_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for must in ("kv_decode_attn", "kv_pack_blocks", "kv_restore_blocks"):
        assert must in names


def test_library_exports_every_declared_function(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_has_the_same_names():
    from paper_2601_22438_amd import kvflow
    for name in declared_functions():
        assert hasattr(kvflow, name), name


def desc(kvflow, base=0x10000, nb=8, hkv=2, bs=16, d=64, dtype=0):
    return kvflow.kv_pool_desc(base, nb, hkv, bs, d, dtype, 1.0, 1.0)


def decode(lib, kvflow, pool, out=0x20000, q=0x30000, table=0x40000, lens=0x50000, mb=4, batch=2, hq=8,
           max_len=64, wgs=0, ws=0x60000, ws_bytes=1 << 30, out_dtype=1):
    return lib.kv_decode_attn(out, out_dtype, q, ctypes.byref(pool), table, mb, lens, batch, hq, max_len,
                              0.125, wgs, ws, ws_bytes, None)


def test_decode_rejects_bad_arguments_before_any_launch(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)
    assert decode(lib, kvflow, desc(kvflow, base=0)) == -1                       # NULL pool
    assert decode(lib, kvflow, ok, out=0) == -1
    assert decode(lib, kvflow, ok, q=0) == -1
    assert decode(lib, kvflow, ok, table=0) == -1
    assert decode(lib, kvflow, ok, lens=0) == -1
    assert decode(lib, kvflow, desc(kvflow, nb=0)) == -2
    assert decode(lib, kvflow, ok, hq=7) == -2                                   # not a multiple of Hkv
    assert decode(lib, kvflow, ok, hq=2 * 17) == -2                              # group > 16
    assert decode(lib, kvflow, ok, max_len=65) == -2                             # beyond the table row
    assert decode(lib, kvflow, ok, wgs=-1) == -2
    assert decode(lib, kvflow, desc(kvflow, d=96)) == -3
    assert decode(lib, kvflow, desc(kvflow, bs=8)) == -3
    assert decode(lib, kvflow, desc(kvflow, dtype=1)) == -3
    assert decode(lib, kvflow, ok, out_dtype=2) == -3
    assert decode(lib, kvflow, desc(kvflow, base=0x10008)) == -4
    assert decode(lib, kvflow, ok, out=0x20004) == -4
    assert decode(lib, kvflow, ok, ws=0x60004) == -4
    assert decode(lib, kvflow, ok, ws=0) == -5
    assert decode(lib, kvflow, ok, ws_bytes=16) == -5
    assert decode(lib, kvflow, ok, batch=0) == 0                                 # nothing to do
    assert decode(lib, kvflow, ok, batch=-1) == -2


def test_pack_restore_reject_bad_arguments_before_any_launch(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)
    for fn, args in ((lib.kv_pack_blocks, lambda p, rep, ids, n: (rep, ctypes.byref(p), ids, n, None)),
                     (lib.kv_restore_blocks, lambda p, rep, ids, n: (ctypes.byref(p), rep, ids, n, None))):
        assert fn(*args(ok, 0x20000, 0x30000, 0)) == 0                           # empty list
        assert fn(*args(ok, 0, 0x30000, 3)) == -1
        assert fn(*args(ok, 0x20000, 0, 3)) == -1
        assert fn(*args(desc(kvflow, base=0), 0x20000, 0x30000, 3)) == -1
        assert fn(*args(ok, 0x20000, 0x30000, -1)) == -2
        assert fn(*args(desc(kvflow, hkv=0), 0x20000, 0x30000, 3)) == -2
        assert fn(*args(desc(kvflow, d=100), 0x20000, 0x30000, 3)) == -3
        assert fn(*args(ok, 0x20008, 0x30000, 3)) == -4


def test_block_bytes_workgroups_and_workspace_size(lib):
    from paper_2601_22438_amd import kvflow
    assert lib.kv_block_bytes(ctypes.byref(desc(kvflow, hkv=8, bs=16, d=128))) == 65536
    assert lib.kv_block_bytes(ctypes.byref(desc(kvflow, hkv=2, bs=16, d=64))) == 8192
    assert lib.kv_block_bytes(None) == 0
    # small problems get fewer workgroups, big ones the full persistent grid; a request is honoured
    assert kvflow.kv_decode_workgroups(4, 2, 256) == 4
    assert kvflow.kv_decode_workgroups(8, 8, 65536) == 256
    assert kvflow.kv_decode_workgroups(8, 8, 65536, 100) == 100
    assert kvflow.kv_decode_workgroups(0, 8, 65536) == 0
    assert kvflow.kv_decode_workgroups(8, 8, 65536, -3) == 0
    # workspace = tile counts (16-byte padded) + (runs + rows) * group * (D + 4) floats
    wgs = 256
    want = 48 + (wgs * 4 + 8 * 8) * 4 * (128 + 4) * 4      # 9 counts = 36 bytes, padded to 48
    assert kvflow.kv_decode_workspace_bytes(8, 32, 8, 128, 65536) == want
    assert kvflow.kv_decode_workspace_bytes(8, 33, 8, 128, 65536) == 0


def test_staged_pack_rejects_bad_arguments_before_any_launch(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)
    sp = lambda dst=0x20000, p=ok, ids=0x30000, n=4, st=0x40000, chunk=2: lib.kv_pack_blocks_staged(
        dst, ctypes.byref(p), ids, n, st, chunk, None, None)
    assert sp(n=0) == 0
    assert sp(dst=0) == -1 and sp(ids=0) == -1 and sp(st=0) == -1 and sp(p=desc(kvflow, base=0)) == -1
    assert sp(n=-1) == -2 and sp(chunk=0) == -2 and sp(chunk=-5) == -2
    assert sp(dst=0x20008) == -4 and sp(st=0x40004) == -4
    assert sp(p=desc(kvflow, d=48)) == -3


def test_status_strings(lib):
    from paper_2601_22438_amd import kvflow
    assert kvflow.kv_status_string(0) == "ok"
    texts = {kvflow.kv_status_string(s) for s in range(-7, 1)}
    assert len(texts) == 8 and "unknown status" not in texts
    assert kvflow.kv_status_string(-99) == "unknown status"


def test_append_collect_counted_pack_reject_bad_arguments(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)
    ap = lambda p=ok, k=0x20000, v=0x30000, tb=0x40000, mb=4, pos=0x50000, b=2, bm=0x60000: \
        lib.kv_append_tokens(ctypes.byref(p), k, v, tb, mb, pos, b, bm, None)
    assert ap(b=0) == 0
    assert ap(k=0) == -1 and ap(v=0) == -1 and ap(tb=0) == -1 and ap(pos=0) == -1 and ap(bm=0) == -1
    assert ap(p=desc(kvflow, base=0)) == -1
    assert ap(b=-1) == -2 and ap(mb=0) == -2
    assert ap(p=desc(kvflow, d=48)) == -3
    assert ap(k=0x20008) == -4
    ga = lambda k=0x20000, v=0x30000, tb=0x40000, mb=4, pos=0x50000, b=2: \
        lib.kv_gather_tokens(k, v, ctypes.byref(ok), tb, mb, pos, b, None)
    assert ga(b=0) == 0
    assert ga(k=0) == -1 and ga(v=0) == -1 and ga(tb=0) == -1 and ga(pos=0) == -1
    assert ga(b=-1) == -2 and ga(mb=0) == -2 and ga(v=0x30004) == -4
    co = lambda bm=0x60000, nb=100, ids=0x70000, cap=10, cnt=0x80000: \
        lib.kv_collect_dirty(bm, nb, ids, cap, cnt, 1, None)
    assert co(bm=0) == -1 and co(cnt=0) == -1 and co(ids=0) == -1
    assert co(nb=0) == -2 and co(cap=-1) == -2
    pc = lambda rep=0x20000, ids=0x30000, cnt=0x40000, n=3: \
        lib.kv_pack_blocks_counted(rep, ctypes.byref(ok), ids, cnt, n, None)
    assert pc(n=0) == 0
    assert pc(cnt=0) == -1 and pc(rep=0) == -1 and pc(ids=0) == -1
    assert pc(n=-2) == -2


def test_fp8_pool_descriptor_checks(lib):
    from paper_2601_22438_amd import kvflow
    fp8 = lambda ks=0.25, vs=0.5, **kw: kvflow.kv_pool_desc(kw.get("base", 0x10000), 8, 8, 16, 128, 2, ks, vs)
    assert lib.kv_block_bytes(ctypes.byref(fp8())) == 32768                     # half of the bf16 block
    assert decode(lib, kvflow, fp8(), hq=32, batch=0) == 0
    for bad in (fp8(ks=0.0), fp8(vs=-1.0), fp8(ks=float("inf")), fp8(vs=float("nan"))):
        assert decode(lib, kvflow, bad, hq=32) == -2
    assert decode(lib, kvflow, kvflow.kv_pool_desc(0x10000, 8, 8, 16, 128, 3, 1.0, 1.0), hq=32) == -3
    assert lib.kv_block_bytes(ctypes.byref(kvflow.kv_pool_desc(0x10000, 8, 8, 16, 128, 3, 1.0, 1.0))) == 0


def test_prefill_rejects_bad_arguments_before_any_launch(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)

    def pf(p=ok, out=0x20000, q=0x30000, tb=0x40000, mb=4, lens=0x50000, qs=0x60000, b=2, hq=8, mq=64, od=1,
           tq=100, scale=0.125, ks=1, ws=0, wsb=0):
        return lib.kv_prefill_attn(out, od, q, ctypes.byref(p), tb, mb, lens, qs, b, hq, mq, tq, scale, ks, ws, wsb,
                                   None)
    assert pf(b=0) == 0 and pf(mq=0) == 0 and pf(tq=0) == 0                       # nothing to do
    assert pf(out=0) == -1 and pf(q=0) == -1 and pf(tb=0) == -1 and pf(lens=0) == -1 and pf(qs=0) == -1
    assert pf(p=desc(kvflow, base=0)) == -1
    assert pf(b=-1) == -2 and pf(mq=-1) == -2 and pf(mb=0) == -2 and pf(hq=7) == -2 and pf(tq=-1) == -2
    assert pf(ks=-1) == -2 and pf(ks=17) == -2
    assert pf(p=desc(kvflow, d=96)) == -3 and pf(od=2) == -3 and pf(b=65536) == -3
    assert pf(p=kvflow.kv_pool_desc(0x10000, 8, 2, 16, 64, 2, 0.0, 0.25)) == -2   # FP8 pool with a bad scale
    assert pf(out=0x20008) == -4 and pf(q=0x30004) == -4
    for bad in (0.0, -0.125, float("inf"), float("nan")):
        assert pf(scale=bad) == -2
    # a split key range needs its workspace
    need = kvflow.kv_prefill_workspace_bytes(100, 8, 64, 4)
    assert need == 4 * 100 * 8 * (64 + 4) * 4
    assert pf(ks=4) == -5 and pf(ks=4, ws=0x70000, wsb=need - 1) == -5 and pf(ks=4, ws=0x70004, wsb=need) == -4
    assert kvflow.kv_prefill_workspace_bytes(100, 8, 64, 1) == 0 and kvflow.kv_prefill_workspace_bytes(100, 8, 64, 17) == 0


def test_prefill_key_split_suggestion():
    from paper_2601_22438_amd import kvflow
    # many query tokens: the token ranges fill the chip by themselves
    assert kvflow.kv_prefill_key_splits(8, 32, 8, 8192, 8192) == 1
    # one sequence, a 256-token chunk over 64k tokens: 8 head groups x 4 range pairs = 32 workgroups -> 16 parts
    assert kvflow.kv_prefill_key_splits(1, 32, 8, 256, 65536) == 16
    # short contexts are not cut below 16 tiles per part
    assert kvflow.kv_prefill_key_splits(1, 32, 8, 256, 1024) == 2
    assert kvflow.kv_prefill_key_splits(1, 32, 8, 64, 300) == 1
    assert kvflow.kv_prefill_key_splits(0, 32, 8, 256, 1024) == 0 and kvflow.kv_prefill_key_splits(1, 33, 8, 256, 1024) == 0


def test_append_packed_rejects_bad_arguments_before_any_launch(lib):
    from paper_2601_22438_amd import kvflow
    ok = desc(kvflow)
    ap = lambda p=ok, k=0x20000, v=0x30000, tb=0x40000, mb=4, lens=0x50000, qs=0x60000, b=2, tq=10, bm=0x70000: \
        lib.kv_append_packed(ctypes.byref(p), k, v, tb, mb, lens, qs, b, tq, bm, None)
    assert ap(b=0) == 0 and ap(tq=0) == 0
    assert ap(k=0) == -1 and ap(v=0) == -1 and ap(tb=0) == -1 and ap(lens=0) == -1 and ap(qs=0) == -1 and ap(bm=0) == -1
    assert ap(p=desc(kvflow, base=0)) == -1
    assert ap(b=-1) == -2 and ap(mb=0) == -2 and ap(tq=-1) == -2
    assert ap(p=desc(kvflow, d=48)) == -3
    assert ap(k=0x20008) == -4 and ap(v=0x30004) == -4


def test_probe_rejects_bad_arguments_before_any_launch(lib):
    pr = lambda mode=2, a=0x20000, b=0x30000, n=1 << 20: lib.kv_probe_stream(mode, a, b, n, None)
    assert pr(n=0) == 0
    assert pr(mode=6) == -2 and pr(mode=-1) == -2 and pr(n=24) == -2
    assert pr(n=(32 << 30) + 16) == -2 and pr(mode=5, a=0, n=(32 << 30) + 16) == -1
    assert pr(a=0) == -1 and pr(b=0) == -1 and pr(mode=0, b=0) == -1 and pr(mode=3, b=0) == -1 and pr(mode=4, a=0) == -1
    assert pr(a=0x20008) == -4 and pr(b=0x30004) == -4


def test_matrix_probe_rejects_bad_arguments_before_any_launch(lib):
    need = 256 * 512 * 4
    pm = lambda mode=1, iters=10, sink=0x20000, n=need: lib.kv_probe_matrix(mode, iters, sink, n, None)
    assert pm(mode=6) == -2 and pm(mode=-1) == -2 and pm(iters=-1) == -2
    assert pm(sink=0) == -1 and pm(sink=0x20008) == -4 and pm(n=need - 4) == -5


def test_binding_rejects_host_tensors_before_touching_the_library():
    """The binding's own checks run on the host: a tensor that is not GPU memory never reaches a kernel."""
    import torch
    from paper_2601_22438_amd import kvflow
    q = torch.zeros((2, 8, 64), dtype=torch.bfloat16)
    pool = torch.zeros((8, 2, 2, 16, 64), dtype=torch.bfloat16)
    table = torch.zeros((2, 4), dtype=torch.int32)
    lens = torch.ones(2, dtype=torch.int32)
    with pytest.raises(ValueError, match="GPU memory"):
        kvflow.kv_decode_attn(torch.empty_like(q), q, pool, table, lens, 16, 0.125)
    with pytest.raises(ValueError, match="GPU memory"):
        kvflow.kv_pack_blocks(torch.empty_like(pool), pool, torch.zeros(8, dtype=torch.int32))
    with pytest.raises(ValueError, match="GPU memory"):
        kvflow.kv_restore_blocks(pool, torch.empty_like(pool), torch.zeros(8, dtype=torch.int32))


def test_decode_kernels_need_no_scratch_memory():
    """A decode kernel that spills registers or calls a function with a stack frame makes every dispatch
    reserve scratch memory, which costs tens of microseconds per call on this device: keep them at zero."""
    from paper_2601_22438_amd.build import kernel_resources
    seen = 0
    for source in ("kv_decode.hip", "kv_decode_fp8.hip"):
        for name, use in kernel_resources(source).items():
            if "decode_partition" in name:
                seen += 1
                assert use["scratch"] == 0 and use["spills"] == 0, (name, use)
    assert seen == 4
