"""Thin ctypes binding of libkvflow.so: argument marshalling only.

Every function has the name and argument order of the C entry point it calls
(see include/kvflow.h).  Tensors are torch CUDA tensors used as device memory;
their ``data_ptr()`` and the current HIP stream handle are passed through.  There
is no fallback: if the library is missing or cannot be loaded, every call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

KV_DTYPE_BF16 = 0
KV_DTYPE_F32 = 1
KV_DTYPE_FP8_E4M3 = 2

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvflow.so")
_lib = None


class KvflowError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"kvflow status {status}: {text}")
        self.status = status


class kv_pool_desc(ctypes.Structure):
    _fields_ = [("base", ctypes.c_void_p), ("num_blocks", ctypes.c_int64),
                ("num_kv_heads", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libkvflow.so (built in-tree by paper_2601_22438_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2601_22438_amd.build` first")
    lib = ctypes.CDLL(_LIB_PATH)
    P, I32, I64, SZ, F = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
    PD = ctypes.POINTER(kv_pool_desc)
    lib.kv_block_bytes.restype, lib.kv_block_bytes.argtypes = SZ, [PD]
    lib.kv_decode_workgroups.restype = I32
    lib.kv_decode_workgroups.argtypes = [I32, I32, I32, I32]
    lib.kv_decode_workspace_bytes.restype = SZ
    lib.kv_decode_workspace_bytes.argtypes = [I32, I32, I32, I32, I32, I32]
    lib.kv_decode_attn.restype = ctypes.c_int
    lib.kv_decode_attn.argtypes = [P, I32, P, PD, P, I32, P, I32, I32, I32, F, I32, P, SZ, P]
    lib.kv_decode_attn_static.restype = ctypes.c_int
    lib.kv_decode_attn_static.argtypes = [P, I32, P, PD, P, I32, P, I32, I32, I32, F, I32, P]
    lib.kv_prefill_attn.restype = ctypes.c_int
    lib.kv_prefill_attn.argtypes = [P, I32, P, PD, P, I32, P, P, I32, I32, I32, I64, F, I32, P, SZ, P]
    lib.kv_prefill_key_splits.restype = I32
    lib.kv_prefill_key_splits.argtypes = [I32, I32, I32, I32, I32]
    lib.kv_prefill_workspace_bytes.restype = SZ
    lib.kv_prefill_workspace_bytes.argtypes = [I64, I32, I32, I32]
    lib.kv_pack_blocks.restype = ctypes.c_int
    lib.kv_pack_blocks.argtypes = [P, PD, P, I64, P]
    lib.kv_restore_blocks.restype = ctypes.c_int
    lib.kv_restore_blocks.argtypes = [PD, P, P, I64, P]
    lib.kv_pack_blocks_staged.restype = ctypes.c_int
    lib.kv_pack_blocks_staged.argtypes = [P, PD, P, I64, P, I64, P, P]
    lib.kv_pack_blocks_counted.restype = ctypes.c_int
    lib.kv_pack_blocks_counted.argtypes = [P, PD, P, P, I64, P]
    lib.kv_append_tokens.restype = ctypes.c_int
    lib.kv_append_tokens.argtypes = [PD, P, P, P, I32, P, I32, P, P]
    lib.kv_append_packed.restype = ctypes.c_int
    lib.kv_append_packed.argtypes = [PD, P, P, P, I32, P, P, I32, I64, P, P]
    lib.kv_gather_tokens.restype = ctypes.c_int
    lib.kv_gather_tokens.argtypes = [P, P, PD, P, I32, P, I32, P]
    lib.kv_collect_dirty.restype = ctypes.c_int
    lib.kv_collect_dirty.argtypes = [P, I64, P, I64, P, I32, P]
    lib.kv_validate_decode.restype = ctypes.c_int
    lib.kv_validate_decode.argtypes = [PD, P, I32, P, I32, I32, P]
    lib.kv_validate_prefill.restype = ctypes.c_int
    lib.kv_validate_prefill.argtypes = [PD, P, I32, P, P, I32, I32, I64, P]
    lib.kv_validate_block_ids.restype = ctypes.c_int
    lib.kv_validate_block_ids.argtypes = [PD, P, I64, I32, P]
    lib.kv_probe_stream.restype = ctypes.c_int
    lib.kv_probe_stream.argtypes = [I32, P, P, SZ, P]
    lib.kv_probe_matrix.restype = ctypes.c_int
    lib.kv_probe_matrix.argtypes = [I32, I32, P, SZ, P]
    lib.kv_status_string.restype, lib.kv_status_string.argtypes = ctypes.c_char_p, [ctypes.c_int]
    _lib = lib
    return lib


def kv_status_string(status: int) -> str:
    return load().kv_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise KvflowError(status, kv_status_string(status))


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


# Host-only argument checks (no synchronisation): the kernels read these buffers as raw memory of a
# fixed element type, so a tensor of another dtype, a strided view or a host tensor would make them
# follow garbage indices.
def _dev(t, name, dtype=None, shape=None, numel=None, allow_pinned=False):
    if not torch.is_tensor(t):
        raise ValueError(f"{name} must be a torch tensor")
    if not (t.is_cuda or (allow_pinned and t.is_pinned())):
        raise ValueError(f"{name} must live in GPU memory" + (" or pinned host memory" if allow_pinned else ""))
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} must hold at least {numel} elements, got {t.numel()}")
    return t


def _pool_data(pool):
    return pool.data if isinstance(pool, Fp8Pool) else pool


def _table(block_table, batch):
    _dev(block_table, "block_table", torch.int32)
    if block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError(f"block_table must be int32 [batch={batch}][max_blocks_per_seq]")
    return block_table


def _new_rows(pool, k, v, rows):
    """k, v: [rows][Hkv][D] in the pool's element type."""
    data = _pool_data(pool)
    want = (rows, data.shape[2], data.shape[4])
    for t, name in ((k, "K rows"), (v, "V rows")):
        _dev(t, name, shape=want)
        if t.element_size() != data.element_size():
            raise ValueError(f"{name} must have the pool's element size ({data.element_size()} bytes)")


def _bitmap(dirty_bitmap, pool):
    _dev(dirty_bitmap, "dirty_bitmap", (torch.int32, torch.uint32), numel=(_pool_data(pool).shape[0] + 31) // 32)


def _replica(replica, pool, n, name="replica"):
    _dev(replica, name, allow_pinned=True)
    data = _pool_data(pool)
    need = n * data[0].numel() * data.element_size()
    if replica.numel() * replica.element_size() < need:
        raise ValueError(f"{name} holds {replica.numel() * replica.element_size()} bytes, {need} needed")
    return replica


class Fp8Pool:
    """An FP8 E4M3 pool: a contiguous uint8 (or float8_e4m3fn) tensor [NB][2][Hkv][bs][D] plus its scales."""

    def __init__(self, data: torch.Tensor, k_scale: float, v_scale: float):
        if data.element_size() != 1:
            raise ValueError("FP8 pool data must have 1-byte elements")
        self.data, self.k_scale, self.v_scale = data, float(k_scale), float(v_scale)

    @property
    def shape(self):
        return self.data.shape


def pool_desc(pool) -> kv_pool_desc:
    """Describe a pool of shape [NB][2][Hkv][bs][D]: a bf16 tensor, or an Fp8Pool (contiguous, on the GPU)."""
    data = pool.data if isinstance(pool, Fp8Pool) else pool
    if not torch.is_tensor(data) or data.dim() != 5 or data.shape[1] != 2 or not data.is_contiguous():
        raise ValueError("pool must be a contiguous [NB][2][Hkv][bs][D] tensor")
    if not data.is_cuda:
        raise ValueError("pool must live in GPU memory")
    nb, _, hkv, bs, d = data.shape
    if isinstance(pool, Fp8Pool):
        return kv_pool_desc(data.data_ptr(), nb, hkv, bs, d, KV_DTYPE_FP8_E4M3, pool.k_scale, pool.v_scale)
    if data.dtype != torch.bfloat16:
        raise ValueError("pool must be bfloat16 (or wrapped in Fp8Pool)")
    return kv_pool_desc(data.data_ptr(), nb, hkv, bs, d, KV_DTYPE_BF16, 1.0, 1.0)


def kv_block_bytes(pool) -> int:
    return int(load().kv_block_bytes(ctypes.byref(pool_desc(pool))))


def kv_decode_workgroups(batch, num_kv_heads, max_context_len, num_workgroups=0) -> int:
    return int(load().kv_decode_workgroups(batch, num_kv_heads, max_context_len, num_workgroups))


def kv_decode_workspace_bytes(batch, num_q_heads, num_kv_heads, head_dim, max_context_len,
                              num_workgroups=0) -> int:
    return int(load().kv_decode_workspace_bytes(batch, num_q_heads, num_kv_heads, head_dim,
                                                max_context_len, num_workgroups))


def kv_decode_attn(out, q, pool, block_table, context_lens, max_context_len, scale,
                   num_workgroups=0, workspace=None, stream=None) -> None:
    """Enqueue paged decode attention; ``out`` ([B][Hq][D], bf16 or fp32) is written in place."""
    _dev(q, "q", torch.bfloat16)
    if q.dim() != 3 or q.shape[2] != _pool_data(pool).shape[4]:
        raise ValueError("q must be bf16 [batch][num_q_heads][head_dim of the pool]")
    batch, num_q_heads, _ = q.shape
    _dev(out, "out", (torch.bfloat16, torch.float32), shape=q.shape)
    _table(block_table, batch)
    _dev(context_lens, "context_lens", torch.int32, shape=(batch,))
    if workspace is not None:
        _dev(workspace, "workspace")
    out_dtype = {torch.bfloat16: KV_DTYPE_BF16, torch.float32: KV_DTYPE_F32}[out.dtype]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().kv_decode_attn(
        _ptr(out), out_dtype, _ptr(q), ctypes.byref(pool_desc(pool)), _ptr(block_table),
        block_table.shape[1], _ptr(context_lens), batch, num_q_heads, int(max_context_len),
        float(scale), int(num_workgroups), _ptr(workspace), ws_bytes, _stream_handle(stream)))


KV_DECODE_STATIC_SCRATCH_BYTES = 16 << 20


def kv_decode_attn_static(out, q, pool, block_table, context_lens, max_context_len, scale,
                          num_workgroups=0, stream=None) -> None:
    """kv_decode_attn with the library's fixed per-GPU scratch array as workspace (allocates nothing)."""
    _dev(q, "q", torch.bfloat16)
    if q.dim() != 3 or q.shape[2] != _pool_data(pool).shape[4]:
        raise ValueError("q must be bf16 [batch][num_q_heads][head_dim of the pool]")
    batch, num_q_heads, _ = q.shape
    _dev(out, "out", (torch.bfloat16, torch.float32), shape=q.shape)
    _table(block_table, batch)
    _dev(context_lens, "context_lens", torch.int32, shape=(batch,))
    out_dtype = {torch.bfloat16: KV_DTYPE_BF16, torch.float32: KV_DTYPE_F32}[out.dtype]
    _check(load().kv_decode_attn_static(
        _ptr(out), out_dtype, _ptr(q), ctypes.byref(pool_desc(pool)), _ptr(block_table),
        block_table.shape[1], _ptr(context_lens), batch, num_q_heads, int(max_context_len),
        float(scale), int(num_workgroups), _stream_handle(stream)))


def kv_prefill_key_splits(batch, num_q_heads, num_kv_heads, max_q_len, max_context_len) -> int:
    return int(load().kv_prefill_key_splits(batch, num_q_heads, num_kv_heads, max_q_len, max_context_len))


def kv_prefill_workspace_bytes(total_q, num_q_heads, head_dim, key_splits) -> int:
    return int(load().kv_prefill_workspace_bytes(total_q, num_q_heads, head_dim, key_splits))


def kv_prefill_attn(out, q, pool, block_table, context_lens, q_starts, max_q_len, scale, key_splits=1,
                    workspace=None, stream=None) -> None:
    """Enqueue causal attention of the packed query tokens ``q`` ([T][Hq][D]) over the pool; ``out`` is
    written in place ([T][Hq][D], bf16 or fp32).  ``workspace`` is needed for key_splits > 1."""
    _dev(q, "q", torch.bfloat16)
    if q.dim() != 3 or q.shape[2] != _pool_data(pool).shape[4]:
        raise ValueError("q must be bf16 [total_q][num_q_heads][head_dim of the pool]")
    total_q, num_q_heads, _ = q.shape
    _dev(out, "out", (torch.bfloat16, torch.float32), shape=q.shape)
    _dev(context_lens, "context_lens", torch.int32)
    batch = context_lens.numel()
    _table(block_table, batch)
    _dev(q_starts, "q_starts", torch.int32, shape=(batch + 1,))
    if workspace is not None:
        _dev(workspace, "workspace")
    out_dtype = {torch.bfloat16: KV_DTYPE_BF16, torch.float32: KV_DTYPE_F32}[out.dtype]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().kv_prefill_attn(
        _ptr(out), out_dtype, _ptr(q), ctypes.byref(pool_desc(pool)), _ptr(block_table),
        block_table.shape[1], _ptr(context_lens), _ptr(q_starts), context_lens.numel(), num_q_heads,
        int(max_q_len), int(total_q), float(scale), int(key_splits), _ptr(workspace), ws_bytes,
        _stream_handle(stream)))


def kv_pack_blocks(replica, pool, block_ids, n=None, stream=None) -> None:
    """Enqueue replica[i] <- pool[block_ids[i]] for i < n (default: all of block_ids)."""
    n = block_ids.numel() if n is None else int(n)
    _dev(block_ids, "block_ids", torch.int32, numel=n)
    _replica(replica, pool, n)
    _check(load().kv_pack_blocks(_ptr(replica), ctypes.byref(pool_desc(pool)), _ptr(block_ids), n,
                                 _stream_handle(stream)))


def kv_restore_blocks(pool, replica, block_ids, n=None, stream=None) -> None:
    """Enqueue pool[block_ids[i]] <- replica[i] for i < n (ids pairwise distinct)."""
    n = block_ids.numel() if n is None else int(n)
    _dev(block_ids, "block_ids", torch.int32, numel=n)
    _replica(replica, pool, n)
    _check(load().kv_restore_blocks(ctypes.byref(pool_desc(pool)), _ptr(replica), _ptr(block_ids), n,
                                    _stream_handle(stream)))


def kv_pack_blocks_staged(dst, pool, block_ids, staging, chunk_blocks, pack_stream, copy_stream, n=None) -> None:
    """Enqueue dst[i] <- pool[block_ids[i]] through the double-buffered device staging area: packs on
    pack_stream, copies of the packed chunks to dst (pinned host memory or a peer's buffer) on copy_stream."""
    n = block_ids.numel() if n is None else int(n)
    _dev(block_ids, "block_ids", torch.int32, numel=n)
    _replica(dst, pool, n, "dst")
    _replica(_dev(staging, "staging"), pool, 2 * int(chunk_blocks), "staging")
    _check(load().kv_pack_blocks_staged(_ptr(dst), ctypes.byref(pool_desc(pool)), _ptr(block_ids), n, _ptr(staging),
                                        int(chunk_blocks), _stream_handle(pack_stream), _stream_handle(copy_stream)))


def kv_pack_blocks_counted(replica, pool, block_ids, count, max_n=None, stream=None) -> None:
    """Enqueue replica[i] <- pool[block_ids[i]] for i < min(count[0], max_n); count lives on the device."""
    max_n = block_ids.numel() if max_n is None else int(max_n)
    _dev(block_ids, "block_ids", torch.int32, numel=max_n)
    _dev(count, "count", torch.int32, numel=1)
    _replica(replica, pool, max_n)
    _check(load().kv_pack_blocks_counted(_ptr(replica), ctypes.byref(pool_desc(pool)), _ptr(block_ids),
                                         _ptr(count), max_n, _stream_handle(stream)))


def kv_append_tokens(pool, k_new, v_new, block_table, positions, dirty_bitmap, stream=None) -> None:
    """Enqueue the write of one new K/V token per sequence and the update of the dirty bitmap."""
    batch = _dev(positions, "positions", torch.int32).numel()
    _table(block_table, batch)
    _new_rows(pool, k_new, v_new, batch)
    _bitmap(dirty_bitmap, pool)
    _check(load().kv_append_tokens(ctypes.byref(pool_desc(pool)), _ptr(k_new), _ptr(v_new), _ptr(block_table),
                                   block_table.shape[1], _ptr(positions), positions.numel(),
                                   _ptr(dirty_bitmap), _stream_handle(stream)))


def kv_append_packed(pool, k_new, v_new, block_table, context_lens, q_starts, dirty_bitmap, stream=None) -> None:
    """Enqueue the write of every sequence's newest q_len K/V rows (packed, [T][Hkv][D]) and the update of
    the dirty bitmap; same conventions as kv_prefill_attn."""
    batch = _dev(context_lens, "context_lens", torch.int32).numel()
    _table(block_table, batch)
    _dev(q_starts, "q_starts", torch.int32, shape=(batch + 1,))
    _new_rows(pool, k_new, v_new, k_new.shape[0])
    _bitmap(dirty_bitmap, pool)
    _check(load().kv_append_packed(ctypes.byref(pool_desc(pool)), _ptr(k_new), _ptr(v_new), _ptr(block_table),
                                   block_table.shape[1], _ptr(context_lens), _ptr(q_starts), context_lens.numel(),
                                   k_new.shape[0], _ptr(dirty_bitmap), _stream_handle(stream)))


def kv_gather_tokens(k_out, v_out, pool, block_table, positions, stream=None) -> None:
    """Enqueue the copy of the K/V rows at positions[b] out of the pool into k_out[b], v_out[b]."""
    batch = _dev(positions, "positions", torch.int32).numel()
    _table(block_table, batch)
    _new_rows(pool, k_out, v_out, batch)
    _check(load().kv_gather_tokens(_ptr(k_out), _ptr(v_out), ctypes.byref(pool_desc(pool)), _ptr(block_table),
                                   block_table.shape[1], _ptr(positions), positions.numel(), _stream_handle(stream)))


def kv_collect_dirty(dirty_bitmap, num_blocks, dirty_ids, dirty_count, clear=True, stream=None) -> None:
    """Enqueue bitmap -> ascending id list (dirty_ids) and its length (dirty_count[0]), both on the device."""
    _dev(dirty_bitmap, "dirty_bitmap", (torch.int32, torch.uint32), numel=(int(num_blocks) + 31) // 32)
    _dev(dirty_ids, "dirty_ids", torch.int32)
    _dev(dirty_count, "dirty_count", torch.int32, numel=1)
    _check(load().kv_collect_dirty(_ptr(dirty_bitmap), int(num_blocks), _ptr(dirty_ids), dirty_ids.numel(),
                                   _ptr(dirty_count), int(bool(clear)), _stream_handle(stream)))


def kv_probe_stream(mode, a, b, nbytes, stream=None) -> None:
    """Enqueue one plain streaming kernel: mode 0 reads b, 1 writes a, 2 copies b to a (nbytes, multiple of 16)."""
    _check(load().kv_probe_stream(int(mode), _ptr(a), _ptr(b), int(nbytes), _stream_handle(stream)))


KV_PROBE_MATRIX_SINK_BYTES = 256 * 512 * 4


def kv_probe_matrix(mode, iters, sink, stream=None) -> None:
    """Enqueue the matrix-core / vector-ALU yardstick kernel (modes 0-5, see the header); sink: device tensor of
    at least KV_PROBE_MATRIX_SINK_BYTES bytes."""
    _dev(sink, "sink")
    _check(load().kv_probe_matrix(int(mode), int(iters), _ptr(sink), sink.numel() * sink.element_size(),
                                  _stream_handle(stream)))


def kv_validate_decode(pool, block_table, context_lens, max_context_len, stream=None) -> int:
    return int(load().kv_validate_decode(
        ctypes.byref(pool_desc(pool)), _ptr(block_table), block_table.shape[1], _ptr(context_lens),
        context_lens.numel(), int(max_context_len), _stream_handle(stream)))


def kv_validate_prefill(pool, block_table, context_lens, q_starts, max_q_len, total_q, stream=None) -> int:
    return int(load().kv_validate_prefill(
        ctypes.byref(pool_desc(pool)), _ptr(block_table), block_table.shape[1], _ptr(context_lens), _ptr(q_starts),
        context_lens.numel(), int(max_q_len), int(total_q), _stream_handle(stream)))


def kv_validate_block_ids(pool, block_ids, require_distinct=False, stream=None) -> int:
    return int(load().kv_validate_block_ids(
        ctypes.byref(pool_desc(pool)), _ptr(block_ids), block_ids.numel(), int(bool(require_distinct)),
        _stream_handle(stream)))
