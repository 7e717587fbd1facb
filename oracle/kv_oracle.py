"""ctypes front end of the C oracle in ``kv_oracle.c`` (test infrastructure only).

The arithmetic lives in the C file; this module only compiles it with gcc,
marshals numpy arrays and turns error codes into exceptions.  bf16 tensors are
numpy ``uint16`` arrays holding the bit patterns.

Operations (paper Sec. 3.2 item 3, Background KV Cache Replication):
``decode_attn``  attention of one query token per sequence over a block-paged cache;
``prefill_attn`` causal attention of many query tokens per sequence over the same cache (recomputation);
``pack_blocks``  replica[i] <- pool[ids[i]] (block-by-block replication, gather side);
``restore_blocks`` pool[ids[i]] <- replica[i] (continuing from the replicated state).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kv_oracle.c")
_LIB = os.path.join(_HERE, "libkv_oracle.so")
_lib = None

_ERRORS = {
    -2: "bad shape argument",
    -3: "context length negative or beyond the block-table row",
    -4: "physical block id out of range",
    -5: "duplicate block id in a restore list",
    -6: "out of host memory",
}


class OracleError(RuntimeError):
    pass


def build(force: bool = False) -> str:
    """Compile kv_oracle.c into libkv_oracle.so next to it and return the path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.kvo_decode_attn.restype = ctypes.c_int
        lib.kvo_decode_attn.argtypes = [
            f64p, u16p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_float,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            i32p, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_float,
            i32p, ctypes.c_int64, ctypes.c_int]
        lib.kvo_prefill_attn.restype = ctypes.c_int
        lib.kvo_prefill_attn.argtypes = [
            f64p, u16p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_float,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            i32p, ctypes.c_int, i32p, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_float,
            i32p, ctypes.c_int64, ctypes.c_int]
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.kvo_append_tokens.restype = ctypes.c_int
        lib.kvo_append_tokens.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          u16p, u16p, i32p, ctypes.c_int, i32p, ctypes.c_int, u32p]
        lib.kvo_append_packed.restype = ctypes.c_int
        lib.kvo_append_packed.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          u16p, u16p, i32p, ctypes.c_int, i32p, i32p, ctypes.c_int, u32p]
        lib.kvo_gather_tokens.restype = ctypes.c_int
        lib.kvo_gather_tokens.argtypes = [u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          u16p, u16p, i32p, ctypes.c_int, i32p, ctypes.c_int]
        lib.kvo_collect_dirty.restype = ctypes.c_int64
        lib.kvo_collect_dirty.argtypes = [u32p, ctypes.c_int64, i32p, ctypes.c_int]
        for fn in (lib.kvo_pack_blocks, lib.kvo_restore_blocks):
            fn.restype = ctypes.c_int
            fn.argtypes = [u8p, u8p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int64, ctypes.c_int]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(rc: int) -> int:
    if rc < 0:
        raise OracleError(_ERRORS.get(rc, f"oracle error {rc}"))
    return rc


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def decode_attn(q, pool, block_table, context_lens, scale, rows=None, num_threads=0,
                return_threads=False, k_scale=1.0, v_scale=1.0):
    """fp64 paged decode attention.

    q            uint16 [B][Hq][D]              bf16 bit patterns
    pool         uint16 [NB][2][Hkv][bs][D]     bf16 bit patterns, axis 1: 0 = K, 1 = V; or uint8 of the
                                                same shape: FP8 E4M3 patterns, value = stored * k_scale
                                                (K) or * v_scale (V), scales rounded to fp32
    block_table  int32  [B][MB]                 logical -> physical block, unused entries ignored
    context_lens int32  [B]
    scale        python/np float; rounded to fp32 and then widened to double
    rows         optional int32 [n][2] of (b, h): compute only these rows -> [n][D]
    Returns float64 [B][Hq][D] (or [n][D]).
    """
    q = _c(q, np.uint16)
    pool = np.ascontiguousarray(pool)
    if pool.dtype not in (np.uint16, np.uint8):
        raise TypeError("pool must be uint16 (bf16) or uint8 (FP8 E4M3)")
    fp8 = pool.dtype == np.uint8
    block_table = _c(block_table, np.int32)
    context_lens = _c(context_lens, np.int32)
    B, Hq, D = q.shape
    NB, two, Hkv, bs, D2 = pool.shape
    if two != 2 or D2 != D or block_table.shape[0] != B or context_lens.shape != (B,):
        raise OracleError("inconsistent shapes")
    if rows is None:
        out = np.empty((B, Hq, D), dtype=np.float64)
        rows_p, n_rows = None, 0
    else:
        rows = _c(rows, np.int32).reshape(-1, 2)
        if len(rows) and (rows.min() < 0 or rows[:, 0].max() >= B or rows[:, 1].max() >= Hq):
            raise OracleError("row index out of range")
        out = np.empty((len(rows), D), dtype=np.float64)
        rows_p, n_rows = _ptr(rows, ctypes.c_int32), len(rows)
    used = _check(_load().kvo_decode_attn(
        _ptr(out, ctypes.c_double), _ptr(q, ctypes.c_uint16), pool.ctypes.data_as(ctypes.c_void_p),
        int(fp8), float(np.float32(k_scale)), float(np.float32(v_scale)), NB, Hkv, bs, D, _ptr(block_table, ctypes.c_int32), block_table.shape[1],
        _ptr(context_lens, ctypes.c_int32), B, Hq, float(np.float32(scale)),
        rows_p, n_rows, int(num_threads)))
    return (out, used) if return_threads else out


def prefill_attn(q, pool, block_table, context_lens, q_starts, scale, rows=None, num_threads=0,
                 return_threads=False, k_scale=1.0, v_scale=1.0):
    """fp64 causal attention of many query tokens per sequence over the block-paged cache.

    q            uint16 [T][Hq][D]   bf16 bit patterns; the query tokens of all sequences, packed in batch order
    pool, block_table, context_lens, scale, k_scale, v_scale   as for decode_attn; context_lens[b] counts
                 the query tokens too (their K/V rows are in the pool already)
    q_starts     int32 [B + 1]       q_starts[b] = first packed row of sequence b; q_starts[B] = T
    rows         optional int32 [n][2] of (t, h), t a packed token index: compute only these -> [n][D]
    Query token j of sequence b is at position context_lens[b] - q_len_b + j and sees keys 0 .. position.
    Returns float64 [T][Hq][D] (or [n][D]).
    """
    q = _c(q, np.uint16)
    pool = np.ascontiguousarray(pool)
    if pool.dtype not in (np.uint16, np.uint8):
        raise TypeError("pool must be uint16 (bf16) or uint8 (FP8 E4M3)")
    fp8 = pool.dtype == np.uint8
    block_table = _c(block_table, np.int32)
    context_lens = _c(context_lens, np.int32)
    q_starts = _c(q_starts, np.int32)
    T, Hq, D = q.shape
    NB, two, Hkv, bs, D2 = pool.shape
    B = len(context_lens)
    if two != 2 or D2 != D or block_table.shape[0] != B or q_starts.shape != (B + 1,) or int(q_starts[B]) != T:
        raise OracleError("inconsistent shapes")
    if rows is None:
        out = np.empty((T, Hq, D), dtype=np.float64)
        rows_p, n_rows = None, 0
    else:
        rows = _c(rows, np.int32).reshape(-1, 2)
        if len(rows) and (rows.min() < 0 or rows[:, 0].max() >= T or rows[:, 1].max() >= Hq):
            raise OracleError("row index out of range")
        out = np.empty((len(rows), D), dtype=np.float64)
        rows_p, n_rows = _ptr(rows, ctypes.c_int32), len(rows)
    used = _check(_load().kvo_prefill_attn(
        _ptr(out, ctypes.c_double), _ptr(q, ctypes.c_uint16), pool.ctypes.data_as(ctypes.c_void_p),
        int(fp8), float(np.float32(k_scale)), float(np.float32(v_scale)), NB, Hkv, bs, D,
        _ptr(block_table, ctypes.c_int32), block_table.shape[1], _ptr(context_lens, ctypes.c_int32),
        _ptr(q_starts, ctypes.c_int32), B, Hq, float(np.float32(scale)), rows_p, n_rows, int(num_threads)))
    return (out, used) if return_threads else out


def _as_bytes(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(a.shape[0], -1)


def pack_blocks(pool, ids, num_threads=0, return_threads=False):
    """replica[i] <- pool[ids[i]].  pool is [NB][...] of any dtype; returns [n][...] of the same."""
    pool = np.ascontiguousarray(pool)
    ids = _c(ids, np.int32).reshape(-1)
    pb = _as_bytes(pool)
    replica = np.empty((len(ids),) + pool.shape[1:], dtype=pool.dtype)
    rb = _as_bytes(replica) if len(ids) else replica.view(np.uint8)
    used = _check(_load().kvo_pack_blocks(
        _ptr(rb, ctypes.c_uint8), _ptr(pb, ctypes.c_uint8), pb.shape[1], pb.shape[0],
        _ptr(ids, ctypes.c_int32), len(ids), int(num_threads)))
    return (replica, used) if return_threads else replica


def restore_blocks(pool, replica, ids, num_threads=0, return_threads=False):
    """pool[ids[i]] <- replica[i], in place on the (C-contiguous, writable) pool array."""
    if not (pool.flags.c_contiguous and pool.flags.writeable):
        raise OracleError("pool must be C-contiguous and writable")
    replica = np.ascontiguousarray(replica)
    ids = _c(ids, np.int32).reshape(-1)
    pb = _as_bytes(pool)
    if len(ids) != replica.shape[0] or (len(ids) and replica[0].nbytes != pb.shape[1]):
        raise OracleError("replica does not match the id list / block size")
    rb = replica.view(np.uint8)
    used = _check(_load().kvo_restore_blocks(
        _ptr(pb, ctypes.c_uint8), _ptr(rb, ctypes.c_uint8), pb.shape[1], pb.shape[0],
        _ptr(ids, ctypes.c_int32), len(ids), int(num_threads)))
    return used if return_threads else None


def bitmap_words(num_blocks: int) -> int:
    return (int(num_blocks) + 31) // 32


def append_tokens(pool, k_new, v_new, block_table, positions, dirty_bitmap):
    """Write one new token per sequence into the pool (in place) and OR its block into dirty_bitmap.

    pool uint16 [NB][2][Hkv][bs][D] (writable), k_new/v_new uint16 [B][Hkv][D], positions int32 [B]
    (< 0: no token for that sequence), dirty_bitmap uint32 [ceil(NB/32)] (in place).
    """
    if not (pool.flags.c_contiguous and pool.flags.writeable and pool.dtype == np.uint16):
        raise OracleError("pool must be a writable C-contiguous uint16 array")
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    block_table, positions = _c(block_table, np.int32), _c(positions, np.int32)
    if not (dirty_bitmap.flags.c_contiguous and dirty_bitmap.dtype == np.uint32):
        raise OracleError("dirty_bitmap must be a C-contiguous uint32 array")
    NB, two, Hkv, bs, D = pool.shape
    B = len(positions)
    if k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D) or block_table.shape[0] != B \
            or len(dirty_bitmap) != bitmap_words(NB):
        raise OracleError("inconsistent shapes")
    _check(_load().kvo_append_tokens(
        _ptr(pool, ctypes.c_uint16), NB, Hkv, bs, D, _ptr(k_new, ctypes.c_uint16), _ptr(v_new, ctypes.c_uint16),
        _ptr(block_table, ctypes.c_int32), block_table.shape[1], _ptr(positions, ctypes.c_int32), B,
        _ptr(dirty_bitmap, ctypes.c_uint32)))


def append_packed(pool, k_new, v_new, block_table, context_lens, q_starts, dirty_bitmap):
    """Write the K/V rows of every sequence's newest q_len tokens into the pool (in place) and OR their
    blocks into dirty_bitmap: the step before prefill_attn, same conventions.

    pool uint16 [NB][2][Hkv][bs][D] (writable), k_new/v_new uint16 [T][Hkv][D] packed in batch order,
    context_lens int32 [B] (counts the new tokens), q_starts int32 [B + 1].
    """
    if not (pool.flags.c_contiguous and pool.flags.writeable and pool.dtype == np.uint16):
        raise OracleError("pool must be a writable C-contiguous uint16 array")
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    block_table, context_lens = _c(block_table, np.int32), _c(context_lens, np.int32)
    q_starts = _c(q_starts, np.int32)
    if not (dirty_bitmap.flags.c_contiguous and dirty_bitmap.dtype == np.uint32):
        raise OracleError("dirty_bitmap must be a C-contiguous uint32 array")
    NB, two, Hkv, bs, D = pool.shape
    B = len(context_lens)
    T = int(q_starts[B]) if q_starts.shape == (B + 1,) else -1
    if k_new.shape != (T, Hkv, D) or v_new.shape != (T, Hkv, D) or block_table.shape[0] != B \
            or len(dirty_bitmap) != bitmap_words(NB):
        raise OracleError("inconsistent shapes")
    _check(_load().kvo_append_packed(
        _ptr(pool, ctypes.c_uint16), NB, Hkv, bs, D, _ptr(k_new, ctypes.c_uint16), _ptr(v_new, ctypes.c_uint16),
        _ptr(block_table, ctypes.c_int32), block_table.shape[1], _ptr(context_lens, ctypes.c_int32),
        _ptr(q_starts, ctypes.c_int32), B, _ptr(dirty_bitmap, ctypes.c_uint32)))


def collect_dirty(dirty_bitmap, num_blocks, clear=True):
    """Ascending ids of the blocks whose bit is set; clears the bitmap in place if asked."""
    if not (dirty_bitmap.flags.c_contiguous and dirty_bitmap.dtype == np.uint32
            and len(dirty_bitmap) == bitmap_words(num_blocks)):
        raise OracleError("dirty_bitmap must be a C-contiguous uint32 array of ceil(NB/32) words")
    ids = np.empty(int(num_blocks), dtype=np.int32)
    n = _load().kvo_collect_dirty(_ptr(dirty_bitmap, ctypes.c_uint32), int(num_blocks),
                                  _ptr(ids, ctypes.c_int32), int(bool(clear)))
    return ids[:n].copy()


def gather_tokens(pool, block_table, positions, k_out=None, v_out=None):
    """Copy the K/V rows of the tokens at positions[b] out of the pool: returns (k, v), each uint16
    [B][Hkv][D]; rows of sequences with positions[b] < 0 keep what k_out / v_out held (zeros by default)."""
    pool = _c(pool, np.uint16)
    block_table, positions = _c(block_table, np.int32), _c(positions, np.int32)
    NB, two, Hkv, bs, D = pool.shape
    B = len(positions)
    k_out = np.zeros((B, Hkv, D), np.uint16) if k_out is None else k_out
    v_out = np.zeros((B, Hkv, D), np.uint16) if v_out is None else v_out
    if k_out.shape != (B, Hkv, D) or v_out.shape != (B, Hkv, D) or block_table.shape[0] != B:
        raise OracleError("inconsistent shapes")
    _check(_load().kvo_gather_tokens(
        _ptr(pool, ctypes.c_uint16), NB, Hkv, bs, D, _ptr(k_out, ctypes.c_uint16), _ptr(v_out, ctypes.c_uint16),
        _ptr(block_table, ctypes.c_int32), block_table.shape[1], _ptr(positions, ctypes.c_int32), B))
    return k_out, v_out
