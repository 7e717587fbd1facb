"""Seeded synthetic inputs for the paged KV-cache data path.

This module only draws random inputs and lays them out; it holds none of the
arithmetic of attention or of block replication, and it is the one module that
both the GPU tests/bench and the CPU oracle's callers use.

The paper (Sec. 4) drives its system with chat requests served by an 8B
Llama-family model; neither is reproduced here.  The cases below stand in for
the *shapes* of that workload: Llama-style grouped-query attention geometry,
block-paged caches with shuffled block tables, and uniform or log-normal
context-length mixes.  All values are bf16 draws of N(0, 1), kept as uint16 bit
patterns in numpy arrays.

Pool layout: [num_blocks][2][num_kv_heads][block_size][head_dim], axis 1 is
(K, V).  Unused pool blocks and unused tail slots are filled with random data
too, so that touching a wrong block shows up as a wrong result.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

_CHUNK_ELEMS = 1 << 22          # elements drawn per child generator
_GEN_THREADS = 8


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed_seq: np.random.SeedSequence, shape) -> np.ndarray:
    """bf16 bit patterns of N(0,1) draws, deterministic for (seed_seq, shape).

    The flat array is cut into fixed-size chunks, each drawn from its own child
    of ``seed_seq``, so the result does not depend on the number of threads.
    """
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.uint16)
    n_chunks = max(1, -(-n // _CHUNK_ELEMS))
    children = seed_seq.spawn(n_chunks)

    def fill(i):
        lo = i * _CHUNK_ELEMS
        hi = min(n, lo + _CHUNK_ELEMS)
        g = np.random.default_rng(children[i])
        out[lo:hi] = f32_to_bf16_bits(g.standard_normal(hi - lo, dtype=np.float32))

    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(_GEN_THREADS) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


def f32_to_fp8_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to OCP FP8 E4M3 (1-4-3, bias 7, no infinities; nearest, ties to even,
    magnitudes beyond 448 saturate to 448); returns uint8 bit patterns.  Inputs must be finite."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = np.signbit(x).astype(np.uint8) << 7
    a = np.minimum(np.abs(x).astype(np.float64), 448.0)
    code = np.zeros(a.shape, dtype=np.int64)
    sub = a < 2.0 ** -6                                   # subnormal range: steps of 2^-9
    code[sub] = np.rint(a[sub] * 2.0 ** 9).astype(np.int64)      # 8 is the smallest normal, as it should be
    nrm = ~sub
    frac, exp = np.frexp(a[nrm])                          # a = frac * 2^exp, frac in [0.5, 1)
    e = exp.astype(np.int64) - 1                          # a = (2 frac) * 2^e, 2 frac in [1, 2)
    m = np.rint((2.0 * frac - 1.0) * 8.0).astype(np.int64)
    carry = m == 8
    e = e + carry
    m = np.where(carry, 0, m)
    code[nrm] = np.minimum(((e + 7) << 3) | m, 0x7E)
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def fp8_e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Decode OCP FP8 E4M3 bit patterns (uint8) to float32 exactly (code 0x7F/0xFF -> NaN)."""
    b = np.ascontiguousarray(b, dtype=np.uint8).astype(np.int64)
    e, m = (b >> 3) & 15, b & 7
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(b & 0x80, -mag, mag).astype(np.float32)


def normal_fp8(seed_seq: np.random.SeedSequence, shape, scale: float = 1.0) -> np.ndarray:
    """FP8 E4M3 bit patterns of N(0,1) draws divided by ``scale`` (the value a consumer multiplies
    back in); chunked like normal_bf16, so the result does not depend on the thread count."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.uint8)
    n_chunks = max(1, -(-n // _CHUNK_ELEMS))
    children = seed_seq.spawn(n_chunks)

    def fill(i):
        lo = i * _CHUNK_ELEMS
        hi = min(n, lo + _CHUNK_ELEMS)
        g = np.random.default_rng(children[i])
        out[lo:hi] = f32_to_fp8_e4m3_bits(g.standard_normal(hi - lo, dtype=np.float32) / np.float32(scale))

    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(_GEN_THREADS) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


@dataclass
class Geometry:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    kv_elt_bytes: int = 2          # 2 = bf16 pool, 1 = FP8 E4M3 pool

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def block_elems(self) -> int:
        return 2 * self.num_kv_heads * self.block_size * self.head_dim

    @property
    def block_bytes(self) -> int:
        return self.kv_elt_bytes * self.block_elems

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.num_kv_heads * self.head_dim * self.kv_elt_bytes

    @property
    def scale(self) -> np.float32:
        return np.float32(1.0 / math.sqrt(self.head_dim))


@dataclass
class DecodeCase:
    """One batch of decode inputs over a block pool, plus a dirty-block list."""
    name: str
    geom: Geometry
    context_lens: np.ndarray            # int32 [B]
    block_table: np.ndarray             # int32 [B][MB], unused entries -1
    num_blocks: int
    q: np.ndarray                       # uint16 [B][Hq][D]
    pool: np.ndarray | None             # uint16 [NB][2][Hkv][bs][D] (None if not materialised)
    dirty_ids: np.ndarray               # int32 [n]
    in_use_ids: np.ndarray = field(default_factory=lambda: np.empty(0, np.int32))
    pool_seed: np.random.SeedSequence | None = None

    @property
    def batch(self) -> int:
        return len(self.context_lens)

    @property
    def max_blocks_per_seq(self) -> int:
        return self.block_table.shape[1]

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if len(self.context_lens) else 0

    @property
    def kv_bytes(self) -> int:
        """Bytes of cached K and V that one decode step has to read (valid tokens only)."""
        return int(self.context_lens.astype(np.int64).sum()) * self.geom.kv_bytes_per_token

    @property
    def pool_shape(self):
        g = self.geom
        return (self.num_blocks, 2, g.num_kv_heads, g.block_size, g.head_dim)


def blocks_needed(context_lens: np.ndarray, block_size: int) -> np.ndarray:
    return (context_lens.astype(np.int64) + block_size - 1) // block_size


def deal_block_table(context_lens, block_size, max_blocks_per_seq, phys_ids) -> np.ndarray:
    """Deal physical ids to sequences in order: sequence b gets the next nb_b ids."""
    nb = blocks_needed(context_lens, block_size)
    if nb.max(initial=0) > max_blocks_per_seq or nb.sum() > len(phys_ids):
        raise ValueError("block table row or id supply too small")
    table = np.full((len(context_lens), max_blocks_per_seq), -1, dtype=np.int32)
    pos = 0
    for b, n in enumerate(nb):
        table[b, :n] = phys_ids[pos:pos + n]
        pos += n
    return table


def make_decode_case(name, seed, geom: Geometry, context_lens, *, num_blocks=None,
                     max_blocks_per_seq=None, pool_factor=1.25, dirty="last",
                     n_dirty=None, materialise_pool=True, phys_id_source=None) -> DecodeCase:
    """Build a decode case from given context lengths.

    Random sub-streams are spawned from ``seed`` in a fixed order: permutation,
    q, pool, dirty list.  ``dirty`` selects the dirty-block list: "last" (the
    block holding each sequence's newest token), "fraction" (n_dirty distinct
    in-use blocks), "any" (n_dirty distinct ids from the whole pool).
    """
    ss_perm, ss_q, ss_pool, ss_dirty = np.random.SeedSequence(seed).spawn(4)
    context_lens = np.asarray(context_lens, dtype=np.int32)
    nb = blocks_needed(context_lens, geom.block_size)
    needed = int(nb.sum())
    if num_blocks is None:
        num_blocks = max(1, math.ceil(pool_factor * needed))
    if max_blocks_per_seq is None:
        max_blocks_per_seq = max(1, int(nb.max(initial=1)))
    if phys_id_source is None:
        perm = np.random.default_rng(ss_perm).permutation(num_blocks).astype(np.int32)
    else:
        src = np.asarray(phys_id_source, dtype=np.int32)
        perm = src[np.random.default_rng(ss_perm).permutation(len(src))]
    in_use = perm[:needed].copy()
    table = deal_block_table(context_lens, geom.block_size, max_blocks_per_seq, in_use)
    q = normal_bf16(ss_q, (len(context_lens), geom.num_q_heads, geom.head_dim))
    pool = None
    if materialise_pool:
        pshape = (num_blocks, 2, geom.num_kv_heads, geom.block_size, geom.head_dim)
        if geom.kv_elt_bytes == 1:
            # K and V are drawn as N(0,1) / scale; the consumer multiplies (k_scale, v_scale) back in
            pool = normal_fp8(ss_pool, pshape, FP8_KV_SCALE)
        else:
            pool = normal_bf16(ss_pool, pshape)
    rng_d = np.random.default_rng(ss_dirty)
    if dirty == "last":
        dirty_ids = np.array([table[b, n - 1] for b, n in enumerate(nb) if n > 0], dtype=np.int32)
    elif dirty == "fraction":
        dirty_ids = rng_d.choice(in_use, size=int(n_dirty), replace=False).astype(np.int32)
    elif dirty == "any":
        dirty_ids = rng_d.choice(num_blocks, size=int(n_dirty), replace=False).astype(np.int32)
    else:
        raise ValueError(dirty)
    return DecodeCase(name, geom, context_lens, table, int(num_blocks), q, pool, dirty_ids,
                      in_use, ss_pool)


def _uniform_lens(seed, batch, lo, hi) -> np.ndarray:
    """Integers uniform on [lo, hi], both ends included."""
    ss = np.random.SeedSequence([seed, 0x6C656E])
    return np.random.default_rng(ss).integers(lo, hi + 1, size=batch).astype(np.int32)


def _lognormal_lens(seed, batch, median, sigma, lo, hi) -> np.ndarray:
    ss = np.random.SeedSequence([seed, 0x6C656E])
    z = np.random.default_rng(ss).standard_normal(batch)
    return np.clip(np.rint(np.exp(math.log(median) + sigma * z)), lo, hi).astype(np.int32)


# ----------------------------------------------------------------------------------------------
# The five serving-shaped cases.  ``shrink`` divides the context-length range (and nothing else)
# so that the CPU oracle can cover a case completely in seconds; shrink=1 is the full size.
# ----------------------------------------------------------------------------------------------

def tiny(seed=0) -> DecodeCase:
    g = Geometry(8, 2, 64, 16)
    lens = _uniform_lens(seed, 4, 1, 256)
    return make_decode_case("tiny", seed, g, lens, num_blocks=128, max_blocks_per_seq=16,
                            dirty="any", n_dirty=32)


def llama8b_layer(seed=1, shrink=1) -> DecodeCase:
    g = Geometry(32, 8, 128, 16)
    lens = _uniform_lens(seed, 32, 512 // shrink, 4096 // shrink)
    return make_decode_case("llama8b_layer", seed, g, lens, max_blocks_per_seq=256 // shrink,
                            dirty="last")


def long_context(seed=2, shrink=1, materialise_pool=True, kv_elt_bytes=2) -> DecodeCase:
    g = Geometry(32, 8, 128, 16, kv_elt_bytes)
    lens = _uniform_lens(seed, 8, 16384 // shrink, 65536 // shrink)
    needed = int(blocks_needed(lens, g.block_size).sum())
    return make_decode_case("long_context", seed, g, lens, max_blocks_per_seq=4096 // shrink,
                            dirty="fraction", n_dirty=round(0.10 * needed),
                            materialise_pool=materialise_pool)


def replication_mix(seed=3, shrink=1, batch=128) -> DecodeCase:
    g = Geometry(64, 8, 128, 32)
    lens = _lognormal_lens(seed, batch, 1024 // shrink, 1.0, 16, 32768 // shrink)
    return make_decode_case("replication_mix", seed, g, lens, max_blocks_per_seq=1024 // shrink,
                            dirty="last")


@dataclass
class RecoveryCase:
    """A full replica to restore into a freshly shuffled pool, then a decode over it."""
    name: str
    geom: Geometry
    num_blocks: int
    restore_ids: np.ndarray             # int32 [num_blocks], a permutation: replica[i] -> pool[ids[i]]
    replica_seed: np.random.SeedSequence
    decode: DecodeCase                  # pool not materialised: it is the restored pool

    def replica_chunk(self, first_block: int, n_blocks: int) -> np.ndarray:
        """Blocks [first_block, first_block+n_blocks) of the replica, uint16 [n][2][Hkv][bs][D].

        Each run of REPLICA_CHUNK_BLOCKS blocks comes from its own child generator, so chunks
        can be produced independently and in any order.
        """
        g = self.geom
        cb = REPLICA_CHUNK_BLOCKS
        if first_block % cb:
            raise ValueError("first_block must be a multiple of REPLICA_CHUNK_BLOCKS")
        n_chunks = -(-self.num_blocks // cb)
        children = self.replica_seed.spawn(n_chunks)
        out = np.empty((n_blocks, 2, g.num_kv_heads, g.block_size, g.head_dim), dtype=np.uint16)
        lo = first_block

        def fill(c):
            a = c * cb
            z = min(self.num_blocks, a + cb, first_block + n_blocks)
            rng = np.random.default_rng(children[c])
            x = rng.standard_normal((min(self.num_blocks, a + cb) - a) * g.block_elems, dtype=np.float32)
            out[a - lo:z - lo] = f32_to_bf16_bits(x).reshape((-1,) + out.shape[1:])[:z - a]

        chunks = range(first_block // cb, -(-(first_block + n_blocks) // cb))
        with ThreadPoolExecutor(_GEN_THREADS) as ex:
            list(ex.map(fill, chunks))
        return out


REPLICA_CHUNK_BLOCKS = 256
# FP8 pools hold value / FP8_KV_SCALE; a power of two other than 1 so that a forgotten scale shows
FP8_KV_SCALE = 0.25


def recovery(seed=4, num_blocks=200_000, shrink=1, batch=64) -> RecoveryCase:
    g = Geometry(64, 8, 128, 16)
    ss_ids, ss_rep = np.random.SeedSequence([seed, 0x726563]).spawn(2)
    restore_ids = np.random.default_rng(ss_ids).permutation(num_blocks).astype(np.int32)
    lens = _uniform_lens(seed, batch, 1024 // shrink, 8192 // shrink)
    dec = make_decode_case("recovery_decode", seed, g, lens, num_blocks=num_blocks,
                           max_blocks_per_seq=512 // shrink, dirty="last",
                           materialise_pool=False, phys_id_source=restore_ids)
    return RecoveryCase("recovery", g, num_blocks, restore_ids, ss_rep, dec)


def materialise_recovered_pool(case: RecoveryCase, first_block=0, n_blocks=None) -> np.ndarray:
    """The pool a correct restore produces, built by plain numpy indexing (for small cases)."""
    n_blocks = case.num_blocks if n_blocks is None else n_blocks
    g = case.geom
    pool = np.zeros((case.num_blocks, 2, g.num_kv_heads, g.block_size, g.head_dim), dtype=np.uint16)
    pool[case.restore_ids[first_block:first_block + n_blocks]] = case.replica_chunk(first_block, n_blocks)
    return pool


# ----------------------------------------------------------------------------------------------
# Prefill / recomputation cases: many query tokens per sequence over the same kind of pool.
# ----------------------------------------------------------------------------------------------

@dataclass
class PrefillCase:
    """A decode case (pool, block table, context lengths) whose last q_lens[b] tokens are queries."""
    name: str
    kv: DecodeCase                      # kv.q is unused here
    q_lens: np.ndarray                  # int32 [B], q_lens[b] <= context_lens[b]
    q_starts: np.ndarray                # int32 [B + 1], exclusive prefix sum of q_lens
    q: np.ndarray                       # uint16 [T][Hq][D], T = q_starts[B]

    @property
    def geom(self) -> Geometry:
        return self.kv.geom

    @property
    def batch(self) -> int:
        return self.kv.batch

    @property
    def total_q(self) -> int:
        return int(self.q_starts[-1])

    @property
    def max_q_len(self) -> int:
        return int(self.q_lens.max()) if len(self.q_lens) else 0

    @property
    def pairs(self) -> int:
        """(query, key) pairs inside the causal mask, per query head."""
        L = self.kv.context_lens.astype(np.int64)
        n = self.q_lens.astype(np.int64)
        # query j of a sequence sees L - n + j + 1 keys
        return int((n * (L - n) + n * (n + 1) // 2).sum())

    @property
    def flops(self) -> int:
        """Multiply-adds of Q K^T and P V counted as 2 flops each."""
        g = self.geom
        return 4 * g.head_dim * g.num_q_heads * self.pairs


def make_prefill_case(name, seed, geom: Geometry, context_lens, q_lens, **kw) -> PrefillCase:
    kv = make_decode_case(name, seed, geom, context_lens, **kw)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    if q_lens.shape != kv.context_lens.shape or (q_lens < 0).any() or (q_lens > kv.context_lens).any():
        raise ValueError("q_lens must lie in [0, context_lens]")
    q_starts = np.zeros(len(q_lens) + 1, dtype=np.int32)
    np.cumsum(q_lens, out=q_starts[1:])
    ss_q = np.random.SeedSequence([seed, 0x7072656669])
    q = normal_bf16(ss_q, (int(q_starts[-1]), geom.num_q_heads, geom.head_dim))
    return PrefillCase(name, kv, q_lens, q_starts, q)


def prefill_tiny(seed=5) -> PrefillCase:
    """Small geometry; sequences recomputed in full, in part, by a single token, and not at all."""
    g = Geometry(8, 2, 64, 16)
    lens = np.array([97, 256, 1, 130, 64, 200], np.int32)
    q_lens = np.array([97, 100, 1, 1, 0, 65], np.int32)
    return make_prefill_case("prefill_tiny", seed, g, lens, q_lens, num_blocks=128, max_blocks_per_seq=16,
                             dirty="any", n_dirty=8)


def recompute(seed=6, shrink=1, batch=8, kv_elt_bytes=2) -> PrefillCase:
    """Whole sequences recomputed after their replicas were dropped: q_len = context length."""
    g = Geometry(32, 8, 128, 16, kv_elt_bytes)
    lens = _uniform_lens(seed, batch, 2048 // shrink, 8192 // shrink)
    return make_prefill_case("recompute", seed, g, lens, lens, max_blocks_per_seq=512 // shrink, dirty="last")


def chunked_recompute(seed=7, shrink=1, batch=8, chunk=2048) -> PrefillCase:
    """The newest ``chunk`` tokens of long sequences recomputed over a restored prefix."""
    g = Geometry(32, 8, 128, 16)
    lens = _uniform_lens(seed, batch, 16384 // shrink, 65536 // shrink)
    q_lens = np.minimum(lens, max(1, chunk // shrink)).astype(np.int32)
    return make_prefill_case("chunked_recompute", seed, g, lens, q_lens, max_blocks_per_seq=4096 // shrink,
                             dirty="last")


def short_chunk_recompute(seed=8) -> PrefillCase:
    """One request whose newest 256 tokens are recomputed over a 40 000-token restored prefix: few query
    tokens, so the work only fills the chip when the key range is cut into parts."""
    g = Geometry(32, 8, 128, 16)
    return make_prefill_case("short_chunk_recompute", seed, g, np.array([40_000], np.int32),
                             np.array([256], np.int32), max_blocks_per_seq=2500, dirty="last")
