"""Seeded synthetic inputs for the tiered-fetch workloads.

This package produces *inputs only*: payload bytes, block tables, residency
draws, sequence lengths and routing traces, shaped like the KV-offload and
expert-offload workloads of the Harvest paper (Sections 4.3-4.4 and 5.2-5.3).
It holds nothing of the fetch method (no directory, no gather) and is the one
module that both the CPU checker and the GPU library's tests may share.
Beside the generators live the harness's own pieces: the scenario drivers
(``scenarios``), the adapter that lets them drive the HIP library
(``hip_engine``) and a checksum with which long runs compare what the two
sides delivered without keeping it (``digest``).

All structure draws use numpy's counter-based Philox generator keyed by
(seed, stream); bulk payload bytes come from ``fill.c`` (splitmix64 on a
per-chunk key), so any chunk can be regenerated on its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

CLS_KV = 0
CLS_EXPERT = 1
CLS_APPEND = 2          # key space of the token rows appended during decode
NO_OBJECT = 0xFFFFFFFF

FILL_NORMAL = 0
FILL_TAG = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwlfill.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile fill.c and digest.c into libwlfill.so (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH,
             os.path.join(_HERE, "fill.c"), os.path.join(_HERE, "digest.c")])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.wl_chunk_key.restype = ctypes.c_uint64
        lib.wl_chunk_key.argtypes = [ctypes.c_uint64] + [ctypes.c_uint32] * 4
        lib.wl_fill_chunk_normal.restype = None
        lib.wl_fill_chunk_normal.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_void_p]
        lib.wl_fill_chunk_tag.restype = None
        lib.wl_fill_chunk_tag.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64] + [ctypes.c_uint32] * 4
        lib.wl_fill_pool.restype = None
        lib.wl_fill_pool.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_size_t,
                                     ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                     ctypes.c_int, ctypes.c_void_p, ctypes.c_uint32]
        _lib = lib
    return _lib


def rng(seed: int, *stream: int) -> np.random.Generator:
    """Philox generator keyed by (seed, stream...) - one independent stream per purpose."""
    key = np.random.SeedSequence([int(seed) & 0xFFFFFFFF, *[int(s) & 0xFFFFFFFF for s in stream]])
    return np.random.Generator(np.random.Philox(key))


_tables: dict[float, np.ndarray] = {}


def normal_table(sigma: float) -> np.ndarray:
    """bf16 bit patterns of sigma * Phi^-1((u + 0.5) / 65536), u = 0..65535 (round to nearest even)."""
    t = _tables.get(sigma)
    if t is None:
        from scipy.special import ndtri
        u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        f = (sigma * ndtri(u)).astype(np.float32)
        bits = f.view(np.uint32)
        bits = bits + 0x7FFF + ((bits >> 16) & 1)
        t = np.ascontiguousarray((bits >> 16).astype(np.uint16))
        _tables[sigma] = t
    return t


def fill_pool(pool_ptr: int, n_layers: int, n_slots: int, chunk_bytes: int, slot_object: np.ndarray,
              seed: int, cls: int, plane: int, mode: int = FILL_NORMAL, sigma: float = 1.0,
              layer_base: int = 0) -> None:
    """Fill a pool plane laid out [layer][slot][chunk_bytes] at raw address ``pool_ptr``.

    ``slot_object[s]`` is the object whose bytes go to slot s (NO_OBJECT = leave untouched); the buffer's first
    layer is model layer ``layer_base``.
    """
    assert chunk_bytes % 16 == 0
    so = np.ascontiguousarray(slot_object, dtype=np.uint32)
    assert so.shape == (n_slots,)
    table = normal_table(sigma) if mode == FILL_NORMAL else None
    _load().wl_fill_pool(ctypes.c_void_p(pool_ptr), n_layers, n_slots, chunk_bytes,
                         so.ctypes.data_as(ctypes.c_void_p), ctypes.c_uint64(seed & (2**64 - 1)), cls, plane, mode,
                         table.ctypes.data_as(ctypes.c_void_p) if table is not None else None, layer_base)


def fill_array(arr: np.ndarray, slot_object, seed: int, cls: int, plane: int,
               mode: int = FILL_NORMAL, sigma: float = 1.0, layer_base: int = 0) -> None:
    """fill_pool on a C-contiguous uint8 array of shape [n_layers, n_slots, chunk_bytes]."""
    assert arr.dtype == np.uint8 and arr.flags.c_contiguous and arr.ndim == 3
    fill_pool(arr.ctypes.data, arr.shape[0], arr.shape[1], arr.shape[2], slot_object, seed, cls, plane, mode, sigma,
              layer_base)


def chunk(seed: int, cls: int, plane: int, layer: int, obj: int, chunk_bytes: int,
          mode: int = FILL_NORMAL, sigma: float = 1.0) -> np.ndarray:
    """Regenerate the bytes of one chunk (same bytes fill_pool writes for that object)."""
    out = np.empty(chunk_bytes, dtype=np.uint8)
    lib = _load()
    if mode == FILL_NORMAL:
        key = lib.wl_chunk_key(ctypes.c_uint64(seed & (2**64 - 1)), cls, plane, layer, obj)
        t = normal_table(sigma)
        lib.wl_fill_chunk_normal(out.ctypes.data_as(ctypes.c_void_p), chunk_bytes // 2, ctypes.c_uint64(key),
                                 t.ctypes.data_as(ctypes.c_void_p))
    else:
        lib.wl_fill_chunk_tag(out.ctypes.data_as(ctypes.c_void_p), chunk_bytes, ctypes.c_uint64(seed & (2**64 - 1)),
                              cls, plane, layer, obj)
    return out


def check_tag(buf: np.ndarray, seed: int, cls: int, plane: int, layer: int, obj: int) -> bool:
    """True iff ``buf`` (uint8, multiple of 16 bytes) is exactly the tag chunk of that object."""
    return bool(np.array_equal(buf, chunk(seed, cls, plane, layer, obj, buf.size, FILL_TAG)))


# ----------------------------------------------------------------------------
# KV workloads (paged KV blocks of decoding sequences; Section 5.2)
# ----------------------------------------------------------------------------

@dataclass
class KVShape:
    n_layers: int = 32
    block_tokens: int = 16
    n_kv_heads: int = 8
    head_dim: int = 128
    elt_bytes: int = 2

    @property
    def row_bytes(self) -> int:          # one token's K (or V) row in one layer
        return self.n_kv_heads * self.head_dim * self.elt_bytes

    @property
    def chunk_bytes(self) -> int:        # one block's K (or V) in one layer
        return self.block_tokens * self.row_bytes


@dataclass
class KVWorkload:
    """Object numbering: closed blocks 0..C-1, then the open tail of each sequence, then the blocks that decode steps
    open, in the order they are opened - i.e. the order in which a harness registers them."""
    shape: KVShape
    seed: int
    seq_lens: np.ndarray                 # tokens per sequence at step 0
    n_objects: int                       # logical blocks, including those that decode steps will open
    tables: list                         # per sequence: int32 block numbers in order; with has_tails the last is the open tail
    has_tails: bool
    future_blocks: list                  # per sequence: numbers of the blocks opened by later steps
    host_slot: np.ndarray                # int64[n_objects]: a seeded permutation, so host slot != block number
    resident: np.ndarray                 # bool[n_objects]: goes to the cache tier once the block is closed
    place_order: np.ndarray              # closed blocks with resident=True, in the seeded order they are placed
    p_cache: float
    fill_mode: int = FILL_NORMAL
    sigma: float = 1.0

    @property
    def n_seq(self) -> int:
        return len(self.tables)

    @property
    def n_closed(self) -> int:
        """Blocks that exist, closed, at step 0 (for the tiny config: the whole pool, requested or not)."""
        return self.n_objects - (self.n_seq if self.has_tails else 0) - sum(len(f) for f in self.future_blocks)

    def n_blocks(self) -> np.ndarray:
        return np.array([len(t) for t in self.tables], dtype=np.int32)


def kv_tiny(seed: int = 0, fill_mode: int = FILL_NORMAL) -> KVWorkload:
    """Tiny KV fetch: 1 layer, 16 sequences x 256 tokens, 1024-block pool, exactly 60% in the cache tier."""
    shape = KVShape(n_layers=1)
    n_pool, n_seq, per_seq = 1024, 16, 16
    perm = rng(seed, 1).permutation(n_pool).astype(np.int32)
    tables = [perm[s * per_seq:(s + 1) * per_seq].copy() for s in range(n_seq)]
    order = rng(seed, 2).permutation(n_pool).astype(np.int32)
    n_res = int(round(0.6 * n_pool))
    resident = np.zeros(n_pool, dtype=bool)
    resident[order[:n_res]] = True
    return KVWorkload(shape=shape, seed=seed, seq_lens=np.full(n_seq, 256, dtype=np.int64), n_objects=n_pool,
                      tables=tables, has_tails=False, future_blocks=[np.zeros(0, np.int32) for _ in range(n_seq)],
                      host_slot=rng(seed, 3).permutation(n_pool).astype(np.int64),
                      resident=resident, place_order=order[:n_res].copy(), p_cache=0.6, fill_mode=fill_mode)


def kv_decode(seed: int = 0, n_layers: int = 32, n_seq: int = 4, min_len: int = 32768, max_len: int = 131072,
              p_cache: float = 0.7, n_steps: int = 200, fill_mode: int = FILL_NORMAL,
              shape: KVShape | None = None, placement: str = "shuffled") -> KVWorkload:
    """Long-context decode: sequence lengths ~U[min_len, max_len], blocks i.i.d. Bernoulli(p_cache) in the cache tier.

    ``placement``: the order in which the resident blocks are placed at start, which (slots being handed out lowest
    first) decides where they sit in the cache tier - "shuffled" (default: a seeded permutation, so a sequence's blocks
    are scattered over the pool) or "in_sequence_order" (sequence after sequence in block order, as a prefill that
    offloads one prompt after the other would leave them: a sequence's blocks are neighbours).

    Every sequence ends in an open tail block (local tier) that decode steps append to.  A step appends one token
    per sequence; a tail that becomes full is closed and a new one opened, so the blocks opened during ``n_steps``
    steps are numbered here in (step, sequence) order.
    """
    shape = shape or KVShape(n_layers=n_layers)
    bt = shape.block_tokens
    lens = rng(seed, 10).integers(min_len, max_len + 1, size=n_seq).astype(np.int64)
    n_closed = [int(l // bt) for l in lens]             # a length that is a multiple of bt owns an empty open tail
    C = sum(n_closed)
    perm = rng(seed, 11).permutation(C).astype(np.int32)
    tables, at = [], 0
    for s, nc in enumerate(n_closed):
        tables.append(np.concatenate([perm[at:at + nc], np.array([C + s], np.int32)])); at += nc
    future = [[] for _ in range(n_seq)]
    nxt = C + n_seq
    for t in range(n_steps):
        for s in range(n_seq):
            if (lens[s] + t + 1) % bt == 0:
                future[s].append(nxt); nxt += 1
    total = nxt
    resident = rng(seed, 12).random(total) < p_cache
    if placement == "shuffled":
        order = rng(seed, 13).permutation(C).astype(np.int32)
    elif placement == "in_sequence_order":
        order = np.concatenate([t[:-1] for t in tables]).astype(np.int32)
    else:
        raise ValueError(placement)
    place_order = order[resident[order]]
    return KVWorkload(shape=shape, seed=seed, seq_lens=lens, n_objects=total, tables=tables, has_tails=True,
                      future_blocks=[np.array(f, np.int32) for f in future],
                      host_slot=rng(seed, 14).permutation(total).astype(np.int64),
                      resident=resident, place_order=place_order, p_cache=p_cache, fill_mode=fill_mode)


def append_rows(wl: KVWorkload, step: int, seq: int) -> np.ndarray:
    """K and V rows of the token that sequence ``seq`` appends at ``step``: uint8 [2 planes][n_layers][row_bytes]."""
    sh = wl.shape
    out = np.empty((2, sh.n_layers, sh.row_bytes), dtype=np.uint8)
    for p in range(2):
        for l in range(sh.n_layers):
            out[p, l] = chunk(wl.seed, CLS_APPEND, p, l, step * 65536 + seq, sh.row_bytes, wl.fill_mode, wl.sigma)
    return out


# ----------------------------------------------------------------------------
# Expert workloads (MoE expert weight matrices; Sections 4.1-4.4)
# ----------------------------------------------------------------------------

@dataclass
class ExpertShape:
    n_layers: int = 32
    n_experts: int = 16
    d_model: int = 4096
    d_ff: int = 6400
    n_mats: int = 3                      # gate, up, down stored back to back
    elt_bytes: int = 2

    @property
    def chunk_bytes(self) -> int:        # one whole expert
        return self.n_mats * self.d_model * self.d_ff * self.elt_bytes


@dataclass
class ExpertWorkload:
    shape: ExpertShape
    seed: int
    n_tokens: int
    top_k: int
    zipf_s: float
    tier0: np.ndarray                    # int8 [n_layers][n_experts]: 2 = local, 1 = cache tier, 0 = host only
    place_order: np.ndarray              # object ids (layer * n_experts + e) with tier0 == 1, seeded order
    rank_to_expert: np.ndarray           # int32 [n_layers][n_experts]
    lru_capacity: int = 0                # > 0: cache tier filled by a per-layer LRU policy instead of tier0
    fill_mode: int = FILL_NORMAL
    sigma: float = 0.02

    @property
    def n_objects(self) -> int:
        return self.shape.n_layers * self.shape.n_experts

    def routing(self, step: int, layer: int) -> np.ndarray:
        """top-k expert ids int32 [n_tokens][k]: each token draws k distinct experts, sequentially, with
        probability proportional to rank^-s (renormalised after each draw)."""
        E, k, T = self.shape.n_experts, self.top_k, self.n_tokens
        g = rng(self.seed, 30, step, layer)
        w = np.tile(np.arange(1, E + 1, dtype=np.float64) ** (-self.zipf_s), (T, 1))
        ranks = np.empty((T, k), dtype=np.int64)
        u = g.random((T, k))
        for j in range(k):
            c = np.cumsum(w, axis=1)
            r = (c < (u[:, j] * c[:, -1])[:, None]).sum(axis=1)
            r = np.minimum(r, E - 1)
            # guard against a zero-weight hit at a boundary: move right to the next live rank
            for t in np.nonzero(w[np.arange(T), r] == 0.0)[0]:
                live = np.nonzero(w[t] > 0)[0]
                r[t] = live[np.searchsorted(live, r[t]) % live.size]
            ranks[:, j] = r
            w[np.arange(T), r] = 0.0
        return self.rank_to_expert[layer][ranks].astype(np.int32)


def expert_offload(seed: int = 0, shape: ExpertShape | None = None, n_tokens: int = 64, top_k: int = 2,
                   zipf_s: float = 1.1, n_local: int = 2, p_cache: float = 0.5,
                   fill_mode: int = FILL_NORMAL) -> ExpertWorkload:
    """Phi-3.5-MoE-shaped expert fetch: n_local experts per layer local, Bernoulli(p_cache) of the rest cached."""
    shape = shape or ExpertShape()
    L, E = shape.n_layers, shape.n_experts
    tier0 = np.zeros((L, E), dtype=np.int8)
    r2e = np.empty((L, E), dtype=np.int32)
    for l in range(L):
        r2e[l] = rng(seed, 20, l).permutation(E)
        loc = rng(seed, 21, l).permutation(E)[:n_local]
        tier0[l, loc] = 2
        draw = rng(seed, 22, l).random(E) < p_cache
        tier0[l, (tier0[l] == 0) & draw] = 1
    ids = np.nonzero(tier0.reshape(-1) == 1)[0].astype(np.int32)
    order = ids[rng(seed, 23).permutation(ids.size)]
    return ExpertWorkload(shape=shape, seed=seed, n_tokens=n_tokens, top_k=top_k, zipf_s=zipf_s, tier0=tier0,
                          place_order=order, rank_to_expert=r2e, fill_mode=fill_mode)


def expert_lru(seed: int = 0, shape: ExpertShape | None = None, n_tokens: int = 256, top_k: int = 4,
               zipf_s: float = 1.0, capacity_frac: float = 0.4, fill_mode: int = FILL_NORMAL) -> ExpertWorkload:
    """Qwen-MoE-shaped fetch: many small experts, cache tier limited to capacity_frac of each layer's experts and
    filled by an LRU policy driven by the routing trace (no local experts, cache starts empty)."""
    shape = shape or ExpertShape(n_layers=24, n_experts=60, d_model=2048, d_ff=1408)
    L, E = shape.n_layers, shape.n_experts
    r2e = np.stack([rng(seed, 20, l).permutation(E) for l in range(L)]).astype(np.int32)
    return ExpertWorkload(shape=shape, seed=seed, n_tokens=n_tokens, top_k=top_k, zipf_s=zipf_s,
                          tier0=np.zeros((L, E), dtype=np.int8), place_order=np.zeros(0, np.int32),
                          rank_to_expert=r2e, lru_capacity=int(np.floor(capacity_frac * E)), fill_mode=fill_mode)


class LRU:
    """Least-recently-used set of fixed capacity (policy code of the harness, not of the library)."""

    def __init__(self, capacity: int):
        from collections import OrderedDict
        self.capacity = capacity
        self._d = OrderedDict()

    def touch(self, key: int) -> None:
        if key in self._d:
            self._d.move_to_end(key)
        else:
            if len(self._d) >= self.capacity:
                self._d.popitem(last=False)
            self._d[key] = True

    def members(self) -> set:
        return set(self._d.keys())


def revoke_draw(seed: int, step: int, cls: int, live_ids, frac: float = 0.25) -> np.ndarray:
    """Seeded choice of round(frac * n) of the live cache-tier allocations (ids are sorted first so the draw
    does not depend on the container's iteration order)."""
    live = np.array(sorted(int(i) for i in live_ids), dtype=np.int32)
    n = int(round(frac * live.size))
    if n == 0:
        return np.zeros(0, np.int32)
    return live[rng(seed, 40, step, cls).permutation(live.size)[:n]]
