"""TEST INFRASTRUCTURE - adapts the CPU oracle to the harness interface the scenario drivers use.

``kv_layers`` restricts the KV class to a subset of model layers (layers are independent in every operation, so an
oracle that materialises only layer L is a complete oracle for the fetches of layer L); this keeps a full-size check
within host memory.  Calls that concern other layers are ignored.
"""
from __future__ import annotations

import numpy as np

import workloads as W
from workloads.digest import digest as _digest
from . import OracleClass, SegPool, HOST, CACHE, LOCAL, NONE, EVICT_DEMOTE, IN_PLACE, STAGED  # noqa: F401

KV, EXPERT = 0, 1


class OracleEngine:
    name = "oracle"

    def __init__(self, kv=None, expert=None, poison=False, kv_layers=None, threads=1, shared_cache_bytes=0,
                 shared_granule=0):
        """kv / expert: objects with n_layers, n_planes, chunk_bytes, max_objects, n_host_slots, n_cache_slots,
        n_local_slots (and n_experts).  shared_cache_bytes: a segment pool from which every class without cache slots
        of its own takes its cache-tier storage."""
        self.spec = {KV: kv, EXPERT: expert}
        self.pool = SegPool(shared_cache_bytes, shared_granule or 4096) if shared_cache_bytes else None
        # an object's segment holds all its layers: a layer subset would change every allocation
        assert not (self.pool and kv is not None and kv_layers is not None and kv.n_cache_slots == 0)
        self.threads = threads
        self.kv_layers = list(range(kv.n_layers)) if (kv is not None and kv_layers is None) else kv_layers
        self.c = {}
        for k, sp in self.spec.items():
            if sp is None:
                continue
            nl = len(self.kv_layers) if k == KV else sp.n_layers
            self.c[k] = OracleClass(nl, sp.n_planes, sp.chunk_bytes, sp.max_objects, sp.n_host_slots,
                                    sp.n_cache_slots, sp.n_local_slots, poison,
                                    segpool=self.pool if sp.n_cache_slots == 0 else None)

    def close(self):
        for c in self.c.values():
            c.close()
        if self.pool:
            self.pool.close()
            self.pool = None

    def shared_plane(self):
        return self.pool.mem()

    def shared_free_runs(self):
        return self.pool.free_runs()

    def _layers(self, cls):
        return self.kv_layers if cls == KV else list(range(self.spec[cls].n_layers))

    # ---- harness-side initialisation -----------------------------------------------------------------------
    def fill_host(self, cls, slot_object, seed, wl_cls, mode, sigma):
        self._fill(cls, HOST, slot_object, seed, wl_cls, mode, sigma)

    def fill_local(self, cls, slot_object, seed, wl_cls, mode, sigma):
        self._fill(cls, LOCAL, slot_object, seed, wl_cls, mode, sigma)

    def _fill(self, cls, tier, slot_object, seed, wl_cls, mode, sigma):
        c = self.c[cls]
        for p in range(c.n_planes):
            plane = c.plane(tier, p)
            for i, layer in enumerate(self._layers(cls)):      # chunks are keyed by their absolute layer number
                W.fill_array(plane[i:i + 1], slot_object, seed, wl_cls, p, mode, sigma, layer_base=layer)

    def adopt(self, cls, ids):
        self.c[cls].adopt(ids)

    def write_local(self, cls, obj, plane, layer, offset, data):
        if layer in self._layers(cls):
            self.c[cls].write_local(obj, plane, self._layers(cls).index(layer), offset, data)

    # ---- directory ---------------------------------------------------------------------------------------------
    def register(self, cls, n, host_slots=None, tier=HOST):
        return self.c[cls].register(n, host_slots, tier)

    def lookup(self, cls, obj):
        return self.c[cls].lookup(obj)

    def place(self, cls, ids):
        return self.c[cls].place(ids)

    def place_from(self, cls, ids, src0, src1, src_block, stride):
        """src planes: numpy uint8 [n_layers][stride][chunk]; object i sits at block src_block[i] of every layer."""
        assert cls != KV or self.kv_layers == list(range(self.spec[KV].n_layers))
        return self.c[cls].place_from(ids, src0, src1, src_block, stride)

    def last_staging(self):
        """The staging buffer of the latest expert fetch."""
        return self._last_expert_fetch[0]

    def revoke(self, cls, ids):
        c = self.c[cls]
        n0 = len(c.revoked_log)
        c.revoke(ids)
        return c.revoked_log[n0:]

    # ---- data path -------------------------------------------------------------------------------------------
    def has_layer(self, layer):
        return layer in self.kv_layers

    def fetch_kv_again(self, layer, dst_fill=0):
        """The latest single-layer fetch once more, for another layer: plainly a fetch with the same arguments."""
        form, args = self._last_kv
        if form == "token-major":
            return self.fetch_kv(layer, *args)
        return self.fetch_kv_head_major(layer, *args, dst_fill=dst_fill)

    def fetch_kv(self, layer, table, n_blocks, seq_dst_block, cap):
        """-> (k bytes, v bytes, sorted miss list, counts) as numpy / dict."""
        self._last_kv = ("token-major", (table, n_blocks, seq_dst_block, cap))
        c = self.c[KV]
        k, v, miss, counts = c.fetch_kv(self.kv_layers.index(layer), table, n_blocks, seq_dst_block, cap,
                                        threads=self.threads)
        return k, v, np.sort(miss), counts

    def fetch_kv_head_major(self, layer, table, n_blocks, seq_dst_block, seq_cap_blocks, cap, n_heads, block_tokens,
                            dst_fill=0):
        self._last_kv = ("head-major", (table, n_blocks, seq_dst_block, seq_cap_blocks, cap, n_heads, block_tokens))
        c = self.c[KV]
        n = cap * c.chunk_bytes
        k, v, miss, counts = c.fetch_kv_head_major(self.kv_layers.index(layer), table, n_blocks, seq_dst_block,
                                                   seq_cap_blocks, cap, n_heads, block_tokens,
                                                   dst_k=np.full(n, dst_fill, np.uint8), dst_v=np.full(n, dst_fill, np.uint8))
        return k, (v if c.n_planes == 2 else None), np.sort(miss), counts

    def fetch_experts(self, layer, topk, n_staging, digest=False):
        """-> (list over experts: None or the expert's bytes as the FFN would see them, kinds, sorted miss, counts).
        digest: the first element is the checksum of the staging slots in use instead (long runs at full size)."""
        c = self.c[EXPERT]
        E = self.spec[EXPERT].n_experts
        buf = None
        if digest:               # one staging buffer for the whole run: only the slots a fetch fills are looked at
            buf = getattr(self, "_staging_buf", None)
            if buf is None or buf.size != n_staging * c.chunk_bytes:
                buf = self._staging_buf = np.zeros(n_staging * c.chunk_bytes, dtype=np.uint8)
        staging, kind, where, miss, counts = c.fetch_experts(layer, E, topk, n_staging, staging=buf)
        self._last_expert_fetch = (staging, where, kind, layer)
        if digest:
            n_staged = int((kind == STAGED).sum())
            assert sorted(where[kind == STAGED]) == list(range(n_staged))
            return _digest(staging[:n_staged * c.chunk_bytes]), kind, where, np.sort(miss), counts
        out = []
        for e in range(E):
            if kind[e] == IN_PLACE:
                out.append(c.plane(LOCAL, 0)[0, where[e]].copy())
            elif kind[e] == STAGED:
                out.append(staging[where[e] * c.chunk_bytes:(where[e] + 1) * c.chunk_bytes].copy())
            else:
                out.append(None)
        return out, kind, where, np.sort(miss), counts

    # begin/end pairs: a CPU has nothing in flight, so "begin" does the work
    def fetch_kv_begin(self, *a, **k):
        return self.fetch_kv(*a, **k)

    def fetch_experts_begin(self, *a, **k):
        return self.fetch_experts(*a, **k)

    def fetch_end(self, handle, digest=False):
        if digest and len(handle) == 4:                  # a KV fetch: (k, v, miss, counts)
            k, v, miss, counts = handle
            return _digest(k), (None if v is None else _digest(v)), miss, counts
        return handle

    def evict(self, cls, layer, ids, src0, src1, src_block, stride, flags=0):
        """src planes: numpy uint8, [stride][chunk] (layer >= 0) or [n_layers][stride][chunk] (layer < 0)."""
        c = self.c[cls]
        layers = self._layers(cls)
        if layer >= 0:
            if layer in layers:
                c.evict(layers.index(layer), ids, src0, src1, src_block, stride, flags)
            return
        chunk = c.chunk_bytes
        sel = lambda a: None if a is None else np.ascontiguousarray(
            np.asarray(a, dtype=np.uint8).reshape(self.spec[cls].n_layers, stride, chunk)[layers])
        c.evict(-1, ids, sel(src0), sel(src1), src_block, stride, flags)

    def restore(self, cls, ids):
        self.c[cls].restore(ids)

    def evict_from_local(self, cls, ids, flags=0):
        """Write back local objects, the source being their own local slots (all layers)."""
        c = self.c[cls]
        slots = [c.lookup(i)[1] for i in ids]
        c.evict(-1, ids, c.plane(LOCAL, 0), c.plane(LOCAL, 1) if c.n_planes == 2 else None, slots, c.n_slots[LOCAL],
                flags)

    def tier_plane(self, cls, tier, plane=0):
        if tier == CACHE and self.c[cls].segpool is not None:
            return np.zeros((self.c[cls].n_layers, 0, self.c[cls].chunk_bytes), np.uint8)
        return self.c[cls].plane(tier, plane)
