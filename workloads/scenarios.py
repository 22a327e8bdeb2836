"""Harness drivers: they sequence engine calls for the synthetic workloads and keep the harness's own state
(block tables, sequence lengths, which objects it has placed, the LRU policy).  An *engine* is anything with the
methods used below - the CPU checker's adapter and the HIP library's adapter both qualify - so the same driver runs
against either, and a test compares what the two return.  Nothing here moves or inspects payload bytes.
"""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np

from . import (CLS_APPEND, CLS_EXPERT, CLS_KV, NO_OBJECT, LRU, KVWorkload, ExpertWorkload, append_rows,
               revoke_draw)

KV, EXPERT = 0, 1
HOST, CACHE, LOCAL, NONE = 0, 1, 2, 3
OK, ENOSPC = 0, -2
EVICT_DEMOTE = 1


def kv_spec(wl: KVWorkload, cache_slack: int = 0, local_slack: int = 0, shared: bool = False, n_planes: int = 2):
    """Pool sizes for a KV workload: a host slot for every block, cache slots for every resident block (none when the
    cache tier is carved from a pool shared with the other class)."""
    return SimpleNamespace(n_layers=wl.shape.n_layers, n_planes=n_planes, chunk_bytes=wl.shape.chunk_bytes,
                           max_objects=wl.n_objects, n_host_slots=wl.n_objects,
                           n_cache_slots=0 if shared else int(wl.resident.sum()) + cache_slack,
                           n_local_slots=(wl.n_seq if wl.has_tails else 0) + local_slack, n_experts=0)


def expert_spec(wl: ExpertWorkload, shared: bool = False):
    sh = wl.shape
    n = wl.n_objects
    n_cache = sh.n_layers * wl.lru_capacity if wl.lru_capacity else int((wl.tier0 == 1).sum())
    return SimpleNamespace(n_layers=1, n_planes=1, chunk_bytes=sh.chunk_bytes, max_objects=n, n_host_slots=n,
                           n_cache_slots=0 if shared else max(1, n_cache), n_local_slots=int((wl.tier0 == 2).sum()),
                           n_experts=sh.n_experts)


class KVRun:
    """Decode-step driver for one engine (Section 5.2: consult the block table, reload what is not local, evict the
    blocks that fill up)."""

    def __init__(self, engine, wl: KVWorkload):
        self.e, self.wl = engine, wl
        sh = wl.shape
        C = wl.n_closed
        ids = engine.register(KV, C, wl.host_slot[:C], HOST)
        assert list(ids[:3]) == [0, 1, 2][:C]
        so = np.full(wl.n_objects, NO_OBJECT, dtype=np.uint32)
        so[wl.host_slot[:C]] = np.arange(C)
        engine.fill_host(KV, so, wl.seed, CLS_KV, wl.fill_mode, wl.sigma)
        self.tables = [list(int(b) for b in t) for t in wl.tables]
        self.lens = [int(l) for l in wl.seq_lens]
        self.n_future = [0] * wl.n_seq
        if wl.has_tails:
            tails = engine.register(KV, wl.n_seq, wl.host_slot[C:C + wl.n_seq], LOCAL)
            assert [int(t) for t in tails] == [t[-1] for t in self.tables]
            lo = np.full(wl.n_seq, NO_OBJECT, dtype=np.uint32)
            for t in tails:
                lo[engine.lookup(KV, t)[1]] = t
            lo = np.concatenate([lo, np.full(engine.spec[KV].n_local_slots - wl.n_seq, NO_OBJECT, np.uint32)])
            engine.fill_local(KV, lo, wl.seed, CLS_KV, wl.fill_mode, wl.sigma)
        engine.adopt(KV, np.arange(C + (wl.n_seq if wl.has_tails else 0)))
        self.place_status = engine.place(KV, wl.place_order)
        self.live = set(int(b) for b, s in zip(wl.place_order, self.place_status) if s == OK)   # cache-tier blocks
        self.pending_replace = []
        final = [len(t) + len(f) for t, f in zip(wl.tables, wl.future_blocks)]
        self.max_blocks = max(final)
        self.seq_dst_block = np.concatenate([[0], np.cumsum(final)[:-1]]).astype(np.uint64)
        self.cap = int(sum(final))

    def table_arrays(self):
        table = np.zeros((self.wl.n_seq, self.max_blocks), dtype=np.int32)
        for s, t in enumerate(self.tables):
            table[s, :len(t)] = t
        return table, np.array([len(t) for t in self.tables], dtype=np.int32)

    def fetch(self, layer, digest=False):
        """digest: checksums of the two destination planes instead of the planes themselves."""
        table, nb = self.table_arrays()
        if digest:
            return self.e.fetch_end(self.e.fetch_kv_begin(layer, table, nb, self.seq_dst_block, self.cap), digest=True)
        return self.e.fetch_kv(layer, table, nb, self.seq_dst_block, self.cap)

    def fetch_begin(self, layer):
        table, nb = self.table_arrays()
        return self.e.fetch_kv_begin(layer, table, nb, self.seq_dst_block, self.cap)

    def append(self, t):
        """Every sequence appends one token; full tails are written back, leave local HBM, are placed in the cache
        tier with the configured probability, and a fresh tail is opened."""
        wl, sh = self.wl, self.wl.shape
        for s in range(wl.n_seq):
            tail = self.tables[s][-1]
            rows = append_rows(wl, t, s)
            off = (self.lens[s] % sh.block_tokens) * sh.row_bytes
            for p in range(self.e.spec[KV].n_planes):
                for l in range(sh.n_layers):
                    self.e.write_local(KV, tail, p, l, off, rows[p, l])
            self.lens[s] += 1
            if self.lens[s] % sh.block_tokens == 0:
                self.e.evict_from_local(KV, [tail], EVICT_DEMOTE)
                if wl.resident[tail]:
                    if self.e.place(KV, [tail])[0] == OK:
                        self.live.add(tail)
                new = int(wl.future_blocks[s][self.n_future[s]])
                self.n_future[s] += 1
                got = self.e.register(KV, 1, wl.host_slot[new:new + 1], LOCAL)
                assert int(got[0]) == new
                self.tables[s].append(new)

    def step(self, t):
        out = self.fetch(t % self.wl.shape.n_layers)
        self.append(t)
        return out

    def revoke_quarter(self, t):
        ids = revoke_draw(self.wl.seed, t, KV, self.live)
        called = self.e.revoke(KV, ids)
        self.live -= set(int(i) for i in ids)
        self.pending_replace = [int(i) for i in ids]
        return ids, called

    def replace_revoked(self):
        ids, self.pending_replace = self.pending_replace, []
        st = self.e.place(KV, ids) if ids else np.zeros(0, np.int32)
        self.live |= {i for i, s in zip(ids, st) if s == OK}
        return st


class ExpertRun:
    """Per-layer expert fetch driver (Section 4.3: a fixed subset is local, the rest start on the host and are
    migrated into the cache tier by the harness's policy - static draw, or LRU over the routing trace)."""

    def __init__(self, engine, wl: ExpertWorkload, n_staging=None):
        self.e, self.wl = engine, wl
        sh = wl.shape
        n, E = wl.n_objects, sh.n_experts
        self.host_slot = _perm(wl.seed, n)
        local = (wl.tier0.reshape(-1) == 2)
        i = 0
        while i < n:                                   # registration is in id order: one call per run of equal tier
            j = i
            while j < n and local[j] == local[i]:
                j += 1
            got = engine.register(EXPERT, j - i, self.host_slot[i:j], LOCAL if local[i] else HOST)
            assert int(got[0]) == i
            i = j
        so = np.full(n, NO_OBJECT, dtype=np.uint32)
        so[self.host_slot] = np.arange(n)
        engine.fill_host(EXPERT, so, wl.seed, CLS_EXPERT, wl.fill_mode, wl.sigma)
        n_local = engine.spec[EXPERT].n_local_slots
        if n_local:
            lo = np.full(n_local, NO_OBJECT, dtype=np.uint32)
            for b in np.nonzero(local)[0]:
                lo[engine.lookup(EXPERT, b)[1]] = b
            engine.fill_local(EXPERT, lo, wl.seed, CLS_EXPERT, wl.fill_mode, wl.sigma)
        engine.adopt(EXPERT, np.arange(n))
        self.place_status = engine.place(EXPERT, wl.place_order) if wl.place_order.size else np.zeros(0, np.int32)
        self.live = set(int(b) for b, s in zip(wl.place_order, self.place_status) if s == OK)
        self.pending_replace = []
        self.n_staging = n_staging if n_staging is not None else E
        self.lru = [LRU(wl.lru_capacity) for _ in range(sh.n_layers)] if wl.lru_capacity else None

    def fetch(self, t, layer, digest=False):
        """digest: a checksum of the staged bytes instead of the experts' bytes."""
        if digest:
            return self.e.fetch_end(self.fetch_begin(t, layer, digest=True), digest=True)
        return self.e.fetch_experts(layer, self.wl.routing(t, layer), self.n_staging)

    def fetch_begin(self, t, layer, digest=False):
        if digest and self.e.name == "oracle":           # a CPU has nothing in flight: "begin" does the work
            return self.e.fetch_experts(layer, self.wl.routing(t, layer), self.n_staging, digest=True)
        return self.e.fetch_experts_begin(layer, self.wl.routing(t, layer), self.n_staging)

    def staged_ranks(self, t, layer):
        """expert -> staging slot of the fetch of (t, layer), from what the host knows: routed experts that are not local,
        in ascending order, as far as the staging buffer has room (Section 4.3: whole experts, one staging slot each)."""
        E = self.wl.shape.n_experts
        routed = sorted(set(int(e) for e in self.wl.routing(t, layer).reshape(-1)))
        staged = [e for e in routed if self.e.lookup(EXPERT, layer * E + e)[0] in (HOST, CACHE)]
        return {e: r for r, e in enumerate(staged) if r < self.n_staging}

    def lru_update(self, t, layer, from_staging=False):
        """After the fetch of (t, layer): run the LRU over this step's token-ordered trace and apply the net change
        as revocations followed by placements.  from_staging: an expert that enters the cache tier was routed in this
        very step, so the fetch has just left it in the staging buffer - it is placed from there, not from the host."""
        E = self.wl.shape.n_experts
        ranks = self.staged_ranks(t, layer) if from_staging else {}      # as the fetch saw residency: before any change
        lru = self.lru[layer]
        before = lru.members()
        for row in self.wl.routing(t, layer):
            for e in row:
                lru.touch(int(e))
        after = lru.members()
        out_ids = sorted(layer * E + e for e in before - after)
        in_ids = sorted(layer * E + e for e in after - before)
        called = self.e.revoke(EXPERT, out_ids) if out_ids else []
        if not in_ids:
            st = np.zeros(0, np.int32)
        elif not from_staging:
            st = self.e.place(EXPERT, in_ids)
        else:
            staged = [i for i in in_ids if i - layer * E in ranks]
            rest = [i for i in in_ids if i - layer * E not in ranks]
            got = {}
            if staged:
                got.update(zip(staged, self.e.place_from(EXPERT, staged, self.e.last_staging(), None,
                                                         [ranks[i - layer * E] for i in staged], max(1, self.n_staging))))
            if rest:
                got.update(zip(rest, self.e.place(EXPERT, rest)))
            st = np.array([got[i] for i in in_ids], dtype=np.int32)
        self.live -= set(out_ids)
        self.live |= {i for i, s in zip(in_ids, st) if s == OK}
        return out_ids, called, in_ids, st

    def revoke_quarter(self, t):
        ids = revoke_draw(self.wl.seed, t, EXPERT, self.live)
        called = self.e.revoke(EXPERT, ids)
        self.live -= set(int(i) for i in ids)
        self.pending_replace = [int(i) for i in ids]
        return ids, called

    def replace_revoked(self):
        ids, self.pending_replace = self.pending_replace, []
        st = self.e.place(EXPERT, ids) if ids else np.zeros(0, np.int32)
        self.live |= {i for i, s in zip(ids, st) if s == OK}
        return st


def _perm(seed, n):
    from . import rng
    return rng(seed, 24).permutation(n).astype(np.int64)
