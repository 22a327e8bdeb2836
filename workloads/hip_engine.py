"""Harness-side adapter of the HIP library: numpy in, numpy out, device buffers managed with torch.  It lives with the
harness (scenario drivers, generators), not in the library's package: the library's Python side is the binding alone.

This is what tests and the benchmark drive.  It only marshals: tables, routing ids and sources are copied to device
tensors, the library is called through the C ABI, destinations are copied back for comparison.  No payload byte is
produced or altered here.
"""
from __future__ import annotations

import numpy as np
import torch

import workloads as W
from workloads.digest import digest as _digest
from paper_2602_00328_amd import binding as B
from paper_2602_00328_amd.binding import KV, EXPERT, HOST, CACHE, LOCAL, NONE  # noqa: F401

IN_PLACE, STAGED, OVERFLOW_OR_LOST = 1, 2, 3


class HipEngine:
    name = "hip"

    def __init__(self, kv=None, expert=None, poison=False, device=0, profile=False, gather_wg_per_cu=0, host_wgs=0,
                 two_streams=False, shared_cache_bytes=0, shared_granule=0, general_fetch=False, gather_threads=0, pcie_wgs=0,
                 cache_planes_adjacent=False):
        """two_streams: KV work and expert work are enqueued on two HIP streams of their own (default priority).
        shared_cache_bytes: one cache pool for every class that has no cache slots of its own."""
        flags = (B.FLAG_POISON if poison else 0) | (B.FLAG_PROFILE if profile else 0) | \
            (B.FLAG_GENERAL_FETCH if general_fetch else 0) | (B.FLAG_CACHE_PLANES_ADJACENT if cache_planes_adjacent else 0)
        self.dev = torch.device("cuda", device)
        torch.cuda.set_device(self.dev)
        self.spec = {KV: kv, EXPERT: expert}
        self.streams = {k: (torch.cuda.Stream(self.dev) if two_streams else None) for k in (KV, EXPERT)}
        self.h = B.Harvest(kv=kv, expert=expert, flags=flags, device=device, gather_wg_per_cu=gather_wg_per_cu,
                           host_wgs=host_wgs, shared_cache_bytes=shared_cache_bytes, shared_granule=shared_granule,
                           gather_threads=gather_threads, pcie_wgs=pcie_wgs)
        self._dst = {}

    def _on(self, cls):
        """Context in which torch's own copies and the library call share the stream of this class."""
        s = self.streams[cls]
        return torch.cuda.stream(s if s is not None else torch.cuda.current_stream(self.dev))

    def close(self):
        torch.cuda.synchronize(self.dev)
        self.h.close()
        self._dst.clear()

    # ---- harness-side initialisation -----------------------------------------------------------------------
    def fill_host(self, cls, slot_object, seed, wl_cls, mode, sigma):
        sp = self.spec[cls]
        for p in range(sp.n_planes):
            W.fill_pool(self.h.host_ptr(cls, p), sp.n_layers, sp.n_host_slots, sp.chunk_bytes, slot_object, seed,
                        wl_cls, p, mode, sigma)

    def fill_local(self, cls, slot_object, seed, wl_cls, mode, sigma):
        sp = self.spec[cls]
        for p in range(sp.n_planes):
            t = self.h.dev_plane(cls, LOCAL, p)
            tmp = np.zeros((1, sp.n_local_slots, sp.chunk_bytes), dtype=np.uint8)
            used = torch.from_numpy((np.asarray(slot_object) != W.NO_OBJECT)).to(self.dev)
            for layer in range(sp.n_layers):
                W.fill_array(tmp, slot_object, seed, wl_cls, p, mode, sigma, layer_base=layer)
                up = torch.from_numpy(tmp[0]).to(self.dev)
                t[layer][used] = up[used]
        torch.cuda.synchronize(self.dev)

    def adopt(self, cls, ids):
        pass                                     # the library has no notion of a tier-free value

    def write_local(self, cls, obj, plane, layer, offset, data):
        tier, slot, _, _ = self.h.lookup(cls, obj)
        assert tier == LOCAL
        with self._on(cls):
            d = torch.from_numpy(np.ascontiguousarray(data, dtype=np.uint8)).to(self.dev)
            self.h.dev_plane(cls, LOCAL, plane)[layer, slot, offset:offset + d.numel()] = d

    # ---- directory ---------------------------------------------------------------------------------------------
    def register(self, cls, n, host_slots=None, tier=HOST):
        return self.h.register(cls, n, host_slots, tier)

    def lookup(self, cls, obj):
        return self.h.lookup(cls, obj)

    def restore(self, cls, ids):
        self.h.restore(cls, ids)

    def place(self, cls, ids):
        with self._on(cls):
            return self.h.place(cls, ids)

    def place_from(self, cls, ids, src0, src1, src_block, stride):
        """src planes: device tensors, or numpy arrays that are copied to the device first; [n_layers][stride][chunk]."""
        with self._on(cls):
            up = lambda a: a if a is None or torch.is_tensor(a) else torch.from_numpy(
                np.ascontiguousarray(a, dtype=np.uint8)).to(self.dev)
            d0, d1 = up(src0), up(src1)
            st = self.h.place_from(cls, ids, d0, d1, src_block, stride)
            if d0 is not src0:
                torch.cuda.current_stream().synchronize()       # the uploaded copies are freed when this returns
            return st

    def last_staging(self):
        """The staging buffer of the latest expert fetch (device tensor)."""
        return self._last_staging

    def revoke(self, cls, ids):
        n0 = len(self.h.revoked_log)
        self.h.revoke(cls, ids)
        return [i for c, i in self.h.revoked_log[n0:] if c == cls]      # another thread may be revoking the other class

    # ---- data path -------------------------------------------------------------------------------------------
    def has_layer(self, layer):
        return True

    def _dst_buffers(self, cap, fill=0):
        sp = self.spec[KV]
        key = (cap, sp.chunk_bytes)
        if key not in self._dst:
            self._dst.clear()
            self._dst[key] = [torch.empty(cap * sp.chunk_bytes, dtype=torch.uint8, device=self.dev)
                              for _ in range(sp.n_planes)]
        for t in self._dst[key]:
            t.fill_(fill)
        return self._dst[key]

    def fetch_kv_device(self, layer, d_table, d_n_blocks, d_sdb, cap, dst=None, stream=None):
        """All-device variant (what the benchmark times): nothing is copied to or from the host."""
        dst = dst or self._dst_buffers(cap)
        self.h.fetch_kv(layer, d_table, d_n_blocks, dst[0], dst[1] if len(dst) > 1 else None, d_sdb, cap, stream)
        return dst

    def fetch_kv_begin(self, layer, table, n_blocks, seq_dst_block, cap, dst_fill=0, head_major=None):
        """Enqueue only; fetch_end(handle) waits and copies the results back.  head_major = (seq_cap_blocks, n_heads,
        block_tokens) selects the head-major working layout."""
        sp = self.spec[KV]
        table = np.ascontiguousarray(table, dtype=np.int32)
        with self._on(KV):
            d_table = torch.from_numpy(table).to(self.dev)
            d_nb = torch.from_numpy(np.ascontiguousarray(n_blocks, dtype=np.int32)).to(self.dev)
            d_sdb = torch.from_numpy(np.ascontiguousarray(seq_dst_block, dtype=np.uint64).view(np.int64)).to(self.dev)
            dst = [torch.full((cap * sp.chunk_bytes,), dst_fill, dtype=torch.uint8, device=self.dev)
                   for _ in range(sp.n_planes)]
            d_cap = None
            if head_major is None:
                self.h.fetch_kv(layer, d_table, d_nb, dst[0], dst[1] if len(dst) > 1 else None, d_sdb, cap)
            else:
                caps, n_heads, block_tokens = head_major
                d_cap = torch.from_numpy(np.ascontiguousarray(caps, dtype=np.uint32).view(np.int32)).to(self.dev)
                self.h.fetch_kv_head_major(layer, d_table, d_nb, dst[0], dst[1] if len(dst) > 1 else None, d_sdb, d_cap,
                                           cap, n_heads, block_tokens)
        self._last_kv = (dst[0].numel(), len(dst), table.size, (d_table, d_nb, d_sdb, d_cap))   # the arrays stay alive for "again"
        return ("kv", dst, table.size, (d_table, d_nb, d_sdb, d_cap))

    def fetch_kv_again(self, layer, dst_fill=0):
        """harvest_fetch_kv_again: the latest single-layer fetch of the KV stream for another layer, into fresh buffers."""
        nbytes, n_planes, n_req, keep = self._last_kv
        with self._on(KV):
            dst = [torch.full((nbytes,), dst_fill, dtype=torch.uint8, device=self.dev) for _ in range(n_planes)]
            self.h.fetch_kv_again(layer, dst[0], dst[1] if n_planes > 1 else None)
        return self.fetch_end(("kv", dst, n_req, keep))

    def fetch_kv_head_major(self, layer, table, n_blocks, seq_dst_block, seq_cap_blocks, cap, n_heads, block_tokens,
                            dst_fill=0):
        return self.fetch_end(self.fetch_kv_begin(layer, table, n_blocks, seq_dst_block, cap, dst_fill,
                                                  head_major=(seq_cap_blocks, n_heads, block_tokens)))

    def fetch_kv(self, layer, table, n_blocks, seq_dst_block, cap, dst_fill=0):
        return self.fetch_end(self.fetch_kv_begin(layer, table, n_blocks, seq_dst_block, cap, dst_fill))

    def fetch_kv_layers(self, layer_first, n_layers, table, n_blocks, seq_dst_block, cap, dst_fill=0):
        """One call for n_layers consecutive layers -> ([(k, v) per layer], sorted miss list, counts)."""
        sp = self.spec[KV]
        table = np.ascontiguousarray(table, dtype=np.int32)
        with self._on(KV):
            d_table = torch.from_numpy(table).to(self.dev)
            d_nb = torch.from_numpy(np.ascontiguousarray(n_blocks, dtype=np.int32)).to(self.dev)
            d_sdb = torch.from_numpy(np.ascontiguousarray(seq_dst_block, dtype=np.uint64).view(np.int64)).to(self.dev)
            stride = cap * sp.chunk_bytes + 256               # not a multiple of the chunk size: strides are in bytes
            dst = [torch.full((n_layers * stride,), dst_fill, dtype=torch.uint8, device=self.dev)
                   for _ in range(sp.n_planes)]
            self.h.fetch_kv_layers(layer_first, n_layers, d_table, d_nb, dst[0], dst[1] if sp.n_planes == 2 else None,
                                   stride, d_sdb, cap)
            counts, miss, n_miss = self.h.fetch_info(miss_cap=table.size)
            out = []
            for r in range(n_layers):
                k = dst[0][r * stride:r * stride + cap * sp.chunk_bytes].cpu().numpy()
                v = dst[1][r * stride:r * stride + cap * sp.chunk_bytes].cpu().numpy() if sp.n_planes == 2 else None
                gap = dst[0][r * stride + cap * sp.chunk_bytes:(r + 1) * stride]
                assert bool((gap == dst_fill).all()), "bytes between two layers' destinations were written"
                out.append((k, v))
        return out, np.sort(miss), counts

    def fetch_experts_begin(self, layer, topk, n_staging, staging_fill=0):
        sp = self.spec[EXPERT]
        with self._on(EXPERT):
            d_topk = torch.from_numpy(np.ascontiguousarray(topk, dtype=np.int32)).to(self.dev)
            staging = torch.full((max(1, n_staging) * sp.chunk_bytes,), staging_fill, dtype=torch.uint8,
                                 device=self.dev)
            ptrs = torch.zeros(sp.n_experts, dtype=torch.int64, device=self.dev)
            self.h.fetch_experts(layer, d_topk, staging, n_staging, ptrs)
            self._last_staging = staging
        return ("experts", staging, n_staging, ptrs, d_topk)

    def fetch_experts(self, layer, topk, n_staging, staging_fill=0):
        return self.fetch_end(self.fetch_experts_begin(layer, topk, n_staging, staging_fill))

    def fetch_end(self, handle, digest=False):
        """Waits for a fetch and returns what it delivered.  digest: instead of the delivered bytes, their checksum,
        computed on the device (nothing but counters and the miss list is copied back): KV -> (digest of K, digest of V,
        ...), experts -> (digest of the staging slots in use, ...)."""
        if handle[0] == "kv":
            _, dst, n_req, _keep = handle
            with self._on(KV):
                counts, miss, n_miss = self.h.fetch_info(miss_cap=n_req, cls=KV)
                assert n_miss == miss.size
                if digest:
                    return _digest(dst[0]), (_digest(dst[1]) if len(dst) > 1 else None), np.sort(miss), counts
                k = dst[0].cpu().numpy()
                v = dst[1].cpu().numpy() if len(dst) > 1 else None
            return k, v, np.sort(miss), counts
        _, staging, n_staging, ptrs, _keep = handle
        sp = self.spec[EXPERT]
        E = sp.n_experts
        with self._on(EXPERT):
            counts, miss, n_miss = self.h.fetch_info(miss_cap=E, cls=EXPERT)
            ptrs = ptrs.cpu().numpy()
            local = self.h.dev_plane(EXPERT, LOCAL, 0) if sp.n_local_slots else None
            s0 = staging.data_ptr()
            out, kind, where = [], np.zeros(E, np.int32), np.full(E, -1, np.int64)
            for e in range(E):
                p = int(ptrs[e])
                if p == 0:
                    out.append(None)
                elif s0 <= p < s0 + n_staging * sp.chunk_bytes:
                    r = (p - s0) // sp.chunk_bytes
                    assert (p - s0) % sp.chunk_bytes == 0
                    kind[e], where[e] = STAGED, r
                    out.append(None if digest else staging[r * sp.chunk_bytes:(r + 1) * sp.chunk_bytes].cpu().numpy())
                else:
                    l0 = local.data_ptr()
                    assert l0 <= p < l0 + sp.n_local_slots * sp.chunk_bytes and (p - l0) % sp.chunk_bytes == 0
                    slot = (p - l0) // sp.chunk_bytes
                    kind[e], where[e] = IN_PLACE, slot
                    out.append(None if digest else local[0, slot].cpu().numpy())
            if digest:                           # staged experts fill the slots 0 .. n-1; experts used in place moved no byte
                n_staged = int((kind == STAGED).sum())
                assert sorted(where[kind == STAGED]) == list(range(n_staged))
                out = _digest(staging[:n_staged * sp.chunk_bytes])
        return out, kind, where, np.sort(miss), counts

    def evict(self, cls, layer, ids, src0, src1, src_block, stride, flags=0):
        with self._on(cls):
            d0 = torch.from_numpy(np.ascontiguousarray(src0, dtype=np.uint8)).to(self.dev)
            d1 = None if src1 is None else torch.from_numpy(np.ascontiguousarray(src1, dtype=np.uint8)).to(self.dev)
            self.h.evict(cls, layer, ids, d0, d1, src_block, stride, flags)
            torch.cuda.current_stream().synchronize()          # d0 / d1 are freed when this returns

    def evict_from_local(self, cls, ids, flags=0):
        sp = self.spec[cls]
        slots = [self.h.lookup(cls, i)[1] for i in ids]
        with self._on(cls):
            self.h.evict(cls, -1, ids, self.h.dev_plane(cls, LOCAL, 0),
                         self.h.dev_plane(cls, LOCAL, 1) if sp.n_planes == 2 else None, slots, sp.n_local_slots, flags)

    def tier_plane(self, cls, tier, plane=0):
        if tier == HOST:
            torch.cuda.synchronize(self.dev)
            return self.h.host_plane(cls, plane)
        if tier == CACHE and self.spec[cls].n_cache_slots == 0:
            return np.zeros((self.spec[cls].n_layers, 0, self.spec[cls].chunk_bytes), np.uint8)
        return self.h.dev_plane(cls, tier, plane).cpu().numpy()

    def shared_plane(self):
        torch.cuda.synchronize(self.dev)
        return self.h.shared_cache.cpu().numpy()
