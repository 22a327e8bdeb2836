"""ctypes binding of libharvest.so: the same names as include/harvest.h, argument marshalling only.

Every step of the fetch path runs inside the library's HIP kernels; this module never touches payload bytes.  PyTorch
is used by the ``Harvest`` convenience class for device memory and streams only.  If the library has not been built
the import of this module fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import weakref
import os
from dataclasses import dataclass

import numpy as np
import torch  # noqa: F401  - must be imported BEFORE the library is loaded: PyTorch bundles its own HIP runtime
#                (same SONAME as the system one), and a process must hold exactly one; loading libharvest.so after
#                torch makes the dynamic loader bind it to the runtime torch already mapped, so streams and device
#                pointers are shared.

from . import _build

HOST, CACHE, LOCAL, NONE = 0, 1, 2, 3
OK, EINVAL, ENOSPC, ENOENT, EHIP, ELOST, ENODEV, EBUSY, E2BIG = 0, -1, -2, -3, -4, -5, -6, -7, -8
STATIC_MAX_CELLS = 65536
KV, EXPERT = 0, 1
FLAG_NO_DEVICE, FLAG_POISON, FLAG_PROFILE, FLAG_GENERAL_FETCH, FLAG_CACHE_PLANES_ADJACENT = 1, 2, 4, 8, 16
EVICT_DEMOTE = 1

u32, u64, i32, i64, vp = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p


class harvest_class_config(ctypes.Structure):
    _fields_ = [("n_layers", u32), ("n_planes", u32), ("chunk_bytes", u64), ("max_objects", u32),
                ("n_host_slots", u32), ("n_cache_slots", u32), ("n_local_slots", u32), ("n_experts", u32),
                ("host_pool", vp * 2), ("d_cache_pool", vp * 2), ("d_local_pool", vp * 2)]


class harvest_config(ctypes.Structure):
    _fields_ = [("flags", u32), ("device", i32), ("cls", harvest_class_config * 2),
                ("gather_wg_per_cu", u32), ("host_wgs", u32), ("shared_granule", u32), ("small_fetch_cells", u32), ("gather_threads", u32), ("pcie_wgs", u32), ("reserved", u32 * 2),
                ("d_shared_cache", vp), ("shared_cache_bytes", u64)]


class harvest_fetch_counts(ctypes.Structure):
    _fields_ = [(n, u64) for n in ("n_requests", "n_local", "n_cache", "n_host", "n_lost", "n_invalid")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class harvest_stats_t(ctypes.Structure):
    _fields_ = [("fetch", harvest_fetch_counts * 2), ("n_placed", u64 * 2), ("n_place_enospc", u64 * 2),
                ("n_revoked", u64 * 2), ("n_evicted", u64 * 2), ("n_demoted", u64 * 2),
                ("cache_slots_in_use", u64 * 2), ("local_slots_in_use", u64 * 2),
                ("shared_granules_free", u64), ("shared_free_runs", u64), ("shared_longest_free_run", u64)]


class harvest_profile_t(ctypes.Structure):
    _fields_ = [("hbm_launches", u64), ("hbm_ms", ctypes.c_double), ("host_launches", u64),
                ("host_ms", ctypes.c_double)]


REVOKE_CB = ctypes.CFUNCTYPE(None, ctypes.c_int, u32, vp)

SYMBOLS = {
    "harvest_create": (ctypes.c_int, [ctypes.POINTER(harvest_config), ctypes.POINTER(vp)]),
    "harvest_destroy": (ctypes.c_int, [vp]),
    "harvest_register": (ctypes.c_int, [vp, ctypes.c_int, u32, vp, ctypes.c_int, REVOKE_CB, vp, vp]),
    "harvest_lookup": (ctypes.c_int, [vp, ctypes.c_int, u32, vp, vp, vp, vp]),
    "harvest_restore": (ctypes.c_int, [vp, ctypes.c_int, vp, u32]),
    "harvest_place": (ctypes.c_int, [vp, ctypes.c_int, vp, u32, vp, vp]),
    "harvest_place_from": (ctypes.c_int, [vp, ctypes.c_int, vp, u32, vp, vp, vp, u64, vp, vp]),
    "harvest_revoke": (ctypes.c_int, [vp, ctypes.c_int, vp, u32]),
    "harvest_alloc": (ctypes.c_int, [vp, ctypes.c_int, u32, vp]),
    "harvest_free": (ctypes.c_int, [vp, ctypes.c_int, u32]),
    "harvest_register_cb": (ctypes.c_int, [vp, ctypes.c_int, u32, REVOKE_CB, vp]),
    "harvest_release_stream": (ctypes.c_int, [vp, vp]),
    "harvest_fetch_kv": (ctypes.c_int, [vp, u32, vp, vp, u32, u32, vp, vp, vp, u64, vp]),
    "harvest_fetch_kv_static": (ctypes.c_int, [vp, u32, vp, vp, u32, u32, vp, vp, vp, u64, vp, vp, vp]),
    "harvest_fetch_kv_again": (ctypes.c_int, [vp, u32, vp, vp, vp]),
    "harvest_fetch_kv_layers": (ctypes.c_int, [vp, u32, u32, vp, vp, u32, u32, vp, vp, u64, vp, u64, vp]),
    "harvest_fetch_kv_head_major": (ctypes.c_int, [vp, u32, vp, vp, u32, u32, vp, vp, vp, vp, u64, u32, u32, vp]),
    "harvest_fetch_experts": (ctypes.c_int, [vp, u32, vp, u32, u32, vp, u32, vp, vp]),
    "harvest_prefetcher_create": (ctypes.c_int, [vp, vp * 2, u32, vp * 2, ctypes.POINTER(vp)]),
    "harvest_prefetcher_destroy": (ctypes.c_int, [vp]),
    "harvest_prefetcher_stream": (vp, [vp]),
    "harvest_prefetch_issue": (ctypes.c_int, [vp, u32, vp, u32, u32, vp]),
    "harvest_prefetch_acquire": (ctypes.c_int, [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp)]),
    "harvest_prefetch_release": (ctypes.c_int, [vp, vp]),
    "harvest_fetch_info": (ctypes.c_int, [vp, vp, ctypes.POINTER(harvest_fetch_counts), vp, u32, vp]),
    "harvest_fetch_info_of": (ctypes.c_int, [vp, vp, ctypes.c_int, ctypes.POINTER(harvest_fetch_counts), vp, u32, vp]),
    "harvest_evict": (ctypes.c_int, [vp, ctypes.c_int, ctypes.c_int, vp, u32, vp, vp, vp, u64, ctypes.c_int, vp]),
    "harvest_stats": (ctypes.c_int, [vp, ctypes.POINTER(harvest_stats_t)]),
    "harvest_profile": (ctypes.c_int, [vp, ctypes.POINTER(harvest_profile_t)]),
    "harvest_plain_copy": (ctypes.c_int, [vp, vp, u64, vp]),
    "harvest_plain_read": (ctypes.c_int, [vp, u64, vp, vp]),
    "harvest_plain_write": (ctypes.c_int, [vp, u64, u32, vp]),
    "harvest_pinned_alloc": (vp, [ctypes.c_size_t]),
    "harvest_pinned_free": (ctypes.c_int, [vp]),
    "harvest_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}


def _load():
    if not os.path.exists(_build.LIB_PATH):
        raise ImportError(f"{_build.LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc, gfx950). There is no fallback for the HIP library.")
    lib = ctypes.CDLL(_build.LIB_PATH)
    for name, (res, args) in SYMBOLS.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()
LIB_PATH = _build.LIB_PATH


class HarvestError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {lib.harvest_strerror(code).decode()} ({code})")
        self.code = code


def _chk(rc, what):
    if rc != OK:
        raise HarvestError(rc, what)


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(vp)


def _dev_ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return vp(t)
    return vp(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return vp(stream)
    return vp(stream.cuda_stream)


@dataclass
class ClassSpec:
    n_layers: int
    n_planes: int
    chunk_bytes: int
    max_objects: int
    n_host_slots: int
    n_cache_slots: int
    n_local_slots: int
    n_experts: int = 0


class Harvest:
    """A library context plus the pools it borrows (allocated here with torch / harvest_pinned_alloc)."""

    def __init__(self, kv: ClassSpec | None = None, expert: ClassSpec | None = None, flags: int = 0, device: int = 0,
                 gather_wg_per_cu: int = 0, host_wgs: int = 0, shared_cache_bytes: int = 0, shared_granule: int = 0,
                 small_fetch_cells: int = 0, gather_threads: int = 0, pcie_wgs: int = 0):
        """shared_cache_bytes > 0: one device pool of that size from which every class with n_cache_slots == 0 carves
        its cache-tier segments (best-fit)."""
        self.flags, self.device = flags, device
        self.spec = {KV: kv, EXPERT: expert}
        self.no_device = bool(flags & FLAG_NO_DEVICE)
        self._host_ptr = {}        # (cls, plane) -> address
        self._host_np = {}
        self._dev = {}             # (cls, tier, plane) -> torch tensor
        self.revoked_log = []      # (cls, id) in callback order
        self._prefetchers = []     # weak references: closed with the context, their handles die with it
        self._cb = REVOKE_CB(lambda c, i, _u: self.revoked_log.append((int(c), int(i))))
        cfg = harvest_config()
        cfg.flags, cfg.device = flags, device
        cfg.gather_wg_per_cu, cfg.host_wgs = gather_wg_per_cu, host_wgs
        cfg.small_fetch_cells = small_fetch_cells
        cfg.gather_threads = gather_threads
        cfg.pcie_wgs = pcie_wgs
        adjacent = bool(flags & FLAG_CACHE_PLANES_ADJACENT)
        cfg.shared_cache_bytes, cfg.shared_granule = shared_cache_bytes, shared_granule
        self.shared_cache = None
        if shared_cache_bytes and not self.no_device:
            self.shared_cache = torch.zeros(shared_cache_bytes, dtype=torch.uint8, device=torch.device("cuda", device))
            cfg.d_shared_cache = self.shared_cache.data_ptr()
        for k, sp in self.spec.items():
            if sp is None:
                continue
            cc = cfg.cls[k]
            cc.n_layers, cc.n_planes, cc.chunk_bytes = sp.n_layers, sp.n_planes, sp.chunk_bytes
            cc.max_objects, cc.n_experts = sp.max_objects, sp.n_experts
            cc.n_host_slots, cc.n_cache_slots, cc.n_local_slots = sp.n_host_slots, sp.n_cache_slots, sp.n_local_slots
            if self.no_device:
                continue
            dev = torch.device("cuda", device)
            for p in range(sp.n_planes):
                nbytes = sp.n_layers * sp.n_host_slots * sp.chunk_bytes
                if nbytes:
                    ptr = lib.harvest_pinned_alloc(nbytes)
                    if not ptr:
                        raise HarvestError(EHIP, f"pinned allocation of {nbytes} bytes")
                    self._host_ptr[(k, p)] = ptr
                    ctypes.memset(ptr, 0, nbytes)          # like the device pools: slots nobody has written read as zeros
                    buf = (ctypes.c_uint8 * nbytes).from_address(ptr)
                    self._host_np[(k, p)] = np.frombuffer(buf, dtype=np.uint8).reshape(
                        sp.n_layers, sp.n_host_slots, sp.chunk_bytes)
                    cc.host_pool[p] = ptr
                for tier, n_slots, field in ((CACHE, sp.n_cache_slots, cc.d_cache_pool),
                                             (LOCAL, sp.n_local_slots, cc.d_local_pool)):
                    if not n_slots:
                        continue
                    if tier == CACHE and adjacent and sp.n_planes == 2:
                        # one buffer [layer][slot][plane][chunk]; the planes are strided views of it
                        if p == 0:
                            self._cache_kv = torch.zeros((sp.n_layers, n_slots, 2, sp.chunk_bytes), dtype=torch.uint8, device=dev)
                            field[0] = self._cache_kv.data_ptr()
                        self._dev[(k, tier, p)] = self._cache_kv[:, :, p, :]
                        continue
                    t = torch.zeros((sp.n_layers, n_slots, sp.chunk_bytes), dtype=torch.uint8, device=dev)
                    self._dev[(k, tier, p)] = t
                    field[p] = t.data_ptr()
        h = vp()
        _chk(lib.harvest_create(ctypes.byref(cfg), ctypes.byref(h)), "harvest_create")
        self.h = h

    # ---- pools ------------------------------------------------------------------------------------------------
    def host_plane(self, cls, plane=0) -> np.ndarray:
        return self._host_np[(cls, plane)]

    def host_ptr(self, cls, plane=0) -> int:
        return self._host_ptr[(cls, plane)]

    def dev_plane(self, cls, tier, plane=0):
        return self._dev[(cls, tier, plane)]

    def close(self):
        if getattr(self, "h", None):
            for ref in self._prefetchers:
                pf = ref()
                if pf is not None:
                    pf.close()
            self._prefetchers.clear()
            _chk(lib.harvest_destroy(self.h), "harvest_destroy")
            self.h = None
            self._host_np.clear()
            for ptr in self._host_ptr.values():
                lib.harvest_pinned_free(ptr)
            self._host_ptr.clear()
            self._dev.clear()
            self.shared_cache = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- directory ----------------------------------------------------------------------------------------------
    def register(self, cls, n, host_slots=None, tier=HOST) -> np.ndarray:
        hs = None if host_slots is None else np.ascontiguousarray(host_slots, dtype=np.int64)
        out = np.empty(n, dtype=np.uint32)
        _chk(lib.harvest_register(self.h, cls, n, _np_ptr(hs), tier, self._cb, None, _np_ptr(out)), "harvest_register")
        return out

    def lookup(self, cls, obj):
        t, s, g, hs = ctypes.c_int(), i64(), u32(), i64()
        _chk(lib.harvest_lookup(self.h, cls, int(obj), ctypes.byref(t), ctypes.byref(s), ctypes.byref(g),
                                ctypes.byref(hs)), "harvest_lookup")
        return t.value, s.value, g.value, hs.value

    def alloc(self, cls, obj, stream=None) -> int:
        """harvest_alloc: the status (OK, ENOSPC, ELOST) rather than an exception - a full cache tier is no error."""
        sp = vp(0) if self.no_device else _stream_ptr(stream)
        rc = lib.harvest_alloc(self.h, cls, int(obj), sp)
        if rc not in (OK, ENOSPC, ELOST):
            raise HarvestError(rc, "harvest_alloc")
        return rc

    def free(self, cls, obj):
        _chk(lib.harvest_free(self.h, cls, int(obj)), "harvest_free")

    def register_cb(self, cls, obj, enabled=True):
        """Attach the context's logging callback to the object, or (enabled=False) clear its callback."""
        cb = self._cb if enabled else ctypes.cast(None, REVOKE_CB)
        _chk(lib.harvest_register_cb(self.h, cls, int(obj), cb, None), "harvest_register_cb")

    def restore(self, cls, ids):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        _chk(lib.harvest_restore(self.h, cls, _np_ptr(ids), ids.size), "harvest_restore")

    def place(self, cls, ids, stream=None) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        st = np.zeros(ids.size, dtype=np.int32)
        sp = vp(0) if self.no_device else _stream_ptr(stream)
        _chk(lib.harvest_place(self.h, cls, _np_ptr(ids), ids.size, sp, _np_ptr(st)), "harvest_place")
        return st

    def place_from(self, cls, ids, d_src0, d_src1, src_block, src_layer_stride, stream=None) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        sb = np.ascontiguousarray(src_block, dtype=np.uint64)
        assert sb.shape == ids.shape
        st = np.zeros(ids.size, dtype=np.int32)
        sp = vp(0) if self.no_device else _stream_ptr(stream)
        _chk(lib.harvest_place_from(self.h, cls, _np_ptr(ids), ids.size, _dev_ptr(d_src0), _dev_ptr(d_src1), _np_ptr(sb),
                                    src_layer_stride, sp, _np_ptr(st)), "harvest_place_from")
        return st

    def revoke(self, cls, ids):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        _chk(lib.harvest_revoke(self.h, cls, _np_ptr(ids), ids.size), "harvest_revoke")

    # ---- data path ----------------------------------------------------------------------------------------------
    def fetch_kv(self, layer, d_table, d_n_blocks, d_dst_k, d_dst_v, d_seq_dst_block, dst_capacity_blocks, stream=None):
        """d_table int32 [n_seq][max_blocks], d_n_blocks int32 [n_seq], d_seq_dst_block int64/uint64 [n_seq]: torch
        device tensors."""
        n_seq, max_blocks = d_table.shape
        _chk(lib.harvest_fetch_kv(self.h, layer, _dev_ptr(d_table), _dev_ptr(d_n_blocks), n_seq, max_blocks,
                                  _dev_ptr(d_dst_k), _dev_ptr(d_dst_v), _dev_ptr(d_seq_dst_block), dst_capacity_blocks,
                                  _stream_ptr(stream)), "harvest_fetch_kv")

    def fetch_kv_static(self, layer, d_table, d_n_blocks, d_dst_k, d_dst_v, d_seq_dst_block, dst_capacity_blocks,
                        d_info=None, d_miss_idx=None, stream=None):
        """As fetch_kv, through the entry point that allocates nothing; d_info int32 [8], d_miss_idx int32 [n_seq *
        max_blocks]: torch device tensors or None."""
        n_seq, max_blocks = d_table.shape
        _chk(lib.harvest_fetch_kv_static(self.h, layer, _dev_ptr(d_table), _dev_ptr(d_n_blocks), n_seq, max_blocks,
                                         _dev_ptr(d_dst_k), _dev_ptr(d_dst_v), _dev_ptr(d_seq_dst_block),
                                         dst_capacity_blocks, _dev_ptr(d_info), _dev_ptr(d_miss_idx), _stream_ptr(stream)),
             "harvest_fetch_kv_static")

    def fetch_kv_again(self, layer, d_dst_k, d_dst_v, stream=None):
        _chk(lib.harvest_fetch_kv_again(self.h, layer, _dev_ptr(d_dst_k), _dev_ptr(d_dst_v), _stream_ptr(stream)),
             "harvest_fetch_kv_again")

    def fetch_kv_layers(self, layer_first, n_layers, d_table, d_n_blocks, d_dst_k, d_dst_v, dst_layer_stride_bytes,
                        d_seq_dst_block, cap_blocks, stream=None):
        n_seq, max_blocks = d_table.shape
        _chk(lib.harvest_fetch_kv_layers(self.h, layer_first, n_layers, _dev_ptr(d_table), _dev_ptr(d_n_blocks), n_seq,
                                         max_blocks, _dev_ptr(d_dst_k), _dev_ptr(d_dst_v), dst_layer_stride_bytes,
                                         _dev_ptr(d_seq_dst_block), cap_blocks, _stream_ptr(stream)),
             "harvest_fetch_kv_layers")

    def fetch_kv_head_major(self, layer, d_table, d_n_blocks, d_dst_k, d_dst_v, d_seq_dst_block, d_seq_cap_blocks,
                            dst_capacity_blocks, n_heads, block_tokens, stream=None):
        """As fetch_kv; d_seq_cap_blocks int32/uint32 [n_seq] device tensor."""
        n_seq, max_blocks = d_table.shape
        _chk(lib.harvest_fetch_kv_head_major(self.h, layer, _dev_ptr(d_table), _dev_ptr(d_n_blocks), n_seq, max_blocks,
                                             _dev_ptr(d_dst_k), _dev_ptr(d_dst_v), _dev_ptr(d_seq_dst_block),
                                             _dev_ptr(d_seq_cap_blocks), dst_capacity_blocks, n_heads, block_tokens,
                                             _stream_ptr(stream)), "harvest_fetch_kv_head_major")

    def fetch_experts(self, layer, d_topk, d_staging, n_staging_slots, d_expert_ptr, stream=None):
        n_tokens, k = d_topk.shape
        _chk(lib.harvest_fetch_experts(self.h, layer, _dev_ptr(d_topk), n_tokens, k, _dev_ptr(d_staging),
                                       n_staging_slots, _dev_ptr(d_expert_ptr), _stream_ptr(stream)),
             "harvest_fetch_experts")

    def release_stream(self, stream=None):
        _chk(lib.harvest_release_stream(self.h, _stream_ptr(stream)), "harvest_release_stream")

    def fetch_info(self, stream=None, miss_cap=0, cls=None):
        """cls: the latest fetch of that class on the stream (harvest_fetch_info_of); None: the latest fetch."""
        counts = harvest_fetch_counts()
        miss = np.zeros(max(1, miss_cap), dtype=np.uint32)
        n_miss = u32()
        if cls is None:
            _chk(lib.harvest_fetch_info(self.h, _stream_ptr(stream), ctypes.byref(counts), _np_ptr(miss), miss_cap,
                                        ctypes.byref(n_miss)), "harvest_fetch_info")
        else:
            _chk(lib.harvest_fetch_info_of(self.h, _stream_ptr(stream), cls, ctypes.byref(counts), _np_ptr(miss),
                                           miss_cap, ctypes.byref(n_miss)), "harvest_fetch_info_of")
        return counts.as_dict(), miss[:min(n_miss.value, miss_cap)].copy(), n_miss.value

    def evict(self, cls, layer, ids, d_src0, d_src1, src_block, src_layer_stride, flags=0, stream=None):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        sb = np.ascontiguousarray(src_block, dtype=np.uint64)
        assert sb.shape == ids.shape
        sp = vp(0) if self.no_device else _stream_ptr(stream)
        _chk(lib.harvest_evict(self.h, cls, layer, _np_ptr(ids), ids.size, _dev_ptr(d_src0), _dev_ptr(d_src1),
                               _np_ptr(sb), src_layer_stride, flags, sp), "harvest_evict")

    # ---- introspection ------------------------------------------------------------------------------------------
    def stats(self) -> harvest_stats_t:
        out = harvest_stats_t()
        _chk(lib.harvest_stats(self.h, ctypes.byref(out)), "harvest_stats")
        return out

    def profile(self) -> harvest_profile_t:
        out = harvest_profile_t()
        _chk(lib.harvest_profile(self.h, ctypes.byref(out)), "harvest_profile")
        return out


class Prefetcher:
    """harvest_prefetcher_*: a ring of two staging buffers filled on the library's fetch stream while the caller's
    compute stream uses the other one.  The buffers (torch tensors) are allocated here and lent to the library."""

    def __init__(self, h: Harvest, n_staging_slots: int):
        sp = h.spec[EXPERT]
        dev = torch.device("cuda", h.device)
        self.h = h
        self.staging = [torch.empty(max(1, n_staging_slots) * sp.chunk_bytes, dtype=torch.uint8, device=dev) for _ in range(2)]
        self.ptrs = [torch.zeros(sp.n_experts, dtype=torch.int64, device=dev) for _ in range(2)]
        self.n_staging_slots = n_staging_slots
        st = (vp * 2)(self.staging[0].data_ptr(), self.staging[1].data_ptr())
        pt = (vp * 2)(self.ptrs[0].data_ptr(), self.ptrs[1].data_ptr())
        pf = vp()
        _chk(lib.harvest_prefetcher_create(h.h, st, n_staging_slots, pt, ctypes.byref(pf)), "harvest_prefetcher_create")
        self.pf = pf
        h._prefetchers.append(weakref.ref(self))

    def close(self):
        if getattr(self, "pf", None):
            _chk(lib.harvest_prefetcher_destroy(self.pf), "harvest_prefetcher_destroy")
            self.pf = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def stream(self) -> int:
        return int(lib.harvest_prefetcher_stream(self.pf) or 0)

    def issue(self, layer, d_topk, topk_stream=None):
        n_tokens, k = d_topk.shape
        _chk(lib.harvest_prefetch_issue(self.pf, layer, _dev_ptr(d_topk), n_tokens, k, _stream_ptr(topk_stream)),
             "harvest_prefetch_issue")

    def acquire(self, compute_stream=None):
        """-> (staging tensor, pointer-table tensor) of the oldest issued fetch; compute_stream waits for it."""
        st, pt = vp(), vp()
        _chk(lib.harvest_prefetch_acquire(self.pf, _stream_ptr(compute_stream), ctypes.byref(st), ctypes.byref(pt)),
             "harvest_prefetch_acquire")
        b = 0 if st.value == self.staging[0].data_ptr() else 1
        assert st.value == self.staging[b].data_ptr() and pt.value == self.ptrs[b].data_ptr()
        return self.staging[b], self.ptrs[b]

    def release(self, compute_stream=None):
        _chk(lib.harvest_prefetch_release(self.pf, _stream_ptr(compute_stream)), "harvest_prefetch_release")

    def fetch_info(self, miss_cap=0):
        return self.h.fetch_info(stream=self.stream, miss_cap=miss_cap)


def plain_read(d_src, nbytes, d_sink, stream=None):
    _chk(lib.harvest_plain_read(_dev_ptr(d_src), nbytes, _dev_ptr(d_sink), _stream_ptr(stream)), "harvest_plain_read")


def plain_write(d_dst, nbytes, pattern=0, stream=None):
    _chk(lib.harvest_plain_write(_dev_ptr(d_dst), nbytes, pattern, _stream_ptr(stream)), "harvest_plain_write")


def plain_copy(d_dst, d_src, nbytes, stream=None):
    _chk(lib.harvest_plain_copy(_dev_ptr(d_dst), _dev_ptr(d_src), nbytes, _stream_ptr(stream)), "harvest_plain_copy")
