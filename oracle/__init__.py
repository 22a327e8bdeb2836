"""TEST INFRASTRUCTURE - a plain CPU oracle for Harvest's tiered cache fetch.

Thin ctypes wrapper over ``harvest_oracle.c`` (which states, citing the paper,
what every operation computes).  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package.  It
shares no code with, and never imports, the HIP library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

HOST, CACHE, LOCAL, NONE = 0, 1, 2, 3
OK, EINVAL, ENOSPC, ENOENT, ELOST = 0, -1, -2, -3, -5
EVICT_DEMOTE = 1
POISON = 0xA5
# kinds reported by fetch_experts
UNSELECTED, IN_PLACE, STAGED, OVERFLOW, LOST = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_CB = ctypes.CFUNCTYPE(None, ctypes.c_uint32, ctypes.c_void_p)


class Counts(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in
                ("n_requests", "n_local", "n_cache", "n_host", "n_lost", "n_invalid")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", _LIB_PATH,
                               os.path.join(_HERE, "harvest_oracle.c")])
    return _LIB_PATH


def _bind(path):
    L = ctypes.CDLL(path)
    vp, u32, u64, i32, i64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int, ctypes.c_int64
    L.orc_create.restype = vp
    L.orc_create.argtypes = [u32, u32, u64, u32, u32, u32, u32, i32]
    L.orc_destroy.argtypes = [vp]
    L.orc_plane.restype = vp
    L.orc_plane.argtypes = [vp, i32, u32]
    L.orc_n_objects.restype = u32
    L.orc_n_objects.argtypes = [vp]
    L.orc_register.argtypes = [vp, u32, vp, i32, vp]
    L.orc_lookup.argtypes = [vp, u32, vp, vp, vp, vp]
    L.orc_restore.argtypes = [vp, vp, u32]
    L.orc_set_object.argtypes = [vp, u32, vp, vp]
    L.orc_adopt.argtypes = [vp, u32]
    L.orc_write_local.argtypes = [vp, u32, u32, u32, u64, vp, u64]
    L.orc_place.argtypes = [vp, vp, u32, vp]
    L.orc_place_from.argtypes = [vp, vp, u32, vp, vp, vp, u64, vp]
    L.orc_revoke.argtypes = [vp, vp, u32, _CB, vp]
    L.orc_fetch_kv.argtypes = [vp, u32, vp, vp, u32, u32, vp, vp, vp, u64, vp, vp, vp, i32]
    L.orc_fetch_kv_plain.argtypes = [vp, u32, vp, vp, u32, u32, vp, vp, vp, u64]
    L.orc_fetch_kv_head_major.argtypes = [vp, u32, vp, vp, u32, u32, vp, vp, vp, vp, u64, u32, u32, vp, vp, vp]
    L.orc_fetch_experts.argtypes = [vp, u32, u32, vp, u32, u32, vp, u32, vp, vp, vp, vp, vp]
    L.orc_evict.argtypes = [vp, i32, vp, u32, vp, vp, vp, u64, i32]
    L.orc_segpool_create.restype = vp
    L.orc_segpool_create.argtypes = [u64, u64]
    L.orc_segpool_destroy.argtypes = [vp]
    L.orc_segpool_mem.restype = vp
    L.orc_segpool_mem.argtypes = [vp]
    L.orc_segpool_free_runs.restype = u64
    L.orc_segpool_free_runs.argtypes = [vp, vp, vp, u64]
    L.orc_segpool_alloc.restype = i64
    L.orc_segpool_alloc.argtypes = [vp, u64]
    L.orc_segpool_free.restype = None
    L.orc_segpool_free.argtypes = [vp, u64, u64]
    L.orc_attach_segpool.argtypes = [vp, vp]
    return L


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = _bind(_LIB_PATH)
    return _lib


def use_library(path=None):
    """Tests only: make new OracleClass objects use another build of the oracle (None = the regular one)."""
    global _lib
    _lib = _bind(path) if path else None


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what}: status {code}")
        self.code = code


class SegPool:
    """Cache-tier storage shared by several classes: variable-size segments, best-fit allocation."""

    def __init__(self, n_bytes, granule):
        self.L = _load()
        self.n_bytes, self.granule = int(n_bytes), int(granule)
        self.h = self.L.orc_segpool_create(self.n_bytes, self.granule)
        if not self.h:
            raise OracleError(EINVAL, "segpool create")

    def close(self):
        if self.h:
            self.L.orc_segpool_destroy(self.h)
            self.h = None

    def mem(self) -> np.ndarray:
        buf = (ctypes.c_uint8 * max(1, self.n_bytes)).from_address(self.L.orc_segpool_mem(self.h))
        return np.frombuffer(buf, dtype=np.uint8)[:self.n_bytes]

    def alloc(self, n_granules) -> int:
        return int(self.L.orc_segpool_alloc(self.h, int(n_granules)))

    def free(self, off, n_granules):
        self.L.orc_segpool_free(self.h, int(off), int(n_granules))

    def free_runs(self):
        """[(offset, length)] in granules, ascending."""
        cap = self.n_bytes // self.granule // 2 + 2
        off, ln = np.empty(cap, np.uint64), np.empty(cap, np.uint64)
        n = int(self.L.orc_segpool_free_runs(self.h, _p(off), _p(ln), cap))
        return [(int(off[i]), int(ln[i])) for i in range(n)]


class OracleClass:
    """One class of objects (KV blocks, or expert weights) with its three tiers and directory."""

    def __init__(self, n_layers, n_planes, chunk_bytes, max_objects, n_host_slots, n_cache_slots, n_local_slots,
                 poison=False, segpool=None):
        self.L = _load()
        self.n_layers, self.n_planes, self.chunk_bytes = n_layers, n_planes, chunk_bytes
        self.max_objects = max_objects
        self.n_slots = {HOST: n_host_slots, CACHE: n_cache_slots, LOCAL: n_local_slots}
        self.h = self.L.orc_create(n_layers, n_planes, chunk_bytes, max_objects, n_host_slots, n_cache_slots,
                                   n_local_slots, int(poison))
        if not self.h:
            raise OracleError(EINVAL, "create")
        self.segpool = segpool
        if segpool is not None:
            rc = self.L.orc_attach_segpool(self.h, segpool.h)
            if rc != OK:
                raise OracleError(rc, "attach_segpool")
        self.revoked_log = []          # ids, in callback order
        self._cb = _CB(lambda i, _u: self.revoked_log.append(int(i)))

    def close(self):
        if self.h:
            self.L.orc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- views -----------------------------------------------------------------------------------------
    def plane(self, which, plane=0) -> np.ndarray:
        """uint8 view [n_layers][n_slots][chunk_bytes] of a tier plane (which: HOST/CACHE/LOCAL, or 3 = truth)."""
        n_slots = self.max_objects if which == 3 else self.n_slots[which]
        ptr = self.L.orc_plane(self.h, which, plane)
        n = self.n_layers * n_slots * self.chunk_bytes
        buf = (ctypes.c_uint8 * n).from_address(ptr)
        return np.frombuffer(buf, dtype=np.uint8).reshape(self.n_layers, n_slots, self.chunk_bytes)

    @property
    def n_objects(self):
        return int(self.L.orc_n_objects(self.h))

    # ---- directory -------------------------------------------------------------------------------------
    def register(self, n, host_slots=None, tier=HOST) -> np.ndarray:
        hs = None if host_slots is None else np.ascontiguousarray(host_slots, dtype=np.int64)
        out = np.empty(n, dtype=np.uint32)
        rc = self.L.orc_register(self.h, n, _p(hs), tier, _p(out))
        if rc != OK:
            raise OracleError(rc, "register")
        return out

    def lookup(self, obj):
        t, s, g, hs = ctypes.c_int(), ctypes.c_int64(), ctypes.c_uint32(), ctypes.c_int64()
        rc = self.L.orc_lookup(self.h, int(obj), ctypes.byref(t), ctypes.byref(s), ctypes.byref(g), ctypes.byref(hs))
        if rc != OK:
            raise OracleError(rc, "lookup")
        return t.value, s.value, g.value, hs.value

    def set_object(self, obj, src0, src1=None):
        src0 = np.ascontiguousarray(src0, dtype=np.uint8)
        assert src0.size == self.n_layers * self.chunk_bytes
        if self.n_planes == 2:
            src1 = np.ascontiguousarray(src1, dtype=np.uint8)
            assert src1.size == src0.size
        rc = self.L.orc_set_object(self.h, int(obj), _p(src0), _p(src1))
        if rc != OK:
            raise OracleError(rc, "set_object")

    def adopt(self, ids):
        for i in np.atleast_1d(ids):
            rc = self.L.orc_adopt(self.h, int(i))
            if rc != OK:
                raise OracleError(rc, "adopt")

    def write_local(self, obj, plane, layer, offset, data):
        data = np.ascontiguousarray(data, dtype=np.uint8)
        rc = self.L.orc_write_local(self.h, int(obj), plane, layer, offset, _p(data), data.size)
        if rc != OK:
            raise OracleError(rc, "write_local")

    def place(self, ids) -> np.ndarray:
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        st = np.zeros(ids.size, dtype=np.int32)
        rc = self.L.orc_place(self.h, _p(ids), ids.size, _p(st))
        if rc != OK:
            raise OracleError(rc, "place")
        return st

    def place_from(self, ids, src0, src1, src_block, src_layer_stride) -> np.ndarray:
        """Placement from bytes held elsewhere than the host copy: planes laid out [layer][src_layer_stride][chunk]."""
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        sb = np.ascontiguousarray(src_block, dtype=np.uint64)
        assert sb.shape == ids.shape
        need = self.n_layers * src_layer_stride * self.chunk_bytes
        src0 = np.ascontiguousarray(src0, dtype=np.uint8)
        assert src0.size >= need
        if self.n_planes == 2:
            src1 = np.ascontiguousarray(src1, dtype=np.uint8)
            assert src1.size >= need
        st = np.zeros(ids.size, dtype=np.int32)
        rc = self.L.orc_place_from(self.h, _p(ids), ids.size, _p(src0), _p(src1), _p(sb), src_layer_stride, _p(st))
        if rc != OK:
            raise OracleError(rc, "place_from")
        return st

    def revoke(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        rc = self.L.orc_revoke(self.h, _p(ids), ids.size, self._cb, None)
        if rc != OK:
            raise OracleError(rc, "revoke")

    # ---- data path -------------------------------------------------------------------------------------
    def fetch_kv(self, layer, table, n_blocks, seq_dst_block, dst_capacity_blocks, dst_k=None, dst_v=None,
                 plain=False, threads=1):
        """Returns (dst_k, dst_v, miss_idx, counts).  table int32 [n_seq][max_blocks]."""
        table = np.ascontiguousarray(table, dtype=np.int32)
        n_seq, max_blocks = table.shape
        n_blocks = np.ascontiguousarray(n_blocks, dtype=np.int32)
        sdb = np.ascontiguousarray(seq_dst_block, dtype=np.uint64)
        assert n_blocks.shape == (n_seq,) and sdb.shape == (n_seq,)
        nbytes = dst_capacity_blocks * self.chunk_bytes
        if dst_k is None:
            dst_k = np.zeros(nbytes, dtype=np.uint8)
        if dst_v is None and self.n_planes == 2:
            dst_v = np.zeros(nbytes, dtype=np.uint8)
        assert dst_k.size == nbytes and (dst_v is None or dst_v.size == nbytes)
        if plain:
            rc = self.L.orc_fetch_kv_plain(self.h, layer, _p(table), _p(n_blocks), n_seq, max_blocks, _p(dst_k),
                                           _p(dst_v), _p(sdb), dst_capacity_blocks)
            if rc != OK:
                raise OracleError(rc, "fetch_kv_plain")
            return dst_k, dst_v, None, None
        miss = np.zeros(max(1, n_seq * max_blocks), dtype=np.uint32)
        n_miss = ctypes.c_uint32()
        counts = Counts()
        rc = self.L.orc_fetch_kv(self.h, layer, _p(table), _p(n_blocks), n_seq, max_blocks, _p(dst_k), _p(dst_v),
                                 _p(sdb), dst_capacity_blocks, _p(miss), ctypes.byref(n_miss), ctypes.byref(counts),
                                 threads)
        if rc != OK:
            raise OracleError(rc, "fetch_kv")
        return dst_k, dst_v, miss[:n_miss.value].copy(), counts.as_dict()

    def fetch_kv_head_major(self, layer, table, n_blocks, seq_dst_block, seq_cap_blocks, dst_capacity_blocks, n_heads,
                            block_tokens, dst_k=None, dst_v=None):
        """Returns (dst_k, dst_v, miss_idx, counts); destination per sequence is [n_heads][cap * block_tokens][head_bytes]."""
        table = np.ascontiguousarray(table, dtype=np.int32)
        n_seq, max_blocks = table.shape
        n_blocks = np.ascontiguousarray(n_blocks, dtype=np.int32)
        sdb = np.ascontiguousarray(seq_dst_block, dtype=np.uint64)
        cap = np.ascontiguousarray(seq_cap_blocks, dtype=np.uint32)
        assert n_blocks.shape == (n_seq,) and sdb.shape == (n_seq,) and cap.shape == (n_seq,)
        nbytes = dst_capacity_blocks * self.chunk_bytes
        if dst_k is None:
            dst_k = np.zeros(nbytes, dtype=np.uint8)
        if dst_v is None and self.n_planes == 2:
            dst_v = np.zeros(nbytes, dtype=np.uint8)
        miss = np.zeros(max(1, n_seq * max_blocks), dtype=np.uint32)
        n_miss = ctypes.c_uint32()
        counts = Counts()
        rc = self.L.orc_fetch_kv_head_major(self.h, layer, _p(table), _p(n_blocks), n_seq, max_blocks, _p(dst_k),
                                            _p(dst_v), _p(sdb), _p(cap), dst_capacity_blocks, n_heads, block_tokens,
                                            _p(miss), ctypes.byref(n_miss), ctypes.byref(counts))
        if rc != OK:
            raise OracleError(rc, "fetch_kv_head_major")
        return dst_k, dst_v, miss[:n_miss.value].copy(), counts.as_dict()

    def fetch_experts(self, layer, n_experts, topk, n_staging_slots, staging=None):
        """Returns (staging, kind[n_experts], where[n_experts], miss_idx, counts)."""
        topk = np.ascontiguousarray(topk, dtype=np.int32)
        n_tokens, k = topk.shape
        if staging is None:
            staging = np.zeros(n_staging_slots * self.chunk_bytes, dtype=np.uint8)
        kind = np.zeros(n_experts, dtype=np.int32)
        where = np.zeros(n_experts, dtype=np.int64)
        miss = np.zeros(max(1, n_experts), dtype=np.uint32)
        n_miss = ctypes.c_uint32()
        counts = Counts()
        rc = self.L.orc_fetch_experts(self.h, layer, n_experts, _p(topk), n_tokens, k, _p(staging), n_staging_slots,
                                      _p(kind), _p(where), _p(miss), ctypes.byref(n_miss), ctypes.byref(counts))
        if rc != OK:
            raise OracleError(rc, "fetch_experts")
        return staging, kind, where, miss[:n_miss.value].copy(), counts.as_dict()

    def restore(self, ids):
        """Lost objects come back into local HBM (their bytes are then written by the caller)."""
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        rc = self.L.orc_restore(self.h, _p(ids), ids.size)
        if rc != OK:
            raise OracleError(rc, "restore")

    def evict(self, layer, ids, src_k, src_v, src_block, src_layer_stride, flags=0):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        sb = np.ascontiguousarray(src_block, dtype=np.uint64)
        assert sb.shape == ids.shape
        n_src_layers = self.n_layers if layer < 0 else 1
        need = n_src_layers * src_layer_stride * self.chunk_bytes
        src_k = np.ascontiguousarray(src_k, dtype=np.uint8)
        assert src_k.size >= need
        if self.n_planes == 2:
            src_v = np.ascontiguousarray(src_v, dtype=np.uint8)
            assert src_v.size >= need
        rc = self.L.orc_evict(self.h, layer, _p(ids), ids.size, _p(src_k), _p(src_v), _p(sb), src_layer_stride, flags)
        if rc != OK:
            raise OracleError(rc, "evict")
