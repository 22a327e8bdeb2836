"""A position-dependent 64-bit checksum of a buffer (harness only; see digest.c for the definition and what it is for).

``digest(buf)`` takes a C-contiguous numpy uint8 array (computed by digest.c on the host cores) or a contiguous torch
uint8 tensor on any device (computed where the tensor lives, with the same definition written as tensor operations in
wrapping 64-bit integer arithmetic) and returns a Python int in [0, 2^64).  Buffer sizes must be multiples of 8.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import _load

M = 65536
_MASK = (1 << 64) - 1
_weights = {}


def _host_lib():
    lib = _load()
    if not getattr(lib, "_digest_bound", False):
        lib.wl_digest.restype = ctypes.c_uint64
        lib.wl_digest.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
        lib.wl_digest_weight.restype = ctypes.c_uint64
        lib.wl_digest_weight.argtypes = [ctypes.c_uint64]
        lib.wl_digest_piece_factor.restype = ctypes.c_uint64
        lib.wl_digest_piece_factor.argtypes = [ctypes.c_uint64]
        lib._digest_bound = True
    return lib


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = x + np.uint64(0x9E3779B97F4A7C15)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return x ^ (x >> np.uint64(31))


def weights() -> np.ndarray:
    return _splitmix64(np.arange(M, dtype=np.uint64)) | np.uint64(1)


def piece_factors(n_pieces: int) -> np.ndarray:
    return _splitmix64(np.uint64(1 << 32) + np.arange(n_pieces, dtype=np.uint64)) | np.uint64(1)


def _digest_torch(t) -> int:
    import torch
    assert t.dtype == torch.uint8 and t.is_contiguous() and t.numel() % 8 == 0
    x = t.view(torch.int64)
    n = x.numel()
    key = str(t.device)
    if key not in _weights:
        _weights[key] = torch.from_numpy(weights().view(np.int64)).to(t.device)
    w = _weights[key]
    n_pieces = (n + M - 1) // M
    c = torch.from_numpy(piece_factors(n_pieces).view(np.int64)).to(t.device)
    full = n // M
    total = torch.zeros((), dtype=torch.int64, device=t.device)
    slab = 2048                                        # pieces per step: bounds the temporary at 1 GiB
    for p0 in range(0, full, slab):
        p1 = min(full, p0 + slab)
        sums = (x[p0 * M:p1 * M].view(p1 - p0, M) * w).sum(dim=1)
        total = total + (sums * c[p0:p1]).sum()
    if n > full * M:
        tail = x[full * M:]
        total = total + (tail * w[:tail.numel()]).sum() * c[full]
    return int(total.item()) & _MASK


def digest(buf) -> int:
    if isinstance(buf, np.ndarray):
        assert buf.dtype == np.uint8 and buf.flags.c_contiguous and buf.size % 8 == 0
        return int(_host_lib().wl_digest(buf.ctypes.data_as(ctypes.c_void_p), buf.size // 8))
    return _digest_torch(buf)
