"""TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.

ctypes loader for the single-threaded C++ oracle of the KV-reclaim path
(``warmkv_oracle.cpp``).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
benchmark's CPU-baseline leg may import this package; the HIP library and its
Python binding never do, and this package never imports them.

All functions work on host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC_PATH = os.path.join(_HERE, "warmkv_oracle.cpp")
LIB_PATH = os.path.join(_HERE, "libwarmkv_oracle.so")

OK = 0
E_NULL = -1
E_RANGE = -2
E_TOOBIG = -4
E_OVERLAP = -5
E_NOSPACE = -7


def build(force: bool = False, sanitize: bool = False, out: str | None = None) -> str:
    """Compile the oracle with g++.  ``sanitize`` adds ASan/UBSan (host code only)."""
    out = out or LIB_PATH
    stale = (not os.path.exists(out)) or os.path.getmtime(out) < os.path.getmtime(SRC_PATH)
    if force or stale:
        cmd = ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", SRC_PATH, "-o", out]
        if sanitize:
            cmd[3:3] = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
        subprocess.run(cmd, check=True)
    return out


class _Tensor(ctypes.Structure):
    _fields_ = [("host_ptr", ctypes.c_void_p), ("bytes", ctypes.c_uint64), ("dst_offset", ctypes.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
        L.oracle_plan.restype = ctypes.c_int
        L.oracle_plan.argtypes = [vp, u32, u32, vp, vp, vp, vp, vp]
        L.oracle_compact.restype = ctypes.c_int
        L.oracle_compact.argtypes = [vp, u64, vp, vp, u32]
        L.oracle_remap.restype = ctypes.c_int64
        L.oracle_remap.argtypes = [vp, u64, vp, u32]
        L.oracle_materialize.restype = ctypes.c_int
        L.oracle_materialize.argtypes = [vp, u64, u64, ctypes.POINTER(_Tensor), u32]
        L.oracle_compact_layer_major.restype = ctypes.c_int
        L.oracle_compact_layer_major.argtypes = [vp, u64, u32, u64, vp, vp, u32]
        L.oracle_materialize_strips.restype = ctypes.c_int
        L.oracle_materialize_strips.argtypes = [vp, u64, u32, u32, u32, u64, ctypes.POINTER(_Tensor), u32]
        L.oracle_grow.restype = ctypes.c_int64
        L.oracle_grow.argtypes = [u64, u32, u32, u32, ctypes.POINTER(_Tensor), u32, vp, vp]
        L.oracle_reserve_blocks.restype = ctypes.c_int64
        L.oracle_reserve_blocks.argtypes = [u64, u64, u32, u32]
        L.oracle_grow_strips.restype = ctypes.c_int64
        L.oracle_grow_strips.argtypes = [u64, u32, u32, u64, u32, u32, ctypes.POINTER(_Tensor), u32, vp, vp]
        L.oracle_vmm_select.restype = ctypes.c_int
        L.oracle_vmm_select.argtypes = [vp, u32, u32, vp]
        _lib = L
    return _lib


def _p(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


class Plan:
    """Result of :func:`plan`.  ``status`` is OK or E_NOSPACE; arrays are valid only if OK."""

    def __init__(self, status, src, dst, new_id, live_out, n_moves, num_blocks, boundary):
        self.status = status
        self.src = src
        self.dst = dst
        self.new_id = new_id
        self.live_out = live_out
        self.n_moves = n_moves
        self.num_blocks = num_blocks
        self.boundary = boundary


def plan(live: np.ndarray, num_blocks: int, boundary: int) -> Plan:
    live = np.ascontiguousarray(live, dtype=np.uint64)
    assert live.size == (num_blocks + 63) // 64
    cap = max(1, min(num_blocks - boundary, boundary)) if boundary <= num_blocks else 1
    src = np.full(cap, -1, dtype=np.int32)
    dst = np.full(cap, -1, dtype=np.int32)
    new_id = np.full(max(1, num_blocks), -1, dtype=np.int32)
    live_out = np.zeros(max(1, live.size), dtype=np.uint64)
    n = np.zeros(1, dtype=np.uint32)
    live_arg = live if live.size else np.zeros(1, dtype=np.uint64)
    rc = lib().oracle_plan(_p(live_arg), num_blocks, boundary, _p(src), _p(dst), _p(new_id),
                           _p(live_out), _p(n))
    if rc not in (OK, E_NOSPACE):
        raise ValueError(f"oracle_plan: error {rc}")
    k = int(n[0]) if rc == OK else 0
    return Plan(rc, src[:k], dst[:k], new_id[:num_blocks], live_out[:live.size], k, num_blocks, boundary)


def compact(pool: np.ndarray, block_bytes: int, p: Plan) -> None:
    """In place on a uint8 host pool of num_blocks * block_bytes bytes."""
    assert pool.dtype == np.uint8 and pool.size == p.num_blocks * block_bytes
    if p.status != OK:
        return
    src = np.ascontiguousarray(p.src)
    dst = np.ascontiguousarray(p.dst)
    rc = lib().oracle_compact(_p(pool), block_bytes, _p(src) if p.n_moves else None,
                              _p(dst) if p.n_moves else None, p.n_moves)
    if rc != OK:
        raise ValueError(f"oracle_compact: error {rc}")


def compact_layer_major(pool: np.ndarray, tile_bytes: int, num_layers: int, layer_stride: int, p: Plan) -> None:
    """In place on a uint8 host pool laid out as num_layers slabs of layer_stride bytes."""
    assert pool.dtype == np.uint8 and pool.size >= (num_layers - 1) * layer_stride + p.num_blocks * tile_bytes
    if p.status != OK or p.n_moves == 0:
        return
    src = np.ascontiguousarray(p.src)
    dst = np.ascontiguousarray(p.dst)
    rc = lib().oracle_compact_layer_major(_p(pool), tile_bytes, num_layers, layer_stride, _p(src), _p(dst), p.n_moves)
    if rc != OK:
        raise ValueError(f"oracle_compact_layer_major: error {rc}")


def materialize_strips(pool: np.ndarray, tile_bytes: int, num_layers: int, num_blocks: int, boundary: int,
                       layer_stride: int, tensors) -> int:
    """tensors: iterable of (uint8 host array, region offset).  Returns the oracle's status code."""
    tensors = list(tensors)
    arr = (_Tensor * max(1, len(tensors)))()
    keep = []
    for i, (buf, off) in enumerate(tensors):
        buf = np.ascontiguousarray(buf).view(np.uint8).reshape(-1)
        keep.append(buf)
        arr[i] = _Tensor(buf.ctypes.data if buf.size else None, buf.size, off)
    return int(lib().oracle_materialize_strips(_p(pool), tile_bytes, num_layers, num_blocks, boundary,
                                               layer_stride, arr, len(tensors)))


def remap(tables: np.ndarray, p: Plan) -> int:
    """In place on an int32 table array; returns the number of bad entries left alone."""
    assert tables.dtype == np.int32 and tables.flags["C_CONTIGUOUS"]
    if p.status != OK:
        return 0
    new_id = np.ascontiguousarray(p.new_id) if p.num_blocks else np.zeros(1, dtype=np.int32)
    rc = lib().oracle_remap(_p(tables) if tables.size else None, tables.size, _p(new_id), p.num_blocks)
    if rc < 0:
        raise ValueError(f"oracle_remap: error {rc}")
    return int(rc)


def materialize(pool: np.ndarray, region_offset: int, tensors) -> int:
    """tensors: iterable of (uint8 host array, dst_offset).  Returns the oracle's status code."""
    tensors = list(tensors)
    arr = (_Tensor * max(1, len(tensors)))()
    keep = []
    for i, (buf, off) in enumerate(tensors):
        buf = np.ascontiguousarray(buf).view(np.uint8).reshape(-1)
        keep.append(buf)
        arr[i] = _Tensor(buf.ctypes.data if buf.size else None, buf.size, off)
    return int(lib().oracle_materialize(_p(pool), pool.size, region_offset, arr, len(tensors)))


def reserve_blocks(capacity_blocks: int, used_blocks: int, running: int, max_batch: int) -> int:
    return int(lib().oracle_reserve_blocks(capacity_blocks, used_blocks, running, max_batch))


def grow(block_bytes: int, num_blocks: int, old_boundary: int, new_boundary: int, extents):
    """extents: iterable of (bytes, dst_offset).  Returns (n_lost, evicted uint8[], new_offset uint64[])
    or (negative error, None, None)."""
    extents = list(extents)
    arr = (_Tensor * max(1, len(extents)))()
    for i, (nbytes, off) in enumerate(extents):
        arr[i] = _Tensor(None, nbytes, off)
    ev = np.zeros(max(1, len(extents)), dtype=np.uint8)
    no = np.zeros(max(1, len(extents)), dtype=np.uint64)
    rc = int(lib().oracle_grow(block_bytes, num_blocks, old_boundary, new_boundary, arr, len(extents), _p(ev), _p(no)))
    if rc < 0:
        return rc, None, None
    return rc, ev[:len(extents)], no[:len(extents)]


def grow_strips(tile_bytes: int, num_layers: int, num_blocks: int, layer_stride: int, old_boundary: int,
                new_boundary: int, extents):
    """Reverse switch in a layer-major pool; arguments and result as for :func:`grow`."""
    extents = list(extents)
    arr = (_Tensor * max(1, len(extents)))()
    for i, (nbytes, off) in enumerate(extents):
        arr[i] = _Tensor(None, nbytes, off)
    ev = np.zeros(max(1, len(extents)), dtype=np.uint8)
    no = np.zeros(max(1, len(extents)), dtype=np.uint64)
    rc = int(lib().oracle_grow_strips(tile_bytes, num_layers, num_blocks, layer_stride, old_boundary, new_boundary,
                                      arr, len(extents), _p(ev), _p(no)))
    if rc < 0:
        return rc, None, None
    return rc, ev[:len(extents)], no[:len(extents)]


def vmm_select(live: np.ndarray, num_blocks: int, want: int):
    """Blocks that lend their pages to the slot in the no-move variant, in slot order
    (int32 array), or None if fewer than ``want`` blocks are free."""
    live = np.ascontiguousarray(live, dtype=np.uint64)
    assert live.size == (num_blocks + 63) // 64
    ids = np.full(max(1, want), -1, dtype=np.int32)
    rc = lib().oracle_vmm_select(_p(live if live.size else np.zeros(1, dtype=np.uint64)), num_blocks, want, _p(ids))
    if rc == E_NOSPACE:
        return None
    if rc != OK:
        raise ValueError(f"oracle_vmm_select: error {rc}")
    return ids[:want]
