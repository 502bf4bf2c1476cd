"""Seeded byte content for KV pools and weight tensors.

Content is a pure function of (seed, content id, 64-bit word index), so any
block can be regenerated on its own, on the host (numpy, here) or on the
device (``fill.hip``, same arithmetic), without holding a second copy of a
40-120 GiB pool.  Word ``w`` of item ``cid`` is output ``w+1`` of a SplitMix64
stream seeded with ``mix64(seed + (cid+1)*GOLDEN)``.

Two renderings of a word:
  * ``table is None``: the 8 raw little-endian bytes (fp8-as-bytes pools);
  * ``table`` given: each 16-bit field indexes a 65 536-entry table of bf16 bit
    patterns (quantiles of a normal distribution), giving four bf16 values.
    No transcendental runs on the device, so host and device agree bit for bit.

This is input generation only; it holds none of the reclaim method's logic.
"""
from __future__ import annotations

import ctypes
import hashlib
import os
import re
import subprocess

import numpy as np

from .rng import GOLDEN, MASK64, mix64, mix64_int

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwarmkv_synth.so")
_SRC_PATH = os.path.join(_HERE, "fill.hip")


def normal_bf16_table(sigma: float = 1.0) -> np.ndarray:
    """uint16[65536]: bf16 (round-to-nearest-even) of sigma * Phi^-1((i+0.5)/65536)."""
    from scipy.special import ndtri
    q = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    f32 = (sigma * ndtri(q)).astype(np.float32)
    bits = f32.view(np.uint32).astype(np.uint64)
    rounded = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return rounded.astype(np.uint16)


def item_base(seed: int, cid: int) -> int:
    return mix64_int((seed + (cid + 1) * GOLDEN) & MASK64)


def item_words(seed: int, cid: int, first_word: int, n_words: int) -> np.ndarray:
    """uint64[n_words]: words first_word .. first_word+n_words-1 of item ``cid``."""
    w = np.arange(first_word + 1, first_word + 1 + n_words, dtype=np.uint64)
    return mix64(np.uint64(item_base(seed, cid)) + w * np.uint64(GOLDEN))


def item_bytes_host(seed: int, cid: int, nbytes: int, table: np.ndarray | None,
                    byte_offset: int = 0) -> np.ndarray:
    """uint8[nbytes] of item ``cid`` starting at ``byte_offset`` (both multiples of 8)."""
    assert nbytes % 8 == 0 and byte_offset % 8 == 0
    words = item_words(seed, cid, byte_offset // 8, nbytes // 8)
    if table is None:
        return words.view(np.uint8)
    fields = words.view(np.uint16)          # little-endian: field i = bits 16i..16i+15
    return table[fields].view(np.uint8)


def fill_host(dst: np.ndarray, item_bytes: int, cids, seed: int, table: np.ndarray | None) -> None:
    """Fill a uint8 host buffer holding len(cids) items of item_bytes each."""
    flat = dst.reshape(-1)
    for i, cid in enumerate(cids):
        flat[i * item_bytes:(i + 1) * item_bytes] = item_bytes_host(seed, int(cid), item_bytes, table)


# --------------------------------------------------------------------------
# Device-side generator (same arithmetic, HIP).  Test/bench infrastructure.
# --------------------------------------------------------------------------
def _source_id() -> str:
    with open(_SRC_PATH, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def _built_id() -> str | None:
    if not os.path.exists(_LIB_PATH):
        return None
    with open(_LIB_PATH, "rb") as f:
        m = re.search(rb"SYNTH_BUILD_ID=([0-9a-f]{16})\0", f.read())
    return m.group(1).decode() if m else None


def build_device_fill(force: bool = False) -> str:
    """Compile fill.hip unless the library at hand was built from this very source text."""
    want = _source_id()
    if force or _built_id() != want:
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", f'-DSYNTH_BUILD_ID="{want}"',
               _SRC_PATH, "-o", _LIB_PATH]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_device_fill()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.synth_fill.restype = ctypes.c_int
        lib.synth_fill.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                   ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
        lib.synth_host_alloc.restype = ctypes.c_void_p
        lib.synth_host_alloc.argtypes = [ctypes.c_uint64]
        lib.synth_host_free.restype = ctypes.c_int
        lib.synth_host_free.argtypes = [ctypes.c_void_p]
        lib.synth_copy.restype = ctypes.c_int
        lib.synth_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
        _lib = lib
    return _lib


class PinnedHostBuffer:
    """Pinned host memory of exactly nbytes (torch's pinned allocator rounds sizes up to a power of
    two, which a 40 GiB pool copy cannot afford).  ``array`` is a uint8 numpy view of it."""

    def __init__(self, nbytes: int):
        self.nbytes = nbytes
        self.ptr = _load().synth_host_alloc(nbytes)
        if not self.ptr:
            raise MemoryError(f"cannot pin {nbytes} bytes of host memory")
        self.array = np.ctypeslib.as_array((ctypes.c_uint8 * nbytes).from_address(self.ptr))

    def free(self) -> None:
        if self.ptr:
            self.array = None
            _load().synth_host_free(self.ptr)
            self.ptr = None

    def __del__(self):
        self.free()


def copy_bytes(dst_ptr: int, src_ptr: int, nbytes: int) -> None:
    """Synchronous copy between any two of pinned host and device memory."""
    if nbytes and _load().synth_copy(dst_ptr, src_ptr, nbytes) != 0:
        raise RuntimeError("synth_copy failed")


def fill_device(dst_ptr: int, n_items: int, item_bytes: int, seed: int, *,
                cids_ptr: int = 0, cid0: int = 0, table_ptr: int = 0, byte_offset: int = 0,
                stream: int = 0) -> None:
    """Fill device memory at ``dst_ptr`` with n_items items.  Item i has content
    id ``cids[i]`` (device int32 array) when ``cids_ptr`` is non-zero, else
    ``cid0 + i``; it receives bytes [byte_offset, byte_offset + item_bytes) of that
    content.  ``table_ptr`` is a device uint16[65536] table or 0 for raw bytes."""
    assert byte_offset % 8 == 0
    rc = _load().synth_fill(dst_ptr, n_items, item_bytes, seed & MASK64, cids_ptr, cid0,
                            table_ptr, byte_offset // 8, stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill failed with code {rc}")
