"""ctypes binding of libwarmkv.so: the same names as the C ABI (include/warmkv.h),
argument marshalling only.  Every step runs in the library's HIP kernels; there
is no fallback: if the library is missing or was not built this module raises.

Device and host buffers may be given as integers (raw addresses) or as any
object with a ``data_ptr()`` method (torch tensors); streams and events as
integers (``torch.cuda.Stream.cuda_stream``, ``torch.cuda.Event.cuda_event``)
or 0 / None.
"""
from __future__ import annotations

import ctypes
import os
import re
import sys
from ctypes import POINTER, Structure, byref, c_char_p, c_int, c_int32, c_int64, c_size_t, c_uint32, c_uint64, c_void_p

from . import build as _build

KV_OK = 0
KV_E_NULL = -1
KV_E_RANGE = -2
KV_E_ALIGN = -3
KV_E_TOOBIG = -4
KV_E_OVERLAP = -5
KV_E_HIP = -6
KV_E_NOSPACE = -7
KV_E_BADPLAN = -8
KV_E_NOMEM = -9

_NAMES = {KV_OK: "KV_OK", KV_E_NULL: "KV_E_NULL", KV_E_RANGE: "KV_E_RANGE", KV_E_ALIGN: "KV_E_ALIGN",
          KV_E_TOOBIG: "KV_E_TOOBIG", KV_E_OVERLAP: "KV_E_OVERLAP", KV_E_HIP: "KV_E_HIP",
          KV_E_NOSPACE: "KV_E_NOSPACE", KV_E_BADPLAN: "KV_E_BADPLAN", KV_E_NOMEM: "KV_E_NOMEM"}

EXPORTS = ("kv_plan_workspace_bytes", "kv_plan_bind", "kv_plan_reclaim", "kv_compact", "kv_compact_launch",
           "kv_remap_tables", "kv_reclaim", "kv_plan_fetch", "weights_materialize", "weights_materialize_schedule",
           "weights_materialize_pipelined", "kv_compact_moves", "kv_compact_layers", "kv_movers_in_front", "weights_materialize_front", "weights_materialize_streams",
           "kv_switch", "kv_reclaim_static", "kv_reserve_blocks", "kv_grow", "kv_vmm_pool_create", "kv_vmm_kv_base", "kv_vmm_slot_base",
           "kv_vmm_reclaim", "kv_vmm_reclaim_load", "kv_vmm_lent", "kv_vmm_restore", "kv_vmm_pool_destroy", "ws_predict_load", "ws_replica_scores",
           "ws_place_replicas", "warmkv_version", "warmkv_build_id")


__all__ = [*EXPORTS, "KV_OK", "KV_E_NULL", "KV_E_RANGE", "KV_E_ALIGN", "KV_E_TOOBIG", "KV_E_OVERLAP", "KV_E_HIP",
           "KV_E_NOSPACE", "KV_E_BADPLAN", "KV_E_NOMEM", "KV_STATIC_MAX_BLOCKS", "WarmKVError", "StaleLibraryError", "pool_desc", "make_model"]


class WarmKVError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} failed: {_NAMES.get(code, code)}")
        self.code = code


class kv_pool_desc(Structure):
    _fields_ = [("base", c_void_p), ("num_blocks", c_uint32), ("num_layers", c_uint32), ("tile_bytes", c_uint64),
                ("layer_stride_bytes", c_uint64)]


class kv_plan_state(Structure):
    _fields_ = [("status", c_int32), ("n_moves", c_uint32), ("n_free_below", c_uint32), ("n_bad_entries", c_uint32),
                ("ticket", c_uint32), ("finished", c_uint32), ("bad_plan", c_uint32), ("reserved", c_uint32)]


class kv_plan(Structure):
    _fields_ = [("src", c_void_p), ("dst", c_void_p), ("new_id", c_void_p), ("live_out", c_void_p),
                ("state", c_void_p), ("num_blocks", c_uint32), ("boundary", c_uint32),
                ("capacity", c_uint32), ("reserved", c_uint32)]


class kv_compact_tuning(Structure):
    _fields_ = [("workgroups", c_uint32), ("chunk_bytes", c_uint32), ("flags", c_uint32), ("reserved", c_uint32)]


class wm_tensor(Structure):
    _fields_ = [("host_ptr", c_void_p), ("bytes", c_uint64), ("dst_offset", c_uint64)]


class wm_piece(Structure):
    _fields_ = [("tensor", c_uint32), ("early", c_uint32), ("src_offset", c_uint64), ("dst_offset", c_uint64),
                ("bytes", c_uint64)]


class kv_switch_request(Structure):
    _fields_ = [("pool", POINTER(kv_pool_desc)), ("plan", POINTER(kv_plan)), ("live_in", c_void_p),
                ("live_host", c_void_p), ("tables", c_void_p), ("num_seqs", c_uint32),
                ("max_blocks_per_seq", c_uint32), ("tensors", POINTER(wm_tensor)), ("n_tensors", c_uint32),
                ("reserved", c_uint32), ("early_bytes", c_uint64), ("compute_stream", c_void_p),
                ("copy_stream", c_void_p), ("compaction_done", c_void_p), ("front_done", c_void_p),
                ("copy_stream2", c_void_p)]


class ws_model(Structure):
    _fields_ = [("size_bytes", ctypes.c_double), ("load_avg", ctypes.c_double), ("load_peak", ctypes.c_double),
                ("cold_latency", ctypes.c_double), ("degree", c_uint32), ("batch", c_uint32), ("active", c_uint32),
                ("reserved", c_uint32)]


class ws_placement(Structure):
    _fields_ = [("model", c_uint32), ("replica", c_uint32), ("first_gpu", c_uint32), ("is_burst", c_uint32),
                ("score", ctypes.c_double)]


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


class StaleLibraryError(RuntimeError):
    pass


def _built_id(path: str) -> str | None:
    """Build identifier of the library file at `path`, read from its bytes without loading it
    (a stale library must not enter the process); None if there is no file or no identifier."""
    if not os.path.exists(path):
        return None
    with open(path, "rb") as f:
        m = re.search(rb"WARMKV_BUILD_ID=([0-9a-f]{16})\0", f.read())
    return m.group(1).decode() if m else None


def load():
    """Load libwarmkv.so.  The library carries a hash of the sources it was compiled from; if that
    differs from the sources in the tree (or no library is there) it is built again first, and if
    it still differs (or WARMKV_NO_REBUILD is set, for callers that must not compile) the call
    raises StaleLibraryError: a stale binary is never used."""
    global _lib
    if _lib is not None:
        return _lib
    want = _build.source_id()
    have = _built_id(_build.LIB_PATH)
    if have != want:
        if os.environ.get("WARMKV_NO_REBUILD"):
            raise StaleLibraryError(f"{_build.LIB_PATH}: built from sources {have}, the tree holds {want}")
        print(f"warmkv: library is {have}, sources are {want}: building", file=sys.stderr, flush=True)
        _build.build()
        have = _built_id(_build.LIB_PATH)
        if have != want:
            raise StaleLibraryError(f"{_build.LIB_PATH}: still {have} after a rebuild, the tree holds {want}")
    L = ctypes.CDLL(_build.LIB_PATH)
    L.warmkv_build_id.restype = c_char_p
    L.warmkv_build_id.argtypes = []
    if L.warmkv_build_id().decode() != want:
        raise StaleLibraryError(f"{_build.LIB_PATH}: loaded library says {L.warmkv_build_id().decode()}, wanted {want}")
    L.kv_plan_workspace_bytes.restype = c_size_t
    L.kv_plan_workspace_bytes.argtypes = [c_uint32, c_uint32]
    L.kv_plan_bind.restype = c_int
    L.kv_plan_bind.argtypes = [POINTER(kv_plan), c_void_p, c_size_t, c_uint32, c_uint32]
    L.kv_plan_reclaim.restype = c_int
    L.kv_plan_reclaim.argtypes = [c_void_p, POINTER(kv_plan), c_void_p]
    L.kv_compact.restype = c_int
    L.kv_compact.argtypes = [POINTER(kv_pool_desc), POINTER(kv_plan), c_void_p]
    L.kv_compact_launch.restype = c_int
    L.kv_compact_launch.argtypes = [POINTER(kv_pool_desc), POINTER(kv_plan), POINTER(kv_compact_tuning), c_void_p]
    L.kv_remap_tables.restype = c_int
    L.kv_remap_tables.argtypes = [c_void_p, c_uint32, c_uint32, POINTER(kv_plan), c_void_p]
    L.kv_reclaim.restype = c_int
    L.kv_reclaim.argtypes = [POINTER(kv_pool_desc), POINTER(kv_plan), c_void_p, c_void_p, c_uint32, c_uint32, c_void_p]
    L.kv_plan_fetch.restype = c_int
    L.kv_plan_fetch.argtypes = [POINTER(kv_plan), c_void_p, POINTER(kv_plan_state)]
    L.weights_materialize.restype = c_int
    L.weights_materialize.argtypes = [POINTER(kv_pool_desc), c_uint32, POINTER(wm_tensor), c_uint32, c_void_p, c_void_p]
    L.weights_materialize_schedule.restype = c_int
    L.weights_materialize_schedule.argtypes = [POINTER(kv_pool_desc), c_uint32, c_void_p, POINTER(wm_tensor), c_uint32,
                                               c_uint64, POINTER(wm_piece), c_uint32, POINTER(c_uint32)]
    L.weights_materialize_pipelined.restype = c_int
    L.weights_materialize_pipelined.argtypes = [POINTER(kv_pool_desc), c_uint32, c_void_p, POINTER(wm_tensor), c_uint32,
                                                c_uint64, c_void_p, c_void_p]
    L.kv_compact_moves.restype = c_int
    L.kv_compact_moves.argtypes = [POINTER(kv_pool_desc), POINTER(kv_plan), c_uint32, c_uint32, c_void_p]
    L.kv_compact_layers.restype = c_int
    L.kv_compact_layers.argtypes = [POINTER(kv_pool_desc), POINTER(kv_plan), c_uint32, c_uint32, c_void_p]
    L.kv_movers_in_front.restype = c_uint32
    L.kv_movers_in_front.argtypes = [c_void_p, c_uint32, c_uint32, c_uint32]
    L.weights_materialize_front.restype = c_int
    L.weights_materialize_front.argtypes = [POINTER(kv_pool_desc), c_uint32, c_uint64, POINTER(wm_tensor), c_uint32,
                                            c_void_p, c_void_p, c_void_p]
    L.weights_materialize_streams.restype = c_int
    L.weights_materialize_streams.argtypes = [POINTER(kv_pool_desc), c_uint32, c_uint64, POINTER(wm_tensor), c_uint32,
                                              POINTER(c_void_p), c_uint32, c_void_p, c_void_p]
    L.kv_switch.restype = c_int
    L.kv_switch.argtypes = [POINTER(kv_switch_request), POINTER(kv_plan_state)]
    L.kv_reclaim_static.restype = c_int
    L.kv_reclaim_static.argtypes = [POINTER(kv_pool_desc), c_uint32, c_void_p, c_void_p, c_void_p, c_uint32, c_uint32,
                                    c_void_p, c_void_p]
    L.kv_reserve_blocks.restype = c_int64
    L.kv_reserve_blocks.argtypes = [c_uint64, c_uint64, c_uint32, c_uint32]
    L.kv_grow.restype = c_int64
    L.kv_grow.argtypes = [POINTER(kv_pool_desc), c_uint32, c_uint32, POINTER(wm_tensor), c_uint32, c_void_p, c_void_p]
    L.kv_vmm_pool_create.restype = c_int
    L.kv_vmm_pool_create.argtypes = [c_uint32, c_uint64, POINTER(c_void_p)]
    L.kv_vmm_kv_base.restype = c_void_p
    L.kv_vmm_kv_base.argtypes = [c_void_p]
    L.kv_vmm_slot_base.restype = c_void_p
    L.kv_vmm_slot_base.argtypes = [c_void_p]
    L.kv_vmm_reclaim.restype = c_int
    L.kv_vmm_reclaim.argtypes = [c_void_p, c_void_p, c_uint32, c_void_p]
    L.kv_vmm_reclaim_load.restype = c_int
    L.kv_vmm_reclaim_load.argtypes = [c_void_p, c_void_p, c_uint32, c_uint32, POINTER(wm_tensor), c_uint32, c_void_p,
                                      c_void_p]
    L.kv_vmm_lent.restype = c_uint32
    L.kv_vmm_lent.argtypes = [c_void_p]
    L.kv_vmm_restore.restype = c_int
    L.kv_vmm_restore.argtypes = [c_void_p]
    L.kv_vmm_pool_destroy.restype = c_int
    L.kv_vmm_pool_destroy.argtypes = [c_void_p]
    L.ws_predict_load.restype = c_int
    L.ws_predict_load.argtypes = [c_void_p, c_uint32, c_uint32, c_uint32, c_uint32, c_uint32, c_uint32,
                                  POINTER(ctypes.c_double)]
    L.ws_replica_scores.restype = c_int
    L.ws_replica_scores.argtypes = [POINTER(ws_model), POINTER(c_uint32), POINTER(c_uint32), c_void_p, c_uint32]
    L.ws_place_replicas.restype = c_int
    L.ws_place_replicas.argtypes = [POINTER(ws_model), c_uint32, c_void_p, c_uint32, c_uint32, POINTER(ws_placement),
                                    c_uint32, POINTER(c_uint32)]
    L.warmkv_version.restype = c_char_p
    L.warmkv_version.argtypes = []
    _lib = L
    return L


def _ptr(x) -> int | None:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr() or None
    return int(x) or None


def _check(fn: str, rc: int) -> None:
    if rc != KV_OK:
        raise WarmKVError(fn, rc)


def pool_desc(base, num_blocks: int, num_layers: int, tile_bytes: int, layer_stride_bytes: int = 0) -> kv_pool_desc:
    """layer_stride_bytes = 0: block-major pool; otherwise layer-major with that slab stride."""
    return kv_pool_desc(_ptr(base), num_blocks, num_layers, tile_bytes, layer_stride_bytes)


def kv_plan_workspace_bytes(num_blocks: int, boundary: int) -> int:
    return int(load().kv_plan_workspace_bytes(num_blocks, boundary))


def kv_plan_bind(workspace, workspace_bytes: int, num_blocks: int, boundary: int) -> kv_plan:
    plan = kv_plan()
    _check("kv_plan_bind", load().kv_plan_bind(byref(plan), _ptr(workspace), workspace_bytes, num_blocks, boundary))
    return plan


def kv_plan_reclaim(live_in, plan: kv_plan, stream=0) -> None:
    _check("kv_plan_reclaim", load().kv_plan_reclaim(_ptr(live_in), byref(plan), _ptr(stream)))


def kv_compact(pool: kv_pool_desc, plan: kv_plan, stream=0) -> None:
    _check("kv_compact", load().kv_compact(byref(pool), byref(plan), _ptr(stream)))


def kv_compact_launch(pool: kv_pool_desc, plan: kv_plan, stream=0, *, workgroups: int = 0,
                      chunk_bytes: int = 0, flags: int = 0) -> None:
    t = kv_compact_tuning(workgroups, chunk_bytes, flags, 0)
    _check("kv_compact_launch", load().kv_compact_launch(byref(pool), byref(plan), byref(t), _ptr(stream)))


def kv_remap_tables(tables, num_seqs: int, max_blocks_per_seq: int, plan: kv_plan, stream=0) -> None:
    _check("kv_remap_tables", load().kv_remap_tables(_ptr(tables), num_seqs, max_blocks_per_seq, byref(plan),
                                                      _ptr(stream)))


def kv_reclaim(pool: kv_pool_desc, plan: kv_plan, live_in, tables, num_seqs: int, max_blocks_per_seq: int,
               stream=0) -> None:
    """Plan, block copy and table rewrite as one call (one kernel launch on small pools)."""
    _check("kv_reclaim", load().kv_reclaim(byref(pool), byref(plan), _ptr(live_in), _ptr(tables), num_seqs,
                                            max_blocks_per_seq, _ptr(stream)))


def kv_plan_fetch(plan: kv_plan, stream=0) -> kv_plan_state:
    out = kv_plan_state()
    _check("kv_plan_fetch", load().kv_plan_fetch(byref(plan), _ptr(stream), byref(out)))
    return out


def weights_materialize(pool: kv_pool_desc, boundary: int, tensors, copy_stream=0, compaction_done=None) -> None:
    """tensors: iterable of (host buffer or address, bytes, dst_offset)."""
    arr, n = _tensor_array(tensors)
    _check("weights_materialize", load().weights_materialize(byref(pool), boundary, arr, n,
                                                              _ptr(copy_stream), _ptr(compaction_done)))


def _tensor_array(tensors):
    items = list(tensors)
    arr = (wm_tensor * max(1, len(items)))()
    for i, (host, nbytes, off) in enumerate(items):
        arr[i] = wm_tensor(_ptr(host), nbytes, off)
    return arr, len(items)


def weights_materialize_schedule(pool: kv_pool_desc, boundary: int, live_host, tensors, early_bytes: int = 0):
    """Returns the list of (tensor, early, src_offset, dst_offset, bytes).  live_host: host address or
    a numpy uint64 array."""
    arr, n = _tensor_array(tensors)
    live_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    count = c_uint32(0)
    cap = 64
    while True:
        out = (wm_piece * cap)()
        rc = load().weights_materialize_schedule(byref(pool), boundary, live_ptr, arr, n, early_bytes, out, cap,
                                                 byref(count))
        if rc == KV_E_TOOBIG and count.value > cap:
            cap = count.value
            continue
        _check("weights_materialize_schedule", rc)
        return [(p.tensor, p.early, p.src_offset, p.dst_offset, p.bytes) for p in out[:count.value]]


def weights_materialize_pipelined(pool: kv_pool_desc, boundary: int, live_host, tensors, early_bytes: int = 0,
                                  copy_stream=0, compaction_done=None) -> None:
    arr, n = _tensor_array(tensors)
    live_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    _check("weights_materialize_pipelined",
           load().weights_materialize_pipelined(byref(pool), boundary, live_ptr, arr, n, early_bytes,
                                                _ptr(copy_stream), _ptr(compaction_done)))


def kv_compact_moves(pool: kv_pool_desc, plan: kv_plan, first_move: int, max_moves: int, stream=0) -> None:
    _check("kv_compact_moves", load().kv_compact_moves(byref(pool), byref(plan), first_move, max_moves, _ptr(stream)))


def kv_compact_layers(pool: kv_pool_desc, plan: kv_plan, first_layer: int, max_layers: int, stream=0) -> None:
    _check("kv_compact_layers", load().kv_compact_layers(byref(pool), byref(plan), first_layer, max_layers,
                                                          _ptr(stream)))


def kv_movers_in_front(live_host, num_blocks: int, boundary: int, front_blocks: int) -> int:
    live_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    return int(load().kv_movers_in_front(live_ptr, num_blocks, boundary, front_blocks))


def weights_materialize_front(pool: kv_pool_desc, boundary: int, front_bytes: int, tensors, copy_stream=0,
                              front_done=None, compaction_done=None) -> None:
    arr, n = _tensor_array(tensors)
    _check("weights_materialize_front",
           load().weights_materialize_front(byref(pool), boundary, front_bytes, arr, n, _ptr(copy_stream),
                                            _ptr(front_done), _ptr(compaction_done)))


def weights_materialize_streams(pool: kv_pool_desc, boundary: int, tensors, copy_streams, front_bytes: int = 0,
                                front_done=None, compaction_done=None) -> None:
    """The weight stream dealt out over several copy streams (a sequence of 1 to 4)."""
    arr, n = _tensor_array(tensors)
    streams = (c_void_p * max(1, len(copy_streams)))(*[_ptr(x) for x in copy_streams])
    _check("weights_materialize_streams",
           load().weights_materialize_streams(byref(pool), boundary, front_bytes, arr, n, streams, len(copy_streams),
                                              _ptr(front_done), _ptr(compaction_done)))


def kv_switch(pool: kv_pool_desc, plan: kv_plan, live_in, tables, num_seqs: int, max_blocks_per_seq: int, tensors,
              compute_stream, copy_stream, compaction_done, live_host=None, early_bytes: int = 0,
              front_done=None, copy_stream2=None) -> kv_plan_state:
    """The whole hand-over in one call; returns the plan's header.  Raises WarmKVError (KV_E_NOSPACE) if the
    request is infeasible, in which case nothing was moved or sent."""
    arr, n = _tensor_array(tensors)
    live_host_ptr = None
    if live_host is not None:
        live_host_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    rq = kv_switch_request(ctypes.pointer(pool), ctypes.pointer(plan), _ptr(live_in), live_host_ptr, _ptr(tables),
                           num_seqs, max_blocks_per_seq, arr, n, 0, early_bytes, _ptr(compute_stream),
                           _ptr(copy_stream), _ptr(compaction_done), _ptr(front_done), _ptr(copy_stream2))
    st = kv_plan_state()
    _check("kv_switch", load().kv_switch(byref(rq), byref(st)))
    return st


KV_STATIC_MAX_BLOCKS = 262144


def kv_reclaim_static(pool: kv_pool_desc, boundary: int, live_in, live_out, tables, num_seqs: int,
                      max_blocks_per_seq: int, state_out, stream=0) -> None:
    """Plan, block copy and table rewrite with the plan's workspace inside the library (no allocation).
    live_out and state_out are device buffers of the caller's."""
    _check("kv_reclaim_static", load().kv_reclaim_static(byref(pool), boundary, _ptr(live_in), _ptr(live_out),
                                                          _ptr(tables), num_seqs, max_blocks_per_seq, _ptr(state_out),
                                                          _ptr(stream)))


def kv_reserve_blocks(capacity_blocks: int, used_blocks: int, running: int, max_batch: int) -> int:
    r = int(load().kv_reserve_blocks(capacity_blocks, used_blocks, running, max_batch))
    if r < 0:
        raise WarmKVError("kv_reserve_blocks", r)
    return r


def kv_grow(pool: kv_pool_desc, old_boundary: int, new_boundary: int, tensors):
    """tensors: iterable of (host buffer or address, bytes, dst_offset) as given to weights_materialize.
    Returns (n_evicted, evicted flags, new offsets) as Python lists."""
    arr, n = _tensor_array(tensors)
    ev = (ctypes.c_uint8 * max(1, n))()
    no = (c_uint64 * max(1, n))()
    r = int(load().kv_grow(byref(pool), old_boundary, new_boundary, arr, n, ev, no))
    if r < 0:
        raise WarmKVError("kv_grow", r)
    return r, list(ev[:n]), list(no[:n])


def kv_vmm_pool_create(num_blocks: int, block_bytes: int) -> int:
    """Returns the opaque pool handle (an address)."""
    out = c_void_p()
    _check("kv_vmm_pool_create", load().kv_vmm_pool_create(num_blocks, block_bytes, byref(out)))
    return out.value


def kv_vmm_kv_base(pool: int) -> int:
    return load().kv_vmm_kv_base(pool)


def kv_vmm_slot_base(pool: int) -> int:
    return load().kv_vmm_slot_base(pool)


def kv_vmm_reclaim(pool: int, live_host, want: int) -> list[int]:
    """live_host: numpy uint64 bitmap (host).  Returns the ids whose pages now back the slot, in slot order."""
    ids = (c_int32 * max(1, want))()
    live_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    _check("kv_vmm_reclaim", load().kv_vmm_reclaim(pool, live_ptr, want, ids))
    return list(ids[:want])


def kv_vmm_reclaim_load(pool: int, live_host, want: int, tensors, copy_stream=0, chunk_blocks: int = 0) -> list[int]:
    """kv_vmm_reclaim with the weight stream pipelined behind the mapping.  tensors: iterable of
    (pinned host buffer or address, bytes, offset from the slot's start)."""
    ids = (c_int32 * max(1, want))()
    arr, n = _tensor_array(tensors)
    live_ptr = live_host.ctypes.data if hasattr(live_host, "ctypes") else _ptr(live_host)
    _check("kv_vmm_reclaim_load", load().kv_vmm_reclaim_load(pool, live_ptr, want, chunk_blocks, arr, n,
                                                              _ptr(copy_stream), ids))
    return list(ids[:want])


def kv_vmm_lent(pool: int) -> int:
    return int(load().kv_vmm_lent(pool))


def kv_vmm_restore(pool: int) -> None:
    _check("kv_vmm_restore", load().kv_vmm_restore(pool))


def kv_vmm_pool_destroy(pool: int) -> None:
    _check("kv_vmm_pool_destroy", load().kv_vmm_pool_destroy(pool))


def ws_predict_load(history, day: int, window: int, D: int = 7, N: int = 10) -> float:
    """history: C-contiguous float64 numpy array [n_days][n_windows] (day 0 the oldest)."""
    out = ctypes.c_double()
    _check("ws_predict_load", load().ws_predict_load(history.ctypes.data, history.shape[0], history.shape[1], day,
                                                     window, D, N, byref(out)))
    return out.value


def make_model(size_bytes, load_avg, load_peak, cold_latency, degree, batch, active) -> ws_model:
    return ws_model(size_bytes, load_avg, load_peak, cold_latency, degree, batch, active, 0)


def ws_replica_scores(model: ws_model):
    """Returns (n_basic, n_burst, [scores])."""
    nb, nu = c_uint32(), c_uint32()
    rc = load().ws_replica_scores(byref(model), byref(nb), byref(nu), None, 0)
    if rc not in (KV_OK, KV_E_TOOBIG):
        raise WarmKVError("ws_replica_scores", rc)
    n = nb.value + nu.value
    buf = (ctypes.c_double * max(1, n))()
    _check("ws_replica_scores", load().ws_replica_scores(byref(model), byref(nb), byref(nu), buf, n))
    return nb.value, nu.value, list(buf[:n])


def ws_place_replicas(models, gpu_free_bytes, gpus_per_server: int):
    """models: list of ws_model; gpu_free_bytes: float64 numpy array, updated in place.
    Returns [(model, replica, first_gpu, is_burst, score)] in placement order."""
    arr = (ws_model * max(1, len(models)))(*models)
    count = c_uint32()
    cap = 64
    while True:
        out = (ws_placement * cap)()
        rc = load().ws_place_replicas(arr, len(models), gpu_free_bytes.ctypes.data, gpu_free_bytes.size,
                                      gpus_per_server, out, cap, byref(count))
        if rc == KV_E_TOOBIG and count.value > cap:
            cap = count.value
            continue
        _check("ws_place_replicas", rc)
        return [(p.model, p.replica, p.first_gpu, p.is_burst, p.score) for p in out[:count.value]]


def warmkv_version() -> str:
    return load().warmkv_version().decode()


def warmkv_build_id() -> str:
    return load().warmkv_build_id().decode()
