"""Helpers for the GPU parity tests: drive the C ABI on torch-owned device
memory and bring results back as numpy arrays.  torch is used for allocation,
copies and streams only."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_09472_amd as wk
from synth import content


SUMMARY: list[str] = []      # printed by conftest.pytest_terminal_summary at the end of the run


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Upload a numpy array as raw bytes (uint64/uint16 have no torch dtype on all builds)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1)).to(dev())


def from_dev(t: torch.Tensor, dtype) -> np.ndarray:
    return t.cpu().numpy().view(dtype)


class DevicePlan:
    """Workspace + bound plan on the device."""

    def __init__(self, num_blocks: int, boundary: int):
        self.num_blocks, self.boundary = num_blocks, boundary
        self.bytes = wk.kv_plan_workspace_bytes(num_blocks, boundary)
        assert self.bytes > 0
        # poison so that unwritten outputs cannot pass as zeros
        self.ws = torch.full((self.bytes,), 0xA5, dtype=torch.uint8, device=dev())
        self.plan = wk.kv_plan_bind(self.ws, self.bytes, num_blocks, boundary)

    def _slice(self, ptr: int, nbytes: int) -> torch.Tensor:
        off = ptr - self.ws.data_ptr()
        return self.ws[off:off + nbytes]

    def state(self, stream=0):
        return wk.kv_plan_fetch(self.plan, stream)

    def results(self):
        """(status, n_moves, src, dst, new_id, live_out) as numpy, after a sync."""
        torch.cuda.synchronize()
        st = self.state()
        n = st.n_moves
        src = from_dev(self._slice(self.plan.src, 4 * n), np.int32)
        dst = from_dev(self._slice(self.plan.dst, 4 * n), np.int32)
        new_id = from_dev(self._slice(self.plan.new_id, 4 * self.num_blocks), np.int32)
        live_out = from_dev(self._slice(self.plan.live_out, 8 * ((self.num_blocks + 63) // 64)), np.uint64)
        return st, src, dst, new_id, live_out


def host_pool(cfg, table) -> np.ndarray:
    """Initial pool bytes of a (small) config, block i holding content id i."""
    pool = np.empty(cfg.pool_bytes, dtype=np.uint8)
    content.fill_host(pool, cfg.block_bytes, range(cfg.num_blocks), cfg.seed, table)
    return pool


def content_table(cfg, sigma=1.0):
    return content.normal_bf16_table(sigma) if cfg.content == "bf16_normal" else None


def run_reclaim(cfg, live: np.ndarray, tables: np.ndarray, pool_dev: torch.Tensor, stream=None, tuning=None):
    """plan -> compact -> remap on one stream, no host sync in between.
    Returns (DevicePlan, tables_dev)."""
    s = stream.cuda_stream if stream is not None else 0
    dp = DevicePlan(cfg.num_blocks, cfg.boundary)
    live_dev = to_dev(live) if live.size else torch.zeros(8, dtype=torch.uint8, device=dev())
    tables_dev = torch.from_numpy(tables).to(dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    torch.cuda.synchronize()
    wk.kv_plan_reclaim(live_dev, dp.plan, s)
    if tuning:
        wk.kv_compact_launch(pool, dp.plan, s, **tuning)
    else:
        wk.kv_compact(pool, dp.plan, s)
    wk.kv_remap_tables(tables_dev, tables.shape[0], tables.shape[1], dp.plan, s)
    torch.cuda.synchronize()
    dp.live_dev = live_dev
    return dp, tables_dev


class _RawDeviceBuffer:
    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


def view_device(ptr: int, nbytes: int) -> torch.Tensor:
    """uint8 tensor over device memory the caller owns (no copy, no ownership)."""
    return torch.as_tensor(_RawDeviceBuffer(ptr, nbytes), device=dev())
