"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times (library defaults).

The plan, the id map, the bitmap and the block tables are compared with the
oracle element by element.  The pool is checked in one of two modes, printed by
every test:

* full: where the host has room for a second copy of the pool (MemAvailable >=
  pool + 16 GiB; + 48 GiB for the 120 GiB pool, whose copy is too large to pin and
  stays pageable), the initial pool is brought to host memory, the oracle's block copy (and weight copy) run on that buffer, and the
  device pool is compared with it byte for byte in 1 GiB slices.
* lazy (always run as well): block content is a
  pure function of a content id, the oracle's plan says which content id every
  block must hold afterwards, and the device generator re-creates each 1 GiB
  slab for a byte compare.  A sample of blocks of every kind is brought back to
  the host and compared with what the oracle's block copy produces for it.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import gpu_harness as gh                      # noqa: E402
import paper_2512_09472_amd as wk             # noqa: E402
from synth import CONFIGS, content, dense_offsets, make_workload, weight_shapes_8b   # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    wk.binding.load()


def _say(msg):
    print(msg, flush=True)


FULL_MODE_MAX_POOL = 64 << 30
MODES = {}          # test id -> "full" | "lazy", printed and written out at the end of the module


def _mem_available() -> int:
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            return int(line.split()[1]) * 1024
    return 0


_host_pool_cache = []
PINNED_BUDGET = 60 << 30     # host memory this module keeps pinned at once (the box refused 80 GiB)


class PageableHostBuffer:
    """Plain host memory with the interface of synth.content.PinnedHostBuffer, for a pool copy too
    large to pin (copies to and from it are staged by the runtime and slower)."""

    def __init__(self, nbytes: int):
        self.nbytes = nbytes
        self.array = np.empty(nbytes, dtype=np.uint8)
        self.ptr = self.array.ctypes.data

    def free(self) -> None:
        self.array = None
        self.ptr = None


def _pinned_host_pool(nbytes: int, other_pinned: int = 0):
    """A host buffer of nbytes for the oracle's copy of a pool - pinned (synth.content.PinnedHostBuffer)
    up to 64 GiB, pageable above that - or None where the host has no room for it (then only the lazy
    comparison runs).  A buffer of the same size is reused; one of another size is given back first."""
    if _host_pool_cache and _host_pool_cache[0].nbytes == nbytes:
        return _host_pool_cache[0]
    while _host_pool_cache:
        _host_pool_cache.pop().free()
    if nbytes > FULL_MODE_MAX_POOL:
        if _mem_available() < nbytes + (48 << 30):
            return None
        _host_pool_cache.append(PageableHostBuffer(nbytes))
        return _host_pool_cache[0]
    if nbytes + other_pinned > max(PINNED_BUDGET, nbytes) or _mem_available() < nbytes + (16 << 30):
        return None
    try:
        _host_pool_cache.append(content.PinnedHostBuffer(nbytes))
    except MemoryError:
        return None
    return _host_pool_cache[0]


@pytest.fixture(scope="module", autouse=True)
def _release_host_pools():
    yield
    while _host_pool_cache:
        _host_pool_cache.pop().free()
    if MODES:
        gh.SUMMARY.append("full-size pool comparison against the oracle (full = whole buffer, byte for byte; "
                          "lazy = per-block content ids + sampled blocks): "
                          + ", ".join(f"{k}: {v}" for k, v in MODES.items()))


def _device_equals_host(pool_t, host, what):
    """Byte compare of a device buffer with a pinned host buffer of the same size, 1 GiB at a time."""
    assert pool_t.numel() == host.nbytes
    slab = 1 << 30
    scratch = torch.empty(slab, dtype=torch.uint8, device=gh.dev())
    torch.cuda.synchronize()
    for lo in range(0, pool_t.numel(), slab):
        n = min(slab, pool_t.numel() - lo)
        content.copy_bytes(scratch.data_ptr(), host.ptr + lo, n)
        if not torch.equal(pool_t[lo:lo + n], scratch[:n]):
            bad = (pool_t[lo:lo + n] != scratch[:n]).nonzero().flatten()
            pytest.fail(f"{what}: device pool differs from the oracle's pool at byte {lo + int(bad[0])} "
                        f"({bad.numel()} bytes differ in this GiB)")
    del scratch


def _spot_check_host_copy(host, cfg, table, blocks):
    """The host copy of the initial pool is what the host generator says (the device generator made it)."""
    bb = cfg.block_bytes
    probe = min(bb, 1 << 16)
    for j in blocks:
        want = content.item_bytes_host(cfg.seed, int(j), probe, table)
        assert np.array_equal(host.array[j * bb:j * bb + probe], want), f"host copy of block {j}"


class FullRun:
    """Pool generated on the device, reclaim run once with the default launch shape."""

    def __init__(self, cfg, oracle, full_buffer=True):
        self.cfg, self.oracle = cfg, oracle
        self.w = make_workload(cfg)
        self.p = oracle.plan(self.w.live, cfg.num_blocks, cfg.boundary)
        assert self.p.status == 0 and self.p.n_moves > 0
        self.table = gh.content_table(cfg)
        self.table_d = gh.to_dev(self.table) if self.table is not None else None
        self.tptr = self.table_d.data_ptr() if self.table_d is not None else 0
        _say(f"[full] {cfg.name}: pool {cfg.pool_bytes / 2**30:.0f} GiB, {self.p.n_moves} moves")
        self.pool_t = torch.empty(cfg.pool_bytes, dtype=torch.uint8, device=gh.dev())
        content.fill_device(self.pool_t.data_ptr(), cfg.num_blocks, cfg.block_bytes, cfg.seed, table_ptr=self.tptr)
        torch.cuda.synchronize()
        self.host_pool = None
        if full_buffer:
            self.host_pool = _pinned_host_pool(cfg.pool_bytes)
        if self.host_pool is not None:
            content.copy_bytes(self.host_pool.ptr, self.pool_t.data_ptr(), cfg.pool_bytes)
            rs = np.random.default_rng(cfg.seed + 1)
            _spot_check_host_copy(self.host_pool, cfg, self.table,
                                  [0, cfg.num_blocks - 1, *rs.integers(0, cfg.num_blocks, 6).tolist()])
            oracle.compact(self.host_pool.array, cfg.block_bytes, self.p)       # the oracle, on the whole pool
        self.mode = "full" if self.host_pool is not None else "lazy"
        _say(f"[full] {cfg.name}: comparison mode {self.mode} (MemAvailable {_mem_available() / 2**30:.0f} GiB)")
        self.dp, self.tables_d = gh.run_reclaim(cfg, self.w.live, self.w.tables, self.pool_t)
        # content id every block must hold afterwards, from the oracle's plan
        self.cid = np.arange(cfg.num_blocks, dtype=np.int32)
        self.cid[self.p.dst] = self.p.src

    def check_plan_and_tables(self):
        st, src, dst, new_id, live_out = self.dp.results()
        p = self.p
        assert st.status == 0 and st.n_moves == p.n_moves and st.n_bad_entries == 0
        assert st.ticket == 0 and st.finished == 0
        assert np.array_equal(src, p.src) and np.array_equal(dst, p.dst)
        assert np.array_equal(new_id, p.new_id) and np.array_equal(live_out, p.live_out)
        want = self.w.tables.copy()
        assert self.oracle.remap(want, p) == 0
        assert np.array_equal(self.tables_d.cpu().numpy(), want)

    def check_whole_buffer(self):
        if self.host_pool is not None:
            _device_equals_host(self.pool_t, self.host_pool, self.cfg.name)

    def check_pool(self, first_block=0, end_block=None):
        cfg = self.cfg
        end_block = cfg.num_blocks if end_block is None else end_block
        slab_blocks = max(1, (1 << 30) // cfg.block_bytes)
        scratch = torch.empty(slab_blocks * cfg.block_bytes, dtype=torch.uint8, device=gh.dev())
        cid_d = gh.to_dev(self.cid)
        for j0 in range(first_block, end_block, slab_blocks):
            n = min(slab_blocks, end_block - j0)
            content.fill_device(scratch.data_ptr(), n, cfg.block_bytes, cfg.seed,
                                cids_ptr=cid_d.data_ptr() + 4 * j0, table_ptr=self.tptr)
            got = self.pool_t[j0 * cfg.block_bytes:(j0 + n) * cfg.block_bytes]
            if not torch.equal(got, scratch[:n * cfg.block_bytes]):
                diff = (got.view(n, -1) != scratch[:n * cfg.block_bytes].view(n, -1)).any(dim=1).nonzero().flatten()
                pytest.fail(f"pool blocks differ from the oracle's plan: {(diff[:8] + j0).tolist()}")
        del scratch

    def check_sampled_blocks(self, n_each=6):
        """Bring sampled blocks to the host; expected bytes come from the oracle's block copy."""
        cfg, p = self.cfg, self.p
        rs = np.random.default_rng(cfg.seed)
        live = np.zeros(cfg.num_blocks, dtype=bool)
        live[np.flatnonzero(np.unpackbits(self.w.live.view(np.uint8), bitorder="little")[:cfg.num_blocks])] = True
        is_dst = np.zeros(cfg.num_blocks, dtype=bool)
        is_dst[p.dst] = True
        kinds = {"destination": p.dst, "first/last move": np.array([p.dst[0], p.dst[-1], p.src[0], p.src[-1]]),
                 "vacated source": p.src, "live below boundary": np.flatnonzero(live[:cfg.boundary]),
                 "free, not a destination": np.flatnonzero(~live & ~is_dst)}
        bb = cfg.block_bytes
        for kind, ids in kinds.items():
            for j in rs.choice(ids, size=min(n_each, ids.size), replace=False).tolist():
                got = self.pool_t[j * bb:(j + 1) * bb].cpu().numpy()
                mini = np.empty(2 * bb, dtype=np.uint8)          # [block j before, its source before]
                content.fill_host(mini, bb, [j, int(self.cid[j])], cfg.seed, self.table)
                if is_dst[j]:
                    k = int(np.searchsorted(p.dst, j))
                    assert p.dst[k] == j
                    one = self.oracle.Plan(0, np.array([1], np.int32), np.array([0], np.int32), None, None, 1, 2, 1)
                    self.oracle.compact(mini, bb, one)
                assert np.array_equal(got, mini[:bb]), f"{kind}: block {j}"


@pytest.mark.parametrize("index", [1, 3, 4])
def test_full_size_reclaim(oracle, index):
    cfg = CONFIGS[index]
    free_b, total_b = torch.cuda.mem_get_info()
    if free_b < cfg.pool_bytes + (3 << 30):
        pytest.skip(f"needs {cfg.pool_bytes / 2**30:.0f} GiB of device memory, {free_b / 2**30:.0f} GiB free")
    run = FullRun(cfg, oracle)
    MODES[f"configs[{index}]"] = run.mode
    run.check_plan_and_tables()
    _say("[full] plan and tables match; checking pool")
    run.check_whole_buffer()
    run.check_pool()
    run.check_sampled_blocks()
    # replaying the block copy with the same plan must change nothing
    wk.kv_compact(wk.pool_desc(run.pool_t, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), run.dp.plan)
    torch.cuda.synchronize()
    run.check_pool(0, cfg.boundary)
    del run
    torch.cuda.empty_cache()


def test_byte_offsets_beyond_2_and_4_gib(oracle):
    """A 4.5 GiB pool: source and destination byte offsets cross 2^31 and 2^32 (their low 32-bit
    halves take every sign), which small pools never exercise."""
    cfg = CONFIGS[1].scaled(num_blocks=2304, num_seqs=64)
    run = FullRun(cfg, oracle, full_buffer=False)
    assert int(run.p.src.max()) * cfg.block_bytes > (1 << 32) and int(run.p.dst.max()) * cfg.block_bytes > (1 << 31)
    run.check_plan_and_tables()
    run.check_pool()
    run.check_sampled_blocks(n_each=3)
    del run
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kv_heads", [8, 2, 3])
def test_full_size_layer_major_reclaim(oracle, kv_heads):
    """The 8B-shaped pool kept layer-major (32 slabs of 1.25 GiB): every slab is checked in full
    against the oracle's plan, slab by slab, with the device generator.  With 2 or 3 KV heads per
    block (a tensor-parallel share) the tiles are 16 or 24 KiB and several moves share a ticket."""
    cfg = CONFIGS[1].scaled(kv_heads=kv_heads)
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < cfg.pool_bytes + (4 << 30):
        pytest.skip("not enough device memory")
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    table_d = gh.to_dev(gh.content_table(cfg))
    tile, nb, layers = cfg.tile_bytes, cfg.num_blocks, cfg.num_layers
    stride = nb * tile
    pool_t = torch.empty(layers * stride, dtype=torch.uint8, device=gh.dev())
    for l in range(layers):
        content.fill_device(pool_t.data_ptr() + l * stride, nb, tile, cfg.seed, table_ptr=table_d.data_ptr(),
                            byte_offset=l * tile)
    pool = wk.pool_desc(pool_t, nb, layers, tile, stride)
    dp = gh.DevicePlan(nb, cfg.boundary)
    live_d = gh.to_dev(w.live)
    torch.cuda.synchronize()
    wk.kv_plan_reclaim(live_d, dp.plan)
    wk.kv_compact(pool, dp.plan)
    torch.cuda.synchronize()
    st, src, dst, new_id, live_out = dp.results()
    assert st.status == 0 and np.array_equal(src, p.src) and np.array_equal(dst, p.dst)
    cid = np.arange(nb, dtype=np.int32)
    cid[p.dst] = p.src
    cid_d = gh.to_dev(cid)
    scratch = torch.empty(stride, dtype=torch.uint8, device=gh.dev())
    for l in range(layers):
        content.fill_device(scratch.data_ptr(), nb, tile, cfg.seed, cids_ptr=cid_d.data_ptr(),
                            table_ptr=table_d.data_ptr(), byte_offset=l * tile)
        assert torch.equal(pool_t[l * stride:(l + 1) * stride], scratch), f"slab {l}"
    # sampled tiles against the oracle's layer-major copy on a two-block host pool
    rs = np.random.default_rng(1)
    table = gh.content_table(cfg)
    for k in rs.choice(p.n_moves, size=6, replace=False).tolist():
        l = int(rs.integers(0, layers))
        s_id, d_id = int(p.src[k]), int(p.dst[k])
        mini = np.zeros(2 * tile, dtype=np.uint8)             # one slab of two blocks: [dst, src]
        mini[tile:] = content.item_bytes_host(cfg.seed, s_id, tile, table, byte_offset=l * tile)
        one = oracle.Plan(0, np.array([1], np.int32), np.array([0], np.int32), None, None, 1, 2, 1)
        oracle.compact_layer_major(mini, tile, 1, 2 * tile, one)
        got = pool_t[l * stride + d_id * tile: l * stride + (d_id + 1) * tile].cpu().numpy()
        assert np.array_equal(got, mini[:tile]), (k, l)


class WeightedPool:
    """Third configuration at full size: the 8B-shaped pool, the 225 bf16 tensors (15 009 316 864 B) in
    pinned host memory, and what the oracle says pool and tables must hold after the hand-over.
    Built once per module; every weight path below is run on a freshly generated pool and compared
    with the same expectation (the result does not depend on the order or the timing of the copies)."""

    WSEED = 0x5EED0002

    def __init__(self, oracle):
        cfg = self.cfg = CONFIGS[2]
        self.oracle = oracle
        self.w = make_workload(cfg)
        self.p = oracle.plan(self.w.live, cfg.num_blocks, cfg.boundary)
        assert self.p.status == 0
        self.table = gh.content_table(cfg)
        self.table_d = gh.to_dev(self.table)
        self.wtab = content.normal_bf16_table(0.02)
        self.wtab_d = gh.to_dev(self.wtab)
        bb = self.bb = cfg.block_bytes
        self.pool_t = torch.empty(cfg.pool_bytes, dtype=torch.uint8, device=gh.dev())
        self.sizes = [2 * a * b for _, (a, b) in weight_shapes_8b()]
        self.offs = dense_offsets(self.sizes)
        self.total = sum(self.sizes)
        self.starts = np.concatenate([[0], np.cumsum(self.sizes)[:-1]]).tolist()
        _say(f"[full] weights: {len(self.sizes)} tensors, {self.total} bytes; pinning host memory")
        self.want_pool = _pinned_host_pool(cfg.pool_bytes, other_pinned=16 << 30)   # torch pins 16 GiB for the weights
        self.host = torch.empty(self.total, dtype=torch.uint8, pin_memory=True)
        self.stage = torch.empty(max(self.sizes), dtype=torch.uint8, device=gh.dev())
        for i, (sz, start) in enumerate(zip(self.sizes, self.starts)):
            content.fill_device(self.stage.data_ptr(), 1, sz, self.WSEED, cid0=i, table_ptr=self.wtab_d.data_ptr())
            self.host[start:start + sz].copy_(self.stage[:sz])
        torch.cuda.synchronize()
        # the host copy is what the host generator says (first, one in the middle, last tensor)
        for i in (0, 100, len(self.sizes) - 1):
            want = content.item_bytes_host(self.WSEED, i, 4096, self.wtab)
            assert np.array_equal(self.host[self.starts[i]:self.starts[i] + 4096].numpy(), want)
        self.tensors = [(self.host.data_ptr() + st, sz, off) for st, sz, off in zip(self.starts, self.sizes, self.offs)]
        self.pool = wk.pool_desc(self.pool_t, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        self.live_d = gh.to_dev(self.w.live)
        self.s_compute, self.s_copy, self.s_copy2 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        self.done, self.front = torch.cuda.Event(), torch.cuda.Event()
        self.done.record(self.s_compute)           # torch creates the HIP event on its first record
        self.front.record(self.s_compute)
        self.want_tables = self.w.tables.copy()
        assert oracle.remap(self.want_tables, self.p) == 0
        self.cid = np.arange(cfg.num_blocks, dtype=np.int32)
        self.cid[self.p.dst] = self.p.src
        self.cid_d = gh.to_dev(self.cid)
        # the same pool kept layer-major: 32 slabs of 1.25 GiB, strips of 512 MiB; strip l receives layer
        # l's seven matrices and the l-th of 32 row slices of the embedding matrix (it does not fit a strip)
        self.tile, self.stride = cfg.tile_bytes, cfg.num_blocks * cfg.tile_bytes
        self.strip = (cfg.num_blocks - cfg.boundary) * cfg.tile_bytes
        self.pool_lm = wk.pool_desc(self.pool_t, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes, self.stride)
        emb, emb_slice = len(self.sizes) - 1, self.sizes[-1] // cfg.num_layers
        assert emb_slice * cfg.num_layers == self.sizes[-1] and emb_slice % 256 == 0
        self.lm = []           # (host address, bytes, region offset, content id, byte offset in that content)
        for l in range(cfg.num_layers):
            at = l * self.strip
            for i in range(7 * l, 7 * l + 7):
                self.lm.append((self.host.data_ptr() + self.starts[i], self.sizes[i], at, i, 0))
                at += self.sizes[i]
            self.lm.append((self.host.data_ptr() + self.starts[emb] + l * emb_slice, emb_slice, at, emb, l * emb_slice))
            at += emb_slice
            assert at <= (l + 1) * self.strip
        self.lm_tensors = [(a, n, o) for a, n, o, _, _ in self.lm]
        # full-buffer expectation: the oracle's block copy and weight copy on a host copy of the pool
        self.expectation = None
        self.mode = "full" if self.want_pool is not None else "lazy"
        self.expect("block")
        _say(f"[full] weights: comparison mode {self.mode}")

    def expect(self, layout):
        """Make the pinned host buffer hold what the oracle says the pool must be after the hand-over
        in this layout (recomputed only when the layout changes)."""
        if self.want_pool is None or self.expectation == layout:
            return
        cfg, oracle, bb = self.cfg, self.oracle, self.bb
        self.fresh_pool(layout)
        content.copy_bytes(self.want_pool.ptr, self.pool_t.data_ptr(), cfg.pool_bytes)
        if layout == "block":
            _spot_check_host_copy(self.want_pool, cfg, self.table, [0, 1, cfg.boundary, cfg.num_blocks - 1, 7777])
            oracle.compact(self.want_pool.array, bb, self.p)
            views = [(self.host[st:st + sz].numpy(), off) for st, sz, off in zip(self.starts, self.sizes, self.offs)]
            assert oracle.materialize(self.want_pool.array, cfg.boundary * bb, views) == 0
        else:
            for l, j in ((0, 0), (3, 7777), (cfg.num_layers - 1, cfg.num_blocks - 1)):   # slab l holds bytes [l*tile, (l+1)*tile) of each block
                want = content.item_bytes_host(cfg.seed, j, 4096, self.table, byte_offset=l * self.tile)
                at = l * self.stride + j * self.tile
                assert np.array_equal(self.want_pool.array[at:at + 4096], want), (l, j)
            oracle.compact_layer_major(self.want_pool.array, self.tile, cfg.num_layers, self.stride, self.p)
            base = self.host.data_ptr()
            views = [(self.host[a - base:a - base + n].numpy(), o) for a, n, o, _, _ in self.lm]
            assert oracle.materialize_strips(self.want_pool.array, self.tile, cfg.num_layers, cfg.num_blocks,
                                             cfg.boundary, self.stride, views) == 0
        self.expectation = layout

    def fresh_pool(self, layout="block"):
        cfg = self.cfg
        if layout == "block":
            content.fill_device(self.pool_t.data_ptr(), cfg.num_blocks, self.bb, cfg.seed, table_ptr=self.table_d.data_ptr())
        else:
            for l in range(cfg.num_layers):
                content.fill_device(self.pool_t.data_ptr() + l * self.stride, cfg.num_blocks, self.tile, cfg.seed,
                                    table_ptr=self.table_d.data_ptr(), byte_offset=l * self.tile)
        self.tables_d = torch.from_numpy(self.w.tables).to(gh.dev())
        self.dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        torch.cuda.synchronize()

    def check_layer_major(self, what):
        """As check(), for the layer-major pool: the whole buffer against the oracle (full mode), then
        slab by slab against the oracle's plan, every strip's tensors, and every strip's tail."""
        cfg, p, tile, stride, strip = self.cfg, self.p, self.tile, self.stride, self.strip
        torch.cuda.synchronize()
        st, src, dst, new_id, live_out = self.dp.results()
        assert st.status == 0 and st.n_moves == p.n_moves and st.ticket == 0 and st.finished == 0
        assert np.array_equal(src, p.src) and np.array_equal(dst, p.dst) and np.array_equal(new_id, p.new_id)
        assert np.array_equal(self.tables_d.cpu().numpy(), self.want_tables), f"{what}: tables"
        self.expect_ready("layer")
        if self.want_pool is not None:
            _device_equals_host(self.pool_t, self.want_pool, what)
        nb, b = cfg.num_blocks, cfg.boundary
        scratch = torch.empty(stride, dtype=torch.uint8, device=gh.dev())
        used = [0] * cfg.num_layers
        for a, n, o, cid, off in self.lm:
            l = o // strip
            used[l] = max(used[l], o - l * strip + n)
            content.fill_device(self.stage.data_ptr(), 1, n, self.WSEED, cid0=cid, table_ptr=self.wtab_d.data_ptr(),
                                byte_offset=off)
            at = l * stride + b * tile + (o - l * strip)
            assert torch.equal(self.pool_t[at:at + n], self.stage[:n]), f"{what}: tensor at region offset {o}"
        for l in range(cfg.num_layers):
            content.fill_device(scratch.data_ptr(), nb, tile, cfg.seed, cids_ptr=self.cid_d.data_ptr(),
                                table_ptr=self.table_d.data_ptr(), byte_offset=l * tile)
            slab = self.pool_t[l * stride:(l + 1) * stride]
            assert torch.equal(slab[:b * tile], scratch[:b * tile]), f"{what}: slab {l} below the boundary"
            tail = b * tile + used[l]
            assert torch.equal(slab[tail:], scratch[tail:]), f"{what}: tail of strip {l}"
        del scratch

    def expect_ready(self, layout):
        assert self.want_pool is None or self.expectation == layout, "call expect(layout) before running the path"

    def check(self, what):
        cfg, p, bb = self.cfg, self.p, self.bb
        self.expect_ready("block")
        torch.cuda.synchronize()
        st, src, dst, new_id, live_out = self.dp.results()
        assert st.status == 0 and st.n_moves == p.n_moves and st.ticket == 0 and st.finished == 0
        assert np.array_equal(src, p.src) and np.array_equal(dst, p.dst)
        assert np.array_equal(new_id, p.new_id) and np.array_equal(live_out, p.live_out)
        assert np.array_equal(self.tables_d.cpu().numpy(), self.want_tables), f"{what}: tables"
        if self.want_pool is not None:
            _device_equals_host(self.pool_t, self.want_pool, what)
        # lazy checks, always: below the boundary the oracle's plan decides every block's content
        slab = (1 << 30) // bb
        scratch = torch.empty(slab * bb, dtype=torch.uint8, device=gh.dev())
        for j0 in range(0, cfg.boundary, slab):
            n = min(slab, cfg.boundary - j0)
            content.fill_device(scratch.data_ptr(), n, bb, cfg.seed, cids_ptr=self.cid_d.data_ptr() + 4 * j0,
                                table_ptr=self.table_d.data_ptr())
            assert torch.equal(self.pool_t[j0 * bb:(j0 + n) * bb], scratch[:n * bb]), f"{what}: blocks {j0}..{j0 + n}"
        # the region: every tensor's bytes at its offset (the oracle's weight copy is a memcpy per
        # tensor; the expected bytes are the host tensors, re-created here by the same generator)
        region = cfg.boundary * bb
        for i, (sz, off) in enumerate(zip(self.sizes, self.offs)):
            content.fill_device(self.stage.data_ptr(), 1, sz, self.WSEED, cid0=i, table_ptr=self.wtab_d.data_ptr())
            assert torch.equal(self.pool_t[region + off:region + off + sz], self.stage[:sz]), f"{what}: tensor {i}"
        # bytes of the region past the last tensor keep the old block content
        end = region + self.offs[-1] + self.sizes[-1]
        j0 = end // bb
        n = cfg.num_blocks - j0
        for k0 in range(0, n, slab):
            m = min(slab, n - k0)
            content.fill_device(scratch.data_ptr(), m, bb, cfg.seed, cid0=j0 + k0, table_ptr=self.table_d.data_ptr())
            lo = max(end, (j0 + k0) * bb)
            assert torch.equal(self.pool_t[lo:(j0 + k0 + m) * bb], scratch[lo - (j0 + k0) * bb:m * bb]), f"{what}: tail"
        del scratch

    def check_tensors_on_host(self):
        """Three tensors brought back and compared with the oracle's own weight copy on the host."""
        region = self.cfg.boundary * self.bb
        for i in (0, 6, len(self.sizes) - 1):
            sz, off, st = self.sizes[i], self.offs[i], self.starts[i]
            mini = np.zeros(sz, dtype=np.uint8)
            assert self.oracle.materialize(mini, 0, [(self.host[st:st + sz].numpy(), 0)]) == 0
            assert np.array_equal(self.pool_t[region + off:region + off + sz].cpu().numpy(), mini), f"tensor {i}"


@pytest.fixture(scope="module")
def weighted(oracle):
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < CONFIGS[2].pool_bytes + (4 << 30):
        pytest.skip("not enough device memory")
    wp = WeightedPool(oracle)
    MODES["configs[2] weight paths"] = wp.mode
    yield wp
    del wp
    torch.cuda.empty_cache()


def test_full_size_reclaim_with_weights(weighted):
    """Third configuration through the four separate calls: the copy stream waits for the whole
    block copy (the compaction event), then streams the 225 tensors."""
    wp = weighted
    cfg, w = wp.cfg, wp.w
    wp.expect("block")
    wp.fresh_pool()
    wk.kv_plan_reclaim(wp.live_d, wp.dp.plan, wp.s_compute.cuda_stream)
    wk.kv_compact(wp.pool, wp.dp.plan, wp.s_compute.cuda_stream)
    wp.done.record(wp.s_compute)
    wk.weights_materialize(wp.pool, cfg.boundary, wp.tensors, wp.s_copy.cuda_stream, wp.done.cuda_event)
    wk.kv_remap_tables(wp.tables_d, w.tables.shape[0], w.tables.shape[1], wp.dp.plan, wp.s_compute.cuda_stream)
    wp.check("gated")
    wp.check_tensors_on_host()


# The overlapped paths at the size the benchmark times them.  On this pool the block copy reads the
# reclaimed region for about 3 ms while the weight stream is already writing into it, so an event
# wait that is missing or attached to the wrong piece would leave weight bytes in a moved block (or
# stale KV in a tensor), which the whole-pool compare against the oracle sees.
@pytest.mark.parametrize("order", ["forward", "reverse", "reverse_two_copy_streams"])
@pytest.mark.parametrize("mode", ["front", "block"])
def test_full_size_switch_in_one_call(weighted, mode, order):
    """kv_switch with the front-first and with the block-pipelined weight stream.  `reverse` lists the
    tensors from the end of the region to its start, so the first bytes sent are aimed at the part
    of the region whose movers the block copy reads last."""
    wp = weighted
    cfg, w = wp.cfg, wp.w
    tensors = wp.tensors if order == "forward" else wp.tensors[::-1]
    wp.expect("block")
    wp.fresh_pool()
    st = wk.kv_switch(wp.pool, wp.dp.plan, wp.live_d, wp.tables_d, w.tables.shape[0], w.tables.shape[1], tensors,
                      wp.s_compute.cuda_stream, wp.s_copy.cuda_stream, wp.done.cuda_event, live_host=w.live,
                      front_done=wp.front.cuda_event if mode == "front" else None,
                      copy_stream2=wp.s_copy2.cuda_stream if order.endswith("two_copy_streams") else None)
    assert st.status == 0 and st.n_moves == wp.p.n_moves
    wp.check(f"kv_switch {mode} {order}")


def _front_marks(wp):
    bb = wp.bb
    region_bytes = (wp.cfg.num_blocks - wp.cfg.boundary) * bb
    default = -(-max(64 << 20, 2 * wp.p.n_moves * bb // 64) // bb) * bb          # what kv_switch picks: 294 MiB here
    mid_tensor = wp.offs[11] + wp.sizes[11] // 2 + 256                           # inside a gate matrix, not block-aligned
    return {"zero": 0, "default_294MiB": default, "mid_tensor": mid_tensor, "half_region": region_bytes // 2 + 4096,
            "past_region": region_bytes + bb}


@pytest.mark.parametrize("mark,order", [("zero", "forward"), ("default_294MiB", "forward"), ("default_294MiB", "reverse"),
                                        ("mid_tensor", "forward"), ("mid_tensor", "reverse"), ("half_region", "reverse"),
                                        ("past_region", "forward")])
def test_full_size_front_first_weight_stream(weighted, mark, order):
    """kv_compact_moves in two parts with an event between them, and weights_materialize_front with
    the mark at the start of the region, where kv_switch puts it, inside a tensor, in the middle of
    the region and beyond its end."""
    wp = weighted
    cfg, w, bb = wp.cfg, wp.w, wp.bb
    front_bytes = _front_marks(wp)[mark]
    tensors = wp.tensors if order == "forward" else wp.tensors[::-1]
    s, cs = wp.s_compute.cuda_stream, wp.s_copy.cuda_stream
    wp.expect("block")
    wp.fresh_pool()
    head = wk.kv_movers_in_front(w.live, cfg.num_blocks, cfg.boundary, min(-(-front_bytes // bb), cfg.num_blocks))
    want_head = int(np.count_nonzero(wp.p.src < cfg.boundary + -(-front_bytes // bb)))
    assert head == want_head                    # the oracle's movers below the mark
    wk.kv_plan_reclaim(wp.live_d, wp.dp.plan, s)
    wk.kv_compact_moves(wp.pool, wp.dp.plan, 0, head, s)
    wp.front.record(wp.s_compute)
    wk.kv_compact_moves(wp.pool, wp.dp.plan, head, 0xFFFFFFFF, s)
    wp.done.record(wp.s_compute)
    wk.kv_remap_tables(wp.tables_d, w.tables.shape[0], w.tables.shape[1], wp.dp.plan, s)
    wk.weights_materialize_front(wp.pool, cfg.boundary, front_bytes, tensors, cs, wp.front.cuda_event, wp.done.cuda_event)
    wp.check(f"front-first, mark {mark} ({front_bytes} B, {head} movers in front), {order}")


def test_full_size_block_pipelined_weight_stream(weighted):
    """weights_materialize_pipelined called directly (early pieces before the wait on the compaction
    event), with the default early budget and with the whole region's free blocks sent early."""
    wp = weighted
    cfg, w = wp.cfg, wp.w
    s, cs = wp.s_compute.cuda_stream, wp.s_copy.cuda_stream
    wp.expect("block")
    for early in (0, 1 << 40):
        wp.fresh_pool()
        wk.kv_plan_reclaim(wp.live_d, wp.dp.plan, s)
        wk.kv_compact(wp.pool, wp.dp.plan, s)
        wp.done.record(wp.s_compute)
        wk.weights_materialize_pipelined(wp.pool, cfg.boundary, w.live, wp.tensors[::-1], early, cs, wp.done.cuda_event)
        wk.kv_remap_tables(wp.tables_d, w.tables.shape[0], w.tables.shape[1], wp.dp.plan, s)
        wp.check(f"block-pipelined, early budget {early}")


@pytest.mark.parametrize("path", ["gated", "switch_front", "switch_front_reverse", "switch_block", "front_3_strips_reverse",
                                  "switch_front_two_copy_streams", "front_3_strips_reverse_three_copy_streams"])
def test_full_size_layer_major_weight_paths(weighted, path):
    """The 8B-shaped pool kept layer-major (32 slabs of 1.25 GiB, strips of 512 MiB), with the same
    15 GB of weights placed strip by strip, the table rewrite, and every overlapped weight path."""
    wp = weighted
    cfg, w = wp.cfg, wp.w
    s, cs = wp.s_compute.cuda_stream, wp.s_copy.cuda_stream
    tensors = wp.lm_tensors[::-1] if "reverse" in path else wp.lm_tensors
    wp.expect("layer")
    wp.fresh_pool("layer")
    if path == "gated":
        wk.kv_plan_reclaim(wp.live_d, wp.dp.plan, s)
        wk.kv_compact(wp.pool_lm, wp.dp.plan, s)
        wp.done.record(wp.s_compute)
        wk.weights_materialize(wp.pool_lm, cfg.boundary, tensors, cs, wp.done.cuda_event)
        wk.kv_remap_tables(wp.tables_d, w.tables.shape[0], w.tables.shape[1], wp.dp.plan, s)
    elif path.startswith("switch"):
        st = wk.kv_switch(wp.pool_lm, wp.dp.plan, wp.live_d, wp.tables_d, w.tables.shape[0], w.tables.shape[1], tensors,
                          s, cs, wp.done.cuda_event, live_host=w.live,
                          front_done=wp.front.cuda_event if "front" in path else None,
                          copy_stream2=wp.s_copy2.cuda_stream if path.endswith("two_copy_streams") else None)
        assert st.status == 0 and st.n_moves == wp.p.n_moves
    elif path.startswith("front_3_strips"):
        front_bytes = 2 * wp.strip + 4096           # needs the first three strips
        wk.kv_plan_reclaim(wp.live_d, wp.dp.plan, s)
        wk.kv_compact_layers(wp.pool_lm, wp.dp.plan, 0, 3, s)
        wp.front.record(wp.s_compute)
        wk.kv_compact_layers(wp.pool_lm, wp.dp.plan, 3, 0xFFFFFFFF, s)
        wp.done.record(wp.s_compute)
        wk.kv_remap_tables(wp.tables_d, w.tables.shape[0], w.tables.shape[1], wp.dp.plan, s)
        if path.endswith("three_copy_streams"):
            third = torch.cuda.Stream()
            wk.weights_materialize_streams(wp.pool_lm, cfg.boundary, tensors, [cs, wp.s_copy2.cuda_stream, third.cuda_stream],
                                           front_bytes, wp.front.cuda_event, wp.done.cuda_event)
        else:
            wk.weights_materialize_front(wp.pool_lm, cfg.boundary, front_bytes, tensors, cs, wp.front.cuda_event,
                                         wp.done.cuda_event)
    wp.check_layer_major(f"layer-major {path}")
