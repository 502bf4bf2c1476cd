"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times (library defaults).

The plan, the id map, the bitmap and the block tables are compared with the
oracle element by element.  The pool (40-120 GiB) is checked in full against
the oracle's plan without a second copy: block content is a pure function of a
content id, the oracle's plan says which content id every block must hold
afterwards, and the device generator re-creates each 1 GiB slab for a byte
compare.  In addition a sample of blocks of every kind is brought back to the
host and compared with what the oracle's block copy produces for that block.
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


class FullRun:
    """Pool generated on the device, reclaim run once with the default launch shape."""

    def __init__(self, cfg, oracle):
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
    run.check_plan_and_tables()
    _say("[full] plan and tables match; checking pool")
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
    run = FullRun(cfg, oracle)
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


def test_full_size_reclaim_with_weights(oracle):
    """Third configuration: the 8B-shaped pool plus 225 bf16 tensors (15 009 316 864 B)
    streamed from pinned host memory into the reclaimed region, overlapped with compaction."""
    cfg = CONFIGS[2]
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < cfg.pool_bytes + (4 << 30):
        pytest.skip("not enough device memory")
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    table_d = gh.to_dev(gh.content_table(cfg))
    wtab_d = gh.to_dev(content.normal_bf16_table(0.02))
    bb = cfg.block_bytes
    pool_t = torch.empty(cfg.pool_bytes, dtype=torch.uint8, device=gh.dev())
    content.fill_device(pool_t.data_ptr(), cfg.num_blocks, bb, cfg.seed, table_ptr=table_d.data_ptr())
    sizes = [2 * a * b for _, (a, b) in weight_shapes_8b()]
    offs = dense_offsets(sizes)
    total = sum(sizes)
    wseed = 0x5EED0002
    _say(f"[full] weights: {len(sizes)} tensors, {total} bytes; pinning host memory")
    host = torch.empty(total, dtype=torch.uint8, pin_memory=True)
    stage = torch.empty(max(sizes), dtype=torch.uint8, device=gh.dev())
    pos, tensors = 0, []
    for i, (sz, off) in enumerate(zip(sizes, offs)):
        content.fill_device(stage.data_ptr(), 1, sz, wseed, cid0=i, table_ptr=wtab_d.data_ptr())
        host[pos:pos + sz].copy_(stage[:sz])
        tensors.append((host.data_ptr() + pos, sz, off))
        pos += sz
    torch.cuda.synchronize()
    # the host copy is what the generator says (spot check on the host, first and last tensor)
    for i in (0, len(sizes) - 1):
        start = sum(sizes[:i])
        want = content.item_bytes_host(wseed, i, 4096, content.normal_bf16_table(0.02))
        assert np.array_equal(host[start:start + 4096].numpy(), want)

    pool = wk.pool_desc(pool_t, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live_d = gh.to_dev(w.live)
    tables_d = torch.from_numpy(w.tables).to(gh.dev())
    s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    done = torch.cuda.Event()
    torch.cuda.synchronize()
    wk.kv_plan_reclaim(live_d, dp.plan, s_compute.cuda_stream)
    wk.kv_compact(pool, dp.plan, s_compute.cuda_stream)
    done.record(s_compute)
    wk.weights_materialize(pool, cfg.boundary, tensors, s_copy.cuda_stream, done.cuda_event)
    wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], dp.plan, s_compute.cuda_stream)
    torch.cuda.synchronize()
    _say("[full] reclaim + materialize done; checking")

    st, src, dst, new_id, live_out = dp.results()
    assert st.status == 0 and np.array_equal(src, p.src) and np.array_equal(dst, p.dst)
    want_tables = w.tables.copy()
    oracle.remap(want_tables, p)
    assert np.array_equal(tables_d.cpu().numpy(), want_tables)

    # below the boundary: the oracle's plan decides every block's content
    cid = np.arange(cfg.num_blocks, dtype=np.int32)
    cid[p.dst] = p.src
    cid_d = gh.to_dev(cid)
    slab = (1 << 30) // bb
    scratch = torch.empty(slab * bb, dtype=torch.uint8, device=gh.dev())
    for j0 in range(0, cfg.boundary, slab):
        n = min(slab, cfg.boundary - j0)
        content.fill_device(scratch.data_ptr(), n, bb, cfg.seed, cids_ptr=cid_d.data_ptr() + 4 * j0,
                            table_ptr=table_d.data_ptr())
        assert torch.equal(pool_t[j0 * bb:(j0 + n) * bb], scratch[:n * bb]), f"blocks {j0}..{j0 + n}"
    # the region: every tensor's bytes at its offset (the oracle's materialize is a memcpy per
    # tensor; its expected bytes are the host tensors, re-created here by the same generator)
    region = cfg.boundary * bb
    for i, (sz, off) in enumerate(zip(sizes, offs)):
        content.fill_device(stage.data_ptr(), 1, sz, wseed, cid0=i, table_ptr=wtab_d.data_ptr())
        assert torch.equal(pool_t[region + off:region + off + sz], stage[:sz]), f"tensor {i}"
    # three tensors brought back and compared with the oracle's own materialize on the host
    for i in (0, 6, len(sizes) - 1):
        sz, off = sizes[i], offs[i]
        start = sum(sizes[:i])
        mini = np.zeros(sz, dtype=np.uint8)
        assert oracle.materialize(mini, 0, [(host[start:start + sz].numpy(), 0)]) == 0
        assert np.array_equal(pool_t[region + off:region + off + sz].cpu().numpy(), mini), f"tensor {i}"
    # bytes of the region past the last tensor keep the old block content
    end = region + offs[-1] + sizes[-1]
    j0 = end // bb
    n = cfg.num_blocks - j0
    for k0 in range(0, n, slab):
        m = min(slab, n - k0)
        content.fill_device(scratch.data_ptr(), m, bb, cfg.seed, cid0=j0 + k0, table_ptr=table_d.data_ptr())
        lo = max(end, (j0 + k0) * bb)
        assert torch.equal(pool_t[lo:(j0 + k0 + m) * bb], scratch[lo - (j0 + k0) * bb:m * bb])
