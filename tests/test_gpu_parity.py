"""GPU parity: the HIP path through the C ABI against the CPU oracle, element
by element, on the same seeded inputs.  Integer and byte work: the bar is
bit-exact (no tolerance exists on this path)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import gpu_harness as gh                      # noqa: E402
import pins                                   # noqa: E402
import paper_2512_09472_amd as wk             # noqa: E402
from synth import CONFIGS, bitmap_from_ids, content, make_workload   # noqa: E402
from synth.rng import SplitMix64              # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    wk.binding.load()


def _say(msg):
    print(msg, flush=True)


def _compare_plan(dp, p):
    st, src, dst, new_id, live_out = dp.results()
    assert st.status == p.status
    if p.status != 0:
        assert st.n_moves == 0
        return st
    assert st.n_moves == p.n_moves
    assert np.array_equal(src, p.src), "src"
    assert np.array_equal(dst, p.dst), "dst"
    assert np.array_equal(new_id, p.new_id), "new_id"
    assert np.array_equal(live_out, p.live_out), "live_out"
    return st


SCALED = {
    "cfg1_tiny": CONFIGS[0],
    "cfg2_small": CONFIGS[1].scaled(num_blocks=640, num_layers=3, num_seqs=40),
    "cfg2_ragged_tile": CONFIGS[1].scaled(num_blocks=900, num_layers=5, kv_heads=3, head_dim=40, num_seqs=40),
    "cfg4_odd_boundary": CONFIGS[3].scaled(num_blocks=1536, num_layers=4, num_seqs=128),
    "cfg5_frag": CONFIGS[4].scaled(num_blocks=4096, num_layers=2, num_seqs=1024),
    "cfg5_tiny_tile": CONFIGS[4].scaled(num_blocks=2048, num_layers=1, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=512),
    # blocks of half a ticket or less: several moves share one ticket of the block copy
    "one_layer_16k_blocks": CONFIGS[1].scaled(num_blocks=3000, num_layers=1, kv_heads=2, num_seqs=60),
    "one_layer_7680_blocks": CONFIGS[1].scaled(num_blocks=2500, num_layers=1, kv_heads=3, head_dim=40, num_seqs=50),
    "one_layer_40k_blocks": CONFIGS[1].scaled(num_blocks=1500, num_layers=1, kv_heads=5, num_seqs=50),   # two to a ticket of 20 rows
    "two_layer_288_blocks": CONFIGS[4].scaled(num_blocks=5000, num_layers=2, block_size=1, kv_heads=1, head_dim=72, len_hi=16, num_seqs=900),
    # more than 65 536 blocks: the planner's several-workgroup shape plus its join kernel feed the copy
    "many_small_blocks": CONFIGS[4].scaled(num_blocks=150_000, num_layers=2, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=6000),
}

TUNINGS = [None,                                                        # defaults: 64 KiB units, 16 loads per lane, one WG per CU
           dict(chunk_bytes=4096, flags=2 << 4),                        # units smaller than one step
           dict(chunk_bytes=65536, flags=(8 << 4) | 1),                 # cached accesses
           dict(workgroups=7, chunk_bytes=8192, flags=2 << 4),
           dict(workgroups=3000, chunk_bytes=32768, flags=4 << 4),      # more workgroups than fit at once
           dict(workgroups=5000, chunk_bytes=32768, flags=(4 << 4) | 2),   # next ticket drawn during the copy
           dict(workgroups=256, chunk_bytes=1 << 20, flags=(32 << 4) | 2),
           dict(flags=8),                                               # small blocks: one ticket each, not packed
           dict(workgroups=40, chunk_bytes=16384, flags=1)]             # small blocks packed into 16 KiB tickets


@pytest.mark.parametrize("name", list(SCALED))
def test_reclaim_matches_oracle(oracle, name):
    cfg = SCALED[name]
    w = make_workload(cfg)
    table = gh.content_table(cfg)
    pool0 = gh.host_pool(cfg, table)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert p.status == 0 and p.n_moves > 0
    want_pool = pool0.copy()
    oracle.compact(want_pool, cfg.block_bytes, p)
    want_tables = w.tables.copy()
    assert oracle.remap(want_tables, p) == 0
    for tuning in TUNINGS:
        _say(f"[parity] {name} block_bytes={cfg.block_bytes} NB={cfg.num_blocks} b={cfg.boundary} tuning={tuning}")
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        dp, tables_dev = gh.run_reclaim(cfg, w.live, w.tables, pool_dev, tuning=tuning)
        st = _compare_plan(dp, p)
        assert st.n_bad_entries == 0
        assert st.ticket == 0 and st.finished == 0, "work counters must return to zero"
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), "tables"
        got = pool_dev.cpu().numpy()
        if not np.array_equal(got, want_pool):
            bad = np.flatnonzero(got.reshape(cfg.num_blocks, -1) != want_pool.reshape(cfg.num_blocks, -1))[:5]
            pytest.fail(f"pool differs, first flat positions {bad}")
        del pool_dev


ONE_CALL = {
    # one kernel launch: at most 32 768 blocks, 16 384 table entries, 128 MiB that could move
    "tiny_cfg1": (CONFIGS[0], 0, True),
    "one_word": (CONFIGS[0].scaled(num_blocks=50, boundary=23, num_seqs=5, len_hi=160), 0, True),
    "ragged_tile_3_layers": (CONFIGS[1].scaled(num_blocks=1000, num_layers=3, kv_heads=3, head_dim=40, num_seqs=30, len_hi=4096), 0, True),
    "odd_boundary": (CONFIGS[3].scaled(num_blocks=777, num_layers=2, num_seqs=40, len_hi=4096), 0, True),
    "tiny_tiles_many_blocks": (CONFIGS[4].scaled(num_blocks=32768, num_layers=2, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=1000), 0, True),
    "frag": (CONFIGS[4].scaled(num_blocks=256, num_layers=1, num_seqs=64, len_hi=512), 0, True),
    "layer_major": (CONFIGS[1].scaled(num_blocks=640, num_layers=3, num_seqs=40, len_hi=4096), 512, True),
    "layer_major_small_tile": (CONFIGS[4].scaled(num_blocks=2048, num_layers=6, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=512), 0, True),
    # these take the three launches: too many blocks, too many table entries, too many bytes
    "too_many_blocks": (CONFIGS[4].scaled(num_blocks=32769, num_layers=1, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=1000), 0, False),
    "wide_tables": (CONFIGS[1].scaled(num_blocks=640, num_layers=1, num_seqs=40), 0, False),
    "big_blocks": (CONFIGS[1].scaled(num_blocks=640, num_layers=9, num_seqs=40, len_hi=4096), 0, False),
}


@pytest.mark.parametrize("name", list(ONE_CALL))
def test_reclaim_in_one_call_matches_oracle(oracle, name):
    """kv_reclaim: same plan arrays, header, pool bytes and tables as the oracle's steps, whichever
    way it runs (one launch on small pools, the three launches otherwise), twice in one workspace."""
    cfg, pad, one_launch = ONE_CALL[name]
    w = make_workload(cfg)
    n_entries = w.tables.size
    small = (cfg.num_blocks <= 32768 and n_entries <= 16384
             and min(cfg.boundary, cfg.num_blocks - cfg.boundary) * cfg.block_bytes <= 128 << 20)
    assert small == one_launch, "the case must take the path it is named for"
    layer_major = "layer_major" in name
    if layer_major:
        pool0, stride = _layer_major_pool(cfg, pad)
    else:
        pool0, stride = gh.host_pool(cfg, gh.content_table(cfg)), 0
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert p.status == 0 and p.n_moves > 0
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    if layer_major:
        oracle.compact_layer_major(want_pool, cfg.tile_bytes, cfg.num_layers, stride, p)
    else:
        oracle.compact(want_pool, cfg.block_bytes, p)
    assert oracle.remap(want_tables, p) == 0
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live_dev = gh.to_dev(w.live)
    stream = torch.cuda.Stream()
    for rep in range(2):
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        tables_dev = torch.from_numpy(w.tables).to(gh.dev())
        dp.ws.fill_(0x5A if rep else 0xA5)
        torch.cuda.synchronize()
        wk.kv_reclaim(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes, stride), dp.plan, live_dev,
                      tables_dev, *w.tables.shape, stream.cuda_stream)
        torch.cuda.synchronize()
        st = _compare_plan(dp, p)
        assert (st.n_free_below, st.n_bad_entries, st.ticket, st.finished, st.bad_plan) == \
               (int((~pins.bools_from_words(w.live, cfg.num_blocks)[:cfg.boundary]).sum()), 0, 0, 0, 0)
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), "tables"
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), "pool"


def test_reclaim_in_one_call_special_cases(oracle):
    """Degenerate pools, an infeasible request, bad table entries and a junk-padded bitmap through
    the single-launch path."""
    tile = 4096
    for nb, b, ids in ((0, 0, []), (1, 1, []), (70, 0, []), (70, 70, list(range(70))), (70, 35, list(range(35))),
                       (70, 35, []), (129, 64, [0, 63]), (64, 0, []), (130, 65, [3, 64, 70, 129])):
        live = bitmap_from_ids(np.array(ids, dtype=np.int64), nb)
        if live.size:
            live[-1] |= np.uint64(0xFFFFFFFFFFFFFFFF) << np.uint64(nb % 64) if nb % 64 else np.uint64(0)   # junk past NB
        p = oracle.plan(live, nb, b)
        assert p.status == 0
        pool0 = np.random.default_rng(nb + b).integers(0, 256, max(nb, 1) * tile, dtype=np.uint8)
        want_pool = pool0.copy()
        if nb:
            oracle.compact(want_pool[:nb * tile], tile, p)
        tables = np.array([ids[:4] + [-1] * (4 - len(ids[:4]))], dtype=np.int32)
        want_tables = tables.copy()
        assert oracle.remap(want_tables, p) == 0
        pool_dev, tables_dev = torch.from_numpy(pool0).to(gh.dev()), torch.from_numpy(tables).to(gh.dev())
        dp = gh.DevicePlan(nb, b)
        wk.kv_reclaim(wk.pool_desc(pool_dev, nb, 1, tile), dp.plan, gh.to_dev(live) if live.size else None, tables_dev, 1, 4)
        torch.cuda.synchronize()
        st = _compare_plan(dp, p) if nb else dp.state()
        assert st.status == 0 and st.n_moves == p.n_moves and st.n_bad_entries == 0, (nb, b)
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), (nb, b)
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), (nb, b)
    # infeasible: one more live block than fits below the boundary; nothing may change
    cfg = CONFIGS[0].scaled(num_blocks=300, boundary=100, num_seqs=16, live_budget_override=101)
    w = make_workload(cfg)
    assert oracle.plan(w.live, cfg.num_blocks, cfg.boundary).status == oracle.E_NOSPACE
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_dev, tables_dev = torch.from_numpy(pool0).to(gh.dev()), torch.from_numpy(w.tables).to(gh.dev())
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    wk.kv_reclaim(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), dp.plan, gh.to_dev(w.live),
                  tables_dev, *w.tables.shape)
    torch.cuda.synchronize()
    st = dp.state()
    assert st.status == wk.KV_E_NOSPACE and st.n_moves == 0 and st.ticket == 0 and st.finished == 0
    assert np.array_equal(pool_dev.cpu().numpy(), pool0) and np.array_equal(tables_dev.cpu().numpy(), w.tables)
    # bad table entries: left alone and counted, like the oracle
    cfg = CONFIGS[0].scaled(num_blocks=256, boundary=128, num_seqs=16)
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    free_ids = np.flatnonzero(~pins.bools_from_words(w.live, cfg.num_blocks))
    tables = w.tables.copy()
    tables[0, :4] = [int(free_ids[0]), int(free_ids[-1]), cfg.num_blocks, 2**31 - 1]
    tables[3, 7] = int(p.dst[0])                      # a free id that becomes a destination: still a bad entry
    want_tables = tables.copy()
    n_bad = oracle.remap(want_tables, p)
    assert n_bad == 5
    pool_dev, tables_dev = torch.from_numpy(gh.host_pool(cfg, gh.content_table(cfg))).to(gh.dev()), torch.from_numpy(tables).to(gh.dev())
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    wk.kv_reclaim(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), dp.plan, gh.to_dev(w.live),
                  tables_dev, *tables.shape)
    torch.cuda.synchronize()
    assert dp.state().n_bad_entries == n_bad
    assert np.array_equal(tables_dev.cpu().numpy(), want_tables)


def test_device_fill_matches_host_generator():
    for cfg in (SCALED["cfg2_ragged_tile"], SCALED["cfg5_frag"].scaled(num_blocks=64)):
        table = gh.content_table(cfg)
        n = min(cfg.num_blocks, 48)
        cids = np.array([(7 * i + 3) % 100000 for i in range(n)], dtype=np.int32)
        want = np.empty(n * cfg.block_bytes, dtype=np.uint8)
        content.fill_host(want, cfg.block_bytes, cids, cfg.seed, table)
        buf = torch.zeros(n * cfg.block_bytes, dtype=torch.uint8, device=gh.dev())
        tdev = gh.to_dev(table) if table is not None else None
        content.fill_device(buf.data_ptr(), n, cfg.block_bytes, cfg.seed, cids_ptr=gh.to_dev(cids).data_ptr(),
                            table_ptr=tdev.data_ptr() if tdev is not None else 0)
        torch.cuda.synchronize()
        assert np.array_equal(buf.cpu().numpy(), want)
        content.fill_device(buf.data_ptr(), n, cfg.block_bytes, cfg.seed, cid0=11,
                            table_ptr=tdev.data_ptr() if tdev is not None else 0)
        torch.cuda.synchronize()
        content.fill_host(want, cfg.block_bytes, range(11, 11 + n), cfg.seed, table)
        assert np.array_equal(buf.cpu().numpy(), want)


PLAN_CASES = [(1, 0, 1.0), (1, 1, 1.0), (63, 31, 0.4), (64, 64, 0.3), (65, 64, 0.5), (130, 70, 0.3),
              (1000, 999, 0.5), (4097, 2500, 0.5), (65536, 32768, 0.45), (65536, 65535, 0.5),
              (65537, 40001, 0.5), (70001, 33333, 0.4), (200000, 131072, 0.6), (200000, 77777, 0.35),
              (300000, 0, 0.0), (300000, 300000, 0.7), (1 << 20, 600011, 0.5),
              (1 << 24, 9_000_001, 0.5)]     # the last one is the largest pool the planner accepts


@pytest.mark.parametrize("nb,b,p_live", PLAN_CASES)
def test_planner_matches_oracle(oracle, nb, b, p_live):
    rs = np.random.default_rng(nb * 7 + b)
    for trial in range(2):
        live_bits = rs.random(nb) < p_live
        if trial == 1 and nb > 2:
            live_bits[max(0, b - 1)] = True
            live_bits[min(nb - 1, b)] = True
        live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
        if nb % 64:
            live[-1] |= np.uint64(0xFFFFFFFFFFFFFFFF) << np.uint64(nb % 64)   # junk past NB must be ignored
        p = oracle.plan(bitmap_from_ids(np.flatnonzero(live_bits), nb), nb, b)
        _say(f"[plan] NB={nb} b={b} p={p_live} trial={trial} oracle_status={p.status} n={p.n_moves}")
        dp = gh.DevicePlan(nb, b)
        live_dev = gh.to_dev(live)
        wk.kv_plan_reclaim(live_dev, dp.plan)
        st = _compare_plan(dp, p)
        free_below = int((~live_bits[:b]).sum())
        assert st.n_free_below == free_below


def test_degenerate_pools(oracle):
    """No blocks at all, nothing live, everything below the boundary live, boundary 0 or NB:
    plan, block copy and table rewrite all run, move nothing and report n_moves = 0."""
    tile = 4096
    for nb, b, ids in ((0, 0, []), (1, 1, []), (70, 0, []), (70, 70, list(range(70))), (70, 35, list(range(35))),
                       (70, 35, []), (129, 64, [0, 63]), (64, 0, [])):
        live = bitmap_from_ids(np.array(ids, dtype=np.int64), nb)
        p = oracle.plan(live, nb, b)
        assert p.status == 0 and p.n_moves == 0
        _say(f"[degenerate] NB={nb} b={b} live={len(ids)}")
        pool0 = np.random.default_rng(nb + b).integers(0, 256, max(nb, 1) * tile, dtype=np.uint8)
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        tables = np.array([ids[:4] + [-1] * (4 - len(ids[:4]))], dtype=np.int32)
        tables_dev = torch.from_numpy(tables).to(gh.dev())
        dp = gh.DevicePlan(nb, b)
        live_dev = gh.to_dev(live) if live.size else None
        wk.kv_plan_reclaim(live_dev, dp.plan)
        wk.kv_compact(wk.pool_desc(pool_dev, nb, 1, tile), dp.plan)
        wk.kv_compact_moves(wk.pool_desc(pool_dev, nb, 1, tile), dp.plan, 0, 5)
        wk.kv_remap_tables(tables_dev, 1, 4, dp.plan)
        torch.cuda.synchronize()
        st = _compare_plan(dp, p) if nb else dp.state()
        assert st.status == 0 and st.n_moves == 0 and st.n_bad_entries == 0 and st.ticket == 0 and st.finished == 0
        assert np.array_equal(pool_dev.cpu().numpy(), pool0)
        assert np.array_equal(tables_dev.cpu().numpy(), tables)


def test_planner_on_handworked_fixtures():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "plan_handworked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        nb, b = c["num_blocks"], c["boundary"]
        live = np.array([int(h, 16) for h in c["live_words_hex"]], dtype=np.uint64)
        dp = gh.DevicePlan(nb, b)
        wk.kv_plan_reclaim(gh.to_dev(live), dp.plan)
        st, src, dst, new_id, live_out = dp.results()
        assert st.status == c["status"], c["name"]
        if c["status"] != 0:
            continue
        assert src.tolist() == c["src"] and dst.tolist() == c["dst"], c["name"]
        if "new_id" in c:
            assert new_id.tolist() == c["new_id"]
        assert [f"{int(x):016x}" for x in live_out] == c["live_out_words_hex"]
        t = torch.tensor(c["tables_before"], dtype=torch.int32, device=gh.dev())
        wk.kv_remap_tables(t, t.shape[0], t.shape[1], dp.plan)
        torch.cuda.synchronize()
        assert t.cpu().tolist() == c["tables_after"], c["name"]


def test_infeasible_request_modifies_nothing(oracle):
    """The config's literal 70 % occupancy does not fit under its own boundary."""
    cfg = CONFIGS[1].scaled(num_blocks=2048, num_layers=2, num_seqs=64,
                            live_budget_override=int(0.7 * 2048))
    w = make_workload(cfg)
    assert w.live_count > cfg.boundary
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert p.status == oracle.E_NOSPACE
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    dp, tables_dev = gh.run_reclaim(cfg, w.live, w.tables, pool_dev)
    st = dp.state()
    assert st.status == wk.KV_E_NOSPACE and st.n_moves == 0
    assert np.array_equal(pool_dev.cpu().numpy(), pool0)
    assert np.array_equal(tables_dev.cpu().numpy(), w.tables)
    # one block fewer than the threshold fits exactly
    ids = SplitMix64(4).shuffle(cfg.num_blocks)
    for live_count, ok in ((cfg.boundary, True), (cfg.boundary + 1, False)):
        live = bitmap_from_ids(ids[:live_count], cfg.num_blocks)
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        wk.kv_plan_reclaim(gh.to_dev(live), dp.plan)
        torch.cuda.synchronize()
        assert (dp.state().status == 0) == ok
        _compare_plan(dp, oracle.plan(live, cfg.num_blocks, cfg.boundary))


def test_bad_table_entries_are_counted_and_left(oracle):
    nb, b = 300, 160
    rs = np.random.default_rng(5)
    live_bits = rs.random(nb) < 0.4
    live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
    p = oracle.plan(live, nb, b)
    assert p.status == 0
    t = rs.integers(-1, nb + 40, size=(37, 11)).astype(np.int32)   # many entries name free or outside ids
    want = t.copy()
    bad = oracle.remap(want, p)
    assert bad > 0
    dp = gh.DevicePlan(nb, b)
    wk.kv_plan_reclaim(gh.to_dev(live), dp.plan)
    td = torch.from_numpy(t).to(gh.dev())
    wk.kv_remap_tables(td, t.shape[0], t.shape[1], dp.plan)
    torch.cuda.synchronize()
    assert np.array_equal(td.cpu().numpy(), want)
    assert dp.state().n_bad_entries == bad


def test_remap_table_shapes(oracle):
    """Entry counts around the 4-wide vector path, including odd tails."""
    nb, b = 5000, 2600
    rs = np.random.default_rng(8)
    live_bits = rs.random(nb) < 0.45
    ids = np.flatnonzero(live_bits)
    live = bitmap_from_ids(ids, nb)
    p = oracle.plan(live, nb, b)
    dp = gh.DevicePlan(nb, b)
    wk.kv_plan_reclaim(gh.to_dev(live), dp.plan)
    for rows, cols in ((1, 1), (1, 3), (3, 5), (7, 4), (64, 128), (129, 33), (8192, 16), (5, 2048)):
        t = rs.choice(np.concatenate([ids, np.full(ids.size // 3, -1)]), size=(rows, cols)).astype(np.int32)
        want = t.copy()
        assert oracle.remap(want, p) == 0
        td = torch.from_numpy(t).to(gh.dev())
        wk.kv_remap_tables(td, rows, cols, dp.plan)
        torch.cuda.synchronize()
        assert np.array_equal(td.cpu().numpy(), want), (rows, cols)
    assert dp.state().n_bad_entries == 0


@pytest.mark.parametrize("kv_heads", [8, 1])   # 64 KiB blocks: one ticket each; 8 KiB blocks: both moves in one ticket
def test_hand_built_bad_plan_is_refused_per_move(kv_heads):
    """A move that breaks src >= boundary > dst is skipped and flagged; valid moves still run."""
    cfg = CONFIGS[0].scaled(num_blocks=64, boundary=32, kv_heads=kv_heads)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live = bitmap_from_ids([40, 50], cfg.num_blocks)
    wk.kv_plan_reclaim(gh.to_dev(live), dp.plan)
    torch.cuda.synchronize()
    assert dp.state().n_moves == 2
    # overwrite the lists by hand: first move valid (40 -> 0), second invalid (10 -> 50)
    dp._slice(dp.plan.src, 8).copy_(gh.to_dev(np.array([40, 10], dtype=np.int32)))
    dp._slice(dp.plan.dst, 8).copy_(gh.to_dev(np.array([0, 50], dtype=np.int32)))
    wk.kv_compact(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), dp.plan)
    torch.cuda.synchronize()
    st = dp.state()
    assert st.status == wk.KV_E_BADPLAN and st.ticket == 0 and st.finished == 0
    got = pool_dev.cpu().numpy().reshape(cfg.num_blocks, -1)
    want = pool0.reshape(cfg.num_blocks, -1).copy()
    want[0] = want[40]
    assert np.array_equal(got, want)


@pytest.mark.parametrize("kv_heads,tuning", [(8, dict(workgroups=7, chunk_bytes=4096)),     # ticket kernel, 16 units per move
                                             (1, dict(workgroups=3, chunk_bytes=16384))])   # packed kernel, two moves per ticket
def test_bad_move_among_many_leaves_counters_clean(oracle, kv_heads, tuning):
    """More units than workgroups, so tickets are drawn and every workgroup has to sign out.  One
    move of a planner-made list is corrupted by hand: it is skipped and flagged, every other move
    is copied, both counters are back at zero, and the same workspace then serves a fresh plan."""
    cfg = CONFIGS[0].scaled(num_blocks=256, boundary=128, kv_heads=kv_heads, num_seqs=16)
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert p.status == 0 and p.n_moves >= 12
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live_d = gh.to_dev(w.live)
    wk.kv_plan_reclaim(live_d, dp.plan)
    torch.cuda.synchronize()
    bad_k = 1                                   # an early move: most workgroups start after it was seen
    src = p.src.copy()
    src[bad_k] = int(p.dst[0])                  # a source below the boundary
    dp._slice(dp.plan.src, 4 * p.n_moves).copy_(gh.to_dev(src))
    wk.kv_compact_launch(pool, dp.plan, **tuning)
    torch.cuda.synchronize()
    st = dp.state()
    assert st.status == wk.KV_E_BADPLAN and st.bad_plan == 1 and st.n_moves == p.n_moves
    assert st.ticket == 0 and st.finished == 0
    bb = cfg.block_bytes
    want = pool0.copy()
    good = oracle.Plan(0, np.delete(p.src, bad_k), np.delete(p.dst, bad_k), None, None, p.n_moves - 1,
                       cfg.num_blocks, cfg.boundary)
    oracle.compact(want, bb, good)
    assert np.array_equal(pool_dev.cpu().numpy(), want), "valid moves must still be copied, the bad one skipped"
    # the table rewrite refuses to follow a plan that was not carried out in full
    tables_d = torch.from_numpy(w.tables).to(gh.dev())
    wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], dp.plan)
    torch.cuda.synchronize()
    assert np.array_equal(tables_d.cpu().numpy(), w.tables)
    # a fresh plan in the same workspace: exact against the oracle
    pool_dev.copy_(torch.from_numpy(pool0))
    wk.kv_plan_reclaim(live_d, dp.plan)
    wk.kv_compact_launch(pool, dp.plan, **tuning)
    wk.kv_remap_tables(tables_d, w.tables.shape[0], w.tables.shape[1], dp.plan)
    torch.cuda.synchronize()
    st = _compare_plan(dp, p)
    assert st.bad_plan == 0 and st.ticket == 0 and st.finished == 0
    want = pool0.copy()
    oracle.compact(want, bb, p)
    assert np.array_equal(pool_dev.cpu().numpy(), want)
    want_t = w.tables.copy()
    oracle.remap(want_t, p)
    assert np.array_equal(tables_d.cpu().numpy(), want_t)


def test_materialize_matches_oracle_and_overlaps_compaction(oracle):
    """Weights land byte-exactly in the reclaimed region, with the copy stream
    gated on the compaction event; bytes outside every extent keep their value."""
    cfg = CONFIGS[2].scaled(num_blocks=512, num_layers=4, num_seqs=48)
    w = make_workload(cfg)
    table = gh.content_table(cfg)
    pool0 = gh.host_pool(cfg, table)
    region_bytes = (cfg.num_blocks - cfg.boundary) * cfg.block_bytes
    wtable = content.normal_bf16_table(0.02)
    sizes = [3 * 4096 * 2, 1024 * 512 * 2, 256, 7 * 16, 5 * (1 << 20)]
    offs = [0, 3 * 4096 * 2, 40 << 20, (40 << 20) + 256, region_bytes - 5 * (1 << 20)]
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
        h.numpy()[:] = content.item_bytes_host(0xBEEF, i, -(-sz // 8) * 8, wtable)[:sz]
        hosts.append(h)
    # oracle
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want = pool0.copy()
    oracle.compact(want, cfg.block_bytes, p)
    assert oracle.materialize(want, cfg.boundary * cfg.block_bytes,
                              [(h.numpy(), o) for h, o in zip(hosts, offs)]) == 0
    # device: compaction on one stream, copies on another, event in between
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live_dev = gh.to_dev(w.live)
    s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    done = torch.cuda.Event()
    torch.cuda.synchronize()
    wk.kv_plan_reclaim(live_dev, dp.plan, s_compute.cuda_stream)
    wk.kv_compact(pool, dp.plan, s_compute.cuda_stream)
    done.record(s_compute)
    wk.weights_materialize(pool, cfg.boundary, [(h, h.numel(), o) for h, o in zip(hosts, offs)],
                           s_copy.cuda_stream, done.cuda_event)
    torch.cuda.synchronize()
    assert np.array_equal(pool_dev.cpu().numpy(), want)


def test_materialize_from_one_pinned_buffer(oracle):
    """Tensors cut from one pinned buffer: neighbours that continue each other in host memory
    and in the pool may go out as one request; a gap on either side, or another order, may not
    change a byte."""
    cfg = CONFIGS[2].scaled(num_blocks=256, num_layers=2, num_seqs=32)
    bb = cfg.block_bytes
    region_bytes = (cfg.num_blocks - cfg.boundary) * bb
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    sizes = [4096, 48, 3 * bb + 16, 1 << 20, 256, 2 * bb]
    buf = torch.empty(sum(sizes) + 64, dtype=torch.uint8, pin_memory=True)
    buf.numpy()[:] = content.item_bytes_host(0xC0A1, 0, -(-buf.numel() // 8) * 8, None)[:buf.numel()]
    cuts = np.concatenate([[0], np.cumsum(sizes)])
    cuts[5:] += 64                                  # a gap in host memory before the last two
    views = [buf[int(cuts[i]):int(cuts[i]) + sz] for i, sz in enumerate(sizes)]
    # pool offsets: 0,1,2 back to back; 3 after a gap; 4 right behind 3 (but host memory has the gap); 5 at the end
    offs = [0, 4096, 4096 + 48, 8 * bb, 8 * bb + (1 << 20), region_bytes - 2 * bb]
    for order in ([0, 1, 2, 3, 4, 5], [2, 0, 1, 5, 4, 3]):
        want = pool0.copy()
        assert oracle.materialize(want, cfg.boundary * bb, [(views[i].numpy(), offs[i]) for i in order]) == 0
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        wk.weights_materialize(pool, cfg.boundary, [(views[i], sizes[i], offs[i]) for i in order])
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), order
        live = np.zeros((cfg.num_blocks + 63) // 64, dtype=np.uint64)      # nothing live: every piece is early
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        wk.weights_materialize_pipelined(pool, cfg.boundary, live, [(views[i], sizes[i], offs[i]) for i in order], 1 << 40)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), ("pipelined", order)


def test_pipelined_materialize_matches_oracle(oracle):
    """Block-granular pipelining: early pieces go out before the compaction event, the rest
    after it; the pool must hold exactly what the oracle's plain copy produces."""
    cfg = CONFIGS[2].scaled(num_blocks=768, num_layers=2, num_seqs=64)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    bb = cfg.block_bytes
    region_bytes = (cfg.num_blocks - cfg.boundary) * bb
    wtable = content.normal_bf16_table(0.02)
    sizes = [5 * bb + 4096, 256, 17 * bb, 3 * bb - 512, region_bytes // 4]
    offs = [0, 5 * bb + 4096, 6 * bb, 24 * bb + 512, region_bytes - region_bytes // 4]
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
        h.numpy()[:] = content.item_bytes_host(0xFEED, i, -(-sz // 8) * 8, wtable)[:sz]
        hosts.append(h)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want = pool0.copy()
    oracle.compact(want, bb, p)
    assert oracle.materialize(want, cfg.boundary * bb, [(h.numpy(), o) for h, o in zip(hosts, offs)]) == 0
    tensors = [(h, h.numel(), o) for h, o in zip(hosts, offs)]
    for early_bytes in (0, 3 * bb, 1, 1 << 40):
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        pieces = wk.weights_materialize_schedule(pool, cfg.boundary, w.live, tensors, early_bytes)
        if early_bytes == 0:       # the library's own policy: no early piece that costs more than it hides
            assert all(n >= 2 << 20 for _, e, _, _, n in pieces if e)
        else:
            assert any(e for _, e, *_ in pieces) and any(not e for _, e, *_ in pieces)
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        live_dev = gh.to_dev(w.live)
        s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
        done = torch.cuda.Event()
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_dev, dp.plan, s_compute.cuda_stream)
        wk.kv_compact(pool, dp.plan, s_compute.cuda_stream)
        done.record(s_compute)
        wk.weights_materialize_pipelined(pool, cfg.boundary, w.live, tensors, early_bytes,
                                         s_copy.cuda_stream, done.cuda_event)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), f"early_bytes={early_bytes}"


def test_vmm_variant_lends_pages_without_moving_bytes(oracle):
    """The no-move variant: pages of unused blocks appear back to back in the slot range,
    live KV is untouched, weights written through the slot land in those pages, and a
    restore puts every page back under its block."""
    nb, bb, seed = 160, 2 << 20, 77
    try:
        pool = wk.kv_vmm_pool_create(nb, bb)
    except wk.WarmKVError as e:
        if e.code == wk.KV_E_ALIGN:
            pytest.skip("allocation granularity does not divide 2 MiB")
        raise
    try:
        kv_ptr, slot_ptr = wk.kv_vmm_kv_base(pool), wk.kv_vmm_slot_base(pool)
        content.fill_device(kv_ptr, nb, bb, seed)
        torch.cuda.synchronize()
        rs = np.random.default_rng(3)
        live_bits = rs.random(nb) < 0.55
        live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
        free_desc = np.flatnonzero(~live_bits)[::-1]
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_vmm_reclaim(pool, live, free_desc.size + 1)
        assert e.value.code == wk.KV_E_NOSPACE
        assert oracle.vmm_select(live, nb, free_desc.size + 1) is None
        assert wk.kv_vmm_lent(pool) == 0
        want = 40
        ids = wk.kv_vmm_reclaim(pool, live, want)
        assert ids == oracle.vmm_select(live, nb, want).tolist()      # the oracle's page choice, in slot order
        assert wk.kv_vmm_lent(pool) == want
        kv = gh.view_device(kv_ptr, nb * bb)
        slot = gh.view_device(slot_ptr, want * bb)
        expect = torch.empty(bb, dtype=torch.uint8, device=gh.dev())

        def check_block(t, index, cid):
            content.fill_device(expect.data_ptr(), 1, bb, seed, cid0=cid)
            assert torch.equal(t[index * bb:(index + 1) * bb], expect), (index, cid)

        for k, i in enumerate(ids):                      # pages kept their bytes and their order
            check_block(slot, k, i)
        lent = set(ids)
        for i in range(nb):                              # everything still mapped in the KV range is intact
            if i not in lent:
                check_block(kv, i, i)
        weights = torch.empty(want * bb - 4096, dtype=torch.uint8, pin_memory=True)
        weights.numpy()[:] = content.item_bytes_host(5, 1, weights.numel(), None)
        slot[:weights.numel()].copy_(weights, non_blocking=True)
        torch.cuda.synchronize()
        assert torch.equal(slot[:weights.numel()].cpu(), weights)
        for i in np.flatnonzero(live_bits).tolist():
            check_block(kv, i, i)
        with pytest.raises(wk.WarmKVError) as e:         # pages already lent
            wk.kv_vmm_reclaim(pool, live, 1)
        assert e.value.code == wk.KV_E_RANGE
        del slot
        wk.kv_vmm_restore(pool)
        for i in np.flatnonzero(live_bits).tolist():
            check_block(kv, i, i)
        k = 3                                            # a returned page still holds the weight bytes written to it
        assert torch.equal(kv[ids[k] * bb:(ids[k] + 1) * bb].cpu(), weights[k * bb:(k + 1) * bb])
        ids2 = wk.kv_vmm_reclaim(pool, live, 5)          # and the pool can lend again
        assert ids2 == oracle.vmm_select(live, nb, 5).tolist()
        wk.kv_vmm_restore(pool)
        assert wk.kv_vmm_lent(pool) == 0

        # the same hand-over with the weight stream pipelined behind the mapping, chunk by chunk:
        # the slot must hold what the oracle's weight copy puts into a host buffer of the same size
        content.fill_device(kv_ptr, nb, bb, seed)
        want = 37
        sizes = [5 * bb + 4096, 256, 0, 11 * bb - 8192, 3 * bb // 2]
        offs = [bb // 2, 6 * bb, 6 * bb + 512, 7 * bb, 20 * bb + 256]      # unordered in time: listed shuffled below
        hosts = []
        for i, sz in enumerate(sizes):
            t = torch.empty(max(sz, 8), dtype=torch.uint8, pin_memory=True)
            t.numpy()[:sz] = content.item_bytes_host(9, i, (sz + 7) // 8 * 8, None)[:sz]
            hosts.append(t)
        listed = [3, 0, 4, 2, 1]
        copy_stream = torch.cuda.Stream()
        for chunk in (4, 0, 1000):
            with pytest.raises(wk.WarmKVError) as e:     # an extent past the slot prefix: refused before anything changes
                wk.kv_vmm_reclaim_load(pool, live, want, [(hosts[0], bb, want * bb - 16)], copy_stream.cuda_stream, chunk)
            assert e.value.code == wk.KV_E_TOOBIG and wk.kv_vmm_lent(pool) == 0
            with pytest.raises(wk.WarmKVError) as e:
                wk.kv_vmm_reclaim_load(pool, live, want, [(hosts[0], bb, 0), (hosts[3], bb, bb - 16)],
                                       copy_stream.cuda_stream, chunk)
            assert e.value.code == wk.KV_E_OVERLAP and wk.kv_vmm_lent(pool) == 0
            ids3 = wk.kv_vmm_reclaim_load(pool, live, want, [(hosts[i], sizes[i], offs[i]) for i in listed],
                                          copy_stream.cuda_stream, chunk)
            torch.cuda.synchronize()
            assert ids3 == oracle.vmm_select(live, nb, want).tolist()
            expect_slot = np.empty(want * bb, dtype=np.uint8)
            content.fill_host(expect_slot, bb, ids3, seed, None)           # the pages' old bytes, in slot order
            assert oracle.materialize(expect_slot, 0, [(hosts[i].numpy()[:sizes[i]], offs[i]) for i in listed]) == 0
            slot = gh.view_device(slot_ptr, want * bb)
            assert np.array_equal(slot.cpu().numpy(), expect_slot), f"chunk_blocks={chunk}"
            for i in np.flatnonzero(live_bits).tolist()[::7]:
                check_block(kv, i, i)
            del slot
            wk.kv_vmm_restore(pool)
            content.fill_device(kv_ptr, nb, bb, seed)
            torch.cuda.synchronize()
        del kv
    finally:
        torch.cuda.synchronize()
        wk.kv_vmm_pool_destroy(pool)


LAYER_MAJOR = {
    "lm_small": (CONFIGS[1].scaled(num_blocks=640, num_layers=3, num_seqs=40), 0),
    "lm_padded_slabs": (CONFIGS[3].scaled(num_blocks=1536, num_layers=4, num_seqs=128), 4096),
    "lm_ragged_tile": (CONFIGS[1].scaled(num_blocks=900, num_layers=5, kv_heads=3, head_dim=40, num_seqs=40), 256),
    "lm_tiny_tile": (CONFIGS[4].scaled(num_blocks=2048, num_layers=6, block_size=1, kv_heads=1, head_dim=8, len_hi=16, num_seqs=512), 0),
    # tiles of half a ticket or less: several moves of one slab share a ticket
    "lm_16k_tile": (CONFIGS[1].scaled(num_blocks=1100, num_layers=3, kv_heads=2, num_seqs=50), 0),
    "lm_7680_tile": (CONFIGS[1].scaled(num_blocks=1300, num_layers=4, kv_heads=3, head_dim=40, num_seqs=50), 512),
}


def _layer_major_pool(cfg, pad):
    """Host pool [L][stride]: slab l holds bytes [l*tile, (l+1)*tile) of every block's content."""
    table = gh.content_table(cfg)
    tile, nb, layers = cfg.tile_bytes, cfg.num_blocks, cfg.num_layers
    stride = nb * tile + pad
    pool = np.full(layers * stride, 0x5A, dtype=np.uint8)
    slabs = pool.reshape(layers, stride)
    for i in range(nb):
        blk = content.item_bytes_host(cfg.seed, i, cfg.block_bytes, table).reshape(layers, tile)
        slabs[:, i * tile:(i + 1) * tile] = blk
    return pool, stride


@pytest.mark.parametrize("name", list(LAYER_MAJOR))
def test_layer_major_reclaim_matches_oracle(oracle, name):
    cfg, pad = LAYER_MAJOR[name]
    w = make_workload(cfg)
    pool0, stride = _layer_major_pool(cfg, pad)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert p.status == 0 and p.n_moves > 0
    want = pool0.copy()
    oracle.compact_layer_major(want, cfg.tile_bytes, cfg.num_layers, stride, p)
    # weights into the strips: one tensor per strip start, one that ends exactly at a strip end
    strip = (cfg.num_blocks - cfg.boundary) * cfg.tile_bytes
    sizes = [min(strip, 4096 * 3), min(strip, 100 * 16)]
    offs = [0, (cfg.num_layers - 1) * strip + strip - sizes[1]]
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
        h.numpy()[:] = content.item_bytes_host(0xABCD, i, -(-sz // 8) * 8, None)[:sz]
        hosts.append(h)
    assert oracle.materialize_strips(want, cfg.tile_bytes, cfg.num_layers, cfg.num_blocks, cfg.boundary, stride,
                                     [(h.numpy(), o) for h, o in zip(hosts, offs)]) == 0
    for tuning in (None, dict(chunk_bytes=4096, flags=2 << 4), dict(workgroups=3000, chunk_bytes=16384, flags=4 << 4),
                   dict(workgroups=512, chunk_bytes=32768, flags=(2 << 4) | 2), dict(flags=4),
                   dict(workgroups=100, chunk_bytes=8192, flags=(2 << 4) | 2 | 4), dict(flags=8), dict(flags=8 | 4),
                   dict(workgroups=33, chunk_bytes=32768)):
        _say(f"[layer-major] {name} tile={cfg.tile_bytes} L={cfg.num_layers} NB={cfg.num_blocks} pad={pad} tuning={tuning}")
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes, stride)
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        live_dev = gh.to_dev(w.live)
        wk.kv_plan_reclaim(live_dev, dp.plan)
        if tuning:
            wk.kv_compact_launch(pool, dp.plan, **tuning)
        else:
            wk.kv_compact(pool, dp.plan)
        wk.weights_materialize(pool, cfg.boundary, [(h, h.numel(), o) for h, o in zip(hosts, offs)])
        torch.cuda.synchronize()
        _compare_plan(dp, p)
        assert np.array_equal(pool_dev.cpu().numpy(), want)
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes, stride)
    with pytest.raises(wk.WarmKVError) as e:      # an extent across two strips is not contiguous in memory
        wk.weights_materialize(pool, cfg.boundary, [(hosts[0], 32, strip - 16)])
    assert e.value.code == wk.KV_E_TOOBIG
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_compact(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes,
                                   cfg.num_blocks * cfg.tile_bytes - 256), dp.plan)   # slabs would overlap
    assert e.value.code == wk.KV_E_RANGE


def _strip_tensors(cfg, seed):
    """Weight extents for a layer-major pool: several per strip, never across a strip end; one
    starts a strip, one ends the last strip exactly, one is empty.  Returns (hosts, sizes, offs)."""
    strip = (cfg.num_blocks - cfg.boundary) * cfg.tile_bytes
    tile = cfg.tile_bytes
    sizes, offs = [], []
    for l in range(cfg.num_layers):
        a = min(strip // 3, 5 * tile + 48) // 16 * 16
        sizes += [a, min(strip - strip // 2, 3 * tile) // 16 * 16]
        offs += [l * strip + (16 if l else 0), l * strip + strip // 2 // 16 * 16]
    sizes += [0, min(strip // 4, 2 * tile + 16) // 16 * 16]
    offs += [strip, (cfg.num_layers - 1) * strip + strip - min(strip // 4, 2 * tile + 16) // 16 * 16]
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(max(sz, 16), dtype=torch.uint8, pin_memory=True)
        h.numpy()[:sz] = content.item_bytes_host(seed, i, -(-sz // 8) * 8, None)[:sz]
        hosts.append(h)
    return hosts, sizes, offs


@pytest.mark.parametrize("name", ["lm_small", "lm_padded_slabs", "lm_16k_tile"])
def test_layer_major_pipelined_weight_paths_match_oracle(oracle, name):
    """Layer-major pools through every overlapped weight path: block copy by layer ranges with the
    front-first stream (the region is ready strip by strip), the tile-granular schedule, and
    kv_switch in all three modes.  Pool and tables against the oracle's layer-major steps."""
    cfg, pad = LAYER_MAJOR[name]
    w = make_workload(cfg)
    pool0, stride = _layer_major_pool(cfg, pad)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    hosts, sizes, offs = _strip_tensors(cfg, 0x77)
    want = pool0.copy()
    oracle.compact_layer_major(want, cfg.tile_bytes, cfg.num_layers, stride, p)
    assert oracle.materialize_strips(want, cfg.tile_bytes, cfg.num_layers, cfg.num_blocks, cfg.boundary, stride,
                                     [(h.numpy()[:sz], o) for h, sz, o in zip(hosts, sizes, offs)]) == 0
    want_tables = w.tables.copy()
    assert oracle.remap(want_tables, p) == 0
    strip = (cfg.num_blocks - cfg.boundary) * cfg.tile_bytes
    L = cfg.num_layers
    order = list(range(len(sizes)))[::-1]            # listed from the last strip back to the first
    tensors = [(hosts[i], sizes[i], offs[i]) for i in order]
    s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    done, front_done = torch.cuda.Event(), torch.cuda.Event()
    done.record(s_compute)
    front_done.record(s_compute)
    live_dev = gh.to_dev(w.live)

    def fresh():
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        return (pool_dev, wk.pool_desc(pool_dev, cfg.num_blocks, L, cfg.tile_bytes, stride),
                torch.from_numpy(w.tables).to(gh.dev()), gh.DevicePlan(cfg.num_blocks, cfg.boundary))

    def check(pool_dev, tables_dev, dp, what):
        torch.cuda.synchronize()
        st = _compare_plan(dp, p)
        assert st.ticket == 0 and st.finished == 0 and st.bad_plan == 0
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), what
        assert np.array_equal(pool_dev.cpu().numpy(), want), what

    cs, ss = s_compute.cuda_stream, s_copy.cuda_stream
    # explicit front-first: the first f strips behind the first event
    for front_bytes in (0, 1, strip, strip + 16, (L - 1) * strip + strip // 2, L * strip + 99):
        f = min(L, -(-front_bytes // strip))
        pool_dev, pool, tables_dev, dp = fresh()
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_dev, dp.plan, cs)
        wk.kv_compact_layers(pool, dp.plan, 0, f, cs)
        front_done.record(s_compute)
        wk.kv_compact_layers(pool, dp.plan, f, 0xFFFFFFFF, cs)
        done.record(s_compute)
        wk.kv_remap_tables(tables_dev, *w.tables.shape, dp.plan, cs)
        wk.weights_materialize_front(pool, cfg.boundary, front_bytes, tensors, ss, front_done.cuda_event, done.cuda_event)
        check(pool_dev, tables_dev, dp, f"front {front_bytes} ({f} strips)")
    # tile-granular schedule
    for early in (0, 3 * cfg.tile_bytes, 1 << 40):
        pool_dev, pool, tables_dev, dp = fresh()
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_dev, dp.plan, cs)
        wk.kv_compact(pool, dp.plan, cs)
        done.record(s_compute)
        wk.weights_materialize_pipelined(pool, cfg.boundary, w.live, tensors, early, ss, done.cuda_event)
        wk.kv_remap_tables(tables_dev, *w.tables.shape, dp.plan, cs)
        check(pool_dev, tables_dev, dp, f"pipelined early={early}")
    # one call
    for mode, early in (("gated", 0), ("block", 0), ("front", 0), ("front", strip + 1), ("front", 1 << 40)):
        pool_dev, pool, tables_dev, dp = fresh()
        torch.cuda.synchronize()
        st = wk.kv_switch(pool, dp.plan, live_dev, tables_dev, *w.tables.shape, tensors, cs, ss, done.cuda_event,
                          live_host=None if mode == "gated" else w.live, early_bytes=early,
                          front_done=front_done.cuda_event if mode == "front" else None)
        assert st.status == 0 and st.n_moves == p.n_moves
        check(pool_dev, tables_dev, dp, f"kv_switch {mode} early={early}")


@pytest.mark.parametrize("layer_major", [False, True])
def test_block_copy_of_a_range_of_layers(oracle, layer_major):
    """kv_compact_layers copies exactly the tiles of the chosen layers of every move, in both
    layouts, and consecutive ranges add up to the whole block copy."""
    cfg = CONFIGS[1].scaled(num_blocks=400, num_layers=5, num_seqs=30)
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    tile, L, nb = cfg.tile_bytes, cfg.num_layers, cfg.num_blocks
    if layer_major:
        pool0, stride = _layer_major_pool(cfg, 512)
    else:
        pool0, stride = gh.host_pool(cfg, gh.content_table(cfg)), 0

    def tiles(buf, layer):      # view [num_blocks, tile] of one layer's tiles
        if layer_major:
            return buf[layer * stride:layer * stride + nb * tile].reshape(nb, tile)
        return buf.reshape(nb, L, tile)[:, layer, :]

    dp = gh.DevicePlan(nb, cfg.boundary)
    wk.kv_plan_reclaim(gh.to_dev(w.live), dp.plan)
    for first, count in ((0, 1), (2, 2), (4, 7), (5, 1), (1, 0), (0, 0xFFFFFFFF)):
        want = pool0.copy()
        for l in range(first, min(L, first + count)):
            tiles(want, l)[p.dst] = tiles(pool0, l)[p.src]      # the oracle's moves, these layers only
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        wk.kv_compact_layers(wk.pool_desc(pool_dev, nb, L, tile, stride), dp.plan, first, count)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), (first, count)
        st = dp.state()
        assert st.ticket == 0 and st.finished == 0
    want = pool0.copy()
    if layer_major:
        oracle.compact_layer_major(want, tile, L, stride, p)
    else:
        oracle.compact(want, cfg.block_bytes, p)
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    for first, count in ((0, 2), (2, 1), (3, 9)):
        wk.kv_compact_layers(wk.pool_desc(pool_dev, nb, L, tile, stride), dp.plan, first, count)
    torch.cuda.synchronize()
    assert np.array_equal(pool_dev.cpu().numpy(), want)


def test_two_reclaims_on_two_streams_do_not_interfere(oracle):
    """The library keeps no global state: two pools, two plans, two streams, interleaved calls."""
    cfgs = [CONFIGS[1].scaled(num_blocks=1024, num_layers=4, num_seqs=64),
            CONFIGS[4].scaled(num_blocks=3000, num_layers=3, num_seqs=700)]
    runs = []
    for cfg in cfgs:
        w = make_workload(cfg)
        pool0 = gh.host_pool(cfg, gh.content_table(cfg))
        p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
        want_pool, want_tables = pool0.copy(), w.tables.copy()
        oracle.compact(want_pool, cfg.block_bytes, p)
        oracle.remap(want_tables, p)
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        runs.append(dict(cfg=cfg, w=w, p=p, want_pool=want_pool, want_tables=want_tables, pool_dev=pool_dev,
                         pool=wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes),
                         dp=gh.DevicePlan(cfg.num_blocks, cfg.boundary), live_dev=gh.to_dev(w.live),
                         tables_dev=torch.from_numpy(w.tables).to(gh.dev()), stream=torch.cuda.Stream()))
    torch.cuda.synchronize()
    for r in runs:
        wk.kv_plan_reclaim(r["live_dev"], r["dp"].plan, r["stream"].cuda_stream)
    for r in runs:
        wk.kv_compact(r["pool"], r["dp"].plan, r["stream"].cuda_stream)
    for r in reversed(runs):
        wk.kv_remap_tables(r["tables_dev"], r["w"].tables.shape[0], r["w"].tables.shape[1], r["dp"].plan,
                           r["stream"].cuda_stream)
    torch.cuda.synchronize()
    for r in runs:
        _compare_plan(r["dp"], r["p"])
        assert np.array_equal(r["tables_dev"].cpu().numpy(), r["want_tables"])
        assert np.array_equal(r["pool_dev"].cpu().numpy(), r["want_pool"])


def test_plan_can_be_reused_after_the_pool_changes(oracle):
    """Plan, move, then plan again on the bitmap the first plan produced: nothing is left to move,
    and a third plan after new allocations above the boundary moves exactly those."""
    cfg = CONFIGS[1].scaled(num_blocks=2048, num_layers=2, num_seqs=64)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    dp, tables_dev = gh.run_reclaim(cfg, w.live, w.tables, pool_dev)
    st, src, dst, new_id, live_out = dp.results()
    p1 = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    assert np.array_equal(live_out, p1.live_out)
    dp2 = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    wk.kv_plan_reclaim(gh.to_dev(live_out), dp2.plan)
    wk.kv_compact(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), dp2.plan)
    torch.cuda.synchronize()
    assert dp2.state().n_moves == 0 and dp2.state().status == 0
    grown = live_out.copy()
    for j in (cfg.boundary, cfg.boundary + 65, cfg.num_blocks - 1):
        grown[j // 64] |= np.uint64(1) << np.uint64(j % 64)
    p3 = oracle.plan(grown, cfg.num_blocks, cfg.boundary)
    wk.kv_plan_reclaim(gh.to_dev(grown), dp2.plan)          # same workspace, third use
    _compare_plan(dp2, p3)
    assert p3.n_moves == 3


@pytest.mark.parametrize("kv_heads", [8, 1])     # 128 KiB blocks: ticket kernel; 16 KiB blocks: several moves per ticket
def test_block_copy_of_a_part_of_the_plan(oracle, kv_heads):
    """kv_compact_moves over [first, first + max): exactly those moves, and the parts together
    give the whole block copy."""
    cfg = CONFIGS[1].scaled(num_blocks=1200, num_layers=2, num_seqs=60, kv_heads=kv_heads)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    n = p.n_moves
    assert n > 40
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    wk.kv_plan_reclaim(gh.to_dev(w.live), dp.plan)
    for first, count in ((0, 17), (17, 1), (n - 5, 100), (n, 3), (5, 0), (3, n - 3), (cfg.num_blocks, 9)):
        want = pool0.copy()
        lo, hi = min(first, n), min(first + count, n)
        part = oracle.Plan(0, p.src[lo:hi], p.dst[lo:hi], p.new_id, p.live_out, hi - lo, cfg.num_blocks, cfg.boundary)
        oracle.compact(want, cfg.block_bytes, part)
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        wk.kv_compact_moves(wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), dp.plan, first, count)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), (first, count)
        st = dp.state()
        assert st.ticket == 0 and st.finished == 0
    want = pool0.copy()
    oracle.compact(want, cfg.block_bytes, p)
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    for first, count in ((0, 9), (9, n // 2), (9 + n // 2, 1 << 31)):
        wk.kv_compact_moves(pool, dp.plan, first, count)
    torch.cuda.synchronize()
    assert np.array_equal(pool_dev.cpu().numpy(), want)


def test_front_first_weight_stream_matches_oracle(oracle):
    """The front-first stream writes the same bytes as the plain one wherever the mark falls:
    before every tensor, inside one, on a tensor boundary, beyond the region."""
    cfg = CONFIGS[2].scaled(num_blocks=512, num_layers=2, num_seqs=48)
    w = make_workload(cfg)
    bb = cfg.block_bytes
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    region = (cfg.num_blocks - cfg.boundary) * bb
    sizes = [3 * bb + 48, 4096, 9 * bb, region // 8 // 16 * 16]
    offs = [16, 3 * bb + 64, 4 * bb, region - sizes[3]]
    buf = torch.empty(sum(sizes), dtype=torch.uint8, pin_memory=True)
    buf.numpy()[:] = content.item_bytes_host(0xF0, 0, -(-buf.numel() // 8) * 8, None)[:buf.numel()]
    cuts = np.concatenate([[0], np.cumsum(sizes)])
    views = [buf[int(cuts[i]):int(cuts[i + 1])] for i in range(len(sizes))]
    tensors = [(v, v.numel(), o) for v, o in zip(views, offs)]
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want = pool0.copy()
    oracle.compact(want, bb, p)
    assert oracle.materialize(want, cfg.boundary * bb, [(v.numpy(), o) for v, o in zip(views, offs)]) == 0
    for front_blocks in (0, 1, 3, 4, 13, cfg.num_blocks):
        front_bytes = front_blocks * bb
        head = wk.kv_movers_in_front(w.live, cfg.num_blocks, cfg.boundary, front_blocks)
        assert head == int((p.src < cfg.boundary + front_blocks).sum())
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        live_dev = gh.to_dev(w.live)
        s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
        front_done, done = torch.cuda.Event(), torch.cuda.Event()
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_dev, dp.plan, s_compute.cuda_stream)
        wk.kv_compact_moves(pool, dp.plan, 0, head, s_compute.cuda_stream)
        front_done.record(s_compute)
        wk.kv_compact_moves(pool, dp.plan, head, 1 << 31, s_compute.cuda_stream)
        done.record(s_compute)
        wk.weights_materialize_front(pool, cfg.boundary, front_bytes, tensors, s_copy.cuda_stream,
                                     front_done.cuda_event, done.cuda_event)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want), front_blocks


@pytest.mark.parametrize("n_streams", [1, 2, 3, 4])
def test_weight_stream_over_several_copy_streams_matches_oracle(oracle, n_streams):
    """weights_materialize_streams deals the requests out over 1-4 streams; the pool must hold what the
    oracle's copies produce, with the mark anywhere, the block copy running beside it, and tensors
    that cannot be merged (separate pinned buffers, gaps between them in the region)."""
    cfg = CONFIGS[2].scaled(num_blocks=640, num_layers=2, num_seqs=48)
    w = make_workload(cfg)
    bb = cfg.block_bytes
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    region = (cfg.num_blocks - cfg.boundary) * bb
    rs = np.random.default_rng(n_streams)
    sizes, offs, at = [], [], 0
    while at + 3 * bb < region and len(sizes) < 60:
        sz = int(rs.integers(1, 3 * bb // 16)) * 16
        sizes.append(sz)
        offs.append(at)
        at += sz + int(rs.integers(0, 3)) * 256
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
        h.numpy()[:] = content.item_bytes_host(0xD0, i, -(-sz // 8) * 8, None)[:sz]
        hosts.append(h)
    order = rs.permutation(len(sizes)).tolist()
    tensors = [(hosts[i], sizes[i], offs[i]) for i in order]
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    oracle.compact(want_pool, bb, p)
    assert oracle.remap(want_tables, p) == 0
    assert oracle.materialize(want_pool, cfg.boundary * bb, [(hosts[i].numpy(), offs[i]) for i in order]) == 0
    s_compute = torch.cuda.Stream()
    copies = [torch.cuda.Stream() for _ in range(n_streams)]
    done, front_done = torch.cuda.Event(), torch.cuda.Event()
    done.record(s_compute)
    front_done.record(s_compute)
    live_dev = gh.to_dev(w.live)
    for front_blocks in (0, 5, cfg.num_blocks):
        front_bytes = front_blocks * bb + (4096 if front_blocks == 5 else 0)
        head = wk.kv_movers_in_front(w.live, cfg.num_blocks, cfg.boundary, -(-front_bytes // bb))
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        torch.cuda.synchronize()
        wk.kv_plan_reclaim(live_dev, dp.plan, s_compute.cuda_stream)
        wk.kv_compact_moves(pool, dp.plan, 0, head, s_compute.cuda_stream)
        front_done.record(s_compute)
        wk.kv_compact_moves(pool, dp.plan, head, 1 << 31, s_compute.cuda_stream)
        done.record(s_compute)
        wk.weights_materialize_streams(pool, cfg.boundary, tensors, [c.cuda_stream for c in copies], front_bytes,
                                       front_done.cuda_event if front_blocks else None, done.cuda_event)
        torch.cuda.synchronize()
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), (n_streams, front_blocks)
    # kv_switch with a second copy stream, in its three modes
    for mode in ("gated", "block", "front"):
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
        tables_dev = torch.from_numpy(w.tables).to(gh.dev())
        dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
        torch.cuda.synchronize()
        st = wk.kv_switch(pool, dp.plan, live_dev, tables_dev, *w.tables.shape, tensors, s_compute.cuda_stream,
                          copies[0].cuda_stream, done.cuda_event, live_host=None if mode == "gated" else w.live,
                          early_bytes=(1 << 40) if mode == "block" else 0,
                          front_done=front_done.cuda_event if mode == "front" else None,
                          copy_stream2=copies[-1].cuda_stream if n_streams > 1 else None)
        assert st.status == 0 and st.n_moves == p.n_moves
        torch.cuda.synchronize()
        _compare_plan(dp, p)
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), mode
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), mode
    with pytest.raises(wk.WarmKVError) as e:
        wk.weights_materialize_streams(pool, cfg.boundary, tensors, [c.cuda_stream for c in copies] * 5)
    assert e.value.code == wk.KV_E_RANGE
    with pytest.raises(wk.WarmKVError) as e:
        wk.weights_materialize_streams(pool, cfg.boundary, tensors, [])
    assert e.value.code == wk.KV_E_RANGE


@pytest.mark.parametrize("pipelined", [False, True, "front"])
def test_switch_in_one_call(oracle, pipelined):
    """kv_switch = plan + block copy + table rewrite + weight stream; byte-identical to the
    oracle's steps.  An infeasible request comes back as KV_E_NOSPACE with no pool byte, table
    entry or weight byte moved - the weights must not land on the blocks that could not move."""
    cfg = CONFIGS[2].scaled(num_blocks=640, num_layers=2, num_seqs=48)
    w = make_workload(cfg)
    bb = cfg.block_bytes
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    region = (cfg.num_blocks - cfg.boundary) * bb
    sizes = [region // 2 // 16 * 16, 4096, region // 8 // 16 * 16]
    offs = [0, sizes[0], region - sizes[2]]
    hosts = []
    for i, sz in enumerate(sizes):
        h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
        h.numpy()[:] = content.item_bytes_host(0x51, i, -(-sz // 8) * 8, None)[:sz]
        hosts.append(h)
    tensors = [(h, h.numel(), o) for h, o in zip(hosts, offs)]
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    oracle.compact(want_pool, bb, p)
    assert oracle.remap(want_tables, p) == 0
    assert oracle.materialize(want_pool, cfg.boundary * bb, [(h.numpy(), o) for h, o in zip(hosts, offs)]) == 0

    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    tables_dev = torch.from_numpy(w.tables).to(gh.dev())
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    live_dev = gh.to_dev(w.live)
    s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    done, front_done = torch.cuda.Event(), torch.cuda.Event()
    done.record(s_compute)                 # torch creates the HIP event lazily, on its first record
    front_done.record(s_compute)
    front = front_done.cuda_event if pipelined == "front" else None
    torch.cuda.synchronize()
    st = wk.kv_switch(pool, dp.plan, live_dev, tables_dev, *w.tables.shape, tensors, s_compute.cuda_stream,
                      s_copy.cuda_stream, done.cuda_event, live_host=w.live if pipelined else None, front_done=front)
    assert st.status == 0 and st.n_moves == p.n_moves
    torch.cuda.synchronize()
    _compare_plan(dp, p)
    assert np.array_equal(tables_dev.cpu().numpy(), want_tables)
    assert np.array_equal(pool_dev.cpu().numpy(), want_pool)

    # infeasible: more live blocks than fit under the boundary
    full = cfg.scaled(live_budget_override=cfg.boundary + 7)
    wf = make_workload(full)
    assert oracle.plan(wf.live, cfg.num_blocks, cfg.boundary).status == oracle.E_NOSPACE
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    tables_dev = torch.from_numpy(wf.tables).to(gh.dev())
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_switch(pool, dp.plan, gh.to_dev(wf.live), tables_dev, *wf.tables.shape, tensors, s_compute.cuda_stream,
                     s_copy.cuda_stream, done.cuda_event, live_host=wf.live if pipelined else None, front_done=front)
    assert e.value.code == wk.KV_E_NOSPACE
    torch.cuda.synchronize()
    assert np.array_equal(pool_dev.cpu().numpy(), pool0), "an infeasible hand-over must not write the pool"
    assert np.array_equal(tables_dev.cpu().numpy(), wf.tables)


def test_draining_instance_life_cycle(oracle):
    """The whole scenario of Sec. 3.3 on one small pool, device state chained from step to step
    with no host copy in between: Eq. 4 gives the boundary; reclaim; weights go in; requests
    finish; Eq. 4 gives a lower boundary; reclaim again from the bitmap and tables the first
    round left on the device; more weights; then the reserve proves too small and the boundary
    rises again.  The oracle runs the same chain on the host."""
    cfg = CONFIGS[1].scaled(num_blocks=1024, num_layers=2, num_seqs=64, boundary=1024, live_budget_override=400)
    w = make_workload(cfg)
    nb, bb = cfg.num_blocks, cfg.block_bytes
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    running = int((w.tables[:, 0] >= 0).sum())
    b1 = wk.kv_reserve_blocks(nb, w.live_count, running, 2 * running)
    assert b1 == oracle.reserve_blocks(nb, w.live_count, running, 2 * running) and w.live_count <= b1 < nb

    def weights(seed, sizes):
        out = []
        for i, sz in enumerate(sizes):
            h = torch.empty(sz, dtype=torch.uint8, pin_memory=True)
            h.numpy()[:] = content.item_bytes_host(seed, i, -(-sz // 8) * 8, None)[:sz]
            out.append(h)
        return out

    # ---- host chain (oracle)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    p1 = oracle.plan(w.live, nb, b1)
    assert p1.status == 0 and p1.n_moves > 0
    oracle.compact(want_pool, bb, p1)
    assert oracle.remap(want_tables, p1) == 0
    region1 = (nb - b1) * bb
    sizes1 = [region1 // 3 // 16 * 16, 4096, region1 // 4 // 16 * 16]
    offs1 = [0, sizes1[0], region1 - sizes1[2]]
    hosts1 = weights(0xA1, sizes1)
    assert oracle.materialize(want_pool, b1 * bb, [(h.numpy(), o) for h, o in zip(hosts1, offs1)]) == 0
    # every second running sequence finishes: its blocks become free, its row empty
    done_rows = [r for r in range(want_tables.shape[0]) if want_tables[r, 0] >= 0][::2]
    live2 = p1.live_out.copy()
    for r in done_rows:
        for e in want_tables[r][want_tables[r] >= 0].tolist():
            live2[e // 64] &= ~(np.uint64(1) << np.uint64(e % 64))
        want_tables[r] = -1
    used2 = int(sum(bin(int(x)).count("1") for x in live2))
    b2 = oracle.reserve_blocks(b1, used2, running - len(done_rows), 2 * running)   # capacity is what the first round kept
    assert used2 <= b2 < b1
    p2 = oracle.plan(live2, nb, b2)
    assert p2.status == 0
    oracle.compact(want_pool, bb, p2)
    assert oracle.remap(want_tables, p2) == 0
    sizes2 = [((b1 - b2) * bb) // 2 // 16 * 16]
    hosts2 = weights(0xA2, sizes2)
    assert oracle.materialize(want_pool, b2 * bb, [(hosts2[0].numpy(), 16)]) == 0
    # the reserve proves too small: the boundary rises by 3 blocks; which tensors of the second model survive?
    lost, ev, new_off = oracle.grow(bb, nb, b2, b2 + 3, [(sizes2[0], 16)])

    # ---- device chain
    pool_dev = torch.from_numpy(pool0).to(gh.dev())
    pool = wk.pool_desc(pool_dev, nb, cfg.num_layers, cfg.tile_bytes)
    tables_dev = torch.from_numpy(w.tables).to(gh.dev())
    live_dev = gh.to_dev(w.live)
    s_compute, s_copy = torch.cuda.Stream(), torch.cuda.Stream()
    done = torch.cuda.Event()
    dp1 = gh.DevicePlan(nb, b1)
    torch.cuda.synchronize()
    wk.kv_plan_reclaim(live_dev, dp1.plan, s_compute.cuda_stream)
    wk.kv_compact(pool, dp1.plan, s_compute.cuda_stream)
    done.record(s_compute)
    wk.kv_remap_tables(tables_dev, *w.tables.shape, dp1.plan, s_compute.cuda_stream)
    wk.weights_materialize(pool, b1, [(h, h.numel(), o) for h, o in zip(hosts1, offs1)], s_copy.cuda_stream,
                           done.cuda_event)
    # requests finish: the engine clears their bits and rows on the device (test code, torch ops)
    with torch.cuda.stream(s_compute):
        live_words = gh.view_device(dp1.plan.live_out, 8 * ((nb + 63) // 64)).view(torch.int64)
        ids = tables_dev[done_rows].flatten()
        ids = ids[ids >= 0].to(torch.int64)
        clear = torch.zeros(nb, dtype=torch.bool, device=gh.dev())
        clear[ids] = True
        weights_of_bits = (torch.ones(64, dtype=torch.int64, device=gh.dev()) << torch.arange(64, device=gh.dev()))
        pad = torch.zeros(live_words.numel() * 64, dtype=torch.bool, device=gh.dev())
        pad[:nb] = clear
        mask = (pad.view(-1, 64).to(torch.int64) * weights_of_bits).sum(dim=1)
        live2_dev = live_words & ~mask
        tables_dev[done_rows] = -1
    dp2 = gh.DevicePlan(nb, b2)
    done2 = torch.cuda.Event()
    s_compute.wait_stream(s_copy)          # the second round reads and writes bytes the first weight stream may still touch
    wk.kv_plan_reclaim(live2_dev.data_ptr(), dp2.plan, s_compute.cuda_stream)
    wk.kv_compact(pool, dp2.plan, s_compute.cuda_stream)
    done2.record(s_compute)
    wk.kv_remap_tables(tables_dev, *w.tables.shape, dp2.plan, s_compute.cuda_stream)
    wk.weights_materialize(pool, b2, [(hosts2[0], sizes2[0], 16)], s_copy.cuda_stream, done2.cuda_event)
    torch.cuda.synchronize()
    _compare_plan(dp1, p1)
    _compare_plan(dp2, p2)
    assert np.array_equal(gh.from_dev(live2_dev, np.uint64), live2)
    assert np.array_equal(tables_dev.cpu().numpy(), want_tables)
    assert np.array_equal(pool_dev.cpu().numpy(), want_pool)
    assert int(tables_dev.max()) < b2
    got_lost, got_ev, got_off = wk.kv_grow(pool, b2, b2 + 3, [(hosts2[0], sizes2[0], 16)])
    assert (got_lost, got_ev, got_off) == (lost, ev.tolist(), new_off.tolist()) and lost == 1


def test_reclaim_step_replays_from_a_hip_graph(oracle):
    """plan -> compact -> remap needs no host synchronisation and no memset, so the three launches
    can be captured once and replayed; every replay must give the oracle's result, with eager work
    and synchronisation between replays."""
    cfg = CONFIGS[1].scaled(num_blocks=1536, num_layers=4, num_seqs=96)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    oracle.compact(want_pool, cfg.block_bytes, p)
    oracle.remap(want_tables, p)
    pool0_dev = torch.from_numpy(pool0).to(gh.dev())
    pool_dev = pool0_dev.clone()
    tables0_dev = torch.from_numpy(w.tables).to(gh.dev())
    tables_dev = tables0_dev.clone()
    live_dev = gh.to_dev(w.live)
    dp = gh.DevicePlan(cfg.num_blocks, cfg.boundary)
    pool = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s = torch.cuda.current_stream().cuda_stream
        wk.kv_plan_reclaim(live_dev, dp.plan, s)
        wk.kv_compact(pool, dp.plan, s)
        wk.kv_remap_tables(tables_dev, w.tables.shape[0], w.tables.shape[1], dp.plan, s)
    for replay in range(4):
        pool_dev.copy_(pool0_dev)                       # eager work between replays
        tables_dev.copy_(tables0_dev)
        dp.ws.fill_(0xA5)                               # poison the plan workspace again
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _compare_plan(dp, p)
        st = dp.state()
        assert st.ticket == 0 and st.finished == 0 and st.n_bad_entries == 0
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), f"replay {replay}"
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), f"replay {replay}"


def test_plain_c_client_of_the_abi(tmp_path):
    """tests/c_abi_demo.c: a C99 program (no Python, no C++) drives plan, compact, materialize and
    remap through the shared library and checks the result on the host itself."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "c_abi_demo")
    libdir = os.path.join(root, "paper_2512_09472_amd")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-O1", "-I", os.path.join(root, "include"),
                    "-I", "/opt/rocm/include", os.path.join(root, "tests", "c_abi_demo.c"), "-L", libdir, "-lwarmkv",
                    "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", f"-Wl,-rpath,{libdir}",
                    "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "c_abi_demo ok" in r.stdout, (r.returncode, r.stdout, r.stderr[-500:])


def test_randomized_reclaims_against_the_oracle(oracle):
    """Seventy seeded random pools: sizes, odd tile sizes (small ones that share tickets, large
    ones with ragged tails), layouts, occupancies, boundaries and launch shapes drawn at random,
    the block copy in one launch or in three parts; plan, tables and every pool byte compared
    with the oracle."""
    rs = np.random.default_rng(20251209)
    for case in range(70):
        big_tile = case % 3 == 2
        nb = int(rs.integers(1, 300 if big_tile else 3000))
        b = int(rs.integers(0, nb + 1))
        layers = int(rs.integers(1, 7))
        tile = 16 * int(rs.integers(600, 12000) if big_tile else rs.integers(1, 600))
        layer_major = bool(rs.integers(0, 2))
        pad = 256 * int(rs.integers(0, 4)) if layer_major else 0
        stride = -(-(nb * tile) // 256) * 256 + pad if layer_major else 0
        live_bits = rs.random(nb) < rs.uniform(0.05, 0.6)
        ids = np.flatnonzero(live_bits)
        live = bitmap_from_ids(ids, nb)
        p = oracle.plan(live, nb, b)
        pool_bytes = layers * stride if layer_major else nb * layers * tile
        pool0 = rs.integers(0, 256, pool_bytes, dtype=np.uint8)
        rows = int(rs.integers(1, 20))
        cols = int(rs.integers(1, 40))
        tables = (rs.choice(np.concatenate([ids, [-1]]), size=(rows, cols)) if ids.size else
                  np.full((rows, cols), -1)).astype(np.int32)
        want_pool, want_tables = pool0.copy(), tables.copy()
        if layer_major:
            oracle.compact_layer_major(want_pool, tile, layers, stride, p)
        else:
            oracle.compact(want_pool, layers * tile, p)
        bad = oracle.remap(want_tables, p)
        tuning = dict(workgroups=int(rs.choice([0, 1, 3, 64, 256, 1000])), chunk_bytes=4096 * int(rs.integers(1, 40)),
                      flags=(int(rs.choice([2, 4, 8, 16, 32])) << 4) | int(rs.integers(0, 16)))
        parts = None
        if case % 2 == 1:                      # default launch shape, block copy in three parts
            cut = sorted(int(x) for x in rs.integers(0, max(1, p.n_moves) + 2, size=2))
            parts = [(0, cut[0]), (cut[0], cut[1] - cut[0]), (cut[1], 1 << 31)]
            tuning = None
        _say(f"[random {case}] NB={nb} b={b} L={layers} tile={tile} layer_major={layer_major} stride={stride} "
             f"status={p.status} n={p.n_moves} tuning={tuning} parts={parts}")
        pool_dev = torch.from_numpy(pool0).to(gh.dev())
        pool = wk.pool_desc(pool_dev, nb, layers, tile, stride)
        dp = gh.DevicePlan(nb, b)
        tables_dev = torch.from_numpy(tables).to(gh.dev())
        live_dev = gh.to_dev(live)
        wk.kv_plan_reclaim(live_dev, dp.plan)
        if parts is None:
            wk.kv_compact_launch(pool, dp.plan, **tuning)
        else:
            for first, count in parts:
                wk.kv_compact_moves(pool, dp.plan, first, count)
        wk.kv_remap_tables(tables_dev, rows, cols, dp.plan)
        torch.cuda.synchronize()
        st = _compare_plan(dp, p)
        assert st.n_bad_entries == bad and st.ticket == 0 and st.finished == 0
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), case
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), case
        # the same pool through kv_reclaim (a single launch at these sizes) and through kv_reclaim_static
        for entry in ("kv_reclaim", "kv_reclaim_static"):
            pool_dev.copy_(torch.from_numpy(pool0))
            tables_dev.copy_(torch.from_numpy(tables))
            if entry == "kv_reclaim":
                dp.ws.fill_(0x3C)
                torch.cuda.synchronize()
                wk.kv_reclaim(pool, dp.plan, live_dev, tables_dev, rows, cols)
                torch.cuda.synchronize()
                st = _compare_plan(dp, p)
            else:
                live_out = torch.full((max(1, live.size) * 8,), 0x77, dtype=torch.uint8, device=gh.dev())
                state = torch.zeros(32, dtype=torch.uint8, device=gh.dev())
                wk.kv_reclaim_static(pool, b, live_dev, live_out, tables_dev, rows, cols, state)
                torch.cuda.synchronize()
                st = wk.binding.kv_plan_state.from_buffer_copy(state.cpu().numpy().tobytes())
                assert st.status == p.status and st.n_moves == p.n_moves
                if p.status == 0:
                    assert np.array_equal(gh.from_dev(live_out, np.uint64)[:live.size], p.live_out), (case, entry)
            assert st.n_bad_entries == (bad if p.status == 0 else 0) and st.ticket == 0 and st.finished == 0, (case, entry)
            assert np.array_equal(tables_dev.cpu().numpy(), want_tables), (case, entry)
            assert np.array_equal(pool_dev.cpu().numpy(), want_pool), (case, entry)
