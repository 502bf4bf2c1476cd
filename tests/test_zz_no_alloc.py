"""kv_reclaim_static (the entry point that allocates nothing) against the three existing calls it
stands for, and both against the oracle: two calls in a row on one GPU, the second on a smaller
pool, so that whatever the first left in the library's static workspace is there to be misread."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import gpu_harness as gh                      # noqa: E402
import paper_2512_09472_amd as wk             # noqa: E402
from synth import CONFIGS, make_workload      # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    wk.binding.load()


def _both_ways(cfg, oracle, stream):
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    n_words = (cfg.num_blocks + 63) // 64
    # the existing entry points, workspace from the caller
    pool_a = torch.from_numpy(pool0).to(gh.dev())
    dp, tables_a = gh.run_reclaim(cfg, w.live, w.tables, pool_a, stream=stream)
    st_a, src, dst, new_id, live_out_a = dp.results()
    # the static one: every buffer below exists before the call
    pool_b = torch.from_numpy(pool0).to(gh.dev())
    tables_b = torch.from_numpy(w.tables).to(gh.dev())
    live_in = gh.to_dev(w.live)
    live_out_b = torch.full((n_words * 8,), 0xEE, dtype=torch.uint8, device=gh.dev())
    state_b = torch.full((32,), 0xEE, dtype=torch.uint8, device=gh.dev())
    desc = wk.pool_desc(pool_b, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    wk.kv_reclaim_static(desc, cfg.boundary, live_in, live_out_b, tables_b, w.tables.shape[0], w.tables.shape[1],
                         state_b, stream.cuda_stream)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    st_b = wk.binding.kv_plan_state.from_buffer_copy(state_b.cpu().numpy().tobytes())
    assert (st_b.status, st_b.n_moves, st_b.n_free_below, st_b.n_bad_entries, st_b.ticket, st_b.finished, st_b.bad_plan) == \
           (st_a.status, st_a.n_moves, st_a.n_free_below, st_a.n_bad_entries, 0, 0, 0)
    assert np.array_equal(gh.from_dev(live_out_b, np.uint64), live_out_a), "bitmap after the move"
    assert torch.equal(tables_b, tables_a), "tables"
    assert torch.equal(pool_b, pool_a), "pool"
    # and the oracle
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    oracle.compact(want_pool, cfg.block_bytes, p)
    assert oracle.remap(want_tables, p) == 0
    assert st_b.status == p.status and st_b.n_moves == p.n_moves and p.n_moves > 0
    assert np.array_equal(gh.from_dev(live_out_b, np.uint64), p.live_out)
    assert np.array_equal(tables_b.cpu().numpy(), want_tables)
    assert np.array_equal(pool_b.cpu().numpy(), want_pool)
    return p.n_moves


def test_static_reclaim_matches_the_three_calls_twice_in_a_row(oracle):
    stream = torch.cuda.Stream()
    big = CONFIGS[1].scaled(num_blocks=900, num_layers=5, kv_heads=3, head_dim=40, num_seqs=40)   # ragged tiles
    small = CONFIGS[0].scaled(num_blocks=200, num_seqs=12)
    n_big = _both_ways(big, oracle, stream)
    n_small = _both_ways(small, oracle, stream)
    assert n_small < n_big
    # an infeasible request: verdict reported, nothing moved or rewritten
    cfg = CONFIGS[0].scaled(num_blocks=128, boundary=20, num_seqs=8, live_budget_override=60)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    pool_d, tables_d = torch.from_numpy(pool0).to(gh.dev()), torch.from_numpy(w.tables).to(gh.dev())
    live_out = torch.zeros(16, dtype=torch.uint8, device=gh.dev())
    state = torch.zeros(32, dtype=torch.uint8, device=gh.dev())
    wk.kv_reclaim_static(wk.pool_desc(pool_d, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes), cfg.boundary,
                         gh.to_dev(w.live), live_out, tables_d, *w.tables.shape, state, stream.cuda_stream)
    torch.cuda.synchronize()
    st = wk.binding.kv_plan_state.from_buffer_copy(state.cpu().numpy().tobytes())
    assert st.status == wk.KV_E_NOSPACE and st.n_moves == 0
    assert oracle.plan(w.live, cfg.num_blocks, cfg.boundary).status == oracle.E_NOSPACE
    assert np.array_equal(pool_d.cpu().numpy(), pool0) and np.array_equal(tables_d.cpu().numpy(), w.tables)


def test_static_reclaim_replays_from_a_hip_graph(oracle):
    """The callers this entry point is for: captured once (after one eager call, which also looks up
    the workspace's address on this device), replayed with eager work and synchronisation between
    replays; every replay must give the oracle's result."""
    cfg = CONFIGS[1].scaled(num_blocks=1200, num_layers=3, num_seqs=64)
    w = make_workload(cfg)
    pool0 = gh.host_pool(cfg, gh.content_table(cfg))
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    want_pool, want_tables = pool0.copy(), w.tables.copy()
    oracle.compact(want_pool, cfg.block_bytes, p)
    assert oracle.remap(want_tables, p) == 0
    pool0_dev = torch.from_numpy(pool0).to(gh.dev())
    pool_dev = pool0_dev.clone()
    tables0_dev = torch.from_numpy(w.tables).to(gh.dev())
    tables_dev = tables0_dev.clone()
    live_in = gh.to_dev(w.live)
    live_out = torch.zeros(((cfg.num_blocks + 63) // 64) * 8, dtype=torch.uint8, device=gh.dev())
    state = torch.zeros(32, dtype=torch.uint8, device=gh.dev())
    desc = wk.pool_desc(pool_dev, cfg.num_blocks, cfg.num_layers, cfg.tile_bytes)
    args = (desc, cfg.boundary, live_in, live_out, tables_dev, w.tables.shape[0], w.tables.shape[1], state)
    side = torch.cuda.Stream()
    wk.kv_reclaim_static(*args, side.cuda_stream)          # eager first call, outside any capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wk.kv_reclaim_static(*args, torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        pool_dev.copy_(pool0_dev)                            # eager work between replays
        tables_dev.copy_(tables0_dev)
        live_out.fill_(0xEE)
        state.fill_(0xEE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        st = wk.binding.kv_plan_state.from_buffer_copy(state.cpu().numpy().tobytes())
        assert (st.status, st.n_moves, st.ticket, st.finished, st.n_bad_entries) == (0, p.n_moves, 0, 0, 0)
        assert np.array_equal(gh.from_dev(live_out, np.uint64), p.live_out), f"replay {replay}"
        assert np.array_equal(tables_dev.cpu().numpy(), want_tables), f"replay {replay}"
        assert np.array_equal(pool_dev.cpu().numpy(), want_pool), f"replay {replay}"


def test_static_reclaim_refuses_what_does_not_fit():
    fake = 0x7F0000000000
    too_big = wk.pool_desc(fake, wk.KV_STATIC_MAX_BLOCKS + 1, 1, 4096)
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_reclaim_static(too_big, 10, fake, fake + (1 << 30), fake + (2 << 30), 1, 4, fake + (3 << 30))
    assert e.value.code == wk.KV_E_TOOBIG
    ok = wk.pool_desc(fake, 1024, 1, 4096)
    for args, code in (((ok, 2000, fake, fake, fake, 1, 4, fake), wk.KV_E_RANGE),
                       ((ok, 10, fake, 0, fake, 1, 4, fake), wk.KV_E_NULL),
                       ((ok, 10, fake, fake, fake + 4, 1, 4, fake), wk.KV_E_ALIGN)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_reclaim_static(*args)
        assert e.value.code == code
