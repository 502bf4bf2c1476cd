"""Host-side checks of the seeded input generators (no GPU)."""
import numpy as np
import pytest

from synth import CONFIGS, bitmap_to_bools, dense_offsets, make_workload, weight_shapes_8b
from synth.content import item_bytes_host, normal_bf16_table
from synth.rng import SplitMix64, mix64, mix64_int


def test_splitmix64_published_vector():
    # First outputs for seed 1234567, as listed with the generator's public reference code.
    r = SplitMix64(1234567)
    assert [r.next_u64() for _ in range(5)] == [6457827717110365317, 3203168211198807973,
                                                9817491932198370423, 4593380528125082431,
                                                16408922859458223821]


def test_vector_mix_matches_scalar():
    xs = [0, 1, 2**63, 2**64 - 1, 0x123456789ABCDEF]
    got = mix64(np.array(xs, dtype=np.uint64))
    assert [int(g) for g in got] == [mix64_int(x) for x in xs]


def test_shuffle_is_permutation():
    p = SplitMix64(3).shuffle(1000)
    assert sorted(p) == list(range(1000)) and p != list(range(1000))


def test_config_geometry():
    c1, c2, c3, c4, c5 = CONFIGS
    assert (c1.tile_bytes, c1.block_bytes, c1.num_blocks, c1.boundary) == (65536, 65536, 1024, 512)
    assert (c2.block_bytes, c2.num_blocks, c2.boundary, c2.pool_bytes) == (2 << 20, 20480, 12288, 40 << 30)
    assert (c3.block_bytes, c3.num_blocks, c3.boundary) == (c2.block_bytes, c2.num_blocks, c2.boundary)
    assert (c4.block_bytes, c4.num_blocks, c4.boundary) == (5 << 20, 24576, 18841)
    assert (c5.tile_bytes, c5.block_bytes, c5.num_blocks, c5.boundary) == (32768, 1 << 20, 65536, 32768)
    assert [c.max_blocks_per_seq for c in CONFIGS] == [128, 2048, 2048, 1024, 16]
    assert [c.live_budget for c in CONFIGS] == [480, 11648, 11648, 14746, 30720]


@pytest.mark.parametrize("idx", range(5))
def test_workload_is_consistent_and_feasible(idx):
    cfg = CONFIGS[idx]
    w = make_workload(cfg)
    live = bitmap_to_bools(w.live, cfg.num_blocks)
    ids = w.tables[w.tables >= 0]
    assert ids.size == w.live_count == int(live.sum()) <= cfg.live_budget
    assert np.unique(ids).size == ids.size, "a block belongs to one sequence"
    assert live[ids].all()
    assert w.live_count >= cfg.live_budget - cfg.max_blocks_per_seq
    # rows are left-packed
    counts = (w.tables >= 0).sum(axis=1)
    assert np.array_equal(counts, w.seq_blocks)
    for s in range(0, cfg.num_seqs, max(1, cfg.num_seqs // 50)):
        assert (w.tables[s, :counts[s]] >= 0).all() and (w.tables[s, counts[s]:] == -1).all()
    movers = int(live[cfg.boundary:].sum())
    free_below = int((~live[:cfg.boundary]).sum())
    assert 0 < movers <= free_below
    # scatter: movers within 15 % of the uniform expectation
    expect = w.live_count * (cfg.num_blocks - cfg.boundary) / cfg.num_blocks
    assert abs(movers - expect) < 0.15 * expect
    # same seed, same workload
    w2 = make_workload(cfg)
    assert np.array_equal(w.live, w2.live) and np.array_equal(w.tables, w2.tables)


def test_literal_occupancy_variant_is_infeasible():
    cfg = CONFIGS[1].scaled(live_budget_override=int(0.7 * CONFIGS[1].num_blocks))
    w = make_workload(cfg)
    assert w.live_count > cfg.boundary


def test_scaled_config_keeps_boundary_fraction():
    c = CONFIGS[3].scaled(num_blocks=1000, num_layers=2)
    assert c.boundary == 18841 * 1000 // 24576 and c.block_bytes == 2 * 65536


def test_weight_set_size():
    shapes = weight_shapes_8b()
    sizes = [2 * a * b for _, (a, b) in shapes]
    assert len(shapes) == 225 and sum(sizes) == 15_009_316_864
    offs = dense_offsets(sizes)
    assert offs[0] == 0 and offs[-1] + sizes[-1] == sum(sizes), "every size is a multiple of 256 B"
    assert sum(sizes) <= 16 << 30


def test_normal_table_and_content():
    t = normal_bf16_table(1.0)
    assert t.shape == (65536,) and t.dtype == np.uint16
    f = (t.astype(np.uint32) << 16).view(np.float32)
    assert abs(float(f.mean())) < 1e-3 and abs(float(f.std()) - 1.0) < 5e-3
    assert np.all(np.diff(f) >= 0)
    a = item_bytes_host(5, 3, 4096, t)
    assert np.array_equal(a[1024:2048], item_bytes_host(5, 3, 1024, t, byte_offset=1024))
    assert not np.array_equal(a, item_bytes_host(5, 4, 4096, t))
    assert not np.array_equal(a, item_bytes_host(6, 3, 4096, t))
    raw = item_bytes_host(5, 3, 4096, None)
    assert abs(float(raw.mean()) - 127.5) < 8


def test_bench_threaded_host_copy_equals_the_oracle(oracle):
    """The bench-only all-cores host copy does the same moves as the oracle's block copy."""
    import ctypes
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    so = os.path.join(root, "bench_hostcopy.so")
    subprocess.run(["g++", "-O2", "-std=c++17", "-pthread", "-fPIC", "-shared",
                    os.path.join(root, "bench_hostcopy.cpp"), "-o", so], check=True)
    lib = ctypes.CDLL(so)
    lib.hostcopy_moves.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_uint32, ctypes.c_uint32]
    lib.hostcopy_moves.restype = None
    cfg = CONFIGS[4].scaled(num_blocks=512, num_layers=1, block_size=1, kv_heads=1, head_dim=64, len_hi=16, num_seqs=128)
    w = make_workload(cfg)
    p = oracle.plan(w.live, cfg.num_blocks, cfg.boundary)
    pool = np.random.default_rng(0).integers(0, 256, cfg.pool_bytes, dtype=np.uint8)
    want = pool.copy()
    oracle.compact(want, cfg.block_bytes, p)
    for threads in (1, 3, 8, 1000):
        got = pool.copy()
        src, dst = np.ascontiguousarray(p.src), np.ascontiguousarray(p.dst)
        lib.hostcopy_moves(got.ctypes.data, cfg.block_bytes, src.ctypes.data, dst.ctypes.data, p.n_moves, threads)
        assert np.array_equal(got, want), threads
