"""Host-only checks of the C ABI: the library loads, exports what the header
declares, and rejects bad arguments before touching the device.  No GPU needed:
every call here returns before its first HIP call."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

import paper_2512_09472_amd as wk
from paper_2512_09472_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000   # an aligned address that is never dereferenced


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "warmkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{}]*\)\s*;", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS), names
    lib = binding.load()
    for n in names:
        assert hasattr(lib, n), n
    assert wk.warmkv_version() == "0.2"


def test_loaded_library_was_built_from_the_sources_in_the_tree():
    from paper_2512_09472_amd import build
    binding.load()
    assert binding.warmkv_build_id() == build.source_id() == binding._built_id(build.LIB_PATH)


def test_a_changed_source_is_seen_and_a_stale_library_refused(tmp_path, monkeypatch):
    """The identifier follows the text of every source and header; a library whose identifier
    differs is rebuilt, or refused where rebuilding is switched off - never loaded as it is."""
    import shutil
    from paper_2512_09472_amd import build
    before = build.source_id()
    csrc, inc = tmp_path / "csrc", tmp_path / "include"
    shutil.copytree(build.CSRC, csrc)
    shutil.copytree(build.INCLUDE, inc)
    monkeypatch.setattr(build, "CSRC", str(csrc))
    monkeypatch.setattr(build, "INCLUDE", str(inc))
    assert build.source_id() == before                       # same text, same identifier, wherever it lies
    for touched in (csrc / "compact.hip", csrc / "common.h", inc / "warmkv.h"):
        old = touched.read_bytes()
        touched.write_bytes(old + b"\n// touched\n")
        assert build.source_id() != before, touched
        touched.write_bytes(old)
    assert build.source_id() == before
    (csrc / "remap.hip").write_bytes((csrc / "remap.hip").read_bytes() + b"\n")
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setenv("WARMKV_NO_REBUILD", "1")
    with pytest.raises(binding.StaleLibraryError):
        binding.load()
    monkeypatch.delenv("WARMKV_NO_REBUILD")
    calls = []
    monkeypatch.setattr(build, "build", lambda verbose=False: calls.append(1))   # a build that changes nothing
    with pytest.raises(binding.StaleLibraryError):
        binding.load()
    assert calls == [1]                                      # it did try to rebuild first


def test_struct_sizes_match_the_header():
    assert ctypes.sizeof(binding.kv_pool_desc) == 32
    assert ctypes.sizeof(binding.kv_plan_state) == 32
    assert ctypes.sizeof(binding.kv_plan) == 56
    assert ctypes.sizeof(binding.kv_compact_tuning) == 16
    assert ctypes.sizeof(binding.wm_tensor) == 24
    assert ctypes.sizeof(binding.wm_piece) == 32
    assert ctypes.sizeof(binding.kv_switch_request) == 112


def test_workspace_and_bind():
    nb, b = 20480, 12288
    need = wk.kv_plan_workspace_bytes(nb, b)
    cap = min(nb - b, b)
    assert need >= 16 + nb // 8 + 8 * cap + 4 * nb and need % 256 == 0
    assert wk.kv_plan_workspace_bytes(10, 11) == 0
    assert wk.kv_plan_workspace_bytes((1 << 24) + 1, 0) == 0
    p = wk.kv_plan_bind(FAKE, need, nb, b)
    assert (p.num_blocks, p.boundary, p.capacity) == (nb, b, cap)
    segs = sorted([(p.state, 16), (p.live_out, nb // 8), (p.src, 4 * cap), (p.dst, 4 * cap), (p.new_id, 4 * nb)])
    for (a, n), (a2, _) in zip(segs, segs[1:]):
        assert a + n <= a2 and a % 256 == 0
    assert segs[0][0] == FAKE and segs[-1][0] + segs[-1][1] <= FAKE + need
    for args, code in (((FAKE, need - 1, nb, b), wk.KV_E_TOOBIG), ((FAKE + 8, need, nb, b), wk.KV_E_ALIGN),
                       ((0, need, nb, b), wk.KV_E_NULL), ((FAKE, need, nb, nb + 1), wk.KV_E_RANGE)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_plan_bind(*args)
        assert e.value.code == code


def test_calls_reject_bad_arguments_before_any_launch():
    nb, b = 1024, 512
    plan = wk.kv_plan_bind(FAKE, wk.kv_plan_workspace_bytes(nb, b), nb, b)
    pool = wk.pool_desc(FAKE + (1 << 30), nb, 1, 65536)

    def code(fn, *a, **k):
        with pytest.raises(wk.WarmKVError) as e:
            fn(*a, **k)
        return e.value.code

    assert code(wk.kv_plan_reclaim, 0, plan) == wk.KV_E_NULL
    assert code(wk.kv_plan_reclaim, plan.live_out, plan) == wk.KV_E_OVERLAP
    assert code(wk.kv_plan_reclaim, plan.live_out + 8, plan) == wk.KV_E_OVERLAP
    bad = wk.kv_plan_bind(FAKE, wk.kv_plan_workspace_bytes(nb, b), nb, b)
    bad.boundary = nb + 1
    assert code(wk.kv_plan_reclaim, FAKE + (1 << 20), bad) == wk.KV_E_RANGE
    assert code(wk.kv_compact, pool, bad) == wk.KV_E_RANGE
    assert code(wk.kv_remap_tables, FAKE + (1 << 20), 4, 4, bad) == wk.KV_E_RANGE
    assert code(wk.kv_compact, wk.pool_desc(FAKE, nb + 1, 1, 65536), plan) == wk.KV_E_RANGE
    assert code(wk.kv_compact, wk.pool_desc(FAKE, nb, 1, 65528), plan) == wk.KV_E_ALIGN
    assert code(wk.kv_compact, wk.pool_desc(FAKE + 16, nb, 1, 65536), plan) == wk.KV_E_ALIGN
    assert code(wk.kv_compact, wk.pool_desc(0, nb, 1, 65536), plan) == wk.KV_E_NULL
    assert code(wk.kv_compact, wk.pool_desc(FAKE, nb, 0, 65536), plan) == wk.KV_E_RANGE
    assert code(wk.kv_compact_launch, pool, plan, chunk_bytes=1000) == wk.KV_E_RANGE
    assert code(wk.kv_compact_launch, pool, plan, flags=3 << 4) == wk.KV_E_RANGE
    assert code(wk.kv_remap_tables, 0, 4, 4, plan) == wk.KV_E_NULL
    assert code(wk.kv_remap_tables, FAKE + 4, 4, 4, plan) == wk.KV_E_ALIGN
    wk.kv_remap_tables(0, 0, 128, plan)          # no entries: nothing to do, no launch


def test_materialize_validates_every_extent_first():
    nb, b, tile = 64, 40, 4096
    pool = wk.pool_desc(FAKE, nb, 2, tile)
    region = (nb - b) * 2 * tile

    def code(tensors, boundary=b):
        with pytest.raises(wk.WarmKVError) as e:
            wk.weights_materialize(pool, boundary, tensors)
        return e.value.code

    assert code([(FAKE, 16, 0), (FAKE, region, 1)]) == wk.KV_E_TOOBIG
    assert code([(FAKE, 16, region - 15)]) == wk.KV_E_TOOBIG
    assert code([(FAKE, 16, region + 1)]) == wk.KV_E_TOOBIG
    assert code([(FAKE, 32, 0), (FAKE, 32, 64), (FAKE, 1, 95)]) == wk.KV_E_OVERLAP
    assert code([(FAKE, 32, 64), (FAKE, 65, 0)]) == wk.KV_E_OVERLAP
    assert code([(0, 32, 0)]) == wk.KV_E_NULL
    assert code([(FAKE, 32, 0)], boundary=nb + 1) == wk.KV_E_RANGE
    wk.weights_materialize(pool, b, [])                       # nothing to copy
    wk.weights_materialize(pool, b, [(0, 0, 5), (0, 0, 5)])   # empty extents never overlap


def test_materialize_schedule_partitions_tensors_and_respects_readiness():
    """Early pieces touch only blocks that were free before the move; together with the late
    pieces they cover every tensor byte exactly once, in order."""
    import numpy as np
    from synth import bitmap_from_ids
    nb, b, layers, tile = 96, 40, 2, 512
    bb = layers * tile
    rs = np.random.default_rng(2)
    live_bits = rs.random(nb) < 0.5
    live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
    pool = wk.pool_desc(FAKE, nb, layers, tile)
    region = (nb - b) * bb
    tensors = [(FAKE, 3000, 0), (FAKE, 5 * bb + 17, 3000), (FAKE, 0, 9000), (FAKE, bb, 20 * bb),
               (FAKE, 7, 30 * bb + 5), (FAKE, 10 * bb - 100, region - 10 * bb + 100)]
    for budget in (1, 2 * bb, 6 * bb + 1, 0):
        pieces = wk.weights_materialize_schedule(pool, b, live, tensors, early_bytes=budget)
        flags = [e for _, e, _, _, _ in pieces]
        assert flags == sorted(flags, reverse=True), "early pieces come first"
        early_total = 0
        for i, (_, nbytes, off) in enumerate(tensors):
            mine = sorted((p for p in pieces if p[0] == i), key=lambda p: p[2])
            pos = 0
            for _, early, so, do, n in mine:
                assert so == pos and do == off + so and n > 0
                pos += n
                blocks = range(b + do // bb, b + (do + n - 1) // bb + 1)
                if early:
                    assert not any(live_bits[j] for j in blocks)
                    early_total += n
            assert pos == nbytes
        limit = budget if budget else 128 << 20
        assert early_total < limit + bb
        if budget == 1:
            assert sum(flags) == 1
    # with nothing live above the boundary everything up to the budget is early
    none_live = bitmap_from_ids(np.flatnonzero(live_bits[:b]), nb)
    pieces = wk.weights_materialize_schedule(pool, b, none_live, tensors, early_bytes=1 << 40)
    assert all(e == 1 for _, e, _, _, _ in pieces) and len(pieces) == 5
    with pytest.raises(wk.WarmKVError) as e:
        wk.weights_materialize_schedule(pool, b, 0, tensors)
    assert e.value.code == wk.KV_E_NULL
    with pytest.raises(wk.WarmKVError) as e:
        wk.weights_materialize_pipelined(pool, b, live, [(FAKE, 16, 0), (FAKE, 16, 8)])
    assert e.value.code == wk.KV_E_OVERLAP


def test_materialize_schedule_in_a_layer_major_pool():
    """The unit of readiness is a block's tile in one strip: an early piece touches only tiles of
    blocks that were free before the move, whichever strip it lies in."""
    import numpy as np
    from synth import bitmap_from_ids
    nb, b, layers, tile = 80, 30, 3, 256
    strip = (nb - b) * tile
    rs = np.random.default_rng(5)
    live_bits = rs.random(nb) < 0.5
    live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
    pool = wk.pool_desc(FAKE, nb, layers, tile, nb * tile + 512)
    tensors = [(FAKE, 5 * tile + 9, 100), (FAKE, strip - 7 * tile, strip + 7 * tile), (FAKE, 0, 2 * strip),
               (FAKE, 3 * tile, 2 * strip + 11), (FAKE, tile // 2, 2 * strip + 20 * tile + 3)]
    for budget in (1, 9 * tile, 1 << 40):
        pieces = wk.weights_materialize_schedule(pool, b, live, tensors, early_bytes=budget)
        early_total = 0
        for i, (_, nbytes, off) in enumerate(tensors):
            mine = sorted((p for p in pieces if p[0] == i), key=lambda p: p[2])
            pos = 0
            for _, early, so, do, n in mine:
                assert so == pos and do == off + so and n > 0
                pos += n
                assert do // strip == (do + n - 1) // strip, "a piece stays inside its strip"
                first, last = (do % strip) // tile, ((do + n - 1) % strip) // tile
                if early:
                    assert not live_bits[b + first:b + last + 1].any()
                    early_total += n
                elif budget == 1 << 40:
                    assert live_bits[b + first:b + last + 1].all(), "with no budget limit only live tiles wait"
            assert pos == nbytes
        assert early_total < budget + tile
    with pytest.raises(wk.WarmKVError) as e:      # a tensor across two strips is not contiguous in memory
        wk.weights_materialize_schedule(pool, b, live, [(FAKE, 2, strip - 1)])
    assert e.value.code == wk.KV_E_TOOBIG


def test_default_schedule_sends_no_early_piece_that_costs_more_than_it_hides():
    """With the library's own policy (early_bytes = 0) a free run below 2 MiB stays late; an explicit
    budget takes every free run."""
    import numpy as np
    from synth import bitmap_from_ids
    nb, b = 4096, 2048
    rs = np.random.default_rng(9)
    live_bits = rs.random(nb) < 0.5
    live = bitmap_from_ids(np.flatnonzero(live_bits), nb)
    for layers, tile, stride in ((1, 2 << 20, 0), (4, 65536, nb * 65536), (1, 65536, 0)):
        pool = wk.pool_desc(FAKE, nb, layers, tile, stride)
        strip = (nb - b) * tile * (1 if stride else layers)
        tensors = [(FAKE, strip - 4096, 4096)] + ([(FAKE, strip // 2, strip + 65536)] if stride else [])
        default = wk.weights_materialize_schedule(pool, b, live, tensors)
        explicit = wk.weights_materialize_schedule(pool, b, live, tensors, early_bytes=128 << 20)
        for pieces in (default, explicit):                   # both partition every tensor in order
            for i, (_, nbytes, off) in enumerate(tensors):
                pos = 0
                for _, _, so, do, n in sorted((p for p in pieces if p[0] == i), key=lambda p: p[2]):
                    assert so == pos and do == off + so and n > 0
                    pos += n
                assert pos == nbytes
        assert all(n >= 2 << 20 for _, early, _, _, n in default if early)
        if tile >= 2 << 20:
            assert any(early for _, early, _, _, _ in default)
        else:
            assert sum(1 for p in default if p[1]) < sum(1 for p in explicit if p[1])
            assert any(n < 2 << 20 for _, early, _, _, n in explicit if early)
            lates = [p for p in default if not p[1]]
            assert len(lates) <= len(tensors) + 2 * sum(1 for p in default if p[1])   # late runs are merged again


def test_grow_in_a_layer_major_pool_matches_oracle(oracle):
    import numpy as np
    nb, layers, tile = 50, 4, 128
    pool = wk.pool_desc(FAKE, nb, layers, tile, nb * tile + 256)
    rs = np.random.default_rng(21)
    for _ in range(400):
        old = int(rs.integers(0, nb))
        new = int(rs.integers(old, nb + 1))
        strip = (nb - old) * tile
        ext = []
        for _ in range(int(rs.integers(0, 8))):
            layer, within = int(rs.integers(0, layers)), int(rs.integers(0, strip))
            ext.append((int(rs.integers(0, strip - within + 1)), layer * strip + within))
        if rs.random() < 0.2:
            ext.append((0, layers * strip))                    # an empty extent at the very end
        n, ev, no = wk.kv_grow(pool, old, new, [(FAKE, b, o) for b, o in ext])
        on, oev, ono = oracle.grow_strips(tile, layers, nb, nb * tile + 256, old, new, ext)
        assert n == on and ev == oev.tolist() and no == ono.tolist(), (old, new, ext)
    for ext, code in (([(2, (nb - 10) * tile - 1)], wk.KV_E_TOOBIG), ([(1, layers * (nb - 10) * tile)], wk.KV_E_TOOBIG)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_grow(pool, 10, 20, [(FAKE, b, o) for b, o in ext])
        assert e.value.code == code
        assert oracle.grow_strips(tile, layers, nb, nb * tile + 256, 10, 20, ext)[0] == oracle.E_TOOBIG


def test_reserve_blocks_matches_eq4_fixtures():
    with open(os.path.join(ROOT, "tests", "golden", "eq4_reserve.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        assert wk.kv_reserve_blocks(c["C"], c["T"], c["Q"], c["B"]) == c["R"], c["note"]
    for args in ((10, 11, 1, 32), (10, 1, 1, 0), (1 << 33, 1, 1, 2)):
        with pytest.raises(wk.WarmKVError):
            wk.kv_reserve_blocks(*args)


def test_reserve_blocks_matches_oracle(oracle):
    from synth.rng import SplitMix64
    rng = SplitMix64(99)
    for _ in range(3000):
        C = rng.randint(1, 1 << 22)
        T = rng.randint(0, C)
        B = rng.randint(1, 512)
        Q = rng.randint(0, B + 3)
        assert wk.kv_reserve_blocks(C, T, Q, B) == oracle.reserve_blocks(C, T, Q, B)


def test_grow_matches_oracle_and_hand_cases(oracle):
    """Reverse switch: which tensors are lost when blocks [old, new) go back to the KV cache."""
    import numpy as np
    nb, layers, tile = 100, 2, 512
    bb = layers * tile
    pool = wk.pool_desc(FAKE, nb, layers, tile)
    # hand cases, old boundary 60 (region 40 blocks), 5 blocks returned
    ext = [(bb, 0), (bb, 4 * bb), (1, 5 * bb - 1), (1, 5 * bb), (3 * bb, 10 * bb), (0, 2 * bb), (bb, 39 * bb)]
    n, ev, no = wk.kv_grow(pool, 60, 65, [(FAKE, b, o) for b, o in ext])
    assert (n, ev) == (3, [1, 1, 1, 0, 0, 0, 0])
    assert no[3:] == [0, 5 * bb, 0, 34 * bb]
    assert wk.kv_grow(pool, 60, 60, [(FAKE, b, o) for b, o in ext])[0] == 0
    assert wk.kv_grow(pool, 60, 100, [(FAKE, b, o) for b, o in ext])[0] == 6
    for args, code in (((60, 59), wk.KV_E_RANGE), ((60, 101), wk.KV_E_RANGE)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_grow(pool, *args, [(FAKE, 1, 0)])
        assert e.value.code == code
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_grow(pool, 60, 70, [(FAKE, 2, 40 * bb - 1)])
    assert e.value.code == wk.KV_E_TOOBIG
    # random cases against the oracle and against a per-byte brute force
    rs = np.random.default_rng(12)
    for _ in range(300):
        old = int(rs.integers(0, nb + 1))
        new = int(rs.integers(old, nb + 1))
        region = (nb - old) * bb
        ext = []
        for _ in range(int(rs.integers(0, 8))):
            off = int(rs.integers(0, region + 1))
            ext.append((int(rs.integers(0, region - off + 1)), off))
        n, ev, no = wk.kv_grow(pool, old, new, [(FAKE, b, o) for b, o in ext])
        on, oev, ono = oracle.grow(bb, nb, old, new, ext)
        assert n == on and ev == oev.tolist()
        for i, (b, o) in enumerate(ext):
            first_byte_returned = old * bb + o < new * bb     # extents only extend upwards from o
            assert bool(ev[i]) == (b > 0 and first_byte_returned)
            if not ev[i] and b > 0:
                assert no[i] == ono[i] == old * bb + o - new * bb


def test_product_path_never_touches_the_oracle():
    """The package and the HIP sources must not import, include or load anything of the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2512_09472_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in ("warmkv.h",):
        assert "oracle" not in open(os.path.join(ROOT, "include", f)).read().lower()
    src = open(os.path.join(ROOT, "oracle", "warmkv_oracle.cpp")).read() + open(os.path.join(ROOT, "oracle", "__init__.py")).read()
    assert "warmkv.h" not in src and "paper_2512_09472_amd" not in src and "import synth" not in src


def test_header_is_valid_c99_and_cxx():
    import subprocess
    h = os.path.join(ROOT, "include", "warmkv.h")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", h], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++", h], check=True)


def test_switch_rejects_bad_requests_before_touching_the_device():
    """Every argument error of the one-call hand-over is found on the host, before the planner
    is launched (no GPU here: a launch would fail differently)."""
    nb, b, tile = 64, 40, 4096
    need = wk.kv_plan_workspace_bytes(nb, b)
    plan = wk.kv_plan_bind(FAKE, need, nb, b)
    pool = wk.pool_desc(FAKE + (1 << 20), nb, 2, tile)
    region = (nb - b) * 2 * tile
    ok = dict(pool=pool, plan=plan, live_in=FAKE + 512, tables=FAKE + 1024, num_seqs=4, max_blocks_per_seq=8,
              tensors=[(FAKE, 4096, 0)], compute_stream=0, copy_stream=0, compaction_done=FAKE)
    cases = [
        (dict(compaction_done=None), wk.KV_E_NULL),
        (dict(pool=wk.pool_desc(FAKE + (1 << 20), nb + 1, 2, tile)), wk.KV_E_RANGE),
        (dict(pool=wk.pool_desc(FAKE + (1 << 20), nb, 2, tile + 8)), wk.KV_E_ALIGN),
        (dict(pool=wk.pool_desc(FAKE + (1 << 20) + 16, nb, 2, tile)), wk.KV_E_ALIGN),
        (dict(tables=None), wk.KV_E_NULL),
        (dict(tables=FAKE + 1028), wk.KV_E_ALIGN),
        (dict(tensors=[(FAKE, region + 16, 0)]), wk.KV_E_TOOBIG),
        (dict(tensors=[(FAKE, 4096, 0), (FAKE, 4096, 4095)]), wk.KV_E_OVERLAP),
        (dict(tensors=[(None, 4096, 0)]), wk.KV_E_NULL),
    ]
    for change, code in cases:
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_switch(**{**ok, **change})
        assert e.value.code == code, change


def test_absurd_pool_sizes_are_refused():
    """Sizes whose byte offsets would overflow 64 bits (or leave the 48-bit address space) are
    argument errors, found before any launch."""
    nb, b = 64, 40
    plan = wk.kv_plan_bind(FAKE, wk.kv_plan_workspace_bytes(nb, b), nb, b)
    for pool in (wk.pool_desc(FAKE + (1 << 20), nb, 2, 1 << 60), wk.pool_desc(FAKE + (1 << 20), nb, 1 << 20, 1 << 30),
                 wk.pool_desc(FAKE + (1 << 20), nb, 4, 4096, 1 << 47)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.kv_compact(pool, plan)
        assert e.value.code == wk.KV_E_RANGE
        with pytest.raises(wk.WarmKVError) as e:
            wk.weights_materialize(pool, b, [(FAKE, 16, 0)])
        assert e.value.code == wk.KV_E_RANGE


def test_chained_calls_refuse_too_many_copy_units_before_the_planner_runs():
    """The block copy numbers its units with 32 bits; the calls that chain planner and copy check
    that first, so that a refusal leaves nothing enqueued (they return before any HIP call here)."""
    nb, b = 1 << 20, 1 << 19                      # 524 288 possible moves x 8192 units of a 256 MiB block = 2^32
    plan = wk.kv_plan_bind(FAKE, wk.kv_plan_workspace_bytes(nb, b), nb, b)
    pool = wk.pool_desc(FAKE + (1 << 30), nb, 1, 1 << 28)
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_reclaim(pool, plan, FAKE + (1 << 29), FAKE + (1 << 28), 1, 4)
    assert e.value.code == wk.KV_E_RANGE
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_switch(pool, plan, FAKE + (1 << 29), FAKE + (1 << 28), 1, 4, [], 0, 0, FAKE)
    assert e.value.code == wk.KV_E_RANGE
    small_nb = 1 << 18                             # the static entry point's largest pool, blocks of 1 GiB
    with pytest.raises(wk.WarmKVError) as e:
        wk.kv_reclaim_static(wk.pool_desc(FAKE + (1 << 30), small_nb, 1, 1 << 30), small_nb // 2, FAKE + (1 << 29),
                             FAKE + (1 << 27), FAKE + (1 << 28), 1, 4, FAKE + (1 << 26))
    assert e.value.code == wk.KV_E_RANGE


def test_movers_in_front_counts_live_blocks_above_the_boundary():
    rs = np.random.default_rng(3)
    for nb, b in ((1, 0), (64, 64), (130, 70), (1000, 333), (5000, 4999)):
        bits = rs.random(nb) < 0.5
        words = np.packbits(bits, bitorder="little")
        words = np.concatenate([words, np.zeros((-len(words)) % 8, np.uint8)]).view(np.uint64)
        for front in (0, 1, 7, 64, 65, nb, nb + 100):
            assert wk.kv_movers_in_front(words, nb, b, front) == int(bits[b:b + front].sum()), (nb, b, front)


def test_front_first_stream_validates_like_the_plain_one():
    nb, b, tile = 64, 40, 4096
    pool = wk.pool_desc(FAKE + (1 << 20), nb, 2, tile)
    region = (nb - b) * 2 * tile
    for tensors, code in (([(FAKE, region + 16, 0)], wk.KV_E_TOOBIG),
                          ([(FAKE, 4096, 0), (FAKE, 4096, 4095)], wk.KV_E_OVERLAP),
                          ([(None, 4096, 0)], wk.KV_E_NULL)):
        with pytest.raises(wk.WarmKVError) as e:
            wk.weights_materialize_front(pool, b, 8192, tensors)
        assert e.value.code == code
    with pytest.raises(wk.WarmKVError) as e:      # layer-major pools: a tensor must lie inside one strip
        wk.weights_materialize_front(wk.pool_desc(FAKE + (1 << 20), nb, 2, tile, nb * tile), b, 8192,
                                     [(FAKE, 32, (nb - b) * tile - 16)])
    assert e.value.code == wk.KV_E_TOOBIG


def test_host_code_under_sanitizers(tmp_path):
    """The library's host arithmetic (schedules, validation, Eq. 4, the reverse switch, the
    control-plane formulas) built with ASan + UBSan on the host side and driven by a C++ program
    with exact-size buffers.  Nothing in it reaches a HIP call."""
    import glob
    import subprocess
    from paper_2512_09472_amd import build as lib_build
    exe = str(tmp_path / "host_san")
    srcs = [f for f in sorted(glob.glob(os.path.join(lib_build.CSRC, "*.hip"))) if not f.endswith("vmm.hip")]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", lib_build.INCLUDE, "-I", lib_build.CSRC, os.path.join(ROOT, "tests", "host_san_driver.cpp"), *srcs,
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))      # the HIP runtime keeps its own allocations
    assert r.returncode == 0 and "ok" in r.stdout, (r.stdout + r.stderr)[-3000:]
