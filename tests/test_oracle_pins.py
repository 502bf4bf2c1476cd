"""Pins for the CPU oracle: it is checked against things other than itself.

  * hand-worked fixtures (tests/golden/),
  * exhaustive enumeration of every bitmap up to 12 blocks x every boundary
    against properties that determine the result uniquely,
  * an independently written rank/select formulation,
  * closed forms: nothing to move; a full upper half onto an empty lower half
    is one memmove; the exact feasibility threshold; idempotence,
  * weight placement against numpy slicing; Eq. 4 against hand-evaluated cases,
  * mutants: plausible mistakes planted in the oracle's results (on the CPU)
    must each be rejected by the property checks.
"""
import json
import os

import numpy as np
import pytest

import pins
from synth import bitmap_from_ids, bitmap_to_bools
from synth.rng import SplitMix64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _words(hexes):
    return np.array([int(h, 16) for h in hexes], dtype=np.uint64)


def _random_case(rng, num_blocks, boundary, p_live, block_bytes=32, n_seqs=5):
    live = np.array([rng.uniform() < p_live for _ in range(num_blocks)], dtype=bool)
    ids = np.flatnonzero(live).tolist()
    order = [ids[i] for i in rng.shuffle(len(ids))] if ids else []
    width = max(1, -(-len(order) // n_seqs) + 1)
    tables = np.full((n_seqs, width), -1, dtype=np.int32)
    pos = 0
    for s in range(n_seqs):
        k = min(len(order) - pos, rng.below(width + 1))
        tables[s, :k] = order[pos:pos + k]
        pos += k
    pool = np.frombuffer(bytes(rng.below(256) for _ in range(num_blocks * block_bytes)), dtype=np.uint8).copy()
    return live, tables, pool


def _run(oracle, live, num_blocks, boundary, tables, pool, block_bytes):
    p = oracle.plan(bitmap_from_ids(np.flatnonzero(live), num_blocks), num_blocks, boundary)
    pool1, tables1 = pool.copy(), tables.copy()
    oracle.compact(pool1, block_bytes, p)
    bad = oracle.remap(tables1, p)
    return p, pool1, tables1, bad


# ---------------------------------------------------------------- fixtures
def test_handworked_fixtures(oracle):
    with open(os.path.join(GOLDEN, "plan_handworked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        nb, b = c["num_blocks"], c["boundary"]
        words = _words(c["live_words_hex"])
        assert np.array_equal(words, bitmap_from_ids(c["live_ids"], nb)), c["name"]
        p = oracle.plan(words, nb, b)
        assert p.status == c["status"], c["name"]
        if c["status"] != 0:
            continue
        assert p.src.tolist() == c["src"] and p.dst.tolist() == c["dst"], c["name"]
        if "new_id" in c:
            assert p.new_id.tolist() == c["new_id"], c["name"]
        assert np.array_equal(p.live_out, _words(c["live_out_words_hex"])), c["name"]
        t = np.array(c["tables_before"], dtype=np.int32)
        assert oracle.remap(t, p) == 0
        assert t.tolist() == c["tables_after"], c["name"]


def test_eq4_fixtures(oracle):
    with open(os.path.join(GOLDEN, "eq4_reserve.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        assert oracle.reserve_blocks(c["C"], c["T"], c["Q"], c["B"]) == c["R"], c["note"]
    assert oracle.reserve_blocks(10, 11, 1, 32) < 0 and oracle.reserve_blocks(10, 1, 1, 0) < 0


def test_eq4_against_real_arithmetic(oracle):
    """R is the ceiling of the real-valued maximum, capped at C (fractions.Fraction, exact)."""
    from fractions import Fraction
    from math import ceil
    rng = SplitMix64(7)
    for _ in range(2000):
        C = rng.randint(1, 200000)
        T = rng.randint(0, C)
        B = rng.randint(1, 256)
        Q = rng.randint(0, B)
        want = min(C, ceil(max(Fraction(C * Q, B), T + Fraction(C, B))))
        assert oracle.reserve_blocks(C, T, Q, B) == want


# ------------------------------------------------------------- brute force
def test_exhaustive_small_bitmaps(oracle):
    """Every bitmap with <= 12 blocks, every boundary: plan properties + rank/select."""
    for nb in range(0, 13):
        for bits in range(1 << nb):
            live = np.array([(bits >> i) & 1 for i in range(nb)], dtype=bool)
            words = np.array([bits], dtype=np.uint64) if nb else np.zeros(0, dtype=np.uint64)
            for b in range(nb + 1):
                if nb > 9 and b not in (0, 1, nb // 2, nb - 1, nb):
                    continue
                p = oracle.plan(words, nb, b)
                pins.check_plan(live, nb, b, p)
                if p.status == 0:
                    assert np.array_equal(p.new_id, pins.rank_select_new_id(live, nb, b))


def test_exhaustive_small_pools(oracle):
    """Every bitmap with <= 8 blocks, every boundary, with pool bytes and tables."""
    rng = SplitMix64(11)
    bb = 16
    for nb in range(1, 9):
        pool = np.frombuffer(bytes(rng.below(256) for _ in range(nb * bb)), dtype=np.uint8).copy()
        for bits in range(1 << nb):
            live = np.array([(bits >> i) & 1 for i in range(nb)], dtype=bool)
            ids = np.flatnonzero(live)
            perm = [int(ids[i]) for i in rng.shuffle(len(ids))]
            tables = np.full((2, nb), -1, dtype=np.int32)
            cut = len(perm) // 2
            tables[0, :cut] = perm[:cut]
            tables[1, :len(perm) - cut] = perm[cut:]
            for b in range(nb + 1):
                p, pool1, tables1, bad = _run(oracle, live, nb, b, tables, pool, bb)
                pins.check_plan(live, nb, b, p)
                if p.status == 0:
                    assert bad == 0
                    pins.check_pool_and_tables(pool, pool1, tables, tables1, live, nb, b, bb, p)
                else:
                    assert np.array_equal(pool1, pool) and np.array_equal(tables1, tables)


@pytest.mark.parametrize("nb,b,p_live", [(64, 32, 0.4), (65, 33, 0.45), (200, 77, 0.3), (1000, 640, 0.55),
                                         (4097, 2500, 0.5), (129, 128, 0.5), (300, 0, 0.0), (300, 300, 0.6)])
def test_random_cases_against_properties_and_rank_select(oracle, nb, b, p_live):
    rng = SplitMix64(nb * 1000 + b)
    for _ in range(4):
        live, tables, pool = _random_case(rng, nb, b, p_live)
        p, pool1, tables1, bad = _run(oracle, live, nb, b, tables, pool, 32)
        pins.check_plan(live, nb, b, p)
        if p.status == 0:
            assert bad == 0
            assert np.array_equal(p.new_id, pins.rank_select_new_id(live, nb, b))
            pins.check_pool_and_tables(pool, pool1, tables, tables1, live, nb, b, 32, p)


# ------------------------------------------------------------ closed forms
def test_nothing_to_move_is_identity(oracle):
    nb, b = 300, 200
    live = np.zeros(nb, dtype=bool)
    live[[0, 5, 63, 64, 150, 199]] = True
    words = bitmap_from_ids(np.flatnonzero(live), nb)
    p = oracle.plan(words, nb, b)
    assert p.status == 0 and p.n_moves == 0
    assert np.array_equal(p.live_out, words)
    assert np.array_equal(p.new_id, np.where(live, np.arange(nb), -1))
    pool = np.arange(nb * 8, dtype=np.uint64).view(np.uint8).copy()
    before = pool.copy()
    oracle.compact(pool, 64, p)
    assert np.array_equal(pool, before)


def test_full_upper_half_onto_empty_lower_half_is_memmove(oracle):
    nb, bb = 256, 48
    b = nb // 2
    live = np.arange(nb) >= b
    p = oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b)
    assert p.status == 0 and p.n_moves == b
    assert np.array_equal(p.new_id[b:], np.arange(b))
    rng = np.random.default_rng(3)
    pool = rng.integers(0, 256, nb * bb, dtype=np.uint8)
    want = pool.copy()
    want[:b * bb] = pool[b * bb:]          # the library routine this case reduces to
    oracle.compact(pool, bb, p)
    assert np.array_equal(pool, want)


def test_feasibility_threshold(oracle):
    """Feasible exactly when live_count <= boundary (|F| - n = b - live_count)."""
    nb, b = 200, 120
    rng = SplitMix64(5)
    for live_count in (b - 1, b, b + 1):
        ids = rng.shuffle(nb)[:live_count]
        p = oracle.plan(bitmap_from_ids(ids, nb), nb, b)
        assert (p.status == 0) == (live_count <= b)
        if live_count == b:
            assert bitmap_to_bools(p.live_out, nb)[:b].all()


def test_idempotent(oracle):
    rng = SplitMix64(9)
    nb, b = 777, 400
    live, _, _ = _random_case(rng, nb, b, 0.45)
    p = oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b)
    assert p.status == 0 and p.n_moves > 0
    q = oracle.plan(p.live_out, nb, b)
    assert q.status == 0 and q.n_moves == 0 and np.array_equal(q.live_out, p.live_out)


def test_nospace_touches_nothing(oracle):
    nb, b = 64, 10
    live = np.ones(nb, dtype=bool)
    p = oracle.plan(bitmap_from_ids(range(nb), nb), nb, b)
    assert p.status == oracle.E_NOSPACE
    pool = np.arange(nb * 16, dtype=np.uint8)
    t = np.arange(nb, dtype=np.int32).reshape(4, 16)
    pool1, t1 = pool.copy(), t.copy()
    oracle.compact(pool1, 16, p)
    oracle.remap(t1, p)
    assert np.array_equal(pool1, pool) and np.array_equal(t1, t)
    assert live.all()


def test_bad_table_entries_are_counted_and_left(oracle):
    nb, b = 16, 8
    p = oracle.plan(bitmap_from_ids([0, 2, 3, 7, 9, 12, 13, 15], nb), nb, b)
    t = np.array([[9, 1, 16], [12, -1, 1000], [10, 3, -5]], dtype=np.int32)   # 1, 10 free; 16, 1000 outside
    bad = oracle.remap(t, p)
    assert bad == 4
    assert t.tolist() == [[1, 1, 16], [4, -1, 1000], [10, 3, -5]]


# ----------------------------------------------------------------- weights
def test_materialize_matches_slicing(oracle):
    rng = np.random.default_rng(1)
    nb, bb, b = 32, 64, 20
    pool = rng.integers(0, 256, nb * bb, dtype=np.uint8)
    want = pool.copy()
    region = b * bb
    tensors = [(rng.integers(0, 256, 100, dtype=np.uint8), 0),
               (rng.integers(0, 256, 256, dtype=np.uint8), 256),
               (rng.integers(0, 256, 7, dtype=np.uint8), 120),
               (np.zeros(0, dtype=np.uint8), 130),
               (rng.integers(0, 256, 200, dtype=np.uint8), (nb - b) * bb - 200)]
    for buf, off in tensors:
        want[region + off: region + off + buf.size] = buf
    assert oracle.materialize(pool, region, tensors) == 0
    assert np.array_equal(pool, want)
    assert np.array_equal(pool[:region], want[:region])


def test_materialize_rejects_before_writing(oracle):
    nb, bb, b = 8, 32, 4
    pool = np.arange(nb * bb, dtype=np.uint8)
    ref = pool.copy()
    big = np.ones(200, dtype=np.uint8)
    ok = np.ones(16, dtype=np.uint8)
    assert oracle.materialize(pool, b * bb, [(ok, 0), (big, 0)]) in (oracle.E_TOOBIG, oracle.E_OVERLAP)
    assert oracle.materialize(pool, b * bb, [(ok, 0), (big, 64)]) == oracle.E_TOOBIG
    assert oracle.materialize(pool, b * bb, [(ok, 0), (ok, 8)]) == oracle.E_OVERLAP
    assert oracle.materialize(pool, b * bb, [(ok, 112), (ok, 127)]) in (oracle.E_TOOBIG, oracle.E_OVERLAP)
    assert np.array_equal(pool, ref)
    assert oracle.materialize(pool, b * bb, [(ok, 0), (ok, 16), (ok, 112)]) == 0
    assert oracle.materialize(pool, b * bb, [(ok, 0), (np.zeros(0, np.uint8), 5)]) == 0   # an empty extent overlaps nothing


def test_layer_major_compact_is_the_block_major_one_under_a_transpose(oracle):
    """A layer-major pool [L][NB][tile] is the block-major pool [NB][L][tile] with two axes
    swapped; the block copy must commute with that swap (numpy transpose, pinned block-major oracle)."""
    rs = np.random.default_rng(6)
    for nb, b, layers, tile, pad in ((40, 22, 3, 16, 0), (130, 70, 5, 48, 256), (64, 32, 1, 32, 0)):
        live = rs.random(nb) < 0.45
        p = oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b)
        assert p.status == 0 and p.n_moves > 0
        stride = nb * tile + pad
        lm = rs.integers(0, 256, layers * stride, dtype=np.uint8)
        before = lm.copy()
        slabs = lm.reshape(layers, stride)
        bm = np.ascontiguousarray(slabs[:, :nb * tile].reshape(layers, nb, tile).transpose(1, 0, 2)).reshape(-1)
        oracle.compact(bm, layers * tile, p)
        want = before.copy().reshape(layers, stride)
        want[:, :nb * tile] = bm.reshape(nb, layers, tile).transpose(1, 0, 2).reshape(layers, nb * tile)
        oracle.compact_layer_major(lm, tile, layers, stride, p)
        assert np.array_equal(lm, want.reshape(-1))
        assert np.array_equal(lm.reshape(layers, stride)[:, nb * tile:], before.reshape(layers, stride)[:, nb * tile:]), "padding untouched"


def test_materialize_strips_matches_slicing(oracle):
    rs = np.random.default_rng(7)
    nb, b, layers, tile, stride = 20, 12, 3, 32, 20 * 32 + 256
    pool = rs.integers(0, 256, layers * stride, dtype=np.uint8)
    strip = (nb - b) * tile
    tensors = [(rs.integers(0, 256, 100, dtype=np.uint8), 0), (rs.integers(0, 256, strip, dtype=np.uint8), strip),
               (rs.integers(0, 256, 7, dtype=np.uint8), 2 * strip + 249), (np.zeros(0, np.uint8), 3)]
    want = pool.copy().reshape(layers, stride)
    for buf, off in tensors:
        layer, within = (off // strip, off % strip) if buf.size else (0, 0)
        want[layer, b * tile + within: b * tile + within + buf.size] = buf
    assert oracle.materialize_strips(pool, tile, layers, nb, b, stride, tensors) == 0
    assert np.array_equal(pool, want.reshape(-1))
    ref = pool.copy()
    one = np.ones(10, np.uint8)
    assert oracle.materialize_strips(pool, tile, layers, nb, b, stride, [(one, strip - 5)]) == oracle.E_TOOBIG   # straddles
    assert oracle.materialize_strips(pool, tile, layers, nb, b, stride, [(one, 3 * strip - 9)]) == oracle.E_TOOBIG
    assert oracle.materialize_strips(pool, tile, layers, nb, b, stride, [(one, 0), (one, 9)]) == oracle.E_OVERLAP
    assert np.array_equal(pool, ref)


def test_grow_hand_cases_and_byte_brute_force(oracle):
    """Reverse switch: a tensor is lost iff one of its bytes lies in a returned block."""
    bb, nb = 64, 30
    # old boundary 10, 3 blocks returned: pool bytes [640, 832) go back to the KV cache
    ext = [(64, 0), (1, 191), (1, 192), (200, 100), (0, 50), (10, 1270)]
    n, ev, no = oracle.grow(bb, nb, 10, 13, ext)
    assert n == 3 and ev.tolist() == [1, 1, 0, 1, 0, 0]
    assert no.tolist()[2] == 0 and no.tolist()[5] == 1270 - 192
    assert oracle.grow(bb, nb, 10, 13, [(11, 1270)])[0] == oracle.E_TOOBIG
    assert oracle.grow(bb, nb, 13, 10, [])[0] == oracle.E_RANGE
    rs = np.random.default_rng(4)
    for _ in range(200):
        old = int(rs.integers(0, nb + 1))
        new = int(rs.integers(old, nb + 1))
        region = (nb - old) * bb
        ext = []
        for _ in range(5):
            off = int(rs.integers(0, region + 1))
            ext.append((int(rs.integers(0, region - off + 1)), off))
        n, ev, no = oracle.grow(bb, nb, old, new, ext)
        owner = np.zeros(nb * bb, dtype=bool)
        owner[old * bb:new * bb] = True                      # bytes that go back
        for i, (b, o) in enumerate(ext):
            assert bool(ev[i]) == bool(owner[old * bb + o: old * bb + o + b].any())
            if b and not ev[i]:
                assert old * bb + o == new * bb + int(no[i])  # same absolute place, new origin
        assert n == int(ev.sum())


def test_grow_strips_hand_cases_and_byte_brute_force(oracle):
    """Reverse switch in a layer-major pool: every strip loses its first (new - old) tiles.  Checked
    against a per-byte ownership map of the whole pool (slab padding included)."""
    tile, layers, nb = 16, 3, 12
    stride = nb * tile + 32                                   # padded slabs
    # old boundary 4 (strips of 8 tiles = 128 B), 2 tiles returned per strip: slab bytes [64, 96)
    ext = [(16, 0), (1, 31), (1, 32), (96, 32), (0, 5), (40, 128 + 40), (8, 2 * 128 + 24), (128, 2 * 128)]
    n, ev, no = oracle.grow_strips(tile, layers, nb, stride, 4, 6, ext)
    assert n == 4 and ev.tolist() == [1, 1, 0, 0, 0, 0, 1, 1]
    # survivors keep their place: strips shrink to 6 tiles = 96 B
    assert no.tolist()[2:6] == [0, 0, 0, 96 + 8]
    assert oracle.grow_strips(tile, layers, nb, stride, 4, 6, [(2, 127)])[0] == oracle.E_TOOBIG     # straddles two strips
    assert oracle.grow_strips(tile, layers, nb, stride, 4, 6, [(1, 3 * 128)])[0] == oracle.E_TOOBIG
    assert oracle.grow_strips(tile, layers, nb, stride, 6, 4, [])[0] == oracle.E_RANGE
    # one layer, stride = pool: the block-major function on the same numbers
    for old, new in ((0, 0), (3, 9), (5, 12)):
        e1 = [(7, 3), (0, 0), (20, 40)] if old <= 8 else []
        a = oracle.grow_strips(tile, 1, nb, nb * tile, old, new, e1)
        b = oracle.grow(tile, nb, old, new, e1)
        assert a[0] == b[0] and (a[0] < 0 or (a[1].tolist() == b[1].tolist() and a[2].tolist() == b[2].tolist()))
    rs = np.random.default_rng(8)
    for _ in range(300):
        old = int(rs.integers(0, nb))
        new = int(rs.integers(old, nb + 1))
        old_strip, new_strip = (nb - old) * tile, (nb - new) * tile
        ext = []
        for _ in range(5):
            layer = int(rs.integers(0, layers))
            within = int(rs.integers(0, old_strip))
            ext.append((int(rs.integers(0, old_strip - within + 1)), layer * old_strip + within))
        n, ev, no = oracle.grow_strips(tile, layers, nb, stride, old, new, ext)
        returned = np.zeros(layers * stride, dtype=bool)       # bytes that go back to the KV cache
        for l in range(layers):
            returned[l * stride + old * tile:l * stride + new * tile] = True

        def absolute(boundary, strip_bytes, region_offset):     # where a region offset lies in the pool
            l, w = divmod(region_offset, strip_bytes)
            return l * stride + boundary * tile + w

        for i, (b, o) in enumerate(ext):
            lo = absolute(old, old_strip, o)
            assert bool(ev[i]) == bool(returned[lo:lo + b].any())
            if b and not ev[i]:
                assert absolute(new, new_strip, int(no[i])) == lo   # same absolute place under the new boundary
        assert n == int(ev.sum())


def _check_vmm_selection(live, want, ids):
    """Properties that fix the selection uniquely: `want` distinct unused blocks, highest first, and
    no unused block left out is higher than one that was taken."""
    ids = np.asarray(ids, dtype=np.int64)
    assert ids.shape == (want,)
    assert not live[ids].any(), "only unused blocks lend pages"
    assert np.all(np.diff(ids) < 0), "highest first, no block twice"
    if want:
        left_out = np.setdiff1d(np.flatnonzero(~live), ids)
        assert left_out.size == 0 or left_out.max() < ids.min(), "the highest free ids are the ones taken"


def test_vmm_select_fixtures_and_exhaustive(oracle):
    with open(os.path.join(GOLDEN, "vmm_select_handworked.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        words = _words(c["live_words_hex"])
        clean = bitmap_from_ids(c["live_ids"], c["num_blocks"])
        valid = np.uint64((1 << (c["num_blocks"] % 64)) - 1) if c["num_blocks"] % 64 else np.uint64(0xFFFFFFFFFFFFFFFF)
        assert np.array_equal(words[:-1], clean[:-1]) and (words[-1] & valid) == clean[-1], c["name"]
        got = oracle.vmm_select(words, c["num_blocks"], c["want"])
        if c["ids"] is None:
            assert got is None, c["name"]
        else:
            assert got.tolist() == c["ids"], c["name"]
    # every bitmap of up to 10 blocks, every request size
    for nb in range(0, 11):
        for bits in range(1 << nb):
            live = np.array([(bits >> i) & 1 for i in range(nb)], dtype=bool)
            words = bitmap_from_ids(np.flatnonzero(live), nb)
            n_free = int((~live).sum())
            for want in range(0, nb + 2):
                got = oracle.vmm_select(words, nb, want)
                if want > n_free:
                    assert got is None
                else:
                    _check_vmm_selection(live, want, got)
    # the property check itself rejects the plausible mistakes
    live = np.array([0, 1, 0, 0, 1, 1, 0, 0, 0, 1], dtype=bool)
    good = oracle.vmm_select(bitmap_from_ids(np.flatnonzero(live), 10), 10, 3)
    for name, bad in {"ascending": good[::-1], "lowest free ids": np.array([3, 2, 0]), "a live block": np.array([9, 8, 7]),
                      "skipped one": np.array([8, 6, 3]), "twice": np.array([8, 8, 7])}.items():
        with pytest.raises(AssertionError):
            _check_vmm_selection(live, 3, bad)
            pytest.fail(f"mutant accepted: {name}")


# ----------------------------------------------------------------- mutants
class _Mut:
    def __init__(self, p, **kw):
        self.__dict__.update(p.__dict__)
        self.__dict__.update({k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in kw.items()})


def _rebuild_new_id(p, live, src, dst, boundary):
    new_id = np.where(live & (np.arange(p.num_blocks) < boundary), np.arange(p.num_blocks), -1).astype(np.int32)
    new_id[src] = dst
    return new_id


def _plan_mutants(p, live, nb, b):
    out = {}
    if p.n_moves >= 2:
        rd = p.dst[::-1].copy()
        out["descending_pairing"] = _Mut(p, dst=p.dst, new_id=_rebuild_new_id(p, live, p.src, rd, b))
        out["dst_list_reversed"] = _Mut(p, dst=rd, new_id=_rebuild_new_id(p, live, p.src, rd, b))
        out["swapped_src_dst"] = _Mut(p, src=p.dst, dst=p.src)
        out["dropped_last_move"] = _Mut(p, src=p.src[:-1], dst=p.dst[:-1], n_moves=p.n_moves - 1)
    free_below = np.flatnonzero(~live[:b])
    if p.n_moves and free_below.size > p.n_moves:
        hi = free_below[-p.n_moves:].astype(np.int32)
        lo = np.zeros_like(p.live_out)
        for j in np.flatnonzero(live[:b]).tolist() + hi.tolist():
            lo[j // 64] |= np.uint64(1) << np.uint64(j % 64)
        out["largest_free_ids"] = _Mut(p, dst=hi, new_id=_rebuild_new_id(p, live, p.src, hi, b), live_out=lo)
    stale = p.live_out.copy()
    if p.n_moves:
        j = int(p.src[0])
        stale[j // 64] |= np.uint64(1) << np.uint64(j % 64)
        out["source_bit_not_cleared"] = _Mut(p, live_out=stale)
        nid = p.new_id.copy()
        nid[p.src[0]] = p.src[0]
        out["mover_keeps_id"] = _Mut(p, new_id=nid)
    nid = p.new_id.copy()
    nid[~live] = 0
    out["free_maps_to_zero"] = _Mut(p, new_id=nid)
    return out


def test_plan_mutants_are_rejected(oracle):
    rng = SplitMix64(21)
    nb, b = 190, 100
    live, _, _ = _random_case(rng, nb, b, 0.4)
    live[b - 1] = live[b] = True      # so that an off-by-one boundary changes the answer
    p = oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b)
    pins.check_plan(live, nb, b, p)
    muts = _plan_mutants(p, live, nb, b)
    assert len(muts) == 8
    for name, m in muts.items():
        with pytest.raises(AssertionError):
            pins.check_plan(live, nb, b, m)
            pytest.fail(f"mutant {name} passed the pins")
    # wrong boundary and wrong bit order are mistakes in reading the input
    for name, wrong in (("boundary_plus_one", oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b + 1)),
                        ("boundary_minus_one", oracle.plan(bitmap_from_ids(np.flatnonzero(live), nb), nb, b - 1)),
                        ("msb_first_bits", oracle.plan(bitmap_from_ids(63 - (np.flatnonzero(live) % 64) + 64 * (np.flatnonzero(live) // 64), 192), nb, b))):
        with pytest.raises(AssertionError):
            pins.check_plan(live, nb, b, wrong)
            pytest.fail(f"mutant {name} passed the pins")


def test_pool_and_table_mutants_are_rejected(oracle):
    rng = SplitMix64(22)
    nb, b, bb = 150, 80, 32
    live, tables, pool = _random_case(rng, nb, b, 0.4)
    p, pool1, tables1, _ = _run(oracle, live, nb, b, tables, pool, bb)
    assert p.status == 0 and p.n_moves >= 2
    pins.check_pool_and_tables(pool, pool1, tables, tables1, live, nb, b, bb, p)
    blocks0 = pool.reshape(nb, bb)

    def mutated_pool(fn):
        q = pool.copy().reshape(nb, bb)
        fn(q)
        return q.reshape(-1)

    def reverse_copy(q):
        q[p.src] = blocks0[p.dst]

    def half_block(q):
        q[p.dst, :bb // 2] = blocks0[p.src, :bb // 2]

    def shifted_pairs(q):
        q[p.dst] = blocks0[np.roll(p.src, 1)]

    def also_clears_source(q):
        q[p.dst] = blocks0[p.src]
        q[p.src] = 0

    def scribbles_free_block(q):
        q[p.dst] = blocks0[p.src]
        spare = [j for j in range(nb) if not live[j] and j not in set(p.dst.tolist())]
        q[spare[0], 0] ^= 0xFF

    for fn in (reverse_copy, half_block, shifted_pairs, also_clears_source, scribbles_free_block):
        with pytest.raises(AssertionError):
            pins.check_pool_and_tables(pool, mutated_pool(fn), tables, tables1, live, nb, b, bb, p)
            pytest.fail(f"pool mutant {fn.__name__} passed the pins")

    t_identity = tables.copy()
    t_all = np.where(tables >= 0, 0, tables).astype(np.int32)
    t_padlost = tables1.copy()
    t_padlost[tables1 < 0] = 0
    t_below_touched = tables1.copy()
    keep = np.argwhere((tables >= 0) & (tables < b))
    t_below_touched[tuple(keep[0])] = int(p.dst[0])
    for name, t in (("not_remapped", t_identity), ("all_zero", t_all), ("padding_lost", t_padlost),
                    ("entry_below_boundary_changed", t_below_touched)):
        with pytest.raises(AssertionError):
            pins.check_pool_and_tables(pool, pool1, tables, t, live, nb, b, bb, p)
            pytest.fail(f"table mutant {name} passed the pins")


def test_oracle_under_sanitizers(tmp_path):
    """The oracle plus a small C++ driver, built with ASan+UBSan, run as one host program."""
    import subprocess
    import oracle as o
    exe = str(tmp_path / "oracle_san")
    driver = os.path.join(os.path.dirname(__file__), "oracle_san_driver.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", driver, o.SRC_PATH, "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert r.returncode == 0 and "ok" in r.stdout, (r.stdout + r.stderr)[-2000:]
