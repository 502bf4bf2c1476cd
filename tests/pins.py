"""Property checks that pin a relocation result without re-deriving it the way
the oracle does.  Each check raises AssertionError with the failed property.

The rule being pinned: every live block with id >= boundary moves to a free id
below it, ascending free ids paired with ascending moving ids.  Given that rule
the result is unique, and the properties below characterise it:
  * the destinations are exactly the n smallest free ids below the boundary,
  * the map is order preserving on movers and the identity on live ids below,
  * (so) it is injective and lands everything below the boundary,
  * every sequence reads the same bytes through its new table as before,
  * bytes of blocks that are not destinations are untouched.
"""
from __future__ import annotations

import numpy as np

NOSPACE = -7


def bools_from_words(words: np.ndarray, num_blocks: int) -> np.ndarray:
    out = np.zeros(num_blocks, dtype=bool)
    for i in range(num_blocks):
        out[i] = (int(words[i // 64]) >> (i % 64)) & 1
    return out


def check_plan(live: np.ndarray, num_blocks: int, boundary: int, p) -> None:
    """live: bool[num_blocks].  p: object with status, src, dst, new_id, live_out, n_moves."""
    n_movers = int(live[boundary:].sum())
    n_free = int((~live[:boundary]).sum())
    if n_movers > n_free:
        assert p.status == NOSPACE, "infeasible request must report no-space"
        return
    assert p.status == 0, "feasible request must succeed"
    assert p.n_moves == n_movers, "every live block at/above the boundary moves"
    src = np.asarray(p.src, dtype=np.int64)
    dst = np.asarray(p.dst, dtype=np.int64)
    assert src.shape == dst.shape == (n_movers,)
    if n_movers:
        assert np.all(np.diff(src) > 0), "sources ascending"
        assert np.all(np.diff(dst) > 0), "destinations ascending"
        assert src.min() >= boundary and src.max() < num_blocks and live[src].all(), "sources are live ids >= boundary"
        assert dst.min() >= 0 and dst.max() < boundary and not live[dst].any(), "destinations are free ids < boundary"
        # n smallest free ids: no free id below the largest destination is skipped
        assert int((~live[:dst.max() + 1]).sum()) == n_movers, "destinations are the smallest free ids"
    new_id = np.asarray(p.new_id, dtype=np.int64)
    assert new_id.shape == (num_blocks,)
    ids = np.arange(num_blocks)
    below = live & (ids < boundary)
    assert np.array_equal(new_id[below], ids[below]), "live ids below the boundary keep their id"
    assert np.all(new_id[~live] == -1), "free ids map to -1"
    assert np.array_equal(new_id[src], dst), "k-th mover takes k-th destination"
    image = new_id[live]
    assert len(set(image.tolist())) == image.size, "no duplicate physical ids"
    assert image.size == 0 or (image.min() >= 0 and image.max() < boundary), "all ids below the boundary"
    live_after = bools_from_words(np.asarray(p.live_out), num_blocks)
    expect_after = np.zeros(num_blocks, dtype=bool)
    expect_after[image] = True
    assert np.array_equal(live_after, expect_after), "bitmap after = image of the live set"
    assert int(live_after.sum()) == int(live.sum()), "live count conserved"


def gather(pool: np.ndarray, block_bytes: int, row: np.ndarray) -> bytes:
    blocks = pool.reshape(-1, block_bytes)
    return b"".join(blocks[int(e)].tobytes() for e in row if e >= 0)


def check_pool_and_tables(pool0: np.ndarray, pool1: np.ndarray, tables0: np.ndarray, tables1: np.ndarray,
                          live: np.ndarray, num_blocks: int, boundary: int, block_bytes: int, p) -> None:
    """pool0/tables0 before, pool1/tables1 after a successful reclaim."""
    assert p.status == 0
    b0 = pool0.reshape(num_blocks, block_bytes)
    b1 = pool1.reshape(num_blocks, block_bytes)
    dst_set = np.zeros(num_blocks, dtype=bool)
    dst_set[np.asarray(p.dst, dtype=np.int64)] = True
    assert np.array_equal(b1[~dst_set], b0[~dst_set]), "non-destination blocks untouched"
    assert np.array_equal(b1[boundary:], b0[boundary:]), "nothing written at/above the boundary"
    assert tables1.shape == tables0.shape
    assert np.array_equal(tables1 < 0, tables0 < 0), "empty entries stay empty, row lengths kept"
    valid = tables1[tables1 >= 0]
    assert valid.size == 0 or valid.max() < boundary, "all table ids below the boundary"
    keep = (tables0 >= 0) & (tables0 < boundary)
    assert np.array_equal(tables1[keep], tables0[keep]), "entries below the boundary unchanged"
    for s in range(tables0.shape[0]):
        assert gather(pool0, block_bytes, tables0[s]) == gather(pool1, block_bytes, tables1[s]), \
            f"sequence {s}: KV read through the new table differs"


def rank_select_new_id(live: np.ndarray, num_blocks: int, boundary: int) -> np.ndarray:
    """Independent formulation: new_id[e] = select0(live[0:b), rank1(live[b:e))) for live e >= b."""
    ones_above = np.cumsum(live[boundary:].astype(np.int64))           # inclusive rank1
    zeros_below = np.cumsum((~live[:boundary]).astype(np.int64))       # inclusive rank0
    out = np.full(num_blocks, -1, dtype=np.int64)
    for e in range(num_blocks):
        if not live[e]:
            continue
        if e < boundary:
            out[e] = e
        else:
            r = int(ones_above[e - boundary]) - 1                      # movers strictly before e
            out[e] = int(np.searchsorted(zeros_below, r + 1, side="left"))
    return out
