"""Seeded synthetic paged-KV workloads.

Builds, on the host, the inputs of the KV-reclaim path for the five benchmark
configurations: a live/free block bitmap, per-sequence block tables and the
reclaim boundary.  The recipe (budget rule, allocation order, length
distributions) is a property of the test inputs only; none of the relocation
method's arithmetic lives here.

The configurations describe the sequences as an arrival list that demands far
more blocks than the pool holds, so the *live-block budget* is what binds:
budget = min(stated occupancy x num_blocks, boundary - num_blocks/32).  The
second term is the reservation rule of the paper (Sec. 3.3, Eq. 4) with a
maximum batch of 32 (Sec. 4.1): a worker keeps its current usage plus one
average request's share, so it never offers space it could not vacate.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass

import numpy as np

from .rng import SplitMix64

GIB = 1 << 30
MIB = 1 << 20


@dataclass(frozen=True)
class KVConfig:
    name: str
    index: int                 # position in the benchmark's config list (0-based)
    num_layers: int
    block_size: int            # tokens per block
    kv_heads: int
    head_dim: int
    elem_bytes: int            # 2 = bf16, 1 = fp8 stored as raw bytes
    num_blocks: int
    boundary: int              # first reclaimed block id
    num_seqs: int
    len_lo: int
    len_hi: int
    len_dist: str              # "uniform" | "loguniform"
    occupancy: float | None    # stated live fraction of the pool, if any
    alloc: str                 # "shuffled" | "interleaved_free"
    content: str               # "bf16_normal" | "bytes"
    live_budget_override: int | None = None

    @property
    def seed(self) -> int:
        return 0x5EED0000 + self.index

    @property
    def tile_bytes(self) -> int:
        """One block in one layer, K and V."""
        return 2 * self.block_size * self.kv_heads * self.head_dim * self.elem_bytes

    @property
    def block_bytes(self) -> int:
        return self.num_layers * self.tile_bytes

    @property
    def pool_bytes(self) -> int:
        return self.num_blocks * self.block_bytes

    @property
    def max_blocks_per_seq(self) -> int:
        return -(-self.len_hi // self.block_size)

    @property
    def live_budget(self) -> int:
        if self.live_budget_override is not None:
            return self.live_budget_override
        stated = self.num_blocks if self.occupancy is None else int(round(self.occupancy * self.num_blocks))
        return max(0, min(stated, self.boundary - self.num_blocks // 32))

    def scaled(self, **changes) -> "KVConfig":
        """Same recipe at another size.  If ``num_blocks`` changes and no
        ``boundary`` is given, the boundary keeps its fraction of the pool."""
        if "num_blocks" in changes and "boundary" not in changes:
            nb = changes["num_blocks"]
            changes["boundary"] = (self.boundary * nb) // self.num_blocks
        return dataclasses.replace(self, **changes)


def _reclaim_boundary(num_blocks: int, reclaim_bytes: int, block_bytes: int) -> int:
    """Blocks reclaimed = ceil(bytes / block_bytes), taken from the top."""
    return num_blocks - (-(-reclaim_bytes // block_bytes))


def _make_configs() -> list[KVConfig]:
    tile64k = 2 * 16 * 8 * 128 * 2
    c1 = KVConfig("tiny", 0, 1, 16, 8, 128, 2, 1024, 512, 64, 1, 2048, "uniform",
                  None, "shuffled", "bf16_normal")
    nb2 = 40 * GIB // (32 * tile64k)
    c2 = KVConfig("llama3_8b_kv", 1, 32, 16, 8, 128, 2, nb2,
                  _reclaim_boundary(nb2, 16 * GIB, 32 * tile64k),
                  256, 128, 32768, "loguniform", 0.70, "shuffled", "bf16_normal")
    c3 = dataclasses.replace(c2, name="llama3_8b_kv_weights", index=2)
    nb4 = 120 * GIB // (80 * tile64k)
    c4 = KVConfig("llama_70b_share", 3, 80, 16, 8, 128, 2, nb4,
                  _reclaim_boundary(nb4, 28 * GIB, 80 * tile64k),
                  1024, 64, 16384, "loguniform", 0.60, "shuffled", "bf16_normal")
    tile5 = 2 * 32 * 4 * 128 * 1
    nb5 = 64 * GIB // (32 * tile5)
    c5 = KVConfig("frag_fp8", 4, 32, 32, 4, 128, 1, nb5, nb5 // 2,
                  8192, 16, 512, "uniform", None, "interleaved_free", "bytes")
    return [c1, c2, c3, c4, c5]


CONFIGS: list[KVConfig] = _make_configs()


def config(index: int) -> KVConfig:
    return CONFIGS[index]


@dataclass
class Workload:
    cfg: KVConfig
    live: np.ndarray        # uint64[ceil(NB/64)], bit (i % 64) of word (i // 64)
    tables: np.ndarray      # int32[num_seqs, max_blocks_per_seq], -1 = empty
    seq_blocks: np.ndarray  # int32[num_seqs] blocks held by each sequence
    live_count: int


def bitmap_from_ids(ids, num_blocks: int) -> np.ndarray:
    words = np.zeros((num_blocks + 63) // 64, dtype=np.uint64)
    ids = np.asarray(list(ids), dtype=np.int64)
    if ids.size:
        np.bitwise_or.at(words, ids // 64, np.uint64(1) << (ids % 64).astype(np.uint64))
    return words


def bitmap_to_bools(words: np.ndarray, num_blocks: int) -> np.ndarray:
    bits = np.unpackbits(words.view(np.uint8), bitorder="little")
    return bits[:num_blocks].astype(bool)


def _draw_len(rng: SplitMix64, cfg: KVConfig) -> int:
    if cfg.len_dist == "uniform":
        return rng.randint(cfg.len_lo, cfg.len_hi)
    return rng.log_uniform_int(cfg.len_lo, cfg.len_hi)


def make_workload(cfg: KVConfig) -> Workload:
    rng = SplitMix64(cfg.seed)
    width = cfg.max_blocks_per_seq
    tables = np.full((cfg.num_seqs, width), -1, dtype=np.int32)
    seq_blocks = np.zeros(cfg.num_seqs, dtype=np.int32)
    budget = cfg.live_budget
    free = rng.shuffle(cfg.num_blocks)
    lens = [_draw_len(rng, cfg) for _ in range(cfg.num_seqs)]

    if cfg.alloc == "shuffled":
        # Sequences arrive in index order; the one that would exceed the budget
        # is truncated to fit and later ones wait with empty rows.
        head = 0
        for s, ln in enumerate(lens):
            need = min(-(-ln // cfg.block_size), budget - head)
            if need <= 0:
                break
            tables[s, :need] = free[head:head + need]
            seq_blocks[s] = need
            head += need
        live_ids = free[:head]
    elif cfg.alloc == "interleaved_free":
        # Every sequence arrives; before an arrival that would exceed the budget
        # uniformly chosen resident sequences are freed and their ids re-enter
        # the free list at random positions.
        resident: list[int] = []
        live_n = 0
        for s, ln in enumerate(lens):
            need = -(-ln // cfg.block_size)
            while live_n + need > budget and resident:
                victim = resident.pop(rng.below(len(resident)))
                k = int(seq_blocks[victim])
                for bid in tables[victim, :k].tolist():
                    free.insert(rng.below(len(free) + 1), bid)
                tables[victim, :k] = -1
                seq_blocks[victim] = 0
                live_n -= k
            if live_n + need > budget:
                continue
            tables[s, :need] = free[:need]
            del free[:need]
            seq_blocks[s] = need
            resident.append(s)
            live_n += need
        live_ids = tables[tables >= 0].tolist()
    else:
        raise ValueError(cfg.alloc)

    live = bitmap_from_ids(live_ids, cfg.num_blocks)
    return Workload(cfg, live, tables, seq_blocks, len(live_ids))


# Weight set of the third configuration: per layer q, k, v, o, gate, up, down,
# then the embedding matrix; bf16.
def weight_shapes_8b() -> list[tuple[str, tuple[int, int]]]:
    out = []
    for layer in range(32):
        for nm, shp in (("q", (4096, 4096)), ("k", (1024, 4096)), ("v", (1024, 4096)),
                        ("o", (4096, 4096)), ("gate", (14336, 4096)), ("up", (14336, 4096)),
                        ("down", (4096, 14336))):
            out.append((f"layers.{layer}.{nm}", shp))
    out.append(("embed", (128256, 4096)))
    return out


def dense_offsets(sizes: list[int], align: int = 256) -> list[int]:
    """Pack extents back to back from offset 0, each start rounded up to ``align``."""
    offs, cur = [], 0
    for sz in sizes:
        cur = -(-cur // align) * align
        offs.append(cur)
        cur += sz
    return offs
