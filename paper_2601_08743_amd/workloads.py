"""Seeded synthetic schema/query workloads (input generation only).

This module draws the random inputs that both the HIP path and the CPU checker
are fed with.  It holds none of the method's arithmetic: no gather, no block
allocation, no attention.  Everything is derived from one integer seed per
configuration through ``numpy.random.SeedSequence`` so that any single piece
(one table's KV, one layer's suffix activations) can be regenerated on its own
without materialising the rest.

The five configurations follow the workload shapes of the Text-to-SQL serving
setting of the paper (Sec. 3 problem setup: a query touches a set of m tables
of one database; Sec. 5.1: table order inside a prompt is random per sample):
a database of tables with a few hundred schema tokens each, queries that pick
a handful of them in random order, and a short uncached suffix (question plus
instructions, App. C).  The public benchmarks the paper measures on are not
available here; these inputs stand in for them.

Values are drawn in fp32 from N(0, 1) and rounded once to the storage type of
the configuration (fp32 or bf16 with round-to-nearest-even); bf16 tensors are
carried as ``uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BLOCK_SIZE = 16


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                    # "f32" | "bf16"
    n_tables: int
    table_len: Tuple[int, int]    # inclusive range, tokens
    batch: int
    tables_per_query: Tuple[int, int]   # inclusive range
    choice: str                   # "uniform" | "zipf" | "all" | "db"
    suffix_len: Tuple[int, int]   # inclusive range, tokens
    capacity: int                 # device table-cache capacity C, in tables
    seed: int
    block_size: int = BLOCK_SIZE
    zipf_s: float = 1.1
    db_size: int = 0              # choice "db": tables per database (consecutive ids)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def kv_row_bytes(self) -> int:
        """Bytes of one token's K (or V) row in one layer: Hkv * D * e."""
        return self.n_kv_heads * self.head_dim * self.elem_bytes


CONFIGS = {
    # single fp32 layer, small enough for the CPU checker to finish in well under a second
    "c1": WorkloadConfig("c1", 1, 8, 2, 64, "f32", 16, (128, 256), 1, (4, 4), "uniform",
                         (64, 64), 16, 1001),
    # 7B-class GQA decoder, batch 1, everything resident
    "c2": WorkloadConfig("c2", 28, 28, 4, 128, "bf16", 40, (150, 600), 1, (12, 12), "uniform",
                         (128, 128), 40, 1002),
    # batched hotspot workload, variable lengths
    "c3": WorkloadConfig("c3", 28, 28, 4, 128, "bf16", 40, (150, 600), 32, (3, 10), "zipf",
                         (64, 256), 40, 1003),
    # long-schema stress
    "c4": WorkloadConfig("c4", 32, 32, 8, 128, "bf16", 60, (200, 600), 4, (60, 60), "all",
                         (512, 512), 60, 1004),
    # cold-cache loading pipeline: half of the tables fit on the device
    "c5": WorkloadConfig("c5", 48, 40, 8, 128, "bf16", 80, (150, 600), 64, (4, 12), "zipf",
                         (128, 128), 40, 1005),
    # c5 with the structure of a Text-to-SQL service: the 80 tables belong to 8 databases of 10, a
    # request names tables of one database only; 4 databases fit on the device
    "c5db": WorkloadConfig("c5db", 48, 40, 8, 128, "bf16", 80, (150, 600), 64, (4, 10), "db",
                           (128, 128), 40, 1006, db_size=10),
}


def scaled(cfg: WorkloadConfig, **kw) -> WorkloadConfig:
    """A copy of ``cfg`` with some fields replaced (used for reduced test cases)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return WorkloadConfig(**d)


# ----------------------------------------------------------------------------- storage types

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored tensor (fp32, or bf16 bit patterns) to float64."""
    if dtype == "f32":
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# ----------------------------------------------------------------------------- the workload

@dataclass
class Workload:
    cfg: WorkloadConfig
    table_len: np.ndarray                 # int32 [n_tables]
    queries: List[np.ndarray]             # per query: int32 table ids in prompt order
    suffix_len: np.ndarray                # int32 [B]
    _cache: dict = field(default_factory=dict, repr=False)

    # -- integer structure -------------------------------------------------
    @property
    def table_ids(self) -> np.ndarray:
        return np.concatenate(self.queries).astype(np.int32)

    @property
    def cu_tables(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum([len(q) for q in self.queries])]).astype(np.int32)

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.suffix_len)]).astype(np.int32)

    @property
    def total_suffix(self) -> int:
        return int(self.suffix_len.sum())

    # -- tensors (regenerable piecewise) -----------------------------------
    def table_kv(self, t: int) -> Tuple[np.ndarray, np.ndarray]:
        """K and V of table ``t``: two arrays [L][n_t][Hkv][D] in storage type."""
        c = self.cfg
        rng = np.random.default_rng(np.random.SeedSequence([c.seed, 1, int(t)]))
        shape = (c.n_layers, int(self.table_len[t]), c.n_kv_heads, c.head_dim)
        return _draw(rng, shape, c.dtype), _draw(rng, shape, c.dtype)

    def suffix_qkv(self, layer: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """q [sumS][Hq][D], k_new and v_new [sumS][Hkv][D] of one layer, storage type."""
        c = self.cfg
        rng = np.random.default_rng(np.random.SeedSequence([c.seed, 2, int(layer)]))
        n = self.total_suffix
        q = _draw(rng, (n, c.n_q_heads, c.head_dim), c.dtype)
        k = _draw(rng, (n, c.n_kv_heads, c.head_dim), c.dtype)
        v = _draw(rng, (n, c.n_kv_heads, c.head_dim), c.dtype)
        return q, k, v

    def table_tokens(self, t: int, vocab: int = 32000) -> np.ndarray:
        """Token ids of table ``t``'s schema text (what the Table Trie is built from): one id per
        schema token, drawn uniformly from the vocabulary."""
        rng = np.random.default_rng(np.random.SeedSequence([self.cfg.seed, 3, int(t)]))
        return rng.integers(0, vocab, size=int(self.table_len[t])).astype(np.int32)

    def prompt_tokens(self, i: int, vocab: int = 32000) -> np.ndarray:
        """Token ids of query ``i``'s prompt: its tables' schema texts in prompt order, then the
        suffix (instructions and question)."""
        rng = np.random.default_rng(np.random.SeedSequence([self.cfg.seed, 4, int(i)]))
        parts = [self.table_tokens(int(t), vocab) for t in self.queries[i]]
        parts.append(rng.integers(0, vocab, size=int(self.suffix_len[i])).astype(np.int32))
        return np.concatenate(parts) if parts else np.zeros(0, np.int32)

    @property
    def sm_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.cfg.head_dim))


def _zipf_pick(rng: np.random.Generator, n_tables: int, m: int, s: float) -> np.ndarray:
    """m distinct table indices, popularity of index k proportional to (k+1)^-s, shuffled."""
    p = (np.arange(1, n_tables + 1, dtype=np.float64)) ** (-s)
    p /= p.sum()
    ids = rng.choice(n_tables, size=m, replace=False, p=p)
    rng.shuffle(ids)
    return ids.astype(np.int32)


def make_workload(cfg: WorkloadConfig) -> Workload:
    rng = np.random.default_rng(np.random.SeedSequence([cfg.seed, 0]))
    lo, hi = cfg.table_len
    table_len = rng.integers(lo, hi + 1, size=cfg.n_tables).astype(np.int32)
    queries: List[np.ndarray] = []
    for _ in range(cfg.batch):
        mlo, mhi = cfg.tables_per_query
        m = int(rng.integers(mlo, mhi + 1))
        if cfg.choice == "all":
            ids = rng.permutation(cfg.n_tables).astype(np.int32)
        elif cfg.choice == "uniform":
            ids = rng.choice(cfg.n_tables, size=m, replace=False).astype(np.int32)
            rng.shuffle(ids)
        elif cfg.choice == "zipf":
            ids = _zipf_pick(rng, cfg.n_tables, m, cfg.zipf_s)
        elif cfg.choice == "db":
            n_db = cfg.n_tables // cfg.db_size
            db = int(_zipf_pick(rng, n_db, 1, cfg.zipf_s)[0])
            ids = (db * cfg.db_size + rng.choice(cfg.db_size, size=min(m, cfg.db_size), replace=False)).astype(np.int32)
        else:
            raise ValueError(cfg.choice)
        queries.append(ids)
    slo, shi = cfg.suffix_len
    suffix_len = rng.integers(slo, shi + 1, size=cfg.batch).astype(np.int32)
    return Workload(cfg, table_len, queries, suffix_len)


def get(name: str) -> Workload:
    return make_workload(CONFIGS[name])
