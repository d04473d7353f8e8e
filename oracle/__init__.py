"""CPU checker ("oracle") for the TableCache online path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; it is
used by ``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline``
leg of ``bench.py``.  It shares no code with the HIP library: the fp64
arithmetic lives in ``tc_oracle.c`` (gcc, OpenMP), the integer models
(block allocation, cache replacement) are the plain Python below.

Pieces and the passages they follow:

* ``stitch``            Sec. 4.1.2 (matched tables' KV concatenated in match order)
* ``prefill_attn``      App. E.4 (the uncached part attends to all preceding table
                        content) with the suffix causal to itself
* ``SeqBlockModel``     the paged-pool bookkeeping the library documents: lowest
                        free block first, queries in batch order
* ``SlotModel`` / ``alias_block_table``           the same concatenation without a copy: the
                        sequence's block table points at the table slots' blocks
* ``LRUModel`` / ``FIFOModel`` / ``LFUModel``   App. A, the three replacement rules
* ``plan_pipeline`` / ``simulate_pipeline``      Sec. 4.2.2, micro-batches b_c / b_m

Parity status: every function here is pinned by ``tests/test_oracle_*.py``
(library causal attention, closed forms, brute-force masks, position-coded
gathers, hand-worked replacement traces under ``tests/golden/``).  What is
not pinned, because it needs the paper's datasets, weights and engines: any
statement about end-to-end accuracy or TTFT ("parity unpinned").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tc_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile tc_oracle.c with the host compiler (never hipcc)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_concat_tokens.restype = ctypes.c_int64
        lib.orc_concat_tokens.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p]
        lib.orc_prefill_attn.restype = ctypes.c_int
        lib.orc_prefill_attn.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int32] * 5 + \
            [ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_reencode_keys.restype = ctypes.c_int
        lib.orc_reencode_keys.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_void_p, ctypes.c_double]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


# ----------------------------------------------------------------------------- O1: gather

def stitch(tables: Dict[int, np.ndarray], ids: Sequence[int]) -> np.ndarray:
    """Stitched sequence of one query.

    ``tables[t]`` is table t's K (or V) as [L][n_t][Hkv][D] in any storage type;
    the result is [L][P][Hkv][D] with P = sum of the selected tables' lengths,
    segments in the order of ``ids`` (a table listed twice is copied twice).
    Byte copy, token by token, layer by layer.
    """
    lib = _load()
    first = tables[int(ids[0])] if len(ids) else next(iter(tables.values()))
    L = first.shape[0]
    row_shape = first.shape[2:]
    row_bytes = int(np.prod(row_shape)) * first.dtype.itemsize
    n_tok = np.array([tables[int(t)].shape[1] for t in ids], dtype=np.int32)
    P = int(n_tok.sum())
    out = np.empty((L, P) + tuple(row_shape), dtype=first.dtype)
    segs = [np.ascontiguousarray(tables[int(t)]) for t in ids]
    for l in range(L):
        ptrs = (ctypes.c_void_p * max(len(ids), 1))()
        for j, s in enumerate(segs):
            ptrs[j] = s[l].ctypes.data
        n = lib.orc_concat_tokens(ptrs, n_tok.ctypes.data, len(ids), row_bytes,
                                  out[l].ctypes.data if P else None)
        assert n == P
    return out


def reencode_keys(k: np.ndarray, positions: Sequence[int], theta: float) -> np.ndarray:
    """Rotary re-encoding of position-free keys (Sec. 4.1.1): k is [n][H][D] (any float
    type, widened exactly to fp64), positions[t] the global position of token t in the
    concatenated sequence.  Returns the encoded keys, fp64."""
    lib = _load()
    out = np.array(k, dtype=np.float64, order="C", copy=True)
    pos = np.ascontiguousarray(positions, dtype=np.int64)
    n, H, D = out.shape
    assert pos.shape == (n,)
    rc = lib.orc_reencode_keys(out.ctypes.data, n, H, D, pos.ctypes.data, float(theta))
    if rc != 0:
        raise ValueError("orc_reencode_keys: bad arguments")
    return out


# ----------------------------------------------------------------------------- O3: attention

def prefill_attn(q: np.ndarray, k_seq: np.ndarray, v_seq: np.ndarray,
                 k_new: np.ndarray, v_new: np.ndarray, sm_scale: float,
                 return_weights: bool = False):
    """One query, one layer, fp64.  q [S][Hq][D]; k_seq/v_seq [P][Hkv][D];
    k_new/v_new [S][Hkv][D].  Returns out [S][Hq][D] (and the softmax weights
    [S][Hq][P+S] when asked)."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float64)
    k_seq = np.ascontiguousarray(k_seq, dtype=np.float64)
    v_seq = np.ascontiguousarray(v_seq, dtype=np.float64)
    k_new = np.ascontiguousarray(k_new, dtype=np.float64)
    v_new = np.ascontiguousarray(v_new, dtype=np.float64)
    S, Hq, D = q.shape
    P, Hkv, _ = k_seq.shape
    assert k_new.shape == (S, Hkv, D) and v_new.shape == (S, Hkv, D) and v_seq.shape == k_seq.shape
    out = np.zeros((S, Hq, D), dtype=np.float64)
    w = np.zeros((S, Hq, P + S), dtype=np.float64) if return_weights else None
    rc = lib.orc_prefill_attn(q.ctypes.data, k_seq.ctypes.data, v_seq.ctypes.data,
                              k_new.ctypes.data, v_new.ctypes.data, P, S, Hq, Hkv, D,
                              float(sm_scale), out.ctypes.data,
                              w.ctypes.data if w is not None else None)
    if rc != 0:
        raise RuntimeError("orc_prefill_attn failed: %d" % rc)
    return (out, w) if return_weights else out


def attn_row(q_row: np.ndarray, keys: np.ndarray, values: np.ndarray, sm_scale: float) -> np.ndarray:
    """One output row from its visible keys/values ([n][D] each), fp64: the same
    definition for spot checks at sizes where whole layers are too slow."""
    q_row = np.asarray(q_row, dtype=np.float64)
    s = sm_scale * (np.asarray(keys, dtype=np.float64) @ q_row)
    w = np.exp(s - s.max())
    return (w / w.sum()) @ np.asarray(values, dtype=np.float64)


# ----------------------------------------------------------------------------- O2: block tables

class SeqBlockModel:
    """Bookkeeping model of the sequence region of the paged pool.

    Physical blocks ``first .. first+n-1``; an allocation always takes the
    lowest-numbered free block; queries are served in batch order and each
    query's logical blocks in ascending order; a failed batch allocates nothing.
    """

    def __init__(self, first_block: int, n_blocks: int, block_size: int = 16):
        self.free = sorted(range(first_block, first_block + n_blocks))
        self.bs = block_size

    def stitch(self, prefix_len: Sequence[int], suffix_len: Sequence[int], max_blocks: int):
        need = [-(-(int(p) + int(s)) // self.bs) for p, s in zip(prefix_len, suffix_len)]
        if sum(need) > len(self.free) or any(n > max_blocks for n in need):
            return None
        bt = np.full((len(need), max_blocks), -1, dtype=np.int32)
        for i, n in enumerate(need):
            for j in range(n):
                bt[i, j] = self.free.pop(0)
        return bt

    def release(self, block_table: np.ndarray):
        for b in block_table.reshape(-1):
            if b >= 0:
                self.free.append(int(b))
        self.free.sort()


class SlotModel:
    """Which slot of the device cache holds which table, as the library documents it: on a miss the
    table takes the lowest free slot, or, if the rule evicted a table, that table's slot.  Fed with
    the (table, hit, evicted) trace of a replacement model."""

    def __init__(self, capacity: int):
        self.free = list(range(capacity))
        self.slot: Dict[int, int] = {}

    def apply(self, trace) -> None:
        for t, hit, ev in trace:
            if hit:
                continue
            s = self.slot.pop(int(ev)) if ev >= 0 else self.free.pop(0)
            self.slot[int(t)] = s


def alias_block_table(seq_model: "SeqBlockModel", slot_of: Dict[int, int], table_len: Sequence[int],
                      queries: Sequence[Sequence[int]], suffix_len: Sequence[int], slot_blocks: int,
                      max_blocks: int):
    """Sec. 4.1.2's concatenation made in the block table alone (nothing is copied): query i lists,
    table by table in match order, the blocks of the slots holding its tables (slot s owns blocks
    s*slot_blocks ..; a table of n tokens uses the first ceil(n/16)), then ceil(S_i/16) fresh
    sequence blocks for the suffix, lowest free first, queries in batch order.
    Returns (block_table [B][max_blocks] with -1 for unused, padded prefix lengths [B],
    valid [B] lists: how many token positions of each prefix block hold a token)."""
    bs = seq_model.bs
    bt = np.full((len(queries), max_blocks), -1, dtype=np.int32)
    padded, valid = [], []
    for i, q in enumerate(queries):
        row, val = [], []
        for t in q:
            n = int(table_len[int(t)])
            nb = -(-n // bs)
            row += [slot_of[int(t)] * slot_blocks + j for j in range(nb)]
            val += [bs] * (nb - 1) + [n - bs * (nb - 1)]
        padded.append(bs * len(row))
        valid.append(val)
        row += [seq_model.free.pop(0) for _ in range(-(-int(suffix_len[i]) // bs))]
        bt[i, :len(row)] = row
    return bt, np.array(padded, dtype=np.int32), valid


def prefix_lengths(table_len: Sequence[int], table_ids: Sequence[int], cu_tables: Sequence[int]):
    """P_i = sum of the lengths of query i's tables (Sec. 4.1.2 concatenation)."""
    return np.array([sum(int(table_len[int(t)]) for t in table_ids[cu_tables[i]:cu_tables[i + 1]])
                     for i in range(len(cu_tables) - 1)], dtype=np.int32)


# ----------------------------------------------------------------------------- O4: replacement

class LRUModel:
    """App. A, LRU: hit -> move to the front; miss -> evict the end if |cache| >= C,
    insert at the front.  ``access`` returns (hit, evicted or None).

    `pinned` (all three models): tables that may not be evicted now, because a query that is
    about to be stitched uses them (Sec. 4.2.2 loads a micro-batch ahead of its computation;
    all its tables must still be there).  The victim is then the rule's first choice among the
    other tables; with nothing pinned the rule is App. A's as printed."""

    def __init__(self, capacity: int):
        self.C = capacity
        self.items: List[int] = []          # index 0 = front

    def access(self, t: int, pinned=()) -> Tuple[bool, Optional[int]]:
        if t in self.items:
            self.items.remove(t)
            self.items.insert(0, t)
            return True, None
        ev = None
        if len(self.items) >= self.C:
            ev = [x for x in self.items if x not in pinned][-1]     # IndexError: everything is pinned
            self.items.remove(ev)
        self.items.insert(0, t)
        return False, ev


class FIFOModel:
    """App. A, FIFO: miss -> evict the head if full, enqueue at the tail; hit -> nothing."""

    def __init__(self, capacity: int):
        self.C = capacity
        self.items: List[int] = []          # index 0 = head

    def access(self, t: int, pinned=()) -> Tuple[bool, Optional[int]]:
        if t in self.items:
            return True, None
        ev = None
        if len(self.items) >= self.C:
            ev = [x for x in self.items if x not in pinned][0]
            self.items.remove(ev)
        self.items.append(t)
        return False, ev


class LFUModel:
    """App. A, LFU: hit -> frequency+1, timestamp=now; miss -> evict the smallest
    frequency (ties: smallest timestamp) if full, insert (1, now).  The timestamp
    is the running access counter."""

    def __init__(self, capacity: int):
        self.C = capacity
        self.items: Dict[int, Tuple[int, int]] = {}
        self.now = 0

    def access(self, t: int, pinned=()) -> Tuple[bool, Optional[int]]:
        self.now += 1
        if t in self.items:
            f, _ = self.items[t]
            self.items[t] = (f + 1, self.now)
            return True, None
        ev = None
        if len(self.items) >= self.C:
            ev = min((x for x in self.items if x not in pinned), key=lambda x: self.items[x])
            del self.items[ev]
        self.items[t] = (1, self.now)
        return False, ev


def replay(model, accesses: Sequence[int]) -> List[Tuple[int, int, int]]:
    """Trace of (table, hit as 0/1, evicted or -1) for an access stream."""
    out = []
    for t in accesses:
        hit, ev = model.access(int(t))
        out.append((int(t), int(hit), -1 if ev is None else int(ev)))
    return out


# ----------------------------------------------------------------------------- Sec. 4.2.2: pipeline schedule

def plan_pipeline(table_sets: Sequence[Sequence[int]], capacity: int, b_c: int, b_m: int,
                  keep_pinned: bool = False, taper: bool = False):
    """Sec. 4.2.2, computation-loading pipeline over an ordered batch: the requests are computed
    b_c at a time, and while a micro-batch is computed the tables of the next b_m requests are
    copied in.  Returns one tuple per micro-batch,
        (compute_begin, compute_end, demand_begin, demand_end, prefetch_begin, prefetch_end):
    `demand` are the requests of this micro-batch nobody has asked for yet (asked for right
    before its stitch), `prefetch` those asked for right after its stitch.  Requests asked for
    but not yet stitched keep their tables pinned, so a prefetch stops early where the union of
    their tables would outgrow the cache; for the same reason a micro-batch holds fewer than b_c
    requests where the tables of b_c would not fit together (the next one starts there).
    `keep_pinned`: the micro-batch being computed keeps its tables pinned as well (a stitch that
    points at the cached tables instead of copying them), so they count while the prefetch is sized.
    `taper`: near the end a micro-batch takes min(b_c, max(1, remaining // 2)) requests, so the
    computation left over when the last copy has landed is that of one request."""
    N, steps, asked, c0 = len(table_sets), [], 0, 0
    uni = lambda a, b: set().union(*[set(map(int, x)) for x in table_sets[a:b]]) if b > a else set()
    while c0 < N:
        size = min(b_c, max(1, (N - c0) // 2)) if taper else b_c
        full = min(N, c0 + size)
        d0 = asked
        # requests c0..asked-1 are here already; ask for more of this micro-batch while they fit
        while asked < full and len(uni(c0, asked + 1)) <= capacity:
            asked += 1
        c1 = min(asked, full)
        if c1 == c0:
            raise ValueError("request %d alone needs more than %d tables" % (c0, capacity))
        d1 = p0 = asked
        while asked < N and asked < c1 + b_m and len(uni(c0 if keep_pinned else c1, asked + 1)) <= capacity:
            asked += 1
        steps.append((c0, c1, d0, d1, p0, asked))
        c0 = c1
    return steps


def simulate_pipeline(model, table_sets: Sequence[Sequence[int]], steps,
                      keep_pinned: bool = False) -> List[Tuple[int, int, int]]:
    """Access trace (table, hit, evicted or -1) of the replacement model when the schedule of
    `plan_pipeline` is carried out: a range of requests is asked for by pinning all its tables
    and then requesting them in order; a micro-batch is unpinned once it is stitched (or, with
    `keep_pinned`, after the prefetch behind it has been asked for)."""
    pins: Dict[int, int] = {}
    out = []

    def ask(a, b):
        ids = [int(t) for q in table_sets[a:b] for t in q]
        for t in ids:
            pins[t] = pins.get(t, 0) + 1
        for t in ids:
            hit, ev = model.access(t, pinned=pins)
            out.append((t, int(hit), -1 if ev is None else int(ev)))

    def unpin(a, b):
        for q in table_sets[a:b]:
            for t in q:
                pins[int(t)] -= 1
                if pins[int(t)] == 0:
                    del pins[int(t)]

    for c0, c1, d0, d1, p0, p1 in steps:
        ask(d0, d1)
        if not keep_pinned:
            unpin(c0, c1)
        ask(p0, p1)
        if keep_pinned:
            unpin(c0, c1)
    return out


# ----------------------------------------------------------------------------- front end (upstream of the path)

def trie_match(tables: Dict[int, Sequence[int]], s: Sequence[int]) -> List[Tuple[int, int]]:
    """Alg. 1 (Table Trie Matching) by brute force, without a trie: scan the prompt's token
    sequence `s` from p = 0; at p, among the tables whose whole token content equals
    s[p : p + len], take the longest (Sec. 4.1.2: longest prefix match, exact match of a table);
    found -> record (table id, p) and continue at the end of the match, else p + 1.
    Returns the matches in order.  `tables` maps table id -> token ids (non-empty, distinct)."""
    s = list(s)
    out, p = [], 0
    while p < len(s):
        best_id, best_len = None, 0
        for tid, toks in tables.items():
            n = len(toks)
            if n > best_len and p + n <= len(s) and all(s[p + k] == toks[k] for k in range(n)):
                best_id, best_len = tid, n
        if best_id is None:
            p += 1
        else:
            out.append((best_id, p))
            p += best_len
    return out


def rerank(table_sets: Sequence[Sequence[int]], anchor: int) -> List[int]:
    """Query reranking (Sec. 4.2.1, Eq. 1-2) by brute force with Python sets: start from the
    anchor query; repeatedly move to the remaining query whose table set differs least from the
    current one's - the distance of Eq. 2 is the size of the symmetric difference - lowest index
    on ties.  Returns the visiting order (a permutation of the query indices)."""
    sets = [frozenset(int(t) for t in ts) for ts in table_sets]
    n = len(sets)
    if n == 0:
        return []
    left = [i for i in range(n) if i != anchor]
    order, cur = [anchor], anchor
    while left:
        best = min(left, key=lambda j: (len(sets[cur] ^ sets[j]), j))
        left.remove(best)
        order.append(best)
        cur = best
    return order
