"""ctypes binding over libtablecache.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/tablecache.h for the semantics).  Device tensors are passed as torch
tensors (their ``data_ptr()`` is used) or raw integer addresses; host integer
arrays are numpy int32.  There is no fallback: if the library has not been
built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np
# torch first, always: the library needs libamdhip64.so.7 and must bind to the copy torch ships and
# has initialised.  Loaded before torch, it would pull in the system's copy instead, the process
# would hold two HIP runtimes, and the second one finds no device.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtablecache.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libtablecache.so is not built (%s). Run `python -m paper_2601_08743_amd.build` "
        "(or __graft_entry__.build()); there is no CPU fallback." % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)

TC_OK = 0
TC_ERR_INVALID, TC_ERR_UNKNOWN_TABLE, TC_ERR_OOM_POOL = -1, -2, -3
TC_ERR_NOT_RESIDENT, TC_ERR_CAPACITY, TC_ERR_HIP = -4, -5, -6
TC_F32, TC_BF16 = 0, 1
TC_POLICY_LRU, TC_POLICY_FIFO, TC_POLICY_LFU = 0, 1, 2
TC_SLOTS_ROWS, TC_SLOTS_BLOCKS = 0, 1

EXPORTS = ["tc_block_bytes", "tc_pool_bytes", "tc_first_seq_block", "tc_create", "tc_destroy",
           "tc_register_table_kv", "tc_load_async", "tc_load_trace", "tc_is_resident",
           "tc_stitch_kv", "tc_stitch_kv_rope", "tc_stitch_alias", "tc_prefill_attn", "tc_prefill_attn_noalloc", "tc_grow_seqs", "tc_release_seqs", "tc_read_seq_kv",
           "tc_kv_splits", "tc_set_kv_splits", "tc_set_row_blocks", "tc_set_attn_kernel", "tc_attn_kernel", "tc_profile_enable", "tc_profile_read", "tc_last_error", "tc_version",
           "tc_trie_create", "tc_trie_destroy", "tc_trie_insert", "tc_trie_match", "tc_rerank",
           "tc_pin_tables", "tc_unpin_tables", "tc_plan_pipeline"]


class tc_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("n_pool_blocks", ctypes.c_int64), ("table_capacity", ctypes.c_int32),
                ("max_table_tokens", ctypes.c_int32), ("policy", ctypes.c_int32),
                ("slot_layout", ctypes.c_int32)]


_vp, _i32, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
_cfgp = ctypes.POINTER(tc_config)
_sig = {
    "tc_block_bytes": (ctypes.c_size_t, [_cfgp]),
    "tc_pool_bytes": (ctypes.c_size_t, [_cfgp]),
    "tc_first_seq_block": (_i64, [_cfgp]),
    "tc_create": (_i32, [_cfgp, _vp, ctypes.c_size_t, ctypes.POINTER(_vp)]),
    "tc_destroy": (_i32, [_vp]),
    "tc_register_table_kv": (_i32, [_vp, _i32, _i32, _vp, _vp]),
    "tc_load_async": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp]),
    "tc_load_trace": (_i32, [_vp, _vp, _i32]),
    "tc_is_resident": (_i32, [_vp, _i32, _i32, _i32]),
    "tc_stitch_kv": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp]),
    "tc_stitch_alias": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp]),
    "tc_stitch_kv_rope": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, ctypes.c_double, _vp, _i32, _vp, _vp]),
    "tc_prefill_attn": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32,
                               ctypes.c_float, _vp]),
    "tc_prefill_attn_noalloc": (_i32, [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32,
                                       ctypes.c_float, _vp]),
    "tc_grow_seqs": (_i32, [_vp, _vp, _i32, _i32, _vp]),
    "tc_release_seqs": (_i32, [_vp, _vp, _i32, _i32]),
    "tc_read_seq_kv": (_i32, [_vp, _i32, _vp, _i32, _vp, _vp, _vp]),
    "tc_kv_splits": (_i32, [_vp]),
    "tc_set_kv_splits": (_i32, [_vp, _i32]),
    "tc_set_row_blocks": (_i32, [_vp, _i32]),
    "tc_set_attn_kernel": (_i32, [_vp, _i32]),
    "tc_attn_kernel": (_i32, [_vp]),
    "tc_profile_enable": (_i32, [_vp, _i32]),
    "tc_profile_read": (_i32, [_vp, _vp, _vp]),
    "tc_last_error": (ctypes.c_char_p, [_vp]),
    "tc_version": (ctypes.c_char_p, []),
    "tc_trie_create": (_vp, []),
    "tc_trie_destroy": (None, [_vp]),
    "tc_trie_insert": (_i32, [_vp, _i32, _vp, _i32]),
    "tc_trie_match": (_i32, [_vp, _vp, _i32, _vp, _vp, _i32]),
    "tc_rerank": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp]),
    "tc_pin_tables": (_i32, [_vp, _vp, _i32]),
    "tc_unpin_tables": (_i32, [_vp, _vp, _i32]),
    "tc_plan_pipeline": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _i32]),
}
for _n, (_r, _a) in _sig.items():
    getattr(_lib, _n).restype = _r
    getattr(_lib, _n).argtypes = _a


class TcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("tc error %d: %s" % (code, msg))
        self.code = code


def _ptr(x) -> Optional[int]:
    """Address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _i32arr(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.int32)


def _stream(s) -> Optional[int]:
    if s is None or isinstance(s, int):
        return s
    return s.cuda_stream       # torch.cuda.Stream


def make_config(n_layers, n_q_heads, n_kv_heads, head_dim, dtype, n_pool_blocks, table_capacity,
                max_table_tokens, policy=TC_POLICY_LRU, block_size=16, slot_layout=TC_SLOTS_ROWS) -> tc_config:
    return tc_config(n_layers, n_q_heads, n_kv_heads, head_dim, block_size, dtype, n_pool_blocks,
                     table_capacity, max_table_tokens, policy, slot_layout)


def tc_block_bytes(cfg: tc_config) -> int:
    return int(_lib.tc_block_bytes(ctypes.byref(cfg)))


def tc_pool_bytes(cfg: tc_config) -> int:
    return int(_lib.tc_pool_bytes(ctypes.byref(cfg)))


def tc_first_seq_block(cfg: tc_config) -> int:
    return int(_lib.tc_first_seq_block(ctypes.byref(cfg)))


def tc_version() -> str:
    return _lib.tc_version().decode()


class Context:
    """Owner of a tc_ctx*; methods are the C calls of the same name."""

    def __init__(self, cfg: tc_config, kv_pool, pool_bytes: Optional[int] = None):
        self.cfg = cfg
        self._pool = kv_pool                      # keep the caller's buffer alive
        if pool_bytes is None:
            pool_bytes = kv_pool.numel() * kv_pool.element_size()
        h = _vp()
        rc = _lib.tc_create(ctypes.byref(cfg), _ptr(kv_pool), pool_bytes, ctypes.byref(h))
        if rc != TC_OK:
            raise TcError(rc, "tc_create failed")
        self._h = h
        self._keep = []                           # registered host KV

    def _check(self, rc: int):
        if rc != TC_OK:
            raise TcError(rc, _lib.tc_last_error(self._h).decode())

    def tc_destroy(self):
        if self._h:
            _lib.tc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.tc_destroy()
        except Exception:
            pass

    def tc_register_table_kv(self, table_id: int, n_tokens: int, host_k, host_v):
        self._keep.append((host_k, host_v))
        self._check(_lib.tc_register_table_kv(self._h, table_id, n_tokens, _ptr(host_k), _ptr(host_v)))

    def tc_load_async(self, table_ids, l0: int, l1: int, stream=None):
        ids = _i32arr(table_ids)
        self._check(_lib.tc_load_async(self._h, ids.ctypes.data, ids.size, l0, l1, _stream(stream)))

    def tc_pin_tables(self, table_ids):
        ids = _i32arr(table_ids)
        self._check(_lib.tc_pin_tables(self._h, ids.ctypes.data, ids.size))

    def tc_unpin_tables(self, table_ids):
        ids = _i32arr(table_ids)
        self._check(_lib.tc_unpin_tables(self._h, ids.ctypes.data, ids.size))

    def tc_load_trace(self, cap: int = 1 << 16) -> np.ndarray:
        out = np.zeros((cap, 3), dtype=np.int32)
        n = _lib.tc_load_trace(self._h, out.ctypes.data, cap)
        if n < 0:
            raise TcError(n, "tc_load_trace")
        return out[:n]

    def tc_is_resident(self, table_id: int, l0: int, l1: int) -> bool:
        return bool(_lib.tc_is_resident(self._h, table_id, l0, l1))

    def tc_stitch_kv(self, table_ids, cu_tables, suffix_len, max_blocks: int,
                     stream=None) -> Tuple[np.ndarray, np.ndarray]:
        ids, cu, sl = _i32arr(table_ids), _i32arr(cu_tables), _i32arr(suffix_len)
        B = cu.size - 1
        bt = np.full((B, max_blocks), -7, dtype=np.int32)
        pl = np.full((B,), -7, dtype=np.int32)
        self._check(_lib.tc_stitch_kv(self._h, ids.ctypes.data, cu.ctypes.data, B, sl.ctypes.data,
                                      bt.ctypes.data, max_blocks, pl.ctypes.data, _stream(stream)))
        return bt, pl

    def tc_stitch_alias(self, table_ids, cu_tables, suffix_len, max_blocks: int,
                        stream=None) -> Tuple[np.ndarray, np.ndarray]:
        ids, cu, sl = _i32arr(table_ids), _i32arr(cu_tables), _i32arr(suffix_len)
        B = cu.size - 1
        bt = np.full((B, max_blocks), -7, dtype=np.int32)
        pl = np.full((B,), -7, dtype=np.int32)
        self._check(_lib.tc_stitch_alias(self._h, ids.ctypes.data, cu.ctypes.data, B, sl.ctypes.data,
                                         bt.ctypes.data, max_blocks, pl.ctypes.data, _stream(stream)))
        return bt, pl

    def tc_stitch_kv_rope(self, table_ids, cu_tables, suffix_len, pos0, rope_theta: float, max_blocks: int,
                          stream=None) -> Tuple[np.ndarray, np.ndarray]:
        ids, cu, sl = _i32arr(table_ids), _i32arr(cu_tables), _i32arr(suffix_len)
        B = cu.size - 1
        p0 = None if pos0 is None else _i32arr(pos0)
        bt = np.full((B, max_blocks), -7, dtype=np.int32)
        pl = np.full((B,), -7, dtype=np.int32)
        self._check(_lib.tc_stitch_kv_rope(self._h, ids.ctypes.data, cu.ctypes.data, B, sl.ctypes.data,
                                           None if p0 is None else p0.ctypes.data, float(rope_theta),
                                           bt.ctypes.data, max_blocks, pl.ctypes.data, _stream(stream)))
        return bt, pl

    def tc_prefill_attn(self, layer: int, q, k_new, v_new, out, cu_seqlens, block_table,
                        prefix_len, suffix_len, sm_scale: float, stream=None):
        cu, bt = _i32arr(cu_seqlens), _i32arr(block_table)
        pl, sl = _i32arr(prefix_len), _i32arr(suffix_len)
        B = pl.size
        max_blocks = bt.shape[1] if bt.ndim == 2 else (bt.size // B if B else 0)
        self._check(_lib.tc_prefill_attn(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                         cu.ctypes.data, bt.ctypes.data, max_blocks, pl.ctypes.data,
                                         sl.ctypes.data, B, sm_scale, _stream(stream)))

    def tc_prefill_attn_noalloc(self, layer: int, q, k_new, v_new, out, cu_seqlens, block_table,
                                prefix_len, suffix_len, sm_scale: float, stream=None):
        cu, bt = _i32arr(cu_seqlens), _i32arr(block_table)
        pl, sl = _i32arr(prefix_len), _i32arr(suffix_len)
        B = pl.size
        max_blocks = bt.shape[1] if bt.ndim == 2 else (bt.size // B if B else 0)
        self._check(_lib.tc_prefill_attn_noalloc(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                 cu.ctypes.data, bt.ctypes.data, max_blocks, pl.ctypes.data,
                                                 sl.ctypes.data, B, sm_scale, _stream(stream)))

    def tc_grow_seqs(self, block_table: np.ndarray, new_len) -> np.ndarray:
        """Returns the grown block table (a copy; the argument is left alone)."""
        bt = np.ascontiguousarray(block_table, dtype=np.int32).copy()
        nl = _i32arr(new_len)
        self._check(_lib.tc_grow_seqs(self._h, bt.ctypes.data, bt.shape[1], bt.shape[0], nl.ctypes.data))
        return bt

    def tc_release_seqs(self, block_table):
        bt = _i32arr(block_table)
        B = bt.shape[0] if bt.ndim == 2 else 1
        mb = bt.shape[1] if bt.ndim == 2 else bt.size
        self._check(_lib.tc_release_seqs(self._h, bt.ctypes.data, mb, B))

    def tc_read_seq_kv(self, layer: int, blocks, n_tokens: int, np_dtype, stream=None):
        c = self.cfg
        blk = _i32arr(blocks)
        k = np.zeros((n_tokens, c.n_kv_heads, c.head_dim), dtype=np_dtype)
        v = np.zeros_like(k)
        self._check(_lib.tc_read_seq_kv(self._h, layer, blk.ctypes.data, n_tokens, k.ctypes.data,
                                        v.ctypes.data, _stream(stream)))
        return k, v

    def tc_kv_splits(self) -> int:
        return int(_lib.tc_kv_splits(self._h))

    def tc_set_kv_splits(self, n: int):
        self._check(_lib.tc_set_kv_splits(self._h, n))

    def tc_set_row_blocks(self, n: int):
        self._check(_lib.tc_set_row_blocks(self._h, n))

    def tc_attn_kernel(self) -> int:
        return int(_lib.tc_attn_kernel(self._h))

    def tc_set_attn_kernel(self, kind: int):
        self._check(_lib.tc_set_attn_kernel(self._h, kind))

    def tc_profile_enable(self, on: bool):
        self._check(_lib.tc_profile_enable(self._h, int(on)))

    def tc_profile_read(self):
        """{kind: (total ms, launches)} for stitch / append / attn / merge since the last read."""
        ms = np.zeros(4, dtype=np.float64)
        n = np.zeros(4, dtype=np.int64)
        self._check(_lib.tc_profile_read(self._h, ms.ctypes.data, n.ctypes.data))
        return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(("stitch", "append", "attn", "merge"))}

    def tc_last_error(self) -> str:
        return _lib.tc_last_error(self._h).decode()


class Trie:
    """The Table Trie (same-named calls: tc_trie_insert, tc_trie_match)."""

    def __init__(self):
        self._h = _lib.tc_trie_create()
        if not self._h:
            raise MemoryError("tc_trie_create")

    def tc_trie_insert(self, table_id: int, tokens):
        t = _i32arr(tokens)
        rc = _lib.tc_trie_insert(self._h, int(table_id), t.ctypes.data, t.size)
        if rc != TC_OK:
            raise TcError(rc, "tc_trie_insert(%d)" % table_id)

    def tc_trie_match(self, s, cap: int = None):
        """[(table id, start position)] in match order."""
        s = _i32arr(s)
        cap = s.size if cap is None else cap
        ids = np.empty(max(cap, 1), dtype=np.int32)
        st = np.empty(max(cap, 1), dtype=np.int32)
        n = _lib.tc_trie_match(self._h, s.ctypes.data, s.size, ids.ctypes.data, st.ctypes.data, cap)
        if n < 0:
            raise TcError(n, "tc_trie_match")
        k = min(n, cap)
        return list(zip(ids[:k].tolist(), st[:k].tolist())), n

    def tc_trie_destroy(self):
        if self._h:
            _lib.tc_trie_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.tc_trie_destroy()
        except Exception:
            pass


def tc_rerank(table_ids, cu_tables, n_tables: int, anchor: int) -> np.ndarray:
    ids, cu = _i32arr(table_ids), _i32arr(cu_tables)
    n = cu.size - 1
    order = np.full(max(n, 1), -1, dtype=np.int32)
    rc = _lib.tc_rerank(ids.ctypes.data if ids.size else None, cu.ctypes.data, n, int(n_tables), int(anchor),
                        order.ctypes.data)
    if rc != TC_OK:
        raise TcError(rc, "tc_rerank")
    return order[:n]


def tc_plan_pipeline(table_ids, cu_tables, capacity: int, b_c: int, b_m: int, keep_pinned: bool = False,
                     taper: bool = False) -> np.ndarray:
    """Steps as an int32 array [n_steps, 6]: compute, demand and prefetch ranges (begin, end)."""
    ids, cu = _i32arr(table_ids), _i32arr(cu_tables)
    n = cu.size - 1
    cap = max(1, n)
    steps = np.zeros((cap, 6), dtype=np.int32)
    rc = _lib.tc_plan_pipeline(ids.ctypes.data if ids.size else None, cu.ctypes.data, n, int(capacity), int(b_c),
                               int(b_m), int(bool(keep_pinned)), int(bool(taper)), steps.ctypes.data, cap)
    if rc < 0:
        raise TcError(rc, "tc_plan_pipeline")
    return steps[:rc]
