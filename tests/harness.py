"""Shared set-up for the GPU parity tests: put a synthetic workload on the device
through the C ABI, and compute the same thing with the CPU checker."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2601_08743_amd import workloads as W


def np_dtype(cfg):
    return np.float32 if cfg.dtype == "f32" else np.uint16


def to_dev(a: np.ndarray, cfg):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if cfg.dtype == "bf16":
        t = t.view(torch.bfloat16)
    return t.cuda()


def out_to_f64(t: torch.Tensor, cfg) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class DeviceWorkload:
    """A workload registered with a library context; tables loaded into the device cache."""

    def __init__(self, wl: W.Workload, seq_blocks: int = None, capacity: int = None,
                 policy: int = 0, load_all: bool = True, tables=None, slot_layout: int = 0):
        from paper_2601_08743_amd import binding as B
        self.B = B
        self.wl = wl
        c = wl.cfg
        self.cfg = c
        cap = c.capacity if capacity is None else capacity
        max_tok = int(wl.table_len.max())
        slot_blocks = -(-max_tok // 16)
        if seq_blocks is None:
            P = [int(wl.table_len[q].sum()) for q in wl.queries]
            seq_blocks = sum(-(-(p + int(s)) // 16) for p, s in zip(P, wl.suffix_len)) + 8
        n_blocks = cap * slot_blocks + seq_blocks
        self.tc_cfg = B.make_config(c.n_layers, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                    B.TC_F32 if c.dtype == "f32" else B.TC_BF16, n_blocks, cap,
                                    max_tok, policy, slot_layout=slot_layout)
        self.slot_blocks = slot_blocks
        nbytes = B.tc_pool_bytes(self.tc_cfg)
        assert nbytes > 0
        # poison the pool: NaN patterns in both element types, so that any slot read without
        # having been written shows up
        self.pool = torch.full((nbytes // 4,), 0x7FC07FC0, dtype=torch.int32, device="cuda")
        self.ctx = B.Context(self.tc_cfg, self.pool, nbytes)
        self.first_seq = B.tc_first_seq_block(self.tc_cfg)
        self.seq_blocks = seq_blocks
        self.host_kv = {}
        self.tables_np = {}
        ids = range(c.n_tables) if tables is None else tables
        for t in ids:
            k, v = wl.table_kv(t)
            self.tables_np[t] = (k, v)
            hk = torch.from_numpy(k).pin_memory()
            hv = torch.from_numpy(v).pin_memory()
            self.host_kv[t] = (hk, hv)
            self.ctx.tc_register_table_kv(t, int(wl.table_len[t]), hk, hv)
        if load_all:
            self.ctx.tc_load_async(list(ids), 0, c.n_layers, None)
            torch.cuda.synchronize()

    def stitch(self, max_blocks: int = None, stream=None):
        wl = self.wl
        if max_blocks is None:
            P = [int(wl.table_len[q].sum()) for q in wl.queries]
            max_blocks = max(-(-(p + int(s)) // 16) for p, s in zip(P, wl.suffix_len)) + 1
        bt, pl = self.ctx.tc_stitch_kv(wl.table_ids, wl.cu_tables, wl.suffix_len, max_blocks, stream)
        return bt, pl

    def alias(self, max_blocks: int = None, stream=None):
        """The batch's sequences made by pointing at the table slots' blocks (block-format slots)."""
        wl = self.wl
        if max_blocks is None:
            max_blocks = max(sum(-(-int(wl.table_len[t]) // 16) for t in q) + -(-int(s) // 16)
                             for q, s in zip(wl.queries, wl.suffix_len)) + 1
        return self.ctx.tc_stitch_alias(wl.table_ids, wl.cu_tables, wl.suffix_len, max_blocks, stream)

    def attn_layer(self, layer: int, bt, pl, stream=None, qkv=None):
        wl, c = self.wl, self.cfg
        q, k, v = wl.suffix_qkv(layer) if qkv is None else qkv
        dq, dk, dv = to_dev(q, c), to_dev(k, c), to_dev(v, c)
        out = torch.full_like(dq, float("nan"))
        self.ctx.tc_prefill_attn(layer, dq, dk, dv, out, wl.cu_seqlens, bt, pl, wl.suffix_len,
                                 wl.sm_scale, stream)
        torch.cuda.synchronize()
        return out, (q, k, v)

    def close(self):
        torch.cuda.synchronize()
        self.ctx.tc_destroy()


def oracle_sequences(wl: W.Workload, tables_np, layer: int, query: int):
    """Stitched K and V of one query in one layer, storage type, [P][Hkv][D]."""
    ids = wl.queries[query]
    tk = {int(t): tables_np[int(t)][0][layer:layer + 1] for t in ids}
    tv = {int(t): tables_np[int(t)][1][layer:layer + 1] for t in ids}
    if len(ids) == 0:
        c = wl.cfg
        z = np.zeros((0, c.n_kv_heads, c.head_dim), dtype=np_dtype(c))
        return z, z.copy()
    return oracle.stitch(tk, ids)[0], oracle.stitch(tv, ids)[0]


def oracle_attn_layer(wl: W.Workload, tables_np, layer: int, qkv, queries=None) -> dict:
    """fp64 outputs per query: {i: [S_i][Hq][D]}."""
    c = wl.cfg
    q, k, v = qkv
    cu = wl.cu_seqlens
    res = {}
    for i in (range(c.batch) if queries is None else queries):
        ks, vs = oracle_sequences(wl, tables_np, layer, i)
        sl = slice(int(cu[i]), int(cu[i + 1]))
        res[i] = oracle.prefill_attn(W.storage_to_f64(q[sl], c.dtype), W.storage_to_f64(ks, c.dtype),
                                     W.storage_to_f64(vs, c.dtype), W.storage_to_f64(k[sl], c.dtype),
                                     W.storage_to_f64(v[sl], c.dtype), wl.sm_scale)
    return res
