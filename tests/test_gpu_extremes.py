"""GPU: the extremes of size - length, then width.

Length: one query over a single table of 70 001 tokens (1094 key tiles of 64: more than the 1024
tiles the long-launch and the pipelined kernel keep block ids for, more than four times the general
kernel's 256) next to a short one, few heads so that the CPU checker stays fast.  Every kernel must
cut the long query into as many key partitions as its table forces - also when the caller asks for
fewer - and every row of every head must agree with the checker; then one decode step over the
same sequences (the decode kernels' ranges have the 256-tile limit).  Suffixes of 33 key tiles over
short or no prefixes.  Width: 400 short queries in one batch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_08743_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 1e-2
LONG = 70001


@pytest.fixture(scope="module")
def H():
    import harness
    assert torch.cuda.is_available()
    return harness


@pytest.fixture(scope="module")
def setup(H):
    cfg = W.scaled(W.CONFIGS["c2"], name="long", n_layers=1, n_q_heads=4, n_kv_heads=1, n_tables=2, batch=2,
                   tables_per_query=(1, 1), capacity=2, seed=31337)
    wl = W.Workload(cfg, np.asarray([LONG, 100], dtype=np.int32),
                    [np.asarray([0], dtype=np.int32), np.asarray([1], dtype=np.int32)],
                    np.asarray([37, 5], dtype=np.int32))
    qkv = wl.suffix_qkv(0)
    tables = {t: wl.table_kv(t) for t in range(2)}
    ref = H.oracle_attn_layer(wl, tables, 0, qkv)
    return wl, qkv, ref


@pytest.mark.parametrize("kind,forced,least", [(0, 0, 2), (4, 1, 2), (2, 1, 2), (1, 2, 5), (1, 0, 5)])
def test_prefill_over_a_prefix_longer_than_the_block_id_tables(H, setup, kind, forced, least):
    wl, qkv, ref = setup
    dw = H.DeviceWorkload(wl)
    dw.ctx.tc_set_attn_kernel(kind)
    dw.ctx.tc_set_kv_splits(forced)
    bt, pl = dw.stitch()
    np.testing.assert_array_equal(pl, [LONG, 100])
    out, _ = dw.attn_layer(0, bt, pl, qkv=qkv)
    got = H.out_to_f64(out, wl.cfg)
    splits = dw.ctx.tc_kv_splits()
    assert splits >= least, (kind, forced, splits)
    worst = 0.0
    for i, r in ref.items():
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all()
        worst = max(worst, float(np.abs(got[sl] - r).max()))
    print("kernel %d (chosen %d), %d partitions asked, %d made: max-abs err %.2e" % (
        kind, dw.ctx.tc_attn_kernel(), forced, splits, worst))
    assert worst <= TOL
    if kind == 0:                                       # the gather and the append, bit for bit
        for i in range(2):
            n = int(pl[i]) + int(wl.suffix_len[i])
            kk, vv = dw.ctx.tc_read_seq_kv(0, bt[i, :-(-n // 16)], n, np.uint16)
            ks, vs = H.oracle_sequences(wl, dw.tables_np, 0, i)
            sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
            np.testing.assert_array_equal(kk.view(np.uint8), np.concatenate([ks, qkv[1][sl]]).view(np.uint8))
            np.testing.assert_array_equal(vv.view(np.uint8), np.concatenate([vs, qkv[2][sl]]).view(np.uint8))
    dw.ctx.tc_release_seqs(bt)
    dw.close()


def test_decode_step_over_the_long_sequence(H, setup):
    wl, qkv, _ = setup
    c = wl.cfg
    P = np.array([LONG, 100])
    S = wl.suffix_len.astype(int)
    dw = H.DeviceWorkload(wl, seq_blocks=int(sum(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 4)
    max_blocks = int(max(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 1
    bt, pl = dw.stitch(max_blocks=max_blocks)
    dw.attn_layer(0, bt, pl, qkv=qkv)                   # prefill: appends the suffixes to the pool
    cur = (P + S).astype(np.int32)
    bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
    rng = np.random.default_rng(77)
    q, k, v = (W.f32_to_bf16_bits(rng.standard_normal(size=(2, h, c.head_dim), dtype=np.float32))
               for h in (c.n_q_heads, c.n_kv_heads, c.n_kv_heads))
    dq, dk, dv = H.to_dev(q, c), H.to_dev(k, c), H.to_dev(v, c)
    out = torch.full_like(dq, float("nan"))
    dw.ctx.tc_prefill_attn(0, dq, dk, dv, out, np.arange(3, dtype=np.int32), bt, cur, np.ones(2, dtype=np.int32),
                           wl.sm_scale, None)
    torch.cuda.synchronize()
    assert dw.ctx.tc_attn_kernel() == 3
    assert dw.ctx.tc_kv_splits() >= 5                   # 1095 key tiles, at most 256 per work item
    got = H.out_to_f64(out, c)
    worst = 0.0
    for i in range(2):
        ks, vs = H.oracle_sequences(wl, dw.tables_np, 0, i)
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        K = np.concatenate([ks, qkv[1][sl]])
        V = np.concatenate([vs, qkv[2][sl]])
        r = oracle.prefill_attn(W.storage_to_f64(q[i:i + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[i:i + 1], "bf16"),
                                W.storage_to_f64(v[i:i + 1], "bf16"), wl.sm_scale)
        worst = max(worst, float(np.abs(got[i:i + 1] - r).max()))
    print("decode step over %d keys in %d ranges: max-abs err %.2e" % (LONG + 37, dw.ctx.tc_kv_splits(), worst))
    assert worst <= TOL
    dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("kind", [0, 1, 2, 4])
@pytest.mark.parametrize("splits", [0, 3])
def test_long_suffixes(H, kind, splits):
    """The other extreme: suffixes of 33 key tiles (2100 tokens, 8400 rows per KV head in 66 row
    tiles) over no prefix, a prefix shorter than a tile, and one of 1000 tokens - the causal part
    is most of the work, every row tile ends at a different key tile, and the partitions of a split
    query cut through the suffix."""
    cfg = W.scaled(W.CONFIGS["c2"], name="longs", n_layers=1, n_q_heads=8, n_kv_heads=2, n_tables=2, batch=3,
                   tables_per_query=(0, 1), capacity=2, seed=4711)
    wl = W.Workload(cfg, np.asarray([70, 1000], dtype=np.int32),
                    [np.asarray([], dtype=np.int32), np.asarray([0], dtype=np.int32), np.asarray([1], dtype=np.int32)],
                    np.asarray([2100, 1337, 2100], dtype=np.int32))
    dw = H.DeviceWorkload(wl)
    dw.ctx.tc_set_attn_kernel(kind)
    dw.ctx.tc_set_kv_splits(splits)
    bt, pl = dw.stitch()
    np.testing.assert_array_equal(pl, [0, 70, 1000])
    out, qkv = dw.attn_layer(0, bt, pl)
    got = H.out_to_f64(out, wl.cfg)
    ref = H.oracle_attn_layer(wl, dw.tables_np, 0, qkv)
    worst = 0.0
    for i, r in ref.items():
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all()
        # rows that see only a handful of keys have outputs as large as single values: bf16 rounding
        # of the output alone is 2^-9 of that
        vmax = max(float(np.abs(W.storage_to_f64(qkv[2][sl], "bf16")).max()), 1.0)
        err = np.abs(got[sl] - r).max(axis=(1, 2))
        few = np.arange(err.shape[0]) + int(pl[i]) < 64
        assert (err[~few] <= TOL).all(), (i, float(err[~few].max()))
        assert (err[few] <= max(TOL, 2.0 ** -8 * vmax)).all(), (i, float(err[few].max()))
        worst = max(worst, float(err.max()))
    print("kernel %d (chosen %d), partitions asked %d, made %d: max-abs err %.2e" % (
        kind, dw.ctx.tc_attn_kernel(), splits, dw.ctx.tc_kv_splits(), worst))
    dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("kind", [0, 4])
def test_many_short_queries(H, kind):
    """Width instead of length: 400 queries of one or two small tables and a few suffix tokens each
    (1600 work items of a tile or two; more (query, KV head) pairs than CUs), prefill and one decode
    step, every row against the checker."""
    cfg = W.WorkloadConfig(name="wide", n_layers=1, n_q_heads=8, n_kv_heads=4, head_dim=128, dtype="bf16", n_tables=30,
                           table_len=(5, 80), batch=400, tables_per_query=(1, 2), choice="uniform",
                           suffix_len=(1, 20), capacity=30, seed=2024)
    wl = W.make_workload(cfg)
    c = wl.cfg
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S = wl.suffix_len.astype(int)
    dw = H.DeviceWorkload(wl, seq_blocks=int(sum(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 8)
    dw.ctx.tc_set_attn_kernel(kind)
    max_blocks = int(max(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 1
    bt, pl = dw.stitch(max_blocks=max_blocks)
    out, qkv = dw.attn_layer(0, bt, pl)
    got = H.out_to_f64(out, c)
    ref = H.oracle_attn_layer(wl, dw.tables_np, 0, qkv)
    worst = 0.0
    for i, r in ref.items():
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        vmax = max(float(np.abs(W.storage_to_f64(qkv[2][sl], "bf16")).max()),
                   max(float(np.abs(W.storage_to_f64(dw.tables_np[int(t)][1][0], "bf16")).max()) for t in wl.queries[i]))
        e = float(np.abs(got[sl] - r).max())
        assert e <= max(TOL, 2.0 ** -8 * vmax), (i, e)     # sequences of a few dozen keys: outputs as large as single values
        worst = max(worst, e)
    print("prefill of 400 queries, kernel %d: max-abs err %.2e" % (dw.ctx.tc_attn_kernel(), worst))
    # one decode step
    dw.ctx.tc_set_attn_kernel(0)
    cur = (P + S).astype(np.int32)
    bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
    rng = np.random.default_rng(5)
    q, k, v = (W.f32_to_bf16_bits(rng.standard_normal(size=(c.batch, h, c.head_dim), dtype=np.float32))
               for h in (c.n_q_heads, c.n_kv_heads, c.n_kv_heads))
    dq, dk, dv = H.to_dev(q, c), H.to_dev(k, c), H.to_dev(v, c)
    out = torch.full_like(dq, float("nan"))
    dw.ctx.tc_prefill_attn(0, dq, dk, dv, out, np.arange(c.batch + 1, dtype=np.int32), bt, cur,
                           np.ones(c.batch, dtype=np.int32), wl.sm_scale, None)
    torch.cuda.synchronize()
    assert dw.ctx.tc_attn_kernel() == 3
    got = H.out_to_f64(out, c)
    worst = 0.0
    for i in range(c.batch):
        ks, vs = H.oracle_sequences(wl, dw.tables_np, 0, i)
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        K = np.concatenate([ks, qkv[1][sl]])
        V = np.concatenate([vs, qkv[2][sl]])
        r = oracle.prefill_attn(W.storage_to_f64(q[i:i + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[i:i + 1], "bf16"),
                                W.storage_to_f64(v[i:i + 1], "bf16"), wl.sm_scale)
        vmax = max(float(np.abs(W.storage_to_f64(V, "bf16")).max()), float(np.abs(W.storage_to_f64(v[i], "bf16")).max()))
        e = float(np.abs(got[i:i + 1] - r).max())
        assert e <= max(TOL, 2.0 ** -8 * vmax), (i, e)
        worst = max(worst, e)
    print("decode step of 400 queries in %d ranges at most: max-abs err %.2e" % (dw.ctx.tc_kv_splits(), worst))
    dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("kind,forced", [(0, 0), (4, 1), (2, 1), (1, 2)])
def test_long_prefix_read_in_place(H, kind, forced):
    """The long query again, its tables read in place (block-format slots, tc_stitch_alias): three
    tables of 30 011, 39 989 and 7 tokens, so the sequence has unused block tails in the middle of
    a partition, at a partition's end, and a table shorter than a block at the end of the prefix."""
    cfg = W.scaled(W.CONFIGS["c2"], name="longa", n_layers=1, n_q_heads=4, n_kv_heads=1, n_tables=3, batch=2,
                   tables_per_query=(1, 1), capacity=3, seed=31338)
    wl = W.Workload(cfg, np.asarray([30011, 39989, 7], dtype=np.int32),
                    [np.asarray([0, 1, 2], dtype=np.int32), np.asarray([2], dtype=np.int32)],
                    np.asarray([37, 5], dtype=np.int32))
    dw = H.DeviceWorkload(wl, slot_layout=1)
    dw.ctx.tc_set_attn_kernel(kind)
    dw.ctx.tc_set_kv_splits(forced)
    bt, pl = dw.alias()
    assert int(pl[0]) == 16 * (-(-30011 // 16) + -(-39989 // 16) + 1) and int(pl[1]) == 16
    out, qkv = dw.attn_layer(0, bt, pl)
    got = H.out_to_f64(out, wl.cfg)
    ref = H.oracle_attn_layer(wl, dw.tables_np, 0, qkv)
    worst = 0.0
    for i, r in ref.items():
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all()
        e = float(np.abs(got[sl] - r).max())
        # the second query sees 7 + a few keys: outputs as large as single values
        assert e <= (TOL if i == 0 else max(TOL, 2.0 ** -8 * 4.7)), (i, e)
        worst = max(worst, e)
    print("in place, kernel %d (chosen %d), %d partitions asked, %d made: max-abs err %.2e" % (
        kind, dw.ctx.tc_attn_kernel(), forced, dw.ctx.tc_kv_splits(), worst))
    dw.ctx.tc_release_seqs(bt)
    dw.close()
