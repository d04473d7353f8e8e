"""GPU: randomly drawn batches through every way the library can serve them.  Each case draws a
head configuration (1..4 KV heads, 1..8 query heads per KV head), 2..8 tables of a few to a few
hundred tokens, 1..5 queries with 0..5 tables and 0..200 suffix tokens each, the stitch (copying
or in place), the attention kernel (automatic, general, pipelined, alternating wave groups) and the number of key
partitions; runs one prefill layer twice (the two launches must agree bit for bit), checks it
against the CPU checker, then grows every sequence by one token and checks a decode step (decode
kernels or the prefill kernel).  Tolerance: 1e-2 max-abs, scaled by the largest reference value of
the query where that exceeds 1 (a sequence of a handful of keys has outputs of the size of single
values, and bf16 rounding of an output of size 4 is already 8e-3)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_08743_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import harness
    assert torch.cuda.is_available()
    return harness


def _case(H, seed, long_tokens=0):
    """long_tokens > 0: table 0 gets that many tokens and the first query reads it (few heads, so the
    checker stays fast): key ranges of hundreds of tiles, where the kernels' block-id tables decide
    the number of partitions."""
    from paper_2601_08743_amd import binding as B
    rng = np.random.default_rng(seed)
    hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 5, 7, 8]))
    if long_tokens:
        hkv, G = int(rng.choice([1, 2])), int(rng.choice([1, 4, 7]))
    hq = hkv * G
    nt, batch = int(rng.integers(2, 9)), int(rng.integers(1, 6))
    lo, hi = sorted((int(rng.choice([1, 20, 150])), int(rng.choice([40, 300, 700]))))
    cfg = W.WorkloadConfig(name="rnd", n_layers=1, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, dtype="bf16",
                           n_tables=nt, table_len=(lo, hi), batch=batch, tables_per_query=(0, min(nt, 5)),
                           choice="uniform", suffix_len=(0, int(rng.choice([1, 17, 90, 200]))), capacity=nt,
                           seed=1000 + seed)
    wl = W.make_workload(cfg)
    if long_tokens:
        tl = wl.table_len.copy()
        tl[0] = long_tokens
        queries = [np.asarray(q, dtype=np.int32) for q in wl.queries]
        if 0 not in queries[0].tolist():
            queries[0] = np.concatenate([queries[0][:2], np.asarray([0], dtype=np.int32)])
        wl = W.Workload(cfg, tl, queries, wl.suffix_len)
    alias, kind = bool(rng.integers(0, 2)), int(rng.choice([0, 1, 2, 4]))
    splits = int(rng.choice([0, 0, 1, 2, 3, 5]))
    S = wl.suffix_len.astype(int)
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    tag = "seed %d Hq %d Hkv %d in-place %d kernel %d partitions %d P %s S %s" % (seed, hq, hkv, alias, kind, splits,
                                                                                 P.tolist(), S.tolist())
    if alias:
        nbp = [sum(-(-int(wl.table_len[t]) // 16) for t in q) for q in wl.queries]
        seq_blocks = int(sum(-(-(s + 1) // 16) + 1 for s in S)) + 4
        max_blocks = max(n + -(-(int(s) + 1) // 16) for n, s in zip(nbp, S)) + 2
    else:
        seq_blocks = int(sum(-(-(p + s + 1) // 16) + 1 for p, s in zip(P, S))) + 4
        max_blocks = int(max(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 2
    dw = H.DeviceWorkload(wl, seq_blocks=seq_blocks, slot_layout=B.TC_SLOTS_BLOCKS if alias else B.TC_SLOTS_ROWS)
    dw.ctx.tc_set_attn_kernel(kind)
    dw.ctx.tc_set_kv_splits(splits)
    bt, pl = dw.alias(max_blocks) if alias else dw.stitch(max_blocks)
    out, qkv = dw.attn_layer(0, bt, pl)
    again, _ = dw.attn_layer(0, bt, pl)
    assert torch.equal(out.view(torch.int16), again.view(torch.int16)), "two launches differ: " + tag
    ref = H.oracle_attn_layer(wl, dw.tables_np, 0, qkv)
    got = H.out_to_f64(out, cfg)
    worst = 0.0
    for i, r in ref.items():
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all(), "non-finite output: " + tag
        if r.size:
            worst = max(worst, float(np.abs(got[sl] - r).max()) / max(1.0, float(np.abs(r).max())))
    assert worst <= 1e-2, (worst, tag)
    # one decode step: every query brings one token
    cur = (np.asarray(pl) + S).astype(np.int32)
    bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
    q, k, v = (W.f32_to_bf16_bits(rng.standard_normal(size=(batch, h, 128), dtype=np.float32)) for h in (hq, hkv, hkv))
    dq, dk, dv = H.to_dev(q, cfg), H.to_dev(k, cfg), H.to_dev(v, cfg)
    o = torch.full_like(dq, float("nan"))
    dkind = int(rng.choice([0, 1]))
    dw.ctx.tc_set_attn_kernel(dkind)
    dw.ctx.tc_prefill_attn(0, dq, dk, dv, o, np.arange(batch + 1, dtype=np.int32), bt, cur,
                           np.ones(batch, dtype=np.int32), wl.sm_scale, None)
    torch.cuda.synchronize()
    assert dw.ctx.tc_attn_kernel() == (3 if dkind == 0 else 1)
    god = H.out_to_f64(o, cfg)
    for i in range(batch):
        ks, vs = H.oracle_sequences(wl, dw.tables_np, 0, i)
        sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
        K, V = np.concatenate([ks, qkv[1][sl]]), np.concatenate([vs, qkv[2][sl]])
        r = oracle.prefill_attn(W.storage_to_f64(q[i:i + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[i:i + 1], "bf16"),
                                W.storage_to_f64(v[i:i + 1], "bf16"), wl.sm_scale)
        e = float(np.abs(god[i:i + 1] - r).max()) / max(1.0, float(np.abs(r).max()))
        assert np.isfinite(god[i]).all() and e <= 1e-2, ("decode step, kernel %d, query %d: %g; " % (dkind, i, e)) + tag
    dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_with_a_long_table(H, seed):
    """The same draws with one table of 17 000 .. 45 000 tokens in the first query: more key tiles
    than the general kernel's block-id table holds (256), so forced partition counts are raised, the
    pipelined kernel's batch is planned twice, and the merge runs over the replanned groups."""
    rng = np.random.default_rng(31 + seed)
    _case(H, 9000 + seed, long_tokens=int(rng.integers(17000, 45001)))


@pytest.mark.parametrize("block", range(4))
def test_random_batches_every_path(H, block):
    for seed in range(100 * block, 100 * block + 100):
        _case(H, seed)
