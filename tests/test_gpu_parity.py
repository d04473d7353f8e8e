"""GPU parity: the HIP path, through the C ABI, against the CPU checker on the same seeded
inputs.  Gather, append and block tables bit for bit; attention within 1e-5 (fp32) and
1e-2 max-abs (bf16 operands, fp32 accumulation)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_08743_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


@pytest.fixture(scope="module")
def H():
    import harness
    assert torch.cuda.is_available()
    return harness


def _check_pool_against_oracle(H, dw, bt, pl, layers, qkv_of_layer=None):
    """Read every stitched sequence back and compare with the concatenation, bit for bit."""
    wl, c = dw.wl, dw.cfg
    for layer in layers:
        for i in range(c.batch):
            P, S = int(pl[i]), int(wl.suffix_len[i])
            n = P + (S if qkv_of_layer else 0)
            if n == 0:
                continue
            nb = -(-n // 16)
            k, v = dw.ctx.tc_read_seq_kv(layer, bt[i, :nb], n, H.np_dtype(c))
            ks, vs = H.oracle_sequences(wl, dw.tables_np, layer, i)
            assert ks.shape[0] == P
            np.testing.assert_array_equal(k[:P].view(np.uint8), ks.view(np.uint8))
            np.testing.assert_array_equal(v[:P].view(np.uint8), vs.view(np.uint8))
            if qkv_of_layer:
                _, kn, vn = qkv_of_layer[layer]
                sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
                np.testing.assert_array_equal(k[P:].view(np.uint8), kn[sl].view(np.uint8))
                np.testing.assert_array_equal(v[P:].view(np.uint8), vn[sl].view(np.uint8))


def _check_block_table(dw, bt, pl, model):
    wl = dw.wl
    exp_pl = oracle.prefix_lengths(wl.table_len, wl.table_ids, wl.cu_tables)
    np.testing.assert_array_equal(pl, exp_pl)
    exp_bt = model.stitch(exp_pl, wl.suffix_len, bt.shape[1])
    np.testing.assert_array_equal(bt, exp_bt)


def _attn_err(H, dw, bt, pl, layer, queries=None):
    out, qkv = dw.attn_layer(layer, bt, pl)
    ref = H.oracle_attn_layer(dw.wl, dw.tables_np, layer, qkv, queries)
    got = H.out_to_f64(out, dw.cfg)
    err, rel = 0.0, 0.0
    for i, r in ref.items():
        if r.size == 0:
            continue
        sl = slice(int(dw.wl.cu_seqlens[i]), int(dw.wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all()
        d = np.abs(got[sl] - r)
        err = max(err, float(d.max()))
        rel = max(rel, float(d.max() / np.sqrt((r ** 2).mean())))
    return err, rel, qkv


# ------------------------------------------------------------------------------------ c1 in full

def test_c1_fp32_full(H):
    wl = W.get("c1")
    dw = H.DeviceWorkload(wl)
    model = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    bt, pl = dw.stitch()
    _check_block_table(dw, bt, pl, model)
    _check_pool_against_oracle(H, dw, bt, pl, [0])
    err, rel, qkv = _attn_err(H, dw, bt, pl, 0)
    print("c1: max-abs %.3e, max-abs/rms %.3e, splits %d" % (err, rel, dw.ctx.tc_kv_splits()))
    assert err <= TOL["f32"]
    _check_pool_against_oracle(H, dw, bt, pl, [0], {0: qkv})       # suffix K/V appended bit-exact
    dw.close()


# ------------------------------------------------------------------------------------ c2 shape, reduced depth

@pytest.mark.parametrize("splits", [0, 1, 2, 9])
def test_c2_shape_two_layers(H, splits):
    """28q/4kv/d128 bf16, P ~ 4.5k, S = 128: spans ~70 key tiles, 7 row tiles per KV head and a
    ragged tail; 2 of the 28 layers so the checker finishes in seconds."""
    cfg = W.scaled(W.CONFIGS["c2"], n_layers=2)
    wl = W.make_workload(cfg)
    used = sorted(set(wl.table_ids.tolist()))
    dw = H.DeviceWorkload(wl, capacity=len(used), tables=used)
    dw.ctx.tc_set_kv_splits(splits)
    model = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    bt, pl = dw.stitch()
    _check_block_table(dw, bt, pl, model)
    _check_pool_against_oracle(H, dw, bt, pl, [0, 1])
    qkvs = {}
    for layer in (0, 1):
        err, rel, qkvs[layer] = _attn_err(H, dw, bt, pl, layer)
        print("c2/2 layers, splits=%d(%d) layer %d: max-abs %.3e, max-abs/rms %.3e" %
              (splits, dw.ctx.tc_kv_splits(), layer, err, rel))
        assert err <= TOL["bf16"]
        assert rel <= 0.05
    if splits:
        assert dw.ctx.tc_kv_splits() == splits
    _check_pool_against_oracle(H, dw, bt, pl, [0, 1], qkvs)
    dw.close()


# ------------------------------------------------------------------------------------ ragged and degenerate cases

def _small_cfg(dtype, **kw):
    base = dict(name="t", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128 if dtype == "bf16" else 64,
                dtype=dtype, n_tables=8, table_len=(1, 40), batch=5, tables_per_query=(0, 4),
                choice="uniform", suffix_len=(0, 37), capacity=8, seed=77)
    base.update(kw)
    return W.WorkloadConfig(**base)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_batch(H, dtype):
    """Tables of 1..40 tokens (not multiples of 16), queries with no table, with an empty suffix,
    with a repeated table; variable lengths in one batch."""
    wl = W.make_workload(_small_cfg(dtype))
    wl.table_len[:] = [1, 15, 16, 17, 40, 33, 2, 31]
    wl.queries[0] = np.array([], dtype=np.int32)                # no table matched: P = 0
    wl.queries[1] = np.array([3, 3, 0], dtype=np.int32)         # a table twice
    wl.queries[2] = np.array([2], dtype=np.int32)               # P = 16 exactly
    wl.suffix_len[:] = [5, 0, 16, 37, 1]                        # query 1: nothing to compute
    dw = H.DeviceWorkload(wl)
    model = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    bt, pl = dw.stitch()
    _check_block_table(dw, bt, pl, model)
    _check_pool_against_oracle(H, dw, bt, pl, [0, 1])
    qkvs = {}
    for layer in (0, 1):
        err, rel, qkvs[layer] = _attn_err(H, dw, bt, pl, layer)
        print("ragged %s layer %d: max-abs %.3e" % (dtype, layer, err))
        assert err <= TOL[dtype]
    _check_pool_against_oracle(H, dw, bt, pl, [0, 1], qkvs)
    # release and stitch again: the same lowest blocks come back, results identical
    dw.ctx.tc_release_seqs(bt)
    model.release(bt)
    bt2, pl2 = dw.stitch()
    np.testing.assert_array_equal(bt2, bt)
    _check_block_table(dw, bt2, pl2, oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks))
    dw.close()


def test_varlen_batch_c3_shape(H):
    """c3's shape (zipf table choice, suffix 64..256, shared pool) on 8 queries and 2 layers."""
    cfg = W.scaled(W.CONFIGS["c3"], n_layers=2, batch=8)
    wl = W.make_workload(cfg)
    used = sorted(set(wl.table_ids.tolist()))
    dw = H.DeviceWorkload(wl, capacity=len(used), tables=used)
    model = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    bt, pl = dw.stitch()
    _check_block_table(dw, bt, pl, model)
    _check_pool_against_oracle(H, dw, bt, pl, [1])
    P = pl.astype(int)
    pick = sorted({int(P.argmax()), int(P.argmin()), 0})        # longest, shortest, first
    err, rel, _ = _attn_err(H, dw, bt, pl, 1, queries=pick)
    print("c3/8 queries: P=%s, checked %s, max-abs %.3e rel %.3e" % (P.tolist(), pick, err, rel))
    assert err <= TOL["bf16"] and rel <= 0.05
    dw.close()


def test_hand_made_block_table_and_scattered_blocks(H):
    """tc_prefill_attn with a caller-made batch: blocks in reverse order."""
    wl = W.make_workload(_small_cfg("bf16", batch=2, tables_per_query=(2, 3), suffix_len=(20, 30)))
    dw = H.DeviceWorkload(wl, seq_blocks=64)
    bt, pl = dw.stitch()
    out1, qkv = dw.attn_layer(0, bt, pl)
    # move the sequences to other physical blocks through a second stitch, release the first
    bt_b, pl_b = dw.stitch()
    dw.ctx.tc_release_seqs(bt)
    assert not np.array_equal(bt, bt_b)
    out2, _ = dw.attn_layer(0, bt_b, pl_b, qkv=qkv)
    assert torch.equal(out1, out2)
    dw.close()


# ------------------------------------------------------------------------------------ error behaviour

def test_errors_have_no_side_effects(H):
    B = __import__("paper_2601_08743_amd.binding", fromlist=["x"])
    wl = W.make_workload(_small_cfg("f32", batch=2, tables_per_query=(2, 2), suffix_len=(4, 4)))
    dw = H.DeviceWorkload(wl, load_all=False, capacity=3, seq_blocks=12)
    ctx = dw.ctx
    ids = wl.table_ids
    with pytest.raises(B.TcError) as e:
        ctx.tc_stitch_kv(ids, wl.cu_tables, wl.suffix_len, 32)
    assert e.value.code == B.TC_ERR_NOT_RESIDENT
    with pytest.raises(B.TcError) as e:
        ctx.tc_load_async([99], 0, 2)
    assert e.value.code == B.TC_ERR_UNKNOWN_TABLE
    with pytest.raises(B.TcError) as e:
        ctx.tc_load_async([0], 1, 5)
    assert e.value.code == B.TC_ERR_INVALID
    # only layer 0 resident: still refused
    ctx.tc_load_async(sorted(set(ids.tolist()))[:3], 0, 1)
    with pytest.raises(B.TcError) as e:
        ctx.tc_stitch_kv(ids, wl.cu_tables, wl.suffix_len, 32)
    assert e.value.code == B.TC_ERR_NOT_RESIDENT
    with pytest.raises(B.TcError) as e:
        ctx.tc_stitch_kv([99], [0, 1], [1], 32)
    assert e.value.code == B.TC_ERR_UNKNOWN_TABLE
    with pytest.raises(B.TcError) as e:
        ctx.tc_register_table_kv(50, 10 ** 6, dw.host_kv[0][0], dw.host_kv[0][1])
    assert e.value.code == B.TC_ERR_CAPACITY
    # make one query resident and ask for more blocks than the pool has / than max_blocks allows
    q0 = wl.queries[0]
    ctx.tc_load_async(q0, 0, 2)
    big = np.array([16 * 12], dtype=np.int32)
    with pytest.raises(B.TcError) as e:
        ctx.tc_stitch_kv(q0, [0, len(q0)], big, 64)
    assert e.value.code == B.TC_ERR_OOM_POOL
    with pytest.raises(B.TcError) as e:
        ctx.tc_stitch_kv(q0, [0, len(q0)], [4], 0)
    assert e.value.code == B.TC_ERR_OOM_POOL
    # after all these failures the allocator is untouched: the first block handed out is the lowest
    bt, pl = ctx.tc_stitch_kv(q0, [0, len(q0)], [4], 16)
    assert bt[0, 0] == dw.first_seq
    with pytest.raises(B.TcError) as e:
        ctx.tc_release_seqs(np.array([[dw.first_seq + 11]], dtype=np.int32))       # never allocated
    assert e.value.code == B.TC_ERR_INVALID
    with pytest.raises(B.TcError) as e:                                             # block id out of range
        bad = bt.copy(); bad[0, 0] = 0
        dq = torch.zeros((4, 8, 64), device="cuda")
        ctx.tc_prefill_attn(0, dq, dq[:, :2], dq[:, :2], dq.clone(), [0, 4], bad, pl, [4], 0.1)
    assert e.value.code == B.TC_ERR_INVALID
    with pytest.raises(B.TcError) as e:
        dq = torch.zeros((4, 8, 64), device="cuda")
        ctx.tc_prefill_attn(0, dq, dq[:, :2], dq[:, :2], dq.clone(), [0, 4], bt, pl, [4], -1.0)
    assert e.value.code == B.TC_ERR_INVALID
    dw.close()


def test_replacement_trace_matches_app_a_models(H):
    """The library's (table, hit, evicted) trace equals the checker's App. A models, and a table
    evicted and loaded again stitches bit-exact from its new slot."""
    B = __import__("paper_2601_08743_amd.binding", fromlist=["x"])
    rng = np.random.default_rng(5)
    for policy, Model in ((B.TC_POLICY_LRU, oracle.LRUModel), (B.TC_POLICY_FIFO, oracle.FIFOModel),
                          (B.TC_POLICY_LFU, oracle.LFUModel)):
        wl = W.make_workload(_small_cfg("bf16", batch=1, tables_per_query=(3, 3), suffix_len=(3, 3),
                                        n_tables=8, table_len=(5, 40)))
        dw = H.DeviceWorkload(wl, load_all=False, capacity=3, policy=policy)
        acc = rng.integers(0, 8, size=60).tolist()
        for k in range(0, len(acc), 7):
            dw.ctx.tc_load_async(acc[k:k + 7], 0, 2)
        got = [tuple(r) for r in dw.ctx.tc_load_trace().tolist()]
        model = Model(3)
        assert got == oracle.replay(model, acc)
        resident = sorted(int(t) for t in model.items)
        assert len(resident) == 3
        for t in range(8):
            assert dw.ctx.tc_is_resident(t, 0, 2) == (t in resident)
        wl.queries[0] = np.array(resident[::-1], dtype=np.int32)       # stitch what is cached now
        torch.cuda.synchronize()
        bt, pl = dw.stitch()
        _check_pool_against_oracle(H, dw, bt, pl, [0, 1])
        dw.close()


@pytest.mark.parametrize("kind,entry", [(0, "tc_prefill_attn"), (4, "tc_prefill_attn"), (1, "tc_prefill_attn"),
                                        (0, "tc_prefill_attn_noalloc"), (4, "tc_prefill_attn_noalloc")])
def test_layer_loop_replayed_as_a_graph_matches_eager(H, kind, entry):
    """The per-layer calls captured into a HIP graph (kernel launches only: no memset nodes) and
    replayed several times, with eager stitches, releases and synchronisations in between, give
    bit-identical outputs to the eager calls every time - through the pipelined kernel with its
    merge launch (the automatic choice here), the long-launch kernel with its append launch, the
    general kernel, and through the entry point that allocates nothing, which exists for callers
    like this one (the batch's plan is uploaded by the eager call before the capture)."""
    cfg = W.scaled(W.CONFIGS["c2"], n_layers=3, n_tables=8, tables_per_query=(6, 6), capacity=8)
    wl = W.make_workload(cfg)
    dw = H.DeviceWorkload(wl)
    dw.ctx.tc_set_attn_kernel(kind)
    stream = torch.cuda.Stream()
    qkv = [tuple(H.to_dev(x, cfg) for x in wl.suffix_qkv(l)) for l in range(3)]
    outs = [torch.zeros_like(qkv[l][0]) for l in range(3)]
    call = getattr(dw.ctx, entry)

    def layers(bt, pl):
        for l in range(3):
            q, k, v = qkv[l]
            call(l, q, k, v, outs[l], wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale, stream)

    bt, pl = dw.stitch(stream=stream)
    layers(bt, pl)
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        layers(bt, pl)
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))
        if rep % 2:                                  # eager work between replays: release and stitch again
            dw.ctx.tc_release_seqs(bt)
            bt2, pl2 = dw.stitch(stream=stream)
            np.testing.assert_array_equal(bt2, bt)   # same blocks, so the captured pointers stay valid
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(3):
            assert torch.equal(outs[l], eager[l]), (rep, l)
    assert dw.ctx.tc_attn_kernel() == (kind or 2) and dw.ctx.tc_kv_splits() > 1
    ref = H.oracle_attn_layer(wl, dw.tables_np, 2, wl.suffix_qkv(2))
    got = H.out_to_f64(outs[2], cfg)
    assert max(float(np.abs(got[int(wl.cu_seqlens[i]):int(wl.cu_seqlens[i + 1])] - r).max()) for i, r in ref.items()) <= 1e-2
    dw.close()
