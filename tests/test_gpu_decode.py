"""GPU: decode steps over the pool the prefill filled.  A decode step is tc_prefill_attn with one
new token per query and prefix_len = everything already in the pool; tc_grow_seqs gives the
sequences the blocks they need.  Checked against the CPU checker: every step's output is the
attention of the new token over the whole earlier sequence (tables, prompt suffix, generated
tokens) plus itself, and at the end the pool holds that whole sequence bit for bit - which also
checks that every earlier append landed where attention later reads it."""
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


def _draw(seed, *key, shape):
    rng = np.random.default_rng(np.random.SeedSequence([seed, 9, *key]))
    return W.f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


@pytest.mark.parametrize("kind", [0, 1, 4])
@pytest.mark.parametrize("splits", [0, 3])
def test_decode_steps_after_prefill(H, splits, kind):
    cfg = W.WorkloadConfig(name="dec", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", n_tables=6,
                           table_len=(20, 150), batch=3, tables_per_query=(1, 3), choice="uniform",
                           suffix_len=(3, 40), capacity=6, seed=404)
    wl = W.make_workload(cfg)
    c = wl.cfg
    T = 24                                             # crosses block boundaries and a key-tile boundary
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S = wl.suffix_len.astype(int)
    seq_blocks = int(sum(-(-(p + s + T) // 16) for p, s in zip(P, S))) + 4
    dw = H.DeviceWorkload(wl, seq_blocks=seq_blocks)
    if splits:
        dw.ctx.tc_set_kv_splits(splits)
    dw.ctx.tc_set_attn_kernel(kind)                    # 0: the decode kernels serve the steps; 1, 4: a prefill kernel does
                                                       # (4 appends by blocks in a launch of its own: the pool check below covers it)
    max_blocks = int(max(-(-(p + s + T) // 16) for p, s in zip(P, S))) + 1
    bt, pl = dw.stitch(max_blocks=max_blocks)
    # prefill: both layers (appends the prompt's own suffix to the pool)
    pre = {}
    for layer in range(c.n_layers):
        out, qkv = dw.attn_layer(layer, bt, pl)
        pre[layer] = qkv
    # the sequences as the checker sees them: per layer, per query, K and V rows so far (storage bits)
    seq = {}
    for layer in range(c.n_layers):
        for i in range(c.batch):
            ks, vs = H.oracle_sequences(wl, dw.tables_np, layer, i)
            sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
            seq[layer, i] = [np.concatenate([ks, pre[layer][1][sl]]), np.concatenate([vs, pre[layer][2][sl]])]
    model = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    want_bt = model.stitch(P, S, max_blocks)
    np.testing.assert_array_equal(bt, want_bt)
    one = np.ones(c.batch, dtype=np.int32)
    cu1 = np.arange(c.batch + 1, dtype=np.int32)
    worst = 0.0
    for t in range(T):
        cur = (P + S + t).astype(np.int32)             # tokens in the pool before this step
        bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
        # the checker's model: a query gets a new block exactly when its length crosses a block boundary
        for i in range(c.batch):
            if int(cur[i]) % 16 == 0:
                want_bt[i, int(cur[i]) // 16] = model.free.pop(0)
        np.testing.assert_array_equal(bt, want_bt)
        for layer in range(c.n_layers):
            q = _draw(c.seed, layer, t, 0, shape=(c.batch, c.n_q_heads, c.head_dim))
            k = _draw(c.seed, layer, t, 1, shape=(c.batch, c.n_kv_heads, c.head_dim))
            v = _draw(c.seed, layer, t, 2, shape=(c.batch, c.n_kv_heads, c.head_dim))
            dq, dk, dv = H.to_dev(q, c), H.to_dev(k, c), H.to_dev(v, c)
            out = torch.full_like(dq, float("nan"))
            dw.ctx.tc_prefill_attn(layer, dq, dk, dv, out, cu1, bt, cur, one, wl.sm_scale, None)
            torch.cuda.synchronize()
            assert dw.ctx.tc_attn_kernel() == (3 if kind == 0 else kind)
            got = H.out_to_f64(out, c)
            for i in range(c.batch):
                K, V = seq[layer, i]
                ref = oracle.prefill_attn(W.storage_to_f64(q[i:i + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                          W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[i:i + 1], "bf16"),
                                          W.storage_to_f64(v[i:i + 1], "bf16"), wl.sm_scale)
                worst = max(worst, float(np.abs(got[i:i + 1] - ref).max()))
                seq[layer, i] = [np.concatenate([K, k[i:i + 1]]), np.concatenate([V, v[i:i + 1]])]
    assert worst <= 1e-2, worst
    # the pool now holds every sequence in full
    for layer in range(c.n_layers):
        for i in range(c.batch):
            n = int(P[i] + S[i] + T)
            kk, vv = dw.ctx.tc_read_seq_kv(layer, bt[i, :-(-n // 16)], n, np.uint16)
            np.testing.assert_array_equal(kk.view(np.uint8), seq[layer, i][0].view(np.uint8))
            np.testing.assert_array_equal(vv.view(np.uint8), seq[layer, i][1].view(np.uint8))
    dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("kind", [0, 1])
def test_decode_steps_over_tables_read_in_place(H, kind):
    """The same over sequences whose table part was never copied (block-format slots,
    tc_stitch_alias): the decode batches name the table slots' blocks, the library works out from
    the cached tables which positions of those blocks hold tokens, and the result must be the
    attention over the plain concatenation.  Positions are those of the padded sequence (each table
    rounded up to whole blocks); tables of 3 .. 150 tokens, so some are shorter than a block and a
    key tile can hold several unused tails."""
    from paper_2601_08743_amd import binding as B
    cfg = W.WorkloadConfig(name="decal", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", n_tables=7,
                           table_len=(3, 150), batch=4, tables_per_query=(1, 4), choice="uniform",
                           suffix_len=(1, 40), capacity=7, seed=406)
    wl = W.make_workload(cfg)
    c = wl.cfg
    T = 20
    S = wl.suffix_len.astype(int)
    nb_pref = np.array([sum(-(-int(wl.table_len[t]) // 16) for t in q) for q in wl.queries])
    Pp = 16 * nb_pref                                  # padded prefix lengths
    seq_blocks = int(sum(-(-(s + T) // 16) for s in S)) + 4
    dw = H.DeviceWorkload(wl, seq_blocks=seq_blocks, slot_layout=B.TC_SLOTS_BLOCKS)
    dw.ctx.tc_set_attn_kernel(kind)
    max_blocks = int(max(nb + -(-(s + T) // 16) for nb, s in zip(nb_pref, S))) + 1
    bt, pl = dw.alias(max_blocks=max_blocks)
    np.testing.assert_array_equal(pl, Pp)
    pre = {}
    for layer in range(c.n_layers):
        out, qkv = dw.attn_layer(layer, bt, pl)
        pre[layer] = qkv
    seq = {}
    for layer in range(c.n_layers):
        for i in range(c.batch):
            ks, vs = H.oracle_sequences(wl, dw.tables_np, layer, i)
            sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
            seq[layer, i] = [np.concatenate([ks, pre[layer][1][sl]]), np.concatenate([vs, pre[layer][2][sl]])]
    one = np.ones(c.batch, dtype=np.int32)
    cu1 = np.arange(c.batch + 1, dtype=np.int32)
    worst = 0.0
    for t in range(T):
        cur = (Pp + S + t).astype(np.int32)
        grown = dw.ctx.tc_grow_seqs(bt, cur + 1)
        np.testing.assert_array_equal(grown[bt >= 0], bt[bt >= 0])         # what was there stays
        own = grown[grown >= dw.first_seq]
        assert len(set(own.tolist())) == own.size                          # sequence blocks: nobody shares one
        assert ((grown >= 0).sum(axis=1) == -(-(cur + 1) // 16)).all()
        bt = grown
        for layer in range(c.n_layers):
            q = _draw(c.seed, layer, t, 0, shape=(c.batch, c.n_q_heads, c.head_dim))
            k = _draw(c.seed, layer, t, 1, shape=(c.batch, c.n_kv_heads, c.head_dim))
            v = _draw(c.seed, layer, t, 2, shape=(c.batch, c.n_kv_heads, c.head_dim))
            dq, dk, dv = H.to_dev(q, c), H.to_dev(k, c), H.to_dev(v, c)
            out = torch.full_like(dq, float("nan"))
            dw.ctx.tc_prefill_attn(layer, dq, dk, dv, out, cu1, bt, cur, one, wl.sm_scale, None)
            torch.cuda.synchronize()
            assert dw.ctx.tc_attn_kernel() == (3 if kind == 0 else 1)
            got = H.out_to_f64(out, c)
            for i in range(c.batch):
                K, V = seq[layer, i]
                ref = oracle.prefill_attn(W.storage_to_f64(q[i:i + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                          W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[i:i + 1], "bf16"),
                                          W.storage_to_f64(v[i:i + 1], "bf16"), wl.sm_scale)
                worst = max(worst, float(np.abs(got[i:i + 1] - ref).max()))
                seq[layer, i] = [np.concatenate([K, k[i:i + 1]]), np.concatenate([V, v[i:i + 1]])]
    assert worst <= 1e-2, worst
    # the part of every sequence that is its own (prompt suffix, generated tokens) sits behind the
    # table blocks, bit for bit; the table slots were only read
    for layer in range(c.n_layers):
        for i in range(c.batch):
            n = int(S[i] + T)
            kk, vv = dw.ctx.tc_read_seq_kv(layer, bt[i, nb_pref[i]:nb_pref[i] + -(-n // 16)], n, np.uint16)
            P_real = int(wl.table_len[wl.queries[i]].sum())
            np.testing.assert_array_equal(kk.view(np.uint8), seq[layer, i][0][P_real:].view(np.uint8))
            np.testing.assert_array_equal(vv.view(np.uint8), seq[layer, i][1][P_real:].view(np.uint8))
    # a table block may only stand where the whole block is prefix, and only if a table covers it
    bad = bt.copy()
    bad[0, int(cur[0]) // 16] = bt[0, 0]               # the block the new token goes to
    with pytest.raises(B.TcError) as e:
        dw.ctx.tc_prefill_attn(0, dq, dk, dv, out, cu1, bad, cur, one, wl.sm_scale, None)
    assert e.value.code == B.TC_ERR_INVALID
    t0 = int(wl.queries[0][0])
    bad = bt.copy()
    bad[0, 0] = (bt[0, 0] // dw.slot_blocks) * dw.slot_blocks + -(-int(wl.table_len[t0]) // 16)    # behind its table's last block
    if bad[0, 0] % dw.slot_blocks != 0:
        with pytest.raises(B.TcError) as e:
            dw.ctx.tc_prefill_attn(0, dq, dk, dv, out, cu1, bad, cur, one, wl.sm_scale, None)
        assert e.value.code == B.TC_ERR_INVALID
    dw.ctx.tc_release_seqs(bt)
    dw.close()


def test_grow_errors_change_nothing(H):
    from paper_2601_08743_amd import binding as B
    cfg = W.WorkloadConfig(name="dec", n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", n_tables=2,
                           table_len=(20, 30), batch=2, tables_per_query=(1, 1), choice="uniform",
                           suffix_len=(3, 3), capacity=2, seed=405)
    wl = W.make_workload(cfg)
    dw = H.DeviceWorkload(wl, seq_blocks=7)
    bt, pl = dw.stitch(max_blocks=4)
    n0 = [int(pl[i]) + 3 for i in range(2)]
    with pytest.raises(B.TcError) as e:
        dw.ctx.tc_grow_seqs(bt, [16 * 4 + 1, n0[1]])          # a fifth block does not fit max_blocks
    assert e.value.code == B.TC_ERR_OOM_POOL
    with pytest.raises(B.TcError) as e:
        dw.ctx.tc_grow_seqs(bt, [64, 64])                     # 8 blocks wanted, 7 exist
    assert e.value.code == B.TC_ERR_OOM_POOL
    same = dw.ctx.tc_grow_seqs(bt, n0)                         # nothing to do
    np.testing.assert_array_equal(same, bt)
    bad = bt.copy()
    bad[0, 0] = dw.first_seq + 6                               # not allocated
    with pytest.raises(B.TcError) as e:
        dw.ctx.tc_grow_seqs(bad, [40, 40])
    assert e.value.code == B.TC_ERR_INVALID
    grown = dw.ctx.tc_grow_seqs(bt, [33, 33])                  # one more block each: the two lowest free ones
    have = int((bt >= 0).sum())
    assert int((grown >= 0).sum()) == have + (3 - int((bt[0] >= 0).sum())) + (3 - int((bt[1] >= 0).sum()))
    dw.ctx.tc_release_seqs(grown)
    dw.close()


def test_decode_batch_c3_shape(H):
    """c3's batch (32 queries, prefixes of 600 .. 5000 tokens), one decode step on two layers: the
    decode kernels against the checker on every query, against the prefill kernel on the same
    inputs, and bit-identical from launch to launch; queries without a new token are skipped."""
    wl = W.make_workload(W.scaled(W.CONFIGS["c3"], n_layers=2))
    c = wl.cfg
    used = sorted(set(wl.table_ids.tolist()))
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S = wl.suffix_len.astype(int)
    seq_blocks = int(sum(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 8
    dw = H.DeviceWorkload(wl, seq_blocks=seq_blocks, capacity=len(used), tables=used)
    max_blocks = int(max(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 1
    bt, pl = dw.stitch(max_blocks=max_blocks)
    pre = {}
    for layer in range(2):
        _, qkv = dw.attn_layer(layer, bt, pl)
        pre[layer] = qkv
    cur = (P + S).astype(np.int32)
    bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
    new = np.ones(c.batch, dtype=np.int32)
    new[5] = 0                                          # one query sits this step out
    cu1 = np.concatenate([[0], np.cumsum(new)]).astype(np.int32)
    n_tok = int(new.sum())
    for layer in range(2):
        q = _draw(c.seed, layer, 0, 0, shape=(n_tok, c.n_q_heads, c.head_dim))
        k = _draw(c.seed, layer, 0, 1, shape=(n_tok, c.n_kv_heads, c.head_dim))
        v = _draw(c.seed, layer, 0, 2, shape=(n_tok, c.n_kv_heads, c.head_dim))
        dq, dk, dv = H.to_dev(q, c), H.to_dev(k, c), H.to_dev(v, c)
        outs = {}
        for kind in (0, 1):
            dw.ctx.tc_set_attn_kernel(kind)
            reps = []
            for _ in range(3):
                out = torch.full_like(dq, float("nan"))
                dw.ctx.tc_prefill_attn(layer, dq, dk, dv, out, cu1, bt, cur, new, wl.sm_scale, None)
                torch.cuda.synchronize()
                reps.append(out.view(torch.int16).cpu().numpy())
            assert dw.ctx.tc_attn_kernel() == (3 if kind == 0 else 1)
            np.testing.assert_array_equal(reps[0], reps[2])
            np.testing.assert_array_equal(reps[1], reps[2])
            outs[kind] = H.out_to_f64(out, c)
        assert np.abs(outs[0] - outs[1]).max() <= 1e-2
        for i in range(c.batch):
            if not new[i]:
                continue
            ks, vs = H.oracle_sequences(wl, dw.tables_np, layer, i)
            sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
            K = np.concatenate([ks, pre[layer][1][sl]])
            V = np.concatenate([vs, pre[layer][2][sl]])
            n = int(cu1[i])
            ref = oracle.prefill_attn(W.storage_to_f64(q[n:n + 1], "bf16"), W.storage_to_f64(K, "bf16"),
                                      W.storage_to_f64(V, "bf16"), W.storage_to_f64(k[n:n + 1], "bf16"),
                                      W.storage_to_f64(v[n:n + 1], "bf16"), wl.sm_scale)
            assert np.abs(outs[0][n:n + 1] - ref).max() <= 1e-2, (layer, i)
    dw.ctx.tc_release_seqs(bt)
    dw.close()
