"""GPU: sequences made without copying (block-format table slots, tc_stitch_alias) against the
CPU checker.  The block tables must equal the checker's layout; every table must sit in its slot's
blocks bit for bit with a zero tail; attention over the aliased sequence must equal the checker's
attention over the plain concatenation (the unused block tails take no part) within the bf16
tolerance, through both kernels and the split-KV merge."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_08743_amd import workloads as W

pytestmark = pytest.mark.gpu
BLOCKS = 1      # TC_SLOTS_BLOCKS


@pytest.fixture(scope="module")
def H():
    import harness
    assert torch.cuda.is_available()
    return harness


def _check_layout(H, dw, bt, pl, layers):
    """Block table against the checker's; table slots against the registered KV."""
    wl, c = dw.wl, dw.cfg
    if not hasattr(dw, "slot_model"):
        dw.slot_model = oracle.SlotModel(dw.tc_cfg.table_capacity)
    slots = dw.slot_model
    slots.apply([tuple(r) for r in dw.ctx.tc_load_trace().tolist()])      # what was loaded since the last look
    seq = oracle.SeqBlockModel(dw.first_seq, dw.seq_blocks)
    want_bt, want_pl, valid = oracle.alias_block_table(seq, slots.slot, wl.table_len, wl.queries, wl.suffix_len,
                                                       dw.slot_blocks, bt.shape[1])
    np.testing.assert_array_equal(bt, want_bt)
    np.testing.assert_array_equal(pl, want_pl)
    for t in sorted({int(t) for q in wl.queries for t in q}):
        n = int(wl.table_len[t])
        nb = -(-n // 16)
        blocks = slots.slot[t] * dw.slot_blocks + np.arange(nb, dtype=np.int32)
        for layer in layers:
            k, v = dw.ctx.tc_read_seq_kv(layer, blocks, 16 * nb, H.np_dtype(c))
            tk, tv = dw.tables_np[t]
            np.testing.assert_array_equal(k[:n].view(np.uint8), tk[layer].view(np.uint8))
            np.testing.assert_array_equal(v[:n].view(np.uint8), tv[layer].view(np.uint8))
            assert not k[n:].view(np.uint8).any() and not v[n:].view(np.uint8).any()   # the unused tail is zeros
    return valid


def _attn_err(H, dw, bt, pl, layer, qkv=None):
    out, qkv = dw.attn_layer(layer, bt, pl, qkv=qkv)
    ref = H.oracle_attn_layer(dw.wl, dw.tables_np, layer, qkv)
    got = H.out_to_f64(out, dw.cfg)
    err = 0.0
    for i, r in ref.items():
        if r.size == 0:
            continue
        sl = slice(int(dw.wl.cu_seqlens[i]), int(dw.wl.cu_seqlens[i + 1]))
        assert np.isfinite(got[sl]).all()
        err = max(err, float(np.abs(got[sl] - r).max()))
    return err


@pytest.mark.parametrize("kind", [1, 2])
@pytest.mark.parametrize("splits", [0, 1, 3, 8])
def test_alias_c2_shape(H, kind, splits):
    """c2's shape (12 tables, P ~ 4.1k, S = 128): the pipelined kernel takes the unused tails out of
    the row sums analytically, the general kernel masks them."""
    wl = W.make_workload(W.scaled(W.CONFIGS["c2"], n_layers=2))
    used = sorted(set(wl.table_ids.tolist()))
    dw = H.DeviceWorkload(wl, capacity=len(used), tables=used, slot_layout=BLOCKS)
    dw.ctx.tc_set_attn_kernel(kind)
    if splits:
        dw.ctx.tc_set_kv_splits(splits)
    bt, pl = dw.alias()
    assert dw.ctx.tc_attn_kernel() == kind
    _check_layout(H, dw, bt, pl, [0, 1])
    assert int(pl[0]) >= int(wl.table_len[wl.queries[0]].sum())
    for layer in (0, 1):
        err = _attn_err(H, dw, bt, pl, layer)
        assert err <= 1e-2, (kind, splits, layer, err)
    dw.ctx.tc_release_seqs(bt)
    dw.close()


def _small_cfg(**kw):
    base = dict(name="a", n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", n_tables=10,
                table_len=(1, 40), batch=6, tables_per_query=(0, 5), choice="uniform", suffix_len=(0, 37),
                capacity=10, seed=91)
    base.update(kw)
    return W.WorkloadConfig(**base)


@pytest.mark.parametrize("seed", [91, 92, 93])
def test_alias_ragged_batch(H, seed):
    """Tables of 1..40 tokens (most blocks have unused tails, some tables are shorter than a block,
    several tables end inside one key tile), queries without tables, empty suffixes, a table used
    twice in one query."""
    wl = W.make_workload(_small_cfg(seed=seed))
    wl.queries[1] = np.array([3, 3, 5], dtype=np.int32)
    wl.queries[2] = np.array([], dtype=np.int32)
    wl.suffix_len[3] = 0
    wl = W.Workload(wl.cfg, wl.table_len, wl.queries, wl.suffix_len)
    dw = H.DeviceWorkload(wl, slot_layout=BLOCKS)
    for kind in (1, 2):
        dw.ctx.tc_set_attn_kernel(kind)
        bt, pl = dw.alias()
        if kind == 1:
            _check_layout(H, dw, bt, pl, [0, 1])
        for layer in (0, 1):
            # rows that see few keys: outputs as large as single values (the bound of the bf16 tests)
            q, k, v = wl.suffix_qkv(layer)
            vmax = float(np.abs(W.storage_to_f64(v, "bf16")).max())
            err = _attn_err(H, dw, bt, pl, layer, qkv=(q, k, v))
            assert err <= max(1e-2, 2.0 ** -8 * max(vmax, 4.5)), (kind, layer, err)
        dw.ctx.tc_release_seqs(bt)
    dw.close()


@pytest.mark.parametrize("lens", [(200, 300, 180, 250), (17, 640, 33, 1, 480)])
def test_alias_long_runs_with_many_tails(H, lens):
    """Unsplit queries over several hundred keys: the pipelined path runs over tiles that contain
    table ends (including a first tile whose first 32 keys contain an unused tail)."""
    wl = W.make_workload(_small_cfg(n_tables=len(lens), table_len=(1, 700), batch=2, tables_per_query=(1, 1),
                                    suffix_len=(40, 40), capacity=len(lens)))
    for t, n in enumerate(lens):
        wl.table_len[t] = n
    wl.queries[0] = np.arange(len(lens), dtype=np.int32)
    wl.queries[1] = np.arange(len(lens), dtype=np.int32)[::-1].copy()
    wl = W.Workload(wl.cfg, wl.table_len, wl.queries, wl.suffix_len)
    dw = H.DeviceWorkload(wl, slot_layout=BLOCKS)
    for kind, splits in ((2, 1), (2, 2), (1, 1)):
        dw.ctx.tc_set_attn_kernel(kind)
        dw.ctx.tc_set_kv_splits(splits)
        bt, pl = dw.alias()
        _check_layout(H, dw, bt, pl, [1])
        err = _attn_err(H, dw, bt, pl, 1)
        assert err <= 1e-2, (kind, splits, err)
        dw.ctx.tc_release_seqs(bt)
    dw.close()


class _NegativeScores(W.Workload):
    """Every query element positive, every table key element negative: all prefix scores are far
    below zero (about -60 log2 units), where the zero keys of unused block tails score 0."""

    def table_kv(self, t):
        k, v = super().table_kv(t)
        kf = -(np.abs(W.bf16_bits_to_f32(k)) * 0.25 + 0.25)
        return W.f32_to_bf16_bits(kf.astype(np.float32)), v

    def suffix_qkv(self, layer):
        q, k, v = super().suffix_qkv(layer)
        qf = np.abs(W.bf16_bits_to_f32(q)) + 0.5
        return W.f32_to_bf16_bits(qf.astype(np.float32)), k, v


def test_alias_negative_scores_fall_back_to_masking(H):
    """All real prefix scores far below zero: the zero keys of the unused tails would outweigh every
    real key by 2^60, which the pipelined path must notice (its reference is negative) and hand
    to the loop that masks them."""
    cfg = _small_cfg(n_tables=3, table_len=(1, 700), batch=1, tables_per_query=(3, 3), suffix_len=(16, 16),
                     capacity=3, n_layers=1)
    wl = _NegativeScores(cfg, np.asarray([150, 210, 170], dtype=np.int32), [np.asarray([0, 1, 2], dtype=np.int32)],
                         np.asarray([16], dtype=np.int32))
    dw = H.DeviceWorkload(wl, slot_layout=BLOCKS)
    for kind in (1, 2):
        dw.ctx.tc_set_attn_kernel(kind)
        dw.ctx.tc_set_kv_splits(1)
        bt, pl = dw.alias()
        qkv = wl.suffix_qkv(0)
        vmax = max(float(np.abs(W.bf16_bits_to_f32(qkv[2])).max()),
                   max(float(np.abs(W.bf16_bits_to_f32(dw.tables_np[t][1])).max()) for t in range(3)))
        err = _attn_err(H, dw, bt, pl, 0, qkv=qkv)
        assert err <= max(1e-2, 3 * 2.0 ** -9 * vmax), (kind, err)
        dw.ctx.tc_release_seqs(bt)
    dw.close()


class _CountingTables(W.Workload):
    """All scores equal (every key zero) and the value of sequence position p - counted over the real
    tokens of the query's concatenation - is the unit vector e_(p mod 128): output row r then holds,
    in column d, the number of visible positions congruent to d over the number of visible positions.
    The unused block tails score exactly what the real keys score, so a tail that is counted, or a
    correction that is off by one, shows as a whole count."""

    def _offsets(self):
        off, acc = {}, 0
        for t in self.queries[0]:
            off[int(t)] = acc
            acc += int(self.table_len[int(t)])
        return off, acc

    def table_kv(self, t):
        c = self.cfg
        n = int(self.table_len[t])
        off, _ = self._offsets()
        k = np.zeros((c.n_layers, n, c.n_kv_heads, c.head_dim), dtype=np.float32)
        v = np.zeros_like(k)
        v[:, np.arange(n), :, (off.get(int(t), 0) + np.arange(n)) % c.head_dim] = 1.0
        return W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)

    def suffix_qkv(self, layer):
        c = self.cfg
        q, k, v = super().suffix_qkv(layer)
        _, P = self._offsets()
        S = int(self.suffix_len[0])
        vf = np.zeros(v.shape, dtype=np.float32)
        vf[np.arange(S), :, (P + np.arange(S)) % c.head_dim] = 1.0
        return q, W.f32_to_bf16_bits(np.zeros(k.shape, dtype=np.float32)), W.f32_to_bf16_bits(vf)


@pytest.mark.parametrize("lens,S,splits", [((100, 333, 207), 48, 1), ((341,) * 12, 128, 8), ((341,) * 12, 128, 1),
                                           ((5, 1, 250, 17, 600), 31, 2), ((15,) * 40, 20, 1)])
def test_alias_counts_every_real_key_once(H, lens, S, splits):
    cfg = W.scaled(W.CONFIGS["c2"], name="count", n_layers=1, n_tables=len(lens), batch=1,
                   tables_per_query=(len(lens), len(lens)), capacity=len(lens), seed=5)
    wl = _CountingTables(cfg, np.asarray(lens, dtype=np.int32), [np.arange(len(lens), dtype=np.int32)],
                         np.asarray([S], dtype=np.int32))
    P = int(sum(lens))
    n_vis = P + np.arange(S) + 1
    want = np.stack([np.bincount(np.arange(n) % 128, minlength=128) for n in n_vis]).astype(np.float64)   # [S][128]
    for kind in (1, 2):
        dw = H.DeviceWorkload(wl, slot_layout=BLOCKS)
        dw.ctx.tc_set_attn_kernel(kind)
        dw.ctx.tc_set_kv_splits(splits)
        bt, pl = dw.alias()
        out, _ = dw.attn_layer(0, bt, pl)
        got = H.out_to_f64(out, dw.cfg) * n_vis[:, None, None]
        dev = float(np.abs(got - want[:, None, :]).max())
        print("tables %s S %d, %d partitions, kernel %d: largest count error %.3f (counts up to %d)" %
              (lens[:5], S, splits, kind, dev, int(want.max())))
        assert dev < 0.5 * max(1.0, want.max() * 2.0 ** -7)      # a whole count cannot hide in the output rounding
        assert dev <= want.max() * 2.0 ** -8 + 1e-6               # and what is left is that rounding
        dw.close()


def test_alias_errors(H):
    from paper_2601_08743_amd import binding as B
    wl = W.make_workload(_small_cfg(batch=2, tables_per_query=(2, 2)))
    dw = H.DeviceWorkload(wl, slot_layout=BLOCKS, load_all=False)
    with pytest.raises(B.TcError) as e:
        dw.alias()
    assert e.value.code == B.TC_ERR_NOT_RESIDENT
    dw.ctx.tc_load_async(list(range(wl.cfg.n_tables)), 0, wl.cfg.n_layers)
    torch.cuda.synchronize()
    with pytest.raises(B.TcError) as e:
        dw.stitch()                                    # the copying stitch reads token rows
    assert e.value.code == B.TC_ERR_INVALID
    with pytest.raises(B.TcError) as e:
        dw.alias(max_blocks=1)
    assert e.value.code == B.TC_ERR_OOM_POOL
    bt, pl = dw.alias()
    dw.ctx.tc_release_seqs(bt)
    bt2, _ = dw.alias()                                # released suffix blocks are handed out again
    np.testing.assert_array_equal(bt, bt2)
    dw.ctx.tc_release_seqs(bt2)
    dw.close()
    rows = H.DeviceWorkload(wl)
    with pytest.raises(B.TcError) as e:
        rows.alias()
    assert e.value.code == B.TC_ERR_INVALID
    rows.close()
    # fp32 contexts cannot keep block-format slots
    cfg = B.make_config(1, 8, 2, 64, B.TC_F32, 64, 2, 32, slot_layout=B.TC_SLOTS_BLOCKS)
    assert B.tc_pool_bytes(cfg) == 0


@pytest.mark.parametrize("seed", list(range(8)))
def test_alias_random_batches_match_the_copying_stitch(H, seed):
    """Seeded random batches (1..5 queries of 1..5 tables with 1..400 tokens, suffixes of 1..200
    tokens, 0..5 partitions) through the stitch that copies nothing, both kernels, three launches
    each: against the checker, against the copying stitch on the same inputs (which differs in
    rounding only: padded key tiles), and bit-identical from launch to launch."""
    rng = np.random.default_rng(7000 + seed)
    n_tables = 7
    B = int(rng.integers(1, 6))
    cfg = W.scaled(W.CONFIGS["c2"], name="rnd%d" % seed, n_layers=1, n_tables=n_tables, batch=B, capacity=n_tables,
                   seed=7000 + seed)
    table_len = rng.integers(1, 401, size=n_tables).astype(np.int32)
    queries = [rng.choice(n_tables, size=int(rng.integers(1, 6)), replace=True).astype(np.int32) for _ in range(B)]
    suffix = rng.integers(1, 201, size=B).astype(np.int32)
    wl = W.Workload(cfg, table_len, queries, suffix)
    splits = int(rng.choice([0, 1, 2, 3, 5]))
    q, k, v = wl.suffix_qkv(0)
    ref = None
    outs = {}
    for layout in (0, BLOCKS):
        for kind in (1, 2):
            dw = H.DeviceWorkload(wl, slot_layout=layout)
            dw.ctx.tc_set_attn_kernel(kind)
            dw.ctx.tc_set_kv_splits(splits)
            bt, pl = dw.alias() if layout else dw.stitch()
            dq, dk, dv = (H.to_dev(x, cfg) for x in (q, k, v))
            rep = []
            for _ in range(3):
                out = torch.full_like(dq, float("nan"))
                dw.ctx.tc_prefill_attn(0, dq, dk, dv, out, wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale, None)
                torch.cuda.synchronize()
                rep.append(out.view(torch.int16).cpu().numpy())
            np.testing.assert_array_equal(rep[0], rep[2])
            np.testing.assert_array_equal(rep[1], rep[2])
            outs[layout, kind] = H.out_to_f64(out, cfg)
            if ref is None:
                ref = H.oracle_attn_layer(wl, dw.tables_np, 0, (q, k, v))
            dw.close()
    for key, got in outs.items():
        for i, r in ref.items():
            sl = slice(int(wl.cu_seqlens[i]), int(wl.cu_seqlens[i + 1]))
            P = int(table_len[queries[i]].sum())
            tol = 1e-2 if P >= 64 else max(1e-2, 2.0 ** -7 * 4.7)
            assert np.abs(got[sl] - r).max() <= tol, (key, i, P, int(suffix[i]), splits)
    assert np.abs(outs[0, 2] - outs[BLOCKS, 2]).max() <= 1e-2
    assert np.abs(outs[0, 1] - outs[BLOCKS, 1]).max() <= 1e-2
