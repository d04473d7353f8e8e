"""The entry point that allocates nothing (tc_prefill_attn_noalloc): its plan and split-KV partials
live in the library's static workspace instead of allocated buffers.  Same kernels, same plan, so
its output must equal tc_prefill_attn's bit for bit - on two calls in a row, the second with a
smaller batch, which finds whatever the first call left in the workspace."""
import numpy as np
import pytest
import torch

from paper_2601_08743_amd import workloads as W

pytestmark = pytest.mark.gpu


def _case(H, cfg, force_kernel=0):
    wl = W.make_workload(cfg)
    dw = H.DeviceWorkload(wl)
    if force_kernel:
        dw.ctx.tc_set_attn_kernel(force_kernel)
    bt, pl = dw.stitch()
    res = []
    for layer in range(cfg.n_layers):
        q, k, v = (H.to_dev(x, cfg) for x in wl.suffix_qkv(layer))
        ref = torch.full_like(q, float("nan"))
        got = torch.full_like(q, float("nan"))
        dw.ctx.tc_prefill_attn(layer, q, k, v, ref, wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale)
        splits = dw.ctx.tc_kv_splits()
        dw.ctx.tc_prefill_attn_noalloc(layer, q, k, v, got, wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale)
        torch.cuda.synchronize()
        assert dw.ctx.tc_kv_splits() == splits
        assert torch.isfinite(ref.float()).all()
        res.append((splits, bool(torch.equal(ref.view(torch.int16), got.view(torch.int16))),
                    float((ref.float() - got.float()).abs().max())))
    # and against the checker, to the bf16 bar, on the last layer
    layer = cfg.n_layers - 1
    want = H.oracle_attn_layer(wl, dw.tables_np, layer, wl.suffix_qkv(layer))
    g64 = H.out_to_f64(got, cfg)
    err = max(float(np.abs(g64[int(wl.cu_seqlens[i]):int(wl.cu_seqlens[i + 1])] - r).max()) for i, r in want.items())
    dw.close()
    return res, err


def test_noalloc_matches_allocating_entry_point():
    import harness as H
    assert torch.cuda.is_available()
    base = W.CONFIGS["c2"]
    big = W.scaled(base, n_layers=2, n_tables=8, tables_per_query=(6, 6), capacity=8)          # P ~ 2.2k, split-KV
    small = W.scaled(base, n_layers=2, n_tables=8, tables_per_query=(2, 2), capacity=8, batch=3,
                     suffix_len=(17, 90), seed=base.seed + 5)                                   # shorter, three queries
    for name, cfg, kern in (("first call (larger)", big, 0), ("second call (smaller)", small, 0),
                            ("general kernel, split", big, 1)):
        res, err = _case(H, cfg, kern)
        print("no-alloc %s: per layer (splits, identical, max diff) %s; vs checker %.3e" % (name, res, err), flush=True)
        assert all(same for _, same, _ in res), res
        assert err <= 1e-2
        if cfg is big:
            assert all(s > 1 for s, _, _ in res), "the case is meant to use split-KV partials"


def test_noalloc_other_kernels():
    """The same through the long-launch kernel (split, so with partials in the workspace) and for a
    decode step (the decode kernels keep one partial per key range there)."""
    import harness as H
    base = W.CONFIGS["c2"]
    big = W.scaled(base, n_layers=1, n_tables=8, tables_per_query=(6, 6), capacity=8)
    res, err = _case(H, big, 4)
    print("no-alloc long-launch kernel: (splits, identical, max diff) %s; vs checker %.3e" % (res, err), flush=True)
    assert all(same for _, same, _ in res) and err <= 1e-2
    # decode: prefill first, then one token per query through both entry points
    cfg = W.scaled(base, n_layers=1, n_tables=8, tables_per_query=(3, 3), capacity=8, batch=3, suffix_len=(5, 40))
    wl = W.make_workload(cfg)
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S = wl.suffix_len.astype(int)
    dw = H.DeviceWorkload(wl, seq_blocks=int(sum(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 4)
    bt, pl = dw.stitch(max_blocks=int(max(-(-(p + s + 1) // 16) for p, s in zip(P, S))) + 1)
    dw.attn_layer(0, bt, pl)
    cur = (P + S).astype(np.int32)
    bt = dw.ctx.tc_grow_seqs(bt, cur + 1)
    rng = np.random.default_rng(3)
    q, k, v = (H.to_dev(W.f32_to_bf16_bits(rng.standard_normal(size=(cfg.batch, h, cfg.head_dim), dtype=np.float32)), cfg)
               for h in (cfg.n_q_heads, cfg.n_kv_heads, cfg.n_kv_heads))
    cu1, one = np.arange(cfg.batch + 1, dtype=np.int32), np.ones(cfg.batch, dtype=np.int32)
    ref, got = torch.full_like(q, float("nan")), torch.full_like(q, float("nan"))
    dw.ctx.tc_prefill_attn(0, q, k, v, ref, cu1, bt, cur, one, wl.sm_scale)
    assert dw.ctx.tc_attn_kernel() == 3 and dw.ctx.tc_kv_splits() > 1
    dw.ctx.tc_prefill_attn_noalloc(0, q, k, v, got, cu1, bt, cur, one, wl.sm_scale)
    torch.cuda.synchronize()
    assert dw.ctx.tc_attn_kernel() == 3
    assert torch.isfinite(ref.float()).all()
    assert torch.equal(ref.view(torch.int16), got.view(torch.int16))
    dw.ctx.tc_release_seqs(bt)
    dw.close()


def test_noalloc_refuses_what_does_not_fit():
    """A batch whose partials exceed the fixed workspace is refused with TC_ERR_CAPACITY and
    enqueues nothing; the allocating entry point still serves it."""
    import harness as H
    from paper_2601_08743_amd import binding as B
    cfg = W.scaled(W.CONFIGS["c5"], n_layers=1, n_tables=12, tables_per_query=(4, 4), capacity=12, batch=48)
    wl = W.make_workload(cfg)
    dw = H.DeviceWorkload(wl)
    dw.ctx.tc_set_kv_splits(4)                 # 48 queries x 8 KV heads x 5 row tiles x 4 partitions: 65 MB of partials
    dw.ctx.tc_set_attn_kernel(1)
    bt, pl = dw.stitch()
    q, k, v = (H.to_dev(x, cfg) for x in wl.suffix_qkv(0))
    out = torch.full_like(q, float("nan"))
    with pytest.raises(B.TcError) as e:
        dw.ctx.tc_prefill_attn_noalloc(0, q, k, v, out, wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale)
    assert e.value.code == B.TC_ERR_CAPACITY
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all()      # nothing ran
    dw.ctx.tc_prefill_attn(0, q, k, v, out, wl.cu_seqlens, bt, pl, wl.suffix_len, wl.sm_scale)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    dw.close()
