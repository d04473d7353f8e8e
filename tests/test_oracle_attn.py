"""Pins for the fp64 attention checker (oracle.prefill_attn / oracle.attn_row).

None of these re-type the checker's own loop: each compares it with something
fixed from outside - a library causal attention over the whole sequence, closed
forms, a brute-force enumeration of which keys a row may see, and reductions
between head configurations.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _full_causal_sdpa(q_all, k_all, v_all, scale):
    """Library routine: causal attention over one whole sequence, fp64, GQA by
    repeating KV heads.  [N][H][D] in, [N][Hq][D] out."""
    Hq, Hkv = q_all.shape[1], k_all.shape[1]
    G = Hq // Hkv
    q = torch.from_numpy(q_all).permute(1, 0, 2)[None]
    k = torch.from_numpy(k_all).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    v = torch.from_numpy(v_all).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("P,S,Hq,Hkv,D", [(37, 9, 4, 2, 16), (0, 7, 2, 2, 8), (50, 1, 6, 2, 32),
                                          (5, 20, 8, 2, 64), (129, 33, 7, 1, 128)])
def test_stitched_prefix_equals_full_causal(P, S, Hq, Hkv, D):
    """Cached KV taken from the same sequence: the suffix rows of a full causal
    attention must come out (App. E.4: the uncached part attends to everything
    before it; spec: oracle self-check 1)."""
    rng = np.random.default_rng(P * 1000 + S)
    N = P + S
    q_all, k_all, v_all = _rand(rng, N, Hq, D), _rand(rng, N, Hkv, D), _rand(rng, N, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    ref = _full_causal_sdpa(q_all, k_all, v_all, scale)[P:]

    # cut the prefix at random boundaries into "tables", stitch them back in order
    cuts = sorted(rng.choice(np.arange(1, P), size=min(3, max(P - 1, 0)), replace=False)) if P > 1 else []
    bounds = [0] + list(cuts) + [P]
    tables_k = {j: k_all[None, bounds[j]:bounds[j + 1]] for j in range(len(bounds) - 1)}
    tables_v = {j: v_all[None, bounds[j]:bounds[j + 1]] for j in range(len(bounds) - 1)}
    ids = list(range(len(bounds) - 1))
    if P == 0:
        k_seq = np.zeros((0, Hkv, D)); v_seq = np.zeros((0, Hkv, D))
    else:
        k_seq = oracle.stitch(tables_k, ids)[0]
        v_seq = oracle.stitch(tables_v, ids)[0]
    out = oracle.prefill_attn(q_all[P:], k_seq, v_seq, k_all[P:], v_all[P:], scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_wrong_table_order_is_detected():
    """The pin above has teeth: stitching the segments in another order changes
    nothing for attention (softmax is permutation invariant over keys), but swapping
    K segments without V does; and dropping the causal limit does."""
    rng = np.random.default_rng(7)
    P, S, Hq, Hkv, D = 24, 6, 2, 1, 8
    N = P + S
    q_all, k_all, v_all = _rand(rng, N, Hq, D), _rand(rng, N, Hkv, D), _rand(rng, N, Hkv, D)
    scale = 0.3
    ref = _full_causal_sdpa(q_all, k_all, v_all, scale)[P:]
    k_perm = np.concatenate([k_all[12:24], k_all[:12]])
    out = oracle.prefill_attn(q_all[P:], k_perm, v_all[:P], k_all[P:], v_all[P:], scale)
    assert np.abs(out - ref).max() > 1e-3
    v_perm = np.concatenate([v_all[12:24], v_all[:12]])
    out = oracle.prefill_attn(q_all[P:], k_perm, v_perm, k_all[P:], v_all[P:], scale)
    np.testing.assert_allclose(out, ref, atol=1e-12)


def test_softmax_rows_sum_to_one_and_mask_by_enumeration():
    """Self-checks 2 and 3: every row's weights sum to 1; the set of keys with a
    non-zero weight equals the set listed by brute force; its size summed over the
    rows is S*P + S(S+1)/2 (the count used for FLOPs)."""
    rng = np.random.default_rng(3)
    Hq, Hkv, D = 2, 1, 4
    for P, S in itertools.product(range(0, 6), range(1, 6)):
        q = _rand(rng, S, Hq, D)
        ks, vs = _rand(rng, P, Hkv, D), _rand(rng, P, Hkv, D)
        kn, vn = _rand(rng, S, Hkv, D), _rand(rng, S, Hkv, D)
        _, w = oracle.prefill_attn(q, ks, vs, kn, vn, 0.5, return_weights=True)
        assert w.shape == (S, Hq, P + S)
        np.testing.assert_allclose(w.sum(-1), 1.0, atol=1e-12)
        visible = 0
        for r in range(S):
            # brute force: schema positions, then the suffix positions up to and including r
            allowed = set(range(P)) | {P + t for t in range(S) if t <= r}
            for h in range(Hq):
                got = {j for j in range(P + S) if w[r, h, j] != 0.0}
                assert got == allowed, (P, S, r)
            visible += len(allowed)
        assert visible == S * P + S * (S + 1) // 2


def test_closed_forms():
    rng = np.random.default_rng(11)
    P, S, Hq, Hkv, D = 13, 5, 4, 2, 8
    q = _rand(rng, S, Hq, D)
    vs, vn = _rand(rng, P, Hkv, D), _rand(rng, S, Hkv, D)
    # (a) all keys identical -> uniform weights -> mean of the visible values
    kconst = _rand(rng, 1, Hkv, D)
    ks, kn = np.repeat(kconst, P, 0), np.repeat(kconst, S, 0)
    out = oracle.prefill_attn(q, ks, vs, kn, vn, 0.7)
    for r in range(S):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            mean = np.concatenate([vs[:, g], vn[:r + 1, g]]).mean(0)
            np.testing.assert_allclose(out[r, h], mean, atol=1e-13)
    # (b) constant V -> that constant, whatever the keys
    ks, kn = _rand(rng, P, Hkv, D), _rand(rng, S, Hkv, D)
    c = _rand(rng, Hkv, D)
    out = oracle.prefill_attn(q, ks, np.broadcast_to(c, (P, Hkv, D)).copy(), kn,
                              np.broadcast_to(c, (S, Hkv, D)).copy(), 0.7)
    for h in range(Hq):
        np.testing.assert_allclose(out[:, h], np.broadcast_to(c[h // 2], (S, D)), atol=1e-13)
    # (c) one schema key aligned with q and scaled up -> its value dominates
    j = 4
    qq = np.zeros((S, Hq, D)); qq[..., 0] = 1.0
    ks2 = np.zeros((P, Hkv, D)); ks2[j, :, 0] = 200.0
    out = oracle.prefill_attn(qq, ks2, vs, np.zeros((S, Hkv, D)), vn, 1.0)
    for h in range(Hq):
        np.testing.assert_allclose(out[:, h], np.broadcast_to(vs[j, h // 2], (S, D)), atol=1e-12)
    # (d) sm_scale = 0 -> uniform weights regardless of q and k
    out = oracle.prefill_attn(q, ks, vs, kn, vn, 0.0)
    np.testing.assert_allclose(out[2, 3], np.concatenate([vs[:, 1], vn[:3, 1]]).mean(0), atol=1e-13)
    # (e) first suffix row with no prefix sees exactly one key: output = its value
    out = oracle.prefill_attn(q, np.zeros((0, Hkv, D)), np.zeros((0, Hkv, D)), kn, vn, 0.7)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], vn[0, h // 2], atol=1e-15)


def test_two_key_softmax_by_hand():
    """One row, two visible keys, scalar head: weights are the logistic of the
    score difference; numbers worked by hand."""
    q = np.array([[[2.0]]])
    ks = np.array([[[1.0]]]); vs = np.array([[[10.0]]])
    kn = np.array([[[-1.0]]]); vn = np.array([[[20.0]]])
    scale = 0.5
    # scores: 0.5*2*1 = 1, 0.5*2*(-1) = -1 -> w0 = 1/(1+e^-2)
    w0 = 1.0 / (1.0 + np.exp(-2.0))
    out = oracle.prefill_attn(q, ks, vs, kn, vn, scale)
    np.testing.assert_allclose(out[0, 0, 0], 10.0 * w0 + 20.0 * (1 - w0), atol=1e-13)
    assert abs(out[0, 0, 0] - 11.192029220221176) < 1e-12


def test_gqa_reductions():
    rng = np.random.default_rng(5)
    P, S, D = 17, 6, 16
    # G = 1 is plain multi-head attention: each head can be run on its own
    Hq = Hkv = 3
    q, ks, vs = _rand(rng, S, Hq, D), _rand(rng, P, Hkv, D), _rand(rng, P, Hkv, D)
    kn, vn = _rand(rng, S, Hkv, D), _rand(rng, S, Hkv, D)
    out = oracle.prefill_attn(q, ks, vs, kn, vn, 0.25)
    for h in range(Hq):
        o1 = oracle.prefill_attn(q[:, h:h + 1], ks[:, h:h + 1], vs[:, h:h + 1],
                                 kn[:, h:h + 1], vn[:, h:h + 1], 0.25)
        np.testing.assert_array_equal(out[:, h:h + 1], o1)
    # heads of one group given the same q produce the same output; heads of
    # different groups do not
    Hq, Hkv = 6, 2
    q1 = _rand(rng, S, 1, D)
    q = np.repeat(q1, Hq, 1)
    ks, vs = _rand(rng, P, Hkv, D), _rand(rng, P, Hkv, D)
    kn, vn = _rand(rng, S, Hkv, D), _rand(rng, S, Hkv, D)
    out = oracle.prefill_attn(q, ks, vs, kn, vn, 0.25)
    np.testing.assert_array_equal(out[:, 0], out[:, 1]); np.testing.assert_array_equal(out[:, 1], out[:, 2])
    np.testing.assert_array_equal(out[:, 3], out[:, 5])
    assert np.abs(out[:, 2] - out[:, 3]).max() > 1e-3
    # and group g of the GQA run equals an MHA run on KV head g alone
    o_g1 = oracle.prefill_attn(q[:, 3:6], np.repeat(ks[:, 1:2], 3, 1), np.repeat(vs[:, 1:2], 3, 1),
                               np.repeat(kn[:, 1:2], 3, 1), np.repeat(vn[:, 1:2], 3, 1), 0.25)
    np.testing.assert_array_equal(out[:, 3:6], o_g1)


def test_row_helper_agrees_with_library_and_loop():
    rng = np.random.default_rng(9)
    P, S, Hq, Hkv, D = 40, 8, 4, 2, 32
    N = P + S
    q_all, k_all, v_all = _rand(rng, N, Hq, D), _rand(rng, N, Hkv, D), _rand(rng, N, Hkv, D)
    scale = 1 / np.sqrt(D)
    ref = _full_causal_sdpa(q_all, k_all, v_all, scale)
    for (r, h) in [(0, 0), (3, 1), (7, 3)]:
        g = h // 2
        row = oracle.attn_row(q_all[P + r, h], k_all[:P + r + 1, g], v_all[:P + r + 1, g], scale)
        np.testing.assert_allclose(row, ref[P + r, h], atol=1e-13)


def test_large_logits_do_not_overflow():
    """Scores of +-800 would overflow exp() without the max subtraction."""
    q = np.full((2, 1, 4), 10.0)
    ks = np.full((3, 1, 4), 20.0); ks[1] = -20.0
    vs = np.arange(12.0).reshape(3, 1, 4)
    kn = np.full((2, 1, 4), 20.0); vn = np.ones((2, 1, 4))
    out = oracle.prefill_attn(q, ks, vs, kn, vn, 1.0)
    assert np.isfinite(out).all()
    # keys 0, 2 and the visible suffix keys tie at the maximum; key 1 vanishes
    np.testing.assert_allclose(out[0, 0], (vs[0, 0] + vs[2, 0] + 1.0) / 3.0, atol=1e-12)
    np.testing.assert_allclose(out[1, 0], (vs[0, 0] + vs[2, 0] + 2.0) / 4.0, atol=1e-12)
