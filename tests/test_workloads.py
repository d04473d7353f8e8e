"""Host-side checks of the seeded input generator (no GPU, no library)."""
import numpy as np
import torch

from paper_2601_08743_amd import workloads as W


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.3895314e38]      # ties, signed zero, near max
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(W.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_configs_have_the_stated_shapes():
    for name, c in W.CONFIGS.items():
        w = W.get(name)
        assert len(w.queries) == c.batch and w.table_len.shape == (c.n_tables,)
        assert w.table_len.min() >= c.table_len[0] and w.table_len.max() <= c.table_len[1]
        for ids in w.queries:
            assert c.tables_per_query[0] <= len(ids) <= c.tables_per_query[1]
            assert len(set(ids.tolist())) == len(ids)
        assert w.suffix_len.min() >= c.suffix_len[0] and w.suffix_len.max() <= c.suffix_len[1]
        assert w.cu_seqlens[-1] == w.suffix_len.sum() and w.cu_tables[-1] == len(w.table_ids)
    w2 = W.get("c2")
    P = int(w2.table_len[w2.queries[0]].sum())
    assert 3000 < P < 6000                      # "~4.5k schema tokens"
    w4 = W.get("c4")
    assert sorted(w4.queries[0].tolist()) == list(range(60)) and not np.array_equal(w4.queries[0], w4.queries[1])


def test_pieces_are_regenerable_and_deterministic():
    w = W.make_workload(W.scaled(W.CONFIGS["c2"], n_layers=2, n_tables=3, table_len=(5, 9),
                                 tables_per_query=(2, 2)))
    k1, v1 = w.table_kv(1)
    k1b, v1b = W.make_workload(w.cfg).table_kv(1)
    np.testing.assert_array_equal(k1, k1b); np.testing.assert_array_equal(v1, v1b)
    assert k1.dtype == np.uint16 and k1.shape == (2, int(w.table_len[1]), 4, 128)
    assert not np.array_equal(k1, v1) and not np.array_equal(k1, w.table_kv(2)[0][:, :k1.shape[1]])
    q, k, v = w.suffix_qkv(0)
    assert q.shape == (w.total_suffix, 28, 128) and k.shape == (w.total_suffix, 4, 128)
    f = W.storage_to_f64(q, "bf16")
    assert abs(f.std() - 1.0) < 0.02 and abs(f.mean()) < 0.02


def test_zipf_popularity_is_skewed():
    w = W.get("c3")
    counts = np.bincount(w.table_ids, minlength=40)
    assert counts[:10].sum() > counts[30:].sum()
