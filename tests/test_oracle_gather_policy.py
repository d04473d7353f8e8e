"""Pins for the integer side of the checker: gather order, block tables,
replacement rules (App. A)."""
import numpy as np
import pytest

import oracle
from golden_io import read_replacement_traces


def _coded_tables(lens, L, Hkv, D):
    """K whose every element spells (table, token, layer, head, d)."""
    tabs = {}
    for t, n in enumerate(lens):
        a = np.zeros((L, n, Hkv, D), dtype=np.int64)
        tt, ll, uu, hh, dd = np.meshgrid([t], np.arange(L), np.arange(n), np.arange(Hkv), np.arange(D),
                                         indexing="ij")
        a[:] = (((tt * 1000 + uu) * 10 + ll) * 10 + hh)[0] * 100 + dd[0]
        tabs[t] = a
    return tabs


def test_gather_spells_the_concatenation():
    lens = [5, 1, 17, 16, 3]
    L, Hkv, D = 2, 2, 3
    tabs = _coded_tables(lens, L, Hkv, D)
    for ids in ([2, 0, 4], [4, 3, 2, 1, 0], [1], [3, 3, 0]):     # incl. a repeated table
        out = oracle.stitch(tabs, ids)
        assert out.shape == (L, sum(lens[t] for t in ids), Hkv, D)
        p = 0
        for t in ids:
            for u in range(lens[t]):
                for l in range(L):
                    for h in range(Hkv):
                        for d in range(D):
                            assert out[l, p, h, d] == (((t * 1000 + u) * 10 + l) * 10 + h) * 100 + d
                p += 1
        assert p == out.shape[1]


def test_gather_permutation_permutes_segments_and_keeps_bytes():
    rng = np.random.default_rng(0)
    lens = [7, 19, 4]
    tabs = {t: rng.integers(0, 2 ** 16, size=(3, n, 2, 8), dtype=np.uint16) for t, n in enumerate(lens)}
    a = oracle.stitch(tabs, [0, 1, 2])
    b = oracle.stitch(tabs, [2, 0, 1])
    np.testing.assert_array_equal(a[:, :7], b[:, 4:11])
    np.testing.assert_array_equal(a[:, 7:26], b[:, 11:30])
    np.testing.assert_array_equal(a[:, 26:], b[:, :4])
    np.testing.assert_array_equal(a, np.concatenate([tabs[0], tabs[1], tabs[2]], axis=1))


def test_prefix_lengths():
    tl = [10, 20, 30, 40]
    p = oracle.prefix_lengths(tl, [3, 0, 1, 1, 2], [0, 2, 2, 5])
    assert p.tolist() == [50, 0, 70]


def test_block_table_model_invariants():
    m = oracle.SeqBlockModel(first_block=100, n_blocks=40, block_size=16)
    P, S = [33, 0, 15, 160], [5, 1, 1, 16]
    bt = m.stitch(P, S, max_blocks=12)
    need = [3, 1, 1, 11]
    flat = bt[bt >= 0]
    assert sorted(flat.tolist()) == list(range(100, 116))          # lowest blocks first
    assert len(set(flat.tolist())) == flat.size                    # no block twice
    for i, n in enumerate(need):
        assert (bt[i, :n] >= 100).all() and (bt[i, :n] < 140).all()
        assert (bt[i, n:] == -1).all()
        assert (np.diff(bt[i, :n]) > 0).all()
    # batch order: query 0 holds 100..102, query 1 holds 103, ...
    assert bt[0, :3].tolist() == [100, 101, 102] and bt[1, 0] == 103 and bt[3, 0] == 105
    # all or nothing
    assert m.stitch([16 * 25], [0], max_blocks=30) is None and len(m.free) == 24
    assert m.stitch([16], [0], max_blocks=0) is None
    # release returns blocks; the lowest is reused first; two identical runs agree
    m.release(bt[1:3])
    bt2 = m.stitch([1], [0], max_blocks=12)
    assert bt2[0, 0] == 103
    m2 = oracle.SeqBlockModel(100, 40, 16)
    np.testing.assert_array_equal(m2.stitch(P, S, 12), bt)


def test_replacement_rules_against_hand_worked_traces(golden_dir):
    cls = {"lru": oracle.LRUModel, "fifo": oracle.FIFOModel, "lfu": oracle.LFUModel}
    cases = read_replacement_traces(golden_dir)
    assert {c[0] for c in cases} == {"lru", "fifo", "lfu"}
    for policy, cap, accesses, expected in cases:
        assert oracle.replay(cls[policy](cap), accesses) == expected, (policy, cap, accesses)


@pytest.mark.parametrize("policy", ["lru", "fifo", "lfu"])
def test_replacement_invariants(policy):
    cls = {"lru": oracle.LRUModel, "fifo": oracle.FIFOModel, "lfu": oracle.LFUModel}[policy]
    rng = np.random.default_rng(1)
    C = 5
    m = cls(C)
    resident = set()
    for t in rng.integers(0, 12, size=400):
        hit, ev = m.access(int(t))
        assert hit == (int(t) in resident)
        if not hit:
            assert (ev is None) == (len(resident) < C)
            if ev is not None:
                assert ev in resident and ev != t
                resident.remove(ev)
            resident.add(int(t))
        assert len(resident) <= C
    # capacity >= distinct items: nothing is ever evicted
    m = cls(12)
    assert all(e == -1 for _, _, e in oracle.replay(m, rng.integers(0, 12, size=200)))


def test_lru_equals_stack_distance_rule():
    """LRU hits exactly when fewer than C distinct other items were touched since the last access."""
    rng = np.random.default_rng(2)
    acc = rng.integers(0, 9, size=300).tolist()
    C = 4
    tr = oracle.replay(oracle.LRUModel(C), acc)
    for i, (t, hit, _) in enumerate(tr):
        prev = [j for j in range(i) if acc[j] == t]
        if not prev:
            assert hit == 0
        else:
            assert hit == int(len(set(acc[prev[-1] + 1:i])) < C)


def test_alias_block_table_hand_worked():
    """Concatenation by block table alone: slot s owns blocks 3s, 3s+1, 3s+2 (tables of up to 48
    tokens); sequence blocks start at 12.  Tables: 7 -> slot 2 (20 tokens: two blocks, 4 tokens in
    the second), 9 -> slot 0 (16 tokens: one full block), 4 -> slot 3 (1 token)."""
    slots = oracle.SlotModel(4)
    # misses fill slots 0, 1, 2, 3 in order; then table 4 evicts table 5 and inherits its slot
    slots.apply([(9, 0, -1), (8, 0, -1), (7, 0, -1), (5, 0, -1), (9, 1, -1), (4, 0, 5)])
    assert slots.slot == {9: 0, 8: 1, 7: 2, 4: 3}
    seq = oracle.SeqBlockModel(12, 8)
    table_len = {7: 20, 9: 16, 4: 1, 8: 48}
    bt, padded, valid = oracle.alias_block_table(seq, slots.slot, table_len, [[7, 9], [], [4, 7]], [17, 3, 0], 3, 6)
    assert bt.tolist() == [[6, 7, 0, 12, 13, -1], [14, -1, -1, -1, -1, -1], [9, 6, 7, -1, -1, -1]]
    assert padded.tolist() == [48, 0, 48]
    assert valid == [[16, 4, 16], [], [1, 16, 4]]
    assert seq.free == [15, 16, 17, 18, 19]
