"""Pins for the checker's front end: Alg. 1 (Table Trie Matching, Sec. 4.1.2) and the greedy
query reranking of Sec. 4.2.1 (Eq. 1-2).  Hand-worked cases and properties that hold for any
correct implementation."""
import numpy as np

import oracle


def test_alg1_hand_worked_prompt():
    # tables: A = [1 2 3], B = [1 2], C = [7 8 9 7], D = [9]
    tables = {10: [1, 2, 3], 11: [1, 2], 12: [7, 8, 9, 7], 13: [9]}
    #      0  1  2  3  4  5  6  7  8  9 10 11 12 13
    s = [5, 1, 2, 3, 1, 2, 4, 7, 8, 9, 7, 9, 1, 2]
    # p=0: 5 no; p=1: A (longest of A, B) -> p=4: B ([1 2] then 4) -> p=6: 4 no; p=7: C -> p=11: D;
    # p=12: B
    assert oracle.trie_match(tables, s) == [(10, 1), (11, 4), (12, 7), (13, 11), (11, 12)]


def test_alg1_longest_match_wins_and_partial_match_is_no_match():
    tables = {0: [4, 4], 1: [4, 4, 4, 4], 2: [4, 4, 4, 4, 9]}
    assert oracle.trie_match(tables, [4, 4, 4, 4, 4, 4]) == [(1, 0), (0, 4)]
    assert oracle.trie_match(tables, [4, 4, 4, 4, 9]) == [(2, 0)]
    assert oracle.trie_match(tables, [4]) == []                     # a prefix of a table is not a table
    assert oracle.trie_match(tables, []) == []


def test_alg1_matches_are_disjoint_in_order_and_spell_the_tables():
    rng = np.random.default_rng(11)
    tables = {t: rng.integers(0, 6, size=int(rng.integers(1, 6))).tolist() for t in range(12)}
    # make contents distinct
    seen, uniq = set(), {}
    for t, toks in tables.items():
        if tuple(toks) not in seen:
            seen.add(tuple(toks))
            uniq[t] = toks
    s = rng.integers(0, 6, size=400).tolist()
    m = oracle.trie_match(uniq, s)
    end = 0
    for tid, p in m:
        assert p >= end
        assert s[p:p + len(uniq[tid])] == uniq[tid]
        # nothing longer matches there, and every skipped position matches nothing
        assert not any(len(t) > len(uniq[tid]) and s[p:p + len(t)] == t for t in uniq.values())
        for gap in range(end, p):
            assert not any(s[gap:gap + len(t)] == t for t in uniq.values())
        end = p + len(uniq[tid])
    for gap in range(end, len(s)):
        assert not any(s[gap:gap + len(t)] == t for t in uniq.values())


def test_rerank_hand_worked_batch():
    # the cache-unfriendly alternation of Fig. 1(a): two groups of queries over tables {1,2,3} and {4,5,6}
    sets = [[1, 2, 3], [4, 5, 6], [1, 2, 3], [4, 5, 6], [1, 2], [4, 5]]
    # from 0: d(0,2)=0 -> 2; from 2: d(2,4)=1 -> 4; from 4: d(4,1)=5, d(4,3)=5, d(4,5)=4 -> 5;
    # from 5: d(5,1)=1, d(5,3)=1 -> 1 (lowest index); then 3
    assert oracle.rerank(sets, 0) == [0, 2, 4, 5, 1, 3]
    assert oracle.rerank(sets, 3) == [3, 1, 5, 4, 0, 2]


def test_rerank_is_a_greedy_nearest_neighbour_walk():
    rng = np.random.default_rng(5)
    n_tables = 70                                  # spans more than one 64-bit word
    sets = [rng.choice(n_tables, size=int(rng.integers(0, 9)), replace=False).tolist() for _ in range(40)]
    for anchor in (0, 17, 39):
        order = oracle.rerank(sets, anchor)
        assert sorted(order) == list(range(40)) and order[0] == anchor
        bits = np.zeros((40, n_tables), dtype=np.uint8)
        for i, ts in enumerate(sets):
            bits[i, ts] = 1
        for step in range(1, 40):
            cur, nxt = order[step - 1], order[step]
            rest = order[step:]
            d = {j: int((bits[cur] ^ bits[j]).sum()) for j in rest}       # Eq. 2 written with XOR
            assert d[nxt] == min(d.values())
            assert nxt == min(j for j in rest if d[j] == d[nxt])


def test_rerank_trivial_batches():
    assert oracle.rerank([], 0) == []
    assert oracle.rerank([[3]], 0) == [0]
    assert oracle.rerank([[], [], []], 1) == [1, 0, 2]
