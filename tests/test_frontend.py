"""The library's host front end (Table Trie + Alg. 1 matching, greedy reranking) against the
brute-force checker, through the C ABI.  Integer work: results must be identical.  No GPU needed."""
import numpy as np
import pytest

import oracle
from paper_2601_08743_amd import binding as B


def _trie(tables):
    t = B.Trie()
    for tid, toks in tables.items():
        t.tc_trie_insert(tid, toks)
    return t


def test_alg1_hand_worked_prompt_through_the_abi():
    tables = {10: [1, 2, 3], 11: [1, 2], 12: [7, 8, 9, 7], 13: [9]}
    s = [5, 1, 2, 3, 1, 2, 4, 7, 8, 9, 7, 9, 1, 2]
    got, n = _trie(tables).tc_trie_match(s)
    assert n == 5 and got == [(10, 1), (11, 4), (12, 7), (13, 11), (11, 12)]


@pytest.mark.parametrize("seed,vocab,n_tables,max_len,prompt_len", [(1, 4, 30, 6, 3000), (2, 50, 80, 40, 5000),
                                                                     (3, 2, 10, 9, 2000), (4, 32000, 40, 300, 8000)])
def test_alg1_equals_brute_force(seed, vocab, n_tables, max_len, prompt_len):
    """Random tables over a small vocabulary (many accidental and nested matches) and a prompt that
    embeds whole tables, truncated tables and noise."""
    rng = np.random.default_rng(seed)
    tables, seen = {}, set()
    for t in range(n_tables):
        toks = tuple(rng.integers(0, vocab, size=int(rng.integers(1, max_len + 1))).tolist())
        if toks not in seen:
            seen.add(toks)
            tables[t] = list(toks)
    ids = list(tables)
    s = []
    while len(s) < prompt_len:
        r = rng.random()
        if r < 0.5:
            s += tables[ids[int(rng.integers(len(ids)))]]
        elif r < 0.7:
            toks = tables[ids[int(rng.integers(len(ids)))]]
            s += toks[:max(1, len(toks) - 1)]
        else:
            s += rng.integers(0, vocab, size=int(rng.integers(1, 8))).tolist()
    got, n = _trie(tables).tc_trie_match(s)
    want = oracle.trie_match(tables, s)
    assert n == len(want) and got == want


def test_trie_argument_checks():
    t = B.Trie()
    t.tc_trie_insert(3, [1, 2, 3])
    for bad in ((3, [9]), (4, [1, 2, 3]), (5, []), (-1, [7])):           # repeated id, repeated content, empty, negative id
        with pytest.raises(B.TcError):
            t.tc_trie_insert(*bad)
    t.tc_trie_insert(4, [1, 2])                                          # a prefix of another table is fine
    assert t.tc_trie_match([1, 2, 3, 1, 2, 9])[0] == [(3, 0), (4, 3)]
    got, n = t.tc_trie_match([1, 2, 3, 1, 2, 9], cap=1)                   # more matches than room: count still reported
    assert n == 2 and got == [(3, 0)]
    assert t.tc_trie_match([])[0] == []


@pytest.mark.parametrize("seed,n_queries,n_tables", [(1, 64, 80), (2, 200, 130), (3, 1, 5), (4, 33, 64), (5, 50, 1)])
def test_rerank_equals_brute_force(seed, n_queries, n_tables):
    rng = np.random.default_rng(seed)
    sets = [rng.choice(n_tables, size=int(rng.integers(0, min(n_tables, 12) + 1)), replace=False).tolist()
            for _ in range(n_queries)]
    ids = np.concatenate([np.asarray(x, dtype=np.int32) for x in sets]) if any(sets) else np.zeros(0, np.int32)
    cu = np.concatenate([[0], np.cumsum([len(x) for x in sets])]).astype(np.int32)
    for anchor in sorted({0, n_queries // 2, n_queries - 1}):
        got = B.tc_rerank(ids, cu, n_tables, anchor).tolist()
        assert got == oracle.rerank(sets, anchor)


def test_rerank_argument_checks():
    with pytest.raises(B.TcError):
        B.tc_rerank([0, 9], [0, 2], 5, 0)              # table id out of range
    with pytest.raises(B.TcError):
        B.tc_rerank([0, 1], [0, 2], 5, 1)              # anchor out of range
    assert B.tc_rerank([], [0], 5, 0).tolist() == []


def test_reranking_reduces_cache_misses_on_a_grouped_batch():
    """The point of the reranking (Sec. 4.2.1, Fig. 1(a)): a batch that alternates between two
    groups of tables thrashes a small cache; visited in reranked order each group is loaded once."""
    a, b = [0, 1, 2], [3, 4, 5]
    sets = [a, b] * 6
    cu = np.arange(0, 3 * 12 + 1, 3, dtype=np.int32)
    ids = np.asarray(sum(sets, []), dtype=np.int32)
    order = B.tc_rerank(ids, cu, 6, 0).tolist()

    def misses(seq):
        m = oracle.LRUModel(3)
        return sum(1 for q in seq for t in sets[q] if m.access(t)[0] == 0)

    assert misses(range(12)) == 36 and misses(order) == 6


def test_workload_prompts_resolve_to_their_tables():
    """The synthetic prompts (schema texts of the query's tables in prompt order, then the suffix)
    matched against the trie of all tables give back exactly the table ids that drive the stitch,
    with each table starting where the previous one ended."""
    from paper_2601_08743_amd import workloads as W
    wl = W.make_workload(W.scaled(W.CONFIGS["c3"], batch=8))
    trie = B.Trie()
    for t in range(wl.cfg.n_tables):
        trie.tc_trie_insert(t, wl.table_tokens(t))
    for i in range(wl.cfg.batch):
        m, n = trie.tc_trie_match(wl.prompt_tokens(i))
        ids = wl.queries[i].tolist()
        assert [tid for tid, _ in m][:len(ids)] == ids
        starts = np.concatenate([[0], np.cumsum(wl.table_len[wl.queries[i]])[:-1]]).tolist()
        assert [p for _, p in m][:len(ids)] == starts
        assert m == oracle.trie_match({t: wl.table_tokens(t).tolist() for t in range(wl.cfg.n_tables)},
                                      wl.prompt_tokens(i).tolist())


# ------------------------------------------------------------------------------------ pipeline schedule

def _flat(sets):
    ids = np.asarray([t for q in sets for t in q], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum([len(q) for q in sets])]).astype(np.int32)
    return ids, cu


def test_pipeline_plan_equals_the_checker():
    """Sec. 4.2.2: the library's schedule (incremental window bookkeeping) against the checker's
    (set unions written out), on random batches including empty requests, repeated tables inside a
    request, b_m = 0 and windows cut short by the cache size."""
    rng = np.random.default_rng(21)
    n_err = 0
    for trial in range(300):
        n = int(rng.integers(0, 50))
        sets = [rng.integers(0, 14, size=int(rng.integers(0, 5))).tolist() for _ in range(n)]
        b_c, b_m, C = int(rng.integers(1, 7)), int(rng.integers(0, 12)), int(rng.integers(2, 15))
        ids, cu = _flat(sets)
        keep, taper = bool(trial & 1), bool(trial & 2)
        try:
            want = oracle.plan_pipeline(sets, C, b_c, b_m, keep_pinned=keep, taper=taper)
        except ValueError:
            with pytest.raises(B.TcError) as e:
                B.tc_plan_pipeline(ids, cu, C, b_c, b_m, keep, taper)
            assert e.value.code == B.TC_ERR_CAPACITY
            n_err += 1
            continue
        got = B.tc_plan_pipeline(ids, cu, C, b_c, b_m, keep, taper)
        assert [tuple(r) for r in got.tolist()] == want, (trial, sets, C, b_c, b_m)
    assert 3 < n_err < 200           # both outcomes were exercised


def test_pipeline_plan_rejects_bad_arguments():
    ids, cu = _flat([[0, 1], [2]])
    for C, b_c, b_m in ((4, 0, 1), (4, 1, -1), (-1, 1, 1)):
        with pytest.raises(B.TcError) as e:
            B.tc_plan_pipeline(ids, cu, C, b_c, b_m)
        assert e.value.code == B.TC_ERR_INVALID
    with pytest.raises(B.TcError):
        B.tc_plan_pipeline(ids, [1, 2, 3], 4, 1, 1)            # offsets must start at 0
    with pytest.raises(B.TcError):
        B.tc_plan_pipeline(ids, [0, 2, 1], 4, 1, 1)            # and not decrease
