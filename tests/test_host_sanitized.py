"""The library's host-only logic, built with g++ under the address and undefined-behaviour
sanitizers and driven from a script (csrc/host_check.cpp): replacement rules (App. A) with pins,
the sequence-block allocator, the attention planner, the front end (Alg. 1, Eq. 1-2, the
Sec. 4.2.2 schedule).  Every answer is compared with the CPU checker's models or with the
invariants the kernels rely on; any sanitizer report fails the run.  No GPU needed."""
import os
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2601_08743_amd", "csrc")

# key tiles whose block ids one work item may keep in LDS, per kernel (csrc/tc_types.h)
CAP_GENERAL, CAP_PIPE, CAP_PP = 256, 1024, 1024


@pytest.fixture(scope="module")
def exe(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("hc") / "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", out, os.path.join(CSRC, "host_check.cpp")]
    subprocess.check_call(cmd)
    return out


def run(exe, script: str):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], input=script, capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    return r.stdout.splitlines()


@pytest.mark.parametrize("policy,model", [(0, oracle.LRUModel), (1, oracle.FIFOModel), (2, oracle.LFUModel)])
def test_rules_with_pins_equal_the_models(exe, policy, model):
    rng = np.random.default_rng(100 + policy)
    cap = 5
    m = model(cap)
    pins, script, want = {}, ["rule %d %d" % (policy, cap)], []
    for _ in range(3000):
        r = rng.random()
        t = int(rng.integers(0, 14))
        if r < 0.15 and sum(1 for v in pins.values() if v) < cap - 1:
            pins[t] = pins.get(t, 0) + 1
            script.append("p %d" % t)
        elif r < 0.3 and any(pins.values()):
            t = [k for k, v in pins.items() if v][int(rng.integers(0, sum(1 for v in pins.values() if v)))]
            pins[t] -= 1
            script.append("u %d" % t)
        else:
            hit, ev = m.access(t, pinned=[k for k, v in pins.items() if v])
            want.append("r %d %d %d" % (t, 1 if hit else 0, -1 if ev is None else ev))
            script.append("r %d" % t)
    assert run(exe, "\n".join(script) + "\n") == want


def test_rule_refuses_when_everything_is_pinned(exe):
    got = run(exe, "rule 0 2\nr 1\nr 2\np 1\np 2\nr 3\nu 2\nr 3\n")
    assert got == ["r 1 0 -1", "r 2 0 -1", "r 3 0 refused", "r 3 0 2"]


def test_allocator_equals_the_sorted_set_model(exe):
    rng = np.random.default_rng(7)
    first, n = 40, 300
    free = set(range(first, first + n))
    held, script, want = [], ["seq %d %d" % (first, first + n)], []
    for _ in range(400):
        if rng.random() < 0.55 or not held:
            k = int(rng.integers(1, 40))
            script.append("t %d" % k)
            if k > len(free):
                want.append("t oom")
                continue
            got = sorted(free)[:k]
            free -= set(got)
            held.append(got)
            want.append("t " + " ".join(map(str, got)))
        else:
            blk = held.pop(int(rng.integers(0, len(held))))
            free |= set(blk)
            script.append("f %d %s" % (len(blk), " ".join(map(str, blk))))
    script.append("f 1 5")                       # not a sequence block: refused, no crash
    want.append("f bad 5")
    assert run(exe, "\n".join(script) + "\n") == want


def _plan(exe, Hq, Hkv, PS, splits=0, rb=0, kernel=0, dtype=1, D=128):
    lines = run(exe, "plan %d %d %d %d %d %d %d %d %s\n" % (dtype, Hq, Hkv, D, splits, rb, kernel, len(PS),
                                                          " ".join("%d %d" % ps for ps in PS)))
    head = list(map(int, lines[0].split()[1:]))
    rows = [tuple(map(int, l.split()[1:])) for l in lines[1:] if l.startswith("i ")]
    items = [r[:7] for r in rows]
    assert head[0] == len(items)
    ghead = [l for l in lines if l.startswith("groups ")][0].split()
    groups = [tuple(map(int, l.split()[1:])) for l in lines if l.startswith("g ")]
    info = dict(max_splits=head[1], decode=head[2], pingpong=head[3], pipelined=head[4], row_blocks=head[5], ok=head[6],
                n_groups=int(ghead[2]), groups=groups, item_group=[r[7] for r in rows])
    assert int(ghead[1]) == len(groups)
    return info, items


def _check_plan(info, items, Hq, Hkv, PS, dtype=1):
    """What the kernels rely on: every (query, KV head, row tile) is covered by partitions that cut
    its key tiles [0, n_tiles) into consecutive non-empty ranges, and no range is longer than the
    block-id table of the kernel that runs it."""
    assert info["ok"] == 1
    G = Hq // Hkv
    if info["decode"]:
        cap, rt, unified = CAP_GENERAL, None, False
    else:
        cap = 10 ** 9 if dtype == 0 else CAP_PP if info["pingpong"] else CAP_PIPE if info["pipelined"] else CAP_GENERAL
        rt = 4 if dtype == 0 else 128 * info["row_blocks"]
        unified = dtype == 0 or bool(info["pingpong"])
    cover = {}
    if not info["decode"] and dtype == 1:
        # the merge launch goes by the group table: one entry per (query, KV head, row tile), in the
        # order of the items' group numbers, each with the partition count its items carry
        assert len(info["groups"]) == info["n_groups"]
        for (q, kvh, m0, tb, te, split, ns), grp in zip(items, info["item_group"]):
            if q < 0:
                continue
            assert 0 <= grp < info["n_groups"]
            g_kvh, g_m0, g_ns, g_cu, g_S = info["groups"][grp]
            assert (g_kvh, g_m0, g_ns, g_S) == (kvh, m0, ns, PS[q][1]), (q, kvh, m0, ns, info["groups"][grp])
    for q, kvh, m0, tb, te, split, ns in items:
        if q < 0:
            continue
        empty_ok = info["decode"] and PS[q][0] == 0          # a decode step over an empty prefix: the token sees itself only
        assert (0 < te - tb or empty_ok) and te - tb <= cap, (q, tb, te, cap)
        cover.setdefault((q, kvh, m0), []).append((split, tb, te, ns))
    for i, (P, S) in enumerate(PS):
        if S == 0:
            assert not any(k[0] == i for k in cover)
            continue
        if info["decode"]:
            n_tiles, rows = -(-P // 64), [0]
        else:
            n_tiles = -(-(P + S) // 64) if unified else -(-P // 64) + -(-S // 64)
            rows = list(range(0, S * G, rt))
        for kvh in range(Hkv):
            for m0 in rows:
                parts = sorted(cover[(i, kvh, m0)])
                assert [p[0] for p in parts] == list(range(len(parts))) and all(p[3] == len(parts) for p in parts)
                assert parts[0][1] == 0 and parts[-1][2] == n_tiles
                assert all(a[2] == b[1] for a, b in zip(parts, parts[1:]))
    return max([te - tb for q, _, _, tb, te, _, _ in items if q >= 0], default=0)


def test_planner_partition_limit_with_forced_splits(exe):
    """A long prefix with a short suffix and a forced split count: the cut by weight used to leave
    a first partition of 259 tiles, three more than the general kernel's block-id table holds."""
    PS = [(32400, 168)]
    for splits in (1, 2, 3):
        for kernel in (1, 2, 4, 0):
            info, items = _plan(exe, 28, 4, PS, splits=splits, kernel=kernel)
            longest = _check_plan(info, items, 28, 4, PS)
            print("P=32400 S=168 forced splits %d kernel %d -> %d partitions, longest %d tiles" %
                  (splits, kernel, info["max_splits"], longest))
    info, items = _plan(exe, 28, 4, PS, splits=2, kernel=1)
    assert info["max_splits"] >= 3 and not info["pipelined"]
    # longer than every kernel's table (1095 key tiles): the pipelined kernel is planned twice (for
    # the general kernel's 256 tiles first, then for its own 1024), and the merge groups must be
    # those of the second pass - they once were the first pass's, with five partitions each
    PS = [(70001, 37), (100, 5)]
    for kernel, splits, want in ((2, 1, 2), (2, 4, 4), (4, 1, 2), (1, 2, 5), (0, 0, None)):
        info, items = _plan(exe, 4, 1, PS, splits=splits, kernel=kernel)
        _check_plan(info, items, 4, 1, PS)
        if want is not None:
            assert info["max_splits"] == want, (kernel, splits, info["max_splits"])


def test_planner_paper_shapes(exe):
    c4 = [(24625, 512)] * 4
    info, items = _plan(exe, 32, 8, c4)
    _check_plan(info, items, 32, 8, c4)
    assert info["pingpong"] == 1 and info["max_splits"] == 1 and sum(1 for it in items if it[0] >= 0) == 256
    info, items = _plan(exe, 32, 8, c4, kernel=2)              # the pipelined kernel takes c4 unsplit as well
    _check_plan(info, items, 32, 8, c4)
    assert info["pipelined"] == 1 and info["max_splits"] == 1 and sum(1 for it in items if it[0] >= 0) == 512
    info, items = _plan(exe, 32, 8, c4, kernel=1)              # the general kernel must split
    _check_plan(info, items, 32, 8, c4)
    assert info["max_splits"] >= 2
    c2 = [(4086, 128)]
    info, items = _plan(exe, 28, 4, c2)
    _check_plan(info, items, 28, 4, c2)
    assert info["pipelined"] == 1 and info["max_splits"] == 8
    dec = [(5000, 1), (17, 1), (0, 1), (900, 0)]
    info, items = _plan(exe, 28, 4, dec)
    assert info["decode"] == 1
    _check_plan(info, items, 28, 4, dec)


def test_decode_ranges_make_one_round_of_even_work_groups(exe):
    """A decode step is planned for one round of work-groups on the 256 CUs, all about equally long:
    the paper-shaped batches come out as at most 256 items, none longer than the shortest common
    range length that fits, and a long sequence is cut into more ranges than a short one."""
    import sys
    sys.path.insert(0, ROOT)
    from paper_2601_08743_amd import workloads as W
    for name, Hq, Hkv in (("c3", 28, 4), ("c4", 32, 8), ("c2", 28, 4)):
        wl = W.get(name)
        PS = [(int(wl.table_len[q].sum()) + int(s), 1) for q, s in zip(wl.queries, wl.suffix_len)]
        info, items = _plan(exe, Hq, Hkv, PS)
        assert info["decode"] == 1
        longest = _check_plan(info, items, Hq, Hkv, PS)
        real = [it for it in items if it[0] >= 0]
        tiles = [-(-P // 64) for P, _ in PS]
        assert len(real) <= 256, (name, len(real))
        # no shorter common range length would have fitted the 256 CUs (or the floor of six tiles was hit)
        L = longest
        fits = lambda L: sum(Hkv * max(1, -(-t // L)) for t in tiles) <= 256
        assert fits(L) and (L <= 6 or not fits(L - 1)), (name, L)
        per_q = {}
        for q, kvh, m0, tb, te, split, ns in real:
            per_q[q] = ns
        order = sorted(range(len(tiles)), key=lambda i: tiles[i])
        assert all(per_q[a] <= per_q[b] for a, b in zip(order, order[1:])), name
        lens = [te - tb for _, _, _, tb, te, _, _ in real]
        assert lens == sorted(lens, reverse=True), "longest items first"
        print("%s decode: %d items, ranges of %d..%d key tiles, %d..%d ranges per sequence" % (
            name, len(real), min(lens), max(lens), min(per_q.values()), max(per_q.values())))
    # more (query, KV head) pairs than CUs: one range each, several rounds
    PS = [(3000 + 17 * i, 1) for i in range(100)]
    info, items = _plan(exe, 28, 4, PS)
    assert info["decode"] == 1 and info["max_splits"] == 1 and sum(1 for it in items if it[0] >= 0) == 400
    _check_plan(info, items, 28, 4, PS)
    # a sequence longer than one item's block-id table is cut whatever the batch looks like
    PS = [(64 * 700, 1)] + [(500, 1)] * 80
    info, items = _plan(exe, 28, 4, PS)
    _check_plan(info, items, 28, 4, PS)
    assert info["max_splits"] == 3


def test_planner_random_batches(exe):
    rng = np.random.default_rng(11)
    for _ in range(150):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 4, 5, 7, 8]))
        B = int(rng.integers(1, 7))
        PS = [(int(rng.choice([0, 1, 63, 64, 65, int(rng.integers(0, 3000)), int(rng.integers(0, 70000))])),
               int(rng.choice([0, 1, 64, int(rng.integers(0, 600))]))) for _ in range(B)]
        dtype = int(rng.random() < 0.85)
        kw = dict(splits=int(rng.choice([0, 0, 1, 2, 5, 40])), rb=int(rng.choice([0, 0, 0, 1, 2])) if dtype else 0,
                  kernel=int(rng.choice([0, 0, 1, 2, 3, 4])) if dtype else 0)
        info, items = _plan(exe, Hkv * G, Hkv, PS, dtype=dtype, D=128 if dtype else 64, **kw)
        _check_plan(info, items, Hkv * G, Hkv, PS, dtype=dtype)


def test_front_end_equals_the_checker(exe):
    rng = np.random.default_rng(5)
    tables, seen = {}, set()
    for t in range(40):
        toks = tuple(rng.integers(0, 4, size=int(rng.integers(1, 7))).tolist())
        if toks not in seen:
            seen.add(toks)
            tables[t] = list(toks)
    s = rng.integers(0, 4, size=4000).tolist()
    script = ["trie %d" % len(tables)] + ["%d %d %s" % (t, len(v), " ".join(map(str, v))) for t, v in tables.items()]
    script.append("match %d %s" % (len(s), " ".join(map(str, s))))
    sets = [sorted(rng.choice(30, size=int(rng.integers(1, 9)), replace=False).tolist()) for _ in range(120)]
    qs = "\n".join("%d %s" % (len(q), " ".join(map(str, q))) for q in sets)
    script.append("rerank %d 30 3\n%s" % (len(sets), qs))
    cases = [(12, 4, 4, 0, 0), (12, 4, 8, 0, 1), (10, 3, 0, 0, 0), (16, 8, 8, 1, 1)]
    for cap, bc, bm, keep, taper in cases:
        script.append("pipeline %d %d %d %d %d %d\n%s" % (len(sets), cap, bc, bm, keep, taper, qs))
    out = run(exe, "\n".join(script) + "\n")
    want = oracle.trie_match(tables, s)
    assert out[0] == "match %d" % len(want) + "".join(" %d %d" % m for m in want)
    assert out[1] == "rerank " + " ".join(map(str, oracle.rerank(sets, 3)))
    at = 2
    for cap, bc, bm, keep, taper in cases:
        steps = oracle.plan_pipeline(sets, cap, bc, bm, keep_pinned=bool(keep), taper=bool(taper))
        assert out[at] == "pipeline %d" % len(steps)
        got = [tuple(map(int, l.split()[1:])) for l in out[at + 1:at + 1 + len(steps)]]
        assert got == [tuple(st) for st in steps]
        at += 1 + len(steps)
