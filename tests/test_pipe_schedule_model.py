"""Host model of the pipelined attention path's load schedule (csrc/prefill_attn_bf16.hip, fast_tiles).

The pipelined steps stream K and V tiles from global memory straight into LDS with loads the
compiler does not know about; which tiles have landed is established by hand-counted
`s_waitcnt vmcnt(N)` (a wave's loads complete in issue order), followed by a work-group barrier.
This model replays, for runs of n = 3 .. 40 tiles, exactly what the kernel's rules say - the
initial issue order, what each boundary waits for, what it issues afterwards, which LDS buffer
every step reads - and checks the three properties the scheme stands on:

  1. every tile a step reads (K(s+1) for its QK, V(s-1) for its PV; K(0) for the prime step) has
     landed, for every wave, before the barrier that precedes the step;
  2. a load is issued into a buffer only after the barrier that follows the last step reading the
     tile that buffer held;
  3. nothing is still in flight when the run ends (the general loop then reuses the LDS).

It also lists, per step variant, which score registers the unconditional vector work touches, and
checks that each was written earlier in the same run (no read of a register this launch never
wrote).  The rules below are a transcription of the kernel's; the test pins the *design* of the
schedule for short runs, including n = 3, the length that is kept on the general loop.
CPU only."""
import pytest

LOADS_PER_BATCH = 4          # one tile's K or V: 4 load instructions per wave
N_BUFS = 4


def run_model(n):
    issued = []              # batches in issue order: ("K", tile) / ("V", tile)
    landed_upto = 0          # number of leading batches guaranteed complete (in-order completion)
    buf_k, buf_v = {}, {}    # buffer -> tile it holds (or will hold once landed)
    log = []

    def issue(kind, tile, buf):
        holder = buf_k if kind == "K" else buf_v
        issued.append((kind, tile))
        log.append(("issue", kind, tile, buf, holder.get(buf)))
        holder[buf] = tile

    def wait(allow_batches):
        """s_waitcnt vmcnt(4 * allow_batches): at most that many of the youngest batches still fly."""
        nonlocal landed_upto
        landed_upto = max(landed_upto, len(issued) - allow_batches)

    def has_landed(kind, tile):
        return (kind, tile) in issued and issued.index((kind, tile)) < landed_upto

    # ---- start of the run (n >= 3)
    issue("K", 0, 0); issue("K", 1, 1); issue("K", 2, 2); issue("V", 0, 0)
    if 3 < n:
        issue("K", 3, 3)
    issue("V", 1, 1)
    # prime step: reads K(0)
    wait(4 + (1 if 3 < n else 0))
    assert has_landed("K", 0), (n, "prime reads K(0)")
    reads_done = {("K", 0): "prime"}

    def boundary(s):
        if s >= 0 and s + 5 < n:                         # steady state
            wait(4)
        else:
            younger = (3 + (1 if 3 < n else 0)) if s < 0 else sum(1 for d in (1, 2, 3, 4) if s + d < n)
            wait(younger)
        # ---- barrier: every wave has passed its wait and finished step s ----
        nxt = s + 1
        if nxt + 1 < n:
            assert has_landed("K", nxt + 1), (n, s, "step %d reads K(%d)" % (nxt, nxt + 1))
        if 0 <= nxt - 1 < n:
            assert has_landed("V", nxt - 1), (n, s, "step %d reads V(%d)" % (nxt, nxt - 1))
        if s >= 0 and s + 5 < n:
            todo = [("K", s + 5, (s + 1) % N_BUFS), ("V", s + 3, (s + 3) % N_BUFS)]
        elif s + 3 < n:
            todo = ([("K", s + 5, (s + 1) % N_BUFS)] if s + 5 < n else []) + [("V", s + 3, (s + 3) % N_BUFS)]
        else:
            todo = []
        for kind, tile, buf in todo:
            held = (buf_k if kind == "K" else buf_v).get(buf)
            if held is not None:                          # the tile being overwritten must have been read already
                last_reader = held - 1 if kind == "K" else held + 1     # K(t) is read by step t-1, V(t) by step t+1
                assert last_reader <= s, (n, s, "%s(%d) into buffer %d overwrites %s(%d), read by step %d" % (
                    kind, tile, buf, kind, held, last_reader))
            issue(kind, tile, buf)

    boundary(-1)
    for s in range(0, n + 1):                             # steps 0 .. n
        k_tile, v_tile = s + 1, s - 1
        if k_tile < n:
            assert buf_k[(s + 1) % N_BUFS] == k_tile, (n, s, "K buffer of step")
        if 0 <= v_tile < n:
            assert buf_v[(s - 1) % N_BUFS] == v_tile, (n, s, "V buffer of step")
        if s < n:
            boundary(s)
    assert landed_upto == len(issued), (n, "loads still in flight at the end of the run")
    assert sorted(issued) == sorted([("K", t) for t in range(n)] + [("V", t) for t in range(n)]), (n, "every tile loaded once")
    return log


@pytest.mark.parametrize("n", list(range(3, 41)))
def test_load_schedule_covers_every_read(n):
    run_model(n)


def step_variants(n):
    """(parity, QK, PV) of steps 0 .. n as the kernel instantiates them."""
    out = []
    for s in range(n + 1):
        out.append((s & 1, s + 1 < n, s >= 1))
    return out


@pytest.mark.parametrize("n", list(range(3, 12)))
def test_score_registers_are_written_before_the_vector_work_reads_them(n):
    """The vector work of a step runs unconditionally over stream positions -5 .. 31: positions
    0..15 are score set S[2 PAR] (tile s, keys 32..63), 16..31 set S[2 PAR + 1] (tile s+1, keys
    0..31), negative ones the tail of S[3 - 2 PAR] (tile s, keys 0..31).  QK of step s writes
    S[(2 PAR + 1) & 3] (tile s+1, keys 0..31) and S[(2 PAR + 2) & 3] (keys 32..63); the prime step
    writes S[3] and S[0].  Whatever a step's vector work reads must have been written earlier in the
    same run - by the prime step or by the QK of an earlier (or, for positions 16..31, the same)
    step - also in the steps at the end of a run whose QK does not exist."""
    written = {3, 0}                                       # prime: tile 0 keys 0..31 -> S[3], 32..63 -> S[0]
    for s, (par, qk, pv) in enumerate(step_variants(n)):
        reads_first = {2 * par, 3 - 2 * par}               # positions 0..15 and the previous step's tail
        assert reads_first <= written, (n, s, reads_first - written)
        if qk:
            written |= {(2 * par + 1) & 3, (2 * par + 2) & 3}
        assert (2 * par + 1) in written, (n, s, "positions 16..31 read S[%d]" % (2 * par + 1))


def test_variants_cover_what_the_kernel_instantiates():
    """n = 3 takes: step 0 (QK only), step 1 (QK + PV), steps 2 and 3 (PV only) - the same variants
    as every longer run, with no steady-state pair in between."""
    assert step_variants(3) == [(0, True, False), (1, True, True), (0, False, True), (1, False, True)]
    assert step_variants(4)[-2:] == [(1, False, True), (0, False, True)]
    for n in range(3, 30):
        v = step_variants(n)
        assert v[0] == (0, True, False) and all(x[2] for x in v[1:]) and [x[1] for x in v] == [True] * (n - 1) + [False, False]
