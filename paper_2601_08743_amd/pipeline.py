"""Host loop of the computation-loading pipeline (Sec. 4.2.2) over the C ABI.

The schedule comes from ``tc_plan_pipeline``; this module only carries it out: which library call
is made when.  A range of requests is "asked for" by pinning all its tables and then requesting
them, in batch order, on the load stream; a micro-batch is unpinned as soon as its stitch is
enqueued (the library orders later copies into its slots behind that stitch), or, when the stitch
aliases the table slots instead of copying them, as soon as its attention layers are.
"""
from __future__ import annotations

from typing import Callable, Sequence

import numpy as np

from . import binding as B


def flat_tables(queries: Sequence[np.ndarray], a: int, b: int) -> np.ndarray:
    if b <= a:
        return np.zeros(0, dtype=np.int32)
    return np.concatenate([np.asarray(q, dtype=np.int32) for q in queries[a:b]]).astype(np.int32)


def plan(queries: Sequence[np.ndarray], capacity: int, b_c: int, b_m: int, keep_pinned: bool = False,
         taper: bool = False) -> np.ndarray:
    ids = flat_tables(queries, 0, len(queries))
    cu = np.concatenate([[0], np.cumsum([len(q) for q in queries])]).astype(np.int32)
    return B.tc_plan_pipeline(ids, cu, capacity, b_c, b_m, keep_pinned, taper)


def run(ctx: "B.Context", queries: Sequence[np.ndarray], steps: np.ndarray, l0: int, l1: int, load_stream,
        stitch: Callable[[int, int], object], layers: Callable[[int, int, object], None],
        before_demand: Callable[[], None] = None, keep_pinned: bool = False) -> None:
    """Carry out `steps`.  `stitch(c0, c1)` must enqueue the stitch of requests [c0, c1) and return
    whatever `layers(c0, c1, handle)` needs to run their attention layers and release them.
    `before_demand()` is called ahead of each step's demand loads: a baseline without any overlap
    waits there for the device to go idle (the host otherwise runs ahead, and even demand loads
    overlap the previous step's layers).  `keep_pinned` (schedules planned with it; aliasing
    stitch): a micro-batch's tables are unpinned after its layers are enqueued, not after its stitch.
    `load_stream` may be a list of streams: the load calls then take them in turn, so that the copies
    of consecutive requests are handed to the copy engines from two queues and the start-up gap
    between one copy and the next (tens of microseconds on one queue) is covered by the other queue's
    copy; the library orders slots across streams with its own events."""
    streams = list(load_stream) if isinstance(load_stream, (list, tuple)) else [load_stream]
    turn = [0]

    def ask(a: int, b: int) -> None:
        ids = flat_tables(queries, a, b)
        if ids.size:
            ctx.tc_pin_tables(ids)
            # one load call per request: a stitch waits for the copies of the calls that brought its
            # tables, so a micro-batch at the head of a prefetched range need not wait for the rest
            for i in range(a, b):
                if len(queries[i]):
                    ctx.tc_load_async(np.asarray(queries[i], dtype=np.int32), l0, l1, streams[turn[0] % len(streams)])
                    turn[0] += 1

    for c0, c1, d0, d1, p0, p1 in np.asarray(steps).tolist():
        if before_demand is not None:
            before_demand()
        ask(d0, d1)
        handle = stitch(c0, c1)
        if not keep_pinned:
            ctx.tc_unpin_tables(flat_tables(queries, c0, c1))
        ask(p0, p1)
        layers(c0, c1, handle)
        if keep_pinned:
            ctx.tc_unpin_tables(flat_tables(queries, c0, c1))
