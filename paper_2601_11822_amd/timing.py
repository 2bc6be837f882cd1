"""Measurement loops over the C ABI: one side alone, and both sides co-running.

Used by bench.py and by the offline profiler.  `enqueue_prefill` / `enqueue_decode` are
zero-argument callables that enqueue one layer pass on the context `c` (rs_prefill_layer /
rs_decode_layer with the caller's buffers); everything here is host-side pacing and timing.
"""
from __future__ import annotations

import sys
import time
from typing import Callable, List, Tuple

import numpy as np

PREFILL, DECODE = 0, 1


def _log(*a):
    print(*a, file=sys.stderr, flush=True)


def run_alone(c, side: int, enqueue: Callable[[], None], steps: int, warmup: int, kernel_times: bool = False):
    """Back-to-back passes of one side; returns per-pass GPU ms (events on that side's stream)
    and, if asked, the mean per-kernel ms."""
    for _ in range(warmup):
        enqueue()
    c.sync(side)
    kt = []
    if kernel_times:
        c.set_kernel_timing(True)
        per = []
        for i in range(steps):
            c.mark(side, 0)
            enqueue()
            c.mark(side, 1)
            per.append(c.elapsed_ms(side, 0, 1))
            kt.append(c.kernel_times(side))
        c.set_kernel_timing(False)
        return np.array(per), np.mean(kt, axis=0)
    c.mark(side, 0)
    for i in range(steps):
        enqueue()
        c.mark(side, i + 1)
    c.sync(side)
    per = np.array([c.elapsed_ms(side, i, i + 1) for i in range(steps)])
    return per, None


def run_corun(c, enqueue_prefill: Callable[[], None], enqueue_decode: Callable[[], None], steps: int, warmup: int,
              ahead_p: int = 2, ahead_d: int = 3, dump: bool = False):
    """W + K prefill passes on the prefill side while decode steps run back to back on the decode
    side, both fed by one host loop that polls completion marks and keeps at most `ahead_p`
    passes and `ahead_d` decode steps enqueued beyond what the GPU has finished.  (A deep queue is
    no help and can hurt: with a few hundred commands outstanding the runtime's enqueue calls have
    been seen to block for 10-30 ms until a stream drained, starving both streams.)

    The K timed passes are bracketed on the host clock: from the moment warm-up pass W is seen
    complete (pass W+1 is already queued behind it, so the stream does not idle) to the moment pass
    W+K is seen complete; the poll interval (one loop iteration, < 0.1 ms) bounds the error.
    Returns (host ms for the K passes, per-pass HIP-event ms, HIP-event ms of the decode steps that
    fell entirely inside the timed window, decode steps completed inside the host bracket, the
    host calls that took over 2 ms)."""
    P, D = PREFILL, DECODE
    warmup = max(warmup, 1)
    total = warmup + steps
    c.sync(P); c.sync(D)
    c.mark(D, 0)
    c.mark(P, 0)
    p_enq = p_done = d_enq = d_done = 0
    t_a = t_b = None
    d_at_a = d_at_b = 0
    slow: List[Tuple[str, int, int, float]] = []

    def timed(tag, fn, *a):
        # every runtime call of the loop should return in microseconds; record the ones that do not
        t0 = time.perf_counter()
        out = fn(*a)
        dt = time.perf_counter() - t0
        if dt > 2e-3:
            slow.append((tag, p_enq, d_enq, round(dt * 1e3, 2)))
        return out

    while p_done < total and d_enq < 3900:
        if p_enq < total and p_enq - p_done < ahead_p:
            timed("enqueue_prefill", enqueue_prefill)
            p_enq += 1
            timed("mark_p", c.mark, P, p_enq)
        if d_enq - d_done < ahead_d:
            timed("enqueue_decode", enqueue_decode)
            d_enq += 1
            timed("mark_d", c.mark, D, d_enq)
        while d_done < d_enq and timed("query_d", c.mark_done, D, d_done + 1):
            d_done += 1
        while p_done < p_enq and timed("query_p", c.mark_done, P, p_done + 1):
            p_done += 1
            if p_done == warmup:
                t_a, d_at_a = time.perf_counter(), d_done
            if p_done == total:
                t_b, d_at_b = time.perf_counter(), d_done
    c.sync(P); c.sync(D)
    if t_b is None:
        raise RuntimeError("co-run window not covered by decode steps")
    p_start = c.elapsed_ms(D, 0, warmup, side_end=P)       # timed-window start on the decode stream's clock
    p_ms = np.array([c.elapsed_ms(P, warmup + i, warmup + i + 1) for i in range(steps)])
    p_end = p_start + float(p_ms.sum())
    d_ms = np.array([c.elapsed_ms(D, i, i + 1) for i in range(d_enq)])
    d_end = np.cumsum(d_ms)
    d_beg = d_end - d_ms
    inside = (d_beg >= p_start) & (d_end <= p_end)
    if dump:
        _log("[timing] prefill passes under co-run (event ms): " + " ".join("%.2f" % v for v in p_ms))
        _log("[timing] decode steps (event ms): " + " ".join("%.2f" % v for v in d_ms))
    if slow:
        _log("[timing] host calls over 2 ms (call, prefill passes enqueued, decode steps enqueued, ms): %s" % slow)
    return (t_b - t_a) * 1e3, p_ms, d_ms[inside], d_at_b - d_at_a, slow


def precreate_marks(c, n: int = 3904):
    """Creates every timing event now: an event created while kernels run can stall the GPU."""
    for side in (PREFILL, DECODE):
        for i in range(n):
            c.mark(side, i)
    c.sync(PREFILL); c.sync(DECODE)
