"""Plain CPU model of a pipeline of inference engines that passes micro-batches from stage to stage
over slow links: an event-by-event simulation that returns the steady-state time per iteration.

TEST INFRASTRUCTURE.  It shares no code with the library and must not be imported by it.

What it models (paper section 4.1, "Dynamic Micro-batch").  The engines form a chain; every
micro-batch visits them in order, its activations travel to the next engine after each stage, and
after the last stage the chosen tokens travel back to the first, where the micro-batch's next
iteration can begin.  A stage runs one micro-batch at a time, in arrival order; a link carries one
payload at a time (its latency overlaps with the next payload, its serialisation does not).  When the
transfers are not negligible a stage that has finished its micro-batches idles until the next one
arrives - the pipeline bubble - and more micro-batches fill it.

Readings where the section is silent: all micro-batches of an iteration have the same size; the
order of micro-batches on every stage and link is fixed (0, 1, .., N-1, then the next iteration);
compute and transfer times are deterministic.

Pins (tests/test_oracle_pipeline_pins.py): hand-worked schedules of small pipelines, the two closed
forms that bound the period (a micro-batch's round trip; the busiest resource's work per iteration)
and the regimes in which each is attained.
"""
from __future__ import annotations

from typing import List, Sequence


def simulate_period(compute_ms: Sequence[float], link_latency_ms: Sequence[float], link_serial_ms: Sequence[float],
                    num_microbatches: int, iterations: int = 64) -> float:
    """Steady-state milliseconds per iteration.

    compute_ms[p]: time stage p needs for one micro-batch; link p carries a micro-batch's payload from
    stage p to stage p+1 (the last link back to stage 0): it is occupied for link_serial_ms[p] and the
    payload arrives link_latency_ms[p] after the link has sent it.
    """
    p_count, n = len(compute_ms), num_microbatches
    if not (len(link_latency_ms) == len(link_serial_ms) == p_count) or n < 1 or p_count < 1:
        raise ValueError("one link per stage and at least one micro-batch and stage")
    stage_free = [0.0] * p_count
    link_free = [0.0] * p_count
    ready = [0.0] * n                     # when micro-batch j may start its next iteration at stage 0
    done: List[float] = []                # completion time of every iteration (last micro-batch back at stage 0)
    for _ in range(iterations):
        for j in range(n):
            t = ready[j]
            for p in range(p_count):
                start = max(t, stage_free[p])
                finish = start + compute_ms[p]
                stage_free[p] = finish
                send = max(finish, link_free[p])
                link_free[p] = send + link_serial_ms[p]
                t = send + link_serial_ms[p] + link_latency_ms[p]
            ready[j] = t
        done.append(ready[n - 1])
    half = iterations // 2
    return (done[-1] - done[half - 1]) / (iterations - half)


def best_microbatch_count(periods: Sequence[float], rel_tol: float = 1e-9) -> int:
    """1-based index of the first minimum of per-iteration times listed for N = 1, 2, ..."""
    best = min(periods)
    for i, v in enumerate(periods):
        if v <= best * (1.0 + rel_tol):
            return i + 1
    raise AssertionError
