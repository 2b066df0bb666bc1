"""Plain CPU model of the chunked hand-off of a stage's activation payload.

TEST INFRASTRUCTURE.  Slow, written for checking by eye.  It shares no code with
the HIP library and must not be imported by it.

What it models (paper section 4.2, "Chunk Transmission").  A stage's output is
one activation row per processed token; a prefill request therefore hands over
up to a thousand times more bytes than a decode request, and a decode payload
that becomes ready while a prefill payload is on the wire waits behind it.
The remedy: finished requests' volumes go into two queues by phase; the sender
always serves the decode queue first; prefill volumes are cut into chunks of a
fixed size, so a decode volume waits for at most the one chunk that is on the
wire when it arrives.

Readings where the section is silent: a micro-batch's rows are packed sequence
after sequence; a sequence with one new token is a decode request, with more a
prefill request; consecutive decode rows form one transfer; every prefill
request's span is chunked on its own, chunks in address order, the last one
shorter; each queue is first-in first-out across micro-batches; the sender
moves one transfer at a time and chooses the next one when the current one has
finished.

Pins (tests/test_oracle_handoff_pins.py): hand-worked layouts and drain
orders, byte conservation, the at-most-one-chunk bound, and the degenerate
cases (no prefill, no decode, chunk larger than a span).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

DECODE, PREFILL = 0, 1
Transfer = Tuple[int, int, int]            # (kind, byte offset in the payload, bytes)


def split_payload(q_lens: Sequence[int], row_bytes: int, chunk_bytes: int) -> Tuple[List[Transfer], List[Transfer]]:
    """The transfers of one micro-batch: (decode runs, prefill chunks), each in address order."""
    if row_bytes < 1 or chunk_bytes < 1:
        raise ValueError("row_bytes and chunk_bytes must be positive")
    decode: List[Transfer] = []
    prefill: List[Transfer] = []
    row = 0
    run_start = None
    for q in q_lens:
        q = int(q)
        if q < 1:
            raise ValueError("every sequence contributes at least one row")
        if q == 1:
            if run_start is None:
                run_start = row
        else:
            if run_start is not None:
                decode.append((DECODE, run_start * row_bytes, (row - run_start) * row_bytes))
                run_start = None
            begin, end = row * row_bytes, (row + q) * row_bytes
            off = begin
            while off < end:
                n = min(chunk_bytes, end - off)
                prefill.append((PREFILL, off, n))
                off += n
        row += q
    if run_start is not None:
        decode.append((DECODE, run_start * row_bytes, (row - run_start) * row_bytes))
    return decode, prefill


def drain_order(submits: Sequence[Tuple[int, Sequence[int]]], row_bytes: int, chunk_bytes: int):
    """Order in which the sender moves the transfers of several micro-batches.

    submits: (picks_before, q_lens) per micro-batch in submission order; `picks_before` is how many
    transfers the sender had already chosen when the micro-batch was handed to it (non-decreasing).
    Returns [(ticket, kind, offset, bytes)], ticket = index of the micro-batch.
    """
    decode_q: List[Tuple[int, int, int, int]] = []
    prefill_q: List[Tuple[int, int, int, int]] = []
    order = []
    nxt = 0
    last = -1
    for s, _ in submits:
        if s < last:
            raise ValueError("submissions must be ordered in time")
        last = s
    while True:
        while nxt < len(submits) and submits[nxt][0] <= len(order):
            d, p = split_payload(submits[nxt][1], row_bytes, chunk_bytes)
            decode_q.extend((nxt, *t) for t in d)
            prefill_q.extend((nxt, *t) for t in p)
            nxt += 1
        if decode_q:
            order.append(decode_q.pop(0))
        elif prefill_q:
            order.append(prefill_q.pop(0))
        elif nxt < len(submits):
            raise ValueError("a micro-batch is submitted after more picks than its predecessors can supply")
        else:
            return order
