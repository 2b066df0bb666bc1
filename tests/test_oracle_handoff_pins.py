"""Pins of the hand-off model (two queues by phase, decode first, fixed-size prefill chunks) against
hand-worked cases and the properties the method is built for."""
import random

import pytest

from oracle import handoff_oracle as M

D, P = M.DECODE, M.PREFILL


def test_layout_of_a_mixed_micro_batch_worked_by_hand():
    # rows: [prefill 5 rows][decode][decode][prefill 2 rows][decode], 10 bytes per row, chunks of 24 bytes
    decode, prefill = M.split_payload([5, 1, 1, 2, 1], 10, 24)
    assert decode == [(D, 50, 20), (D, 90, 10)]
    assert prefill == [(P, 0, 24), (P, 24, 24), (P, 48, 2), (P, 70, 20)]


def test_degenerate_layouts():
    assert M.split_payload([1, 1, 1], 8, 64) == ([(D, 0, 24)], [])
    assert M.split_payload([4], 8, 1000) == ([], [(P, 0, 32)])              # chunk larger than the span
    assert M.split_payload([4], 8, 32) == ([], [(P, 0, 32)])                # exactly one chunk
    assert M.split_payload([4], 8, 31) == ([], [(P, 0, 31), (P, 31, 1)])
    with pytest.raises(ValueError):
        M.split_payload([2, 0], 8, 32)
    with pytest.raises(ValueError):
        M.split_payload([2], 8, 0)


def test_every_byte_is_transferred_exactly_once():
    rng = random.Random(0)
    for _ in range(50):
        q = [rng.choice([1, 1, 1, rng.randint(2, 40)]) for _ in range(rng.randint(1, 12))]
        row, chunk = rng.choice([2, 16, 100]), rng.choice([1, 7, 64, 4096])
        d, p = M.split_payload(q, row, chunk)
        covered = sorted((o, o + n) for _, o, n in d + p)
        assert covered[0][0] == 0 and covered[-1][1] == sum(q) * row
        assert all(a[1] == b[0] for a, b in zip(covered, covered[1:]))
        assert all(n <= chunk for _, _, n in p)
        assert sum(n for _, _, n in d) == sum(1 for x in q if x == 1) * row


def test_a_decode_payload_overtakes_the_rest_of_a_prefill_payload():
    # the case of the method's figure: a long prefill is being sent when a decode batch finishes
    # micro-batch 0: one prefill of 10 rows -> 5 chunks; micro-batch 1 (4 decode rows) arrives while
    # chunk 1 is on the wire (two picks made): it goes next, the remaining 3 chunks follow
    order = M.drain_order([(0, [10]), (2, [1, 1, 1, 1])], row_bytes=8, chunk_bytes=16)
    assert order == [(0, P, 0, 16), (0, P, 16, 16), (1, D, 0, 32), (0, P, 32, 16), (0, P, 48, 16), (0, P, 64, 16)]
    # without chunking (one chunk = the whole span) the decode payload waits for all 80 bytes
    order = M.drain_order([(0, [10]), (1, [1, 1, 1, 1])], row_bytes=8, chunk_bytes=80)
    assert order == [(0, P, 0, 80), (1, D, 0, 32)]


def test_decode_first_inside_one_micro_batch_and_fifo_inside_each_queue():
    order = M.drain_order([(0, [3, 1, 1]), (0, [1, 2])], row_bytes=4, chunk_bytes=8)
    assert order == [(0, D, 12, 8), (1, D, 0, 4), (0, P, 0, 8), (0, P, 8, 4), (1, P, 4, 8)]


def test_a_decode_transfer_waits_for_at_most_one_prefill_chunk_chosen_after_its_arrival():
    rng = random.Random(1)
    for _ in range(100):
        submits, picks = [], 0
        for _ in range(rng.randint(1, 6)):
            q = [rng.choice([1, 1, rng.randint(2, 30)]) for _ in range(rng.randint(1, 6))]
            submits.append((picks, q))
            d, p = M.split_payload(q, 4, 16)
            picks += rng.randint(0, len(d) + len(p))        # how far the sender gets before the next arrival
        order = M.drain_order(submits, 4, 16)
        arrival = {k: s for k, (s, _) in enumerate(submits)}
        for i, (ticket, kind, _, _) in enumerate(order):
            if kind != D:
                continue
            # prefill chunks chosen at or after this payload's arrival and before this transfer
            late = [j for j in range(arrival[ticket], i) if order[j][1] == P]
            assert late == [], "the sender chose a prefill chunk while a decode transfer was waiting"
        # conservation per micro-batch
        for k, (_, q) in enumerate(submits):
            assert sum(n for t, _, _, n in order if t == k) == sum(q) * 4


def test_submissions_must_be_ordered_and_reachable():
    with pytest.raises(ValueError):
        M.drain_order([(3, [1]), (1, [1])], 4, 16)
    with pytest.raises(ValueError):
        M.drain_order([(0, [1]), (5, [1])], 4, 16)     # only one pick can have happened before the second arrival
