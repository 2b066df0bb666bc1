"""Pins of the pipeline simulation against schedules worked by hand and the closed forms that bound it."""
import random

import pytest

from oracle import pipeline_oracle as M


def test_one_stage_one_micro_batch_is_the_round_trip():
    # compute 3, link occupied 2, latency 5: the micro-batch is back after 10, every iteration
    assert M.simulate_period([3.0], [5.0], [2.0], 1) == pytest.approx(10.0)


def test_two_stages_worked_by_hand():
    # stages 1 and 1, links: serialisation 0, latency 1 -> a micro-batch's round trip is 4
    # N = 1, 2, 3, 4: every stage has at most 4 x 1 of work per round trip, nobody queues: period 4
    for n in (1, 2, 3, 4):
        assert M.simulate_period([1.0, 1.0], [1.0, 1.0], [0.0, 0.0], n) == pytest.approx(4.0)
    # N = 6: a stage has 6 of work per iteration, more than the round trip: period 6
    assert M.simulate_period([1.0, 1.0], [1.0, 1.0], [0.0, 0.0], 6) == pytest.approx(6.0)


def test_the_bubble_of_the_method_figure():
    # two engines, micro-batch count = pipeline degree, transfers as long as the compute: each engine
    # works 2 of every 4 time units (half of it is bubble); a third and fourth micro-batch fill it
    c, x = [1.0, 1.0], [1.0, 1.0]
    busy = lambda n: n * 1.0 / M.simulate_period(c, x, [0.0, 0.0], n)
    assert busy(2) == pytest.approx(0.5)
    assert busy(3) == pytest.approx(0.75)
    assert busy(4) == pytest.approx(1.0)
    assert busy(5) == pytest.approx(1.0)


def test_a_serialising_link_is_a_resource_like_a_stage():
    # link 0 is occupied 3 per payload: with 4 micro-batches it needs 12 per iteration although a round trip is 3+1+1+0.5+0.5 = 6
    p = M.simulate_period([1.0, 1.0], [0.5, 0.5], [3.0, 0.0], 4)
    assert p == pytest.approx(12.0)
    # latency alone never limits the rate: it only lengthens the round trip
    assert M.simulate_period([1.0, 1.0], [50.0, 50.0], [0.0, 0.0], 200) == pytest.approx(200.0)


def test_period_is_the_larger_of_round_trip_and_busiest_resource():
    rng = random.Random(0)
    for _ in range(200):
        p = rng.randint(1, 5)
        c = [rng.uniform(0.5, 5.0) for _ in range(p)]
        lat = [rng.uniform(0.0, 20.0) for _ in range(p)]
        ser = [rng.uniform(0.0, 4.0) for _ in range(p)]
        n = rng.randint(1, 12)
        round_trip = sum(c) + sum(lat) + sum(ser)
        busiest = n * max(max(c), max(ser))
        got = M.simulate_period(c, lat, ser, n, iterations=200)
        assert got == pytest.approx(max(round_trip, busiest), rel=1e-6)


def test_first_minimum():
    assert M.best_microbatch_count([9.0, 6.0, 4.0, 4.0, 5.0]) == 3
    assert M.best_microbatch_count([3.0]) == 1
