"""Host checks of the micro-batch controller against the event-by-event pipeline simulation: the
modelled iteration time, and the count the incremental search settles on."""
import os
import random
import re

import pytest

from oracle import pipeline_oracle as M
from paper_2507_05043_amd import controller as C
from paper_2507_05043_amd import stage as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(S.LIB_PATH):
        from paper_2507_05043_amd import build
        build.build()
    return S.load_library()


def test_library_exports_every_controller_symbol(lib):
    header = open(os.path.join(ROOT, "include", "molink_controller.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(mbc_[a-z_]+)\s*\(", header))
    assert {"mbc_choose", "mbc_evaluate", "mbc_last_error"} <= names
    for n in sorted(names):
        assert hasattr(lib, n)


def _scenario(rng, stages):
    """Profiles with a point at every batch size (no interpolation between the two sides), links, sizes."""
    num_seqs = rng.randint(1, 40)
    profiles = []
    for _ in range(stages):
        fixed, per_seq = rng.uniform(2.0, 20.0), rng.uniform(0.01, 0.5)
        profiles.append([(b, fixed + per_seq * b) for b in range(1, num_seqs + 1)])
    links = [(rng.uniform(0.0, 30.0), rng.choice([12.5e3, 125e3, 1.25e6])) for _ in range(stages)]   # 100 Mbps .. 10 Gbps
    act_bytes = rng.choice([8192.0, 16384.0])
    return profiles, links, num_seqs, act_bytes, 4.0


def _simulated(profiles, links, num_seqs, act_bytes, tok_bytes, n):
    b = -(-num_seqs // n)
    compute = [dict(p)[b] for p in profiles]
    last = len(profiles) - 1
    serial = [(tok_bytes if i == last else act_bytes) * b / links[i][1] for i in range(len(links))]
    return M.simulate_period(compute, [l[0] for l in links], serial, n, iterations=120)


def test_modelled_iteration_time_equals_the_simulation():
    rng = random.Random(0)
    for _ in range(60):
        profiles, links, num_seqs, act, tok = _scenario(rng, rng.randint(1, 5))
        n = rng.randint(1, num_seqs)
        got = C.evaluate(profiles, links, num_seqs, act, tok, n)
        assert got.num_microbatches == n and got.batch_per_microbatch == -(-num_seqs // n)
        assert got.period_ms == pytest.approx(_simulated(profiles, links, num_seqs, act, tok, n), rel=1e-6)
        assert got.period_ms == max(got.round_trip_ms, got.busiest_ms)


def _resource_times(profiles, links, num_seqs, act_bytes, tok_bytes, n):
    """Per micro-batch: how long every stage and every link is occupied (the simulation's inputs)."""
    b = -(-num_seqs // n)
    last = len(profiles) - 1
    return [dict(p)[b] for p in profiles] + [(tok_bytes if i == last else act_bytes) * b / links[i][1]
                                             for i in range(len(links))]


def _expected_choice(profiles, links, num_seqs, act, tok, n0, n_max):
    """The search read off the simulation: counts are visited upwards while the simulated pipeline still has
    bubbles (its period exceeds what the busiest stage or link needs for its n micro-batches); the first
    shortest simulated period among the visited counts wins."""
    sim = {}
    n = n0
    while True:
        sim[n] = _simulated(profiles, links, num_seqs, act, tok, n)
        saturated = sim[n] <= n * max(_resource_times(profiles, links, num_seqs, act, tok, n)) * (1 + 1e-9)
        if saturated or n >= n_max:
            break
        n += 1
    best = min(sim.values())
    return min(k for k, v in sim.items() if v <= best * (1 + 1e-9)), sim


def test_the_search_runs_while_the_simulated_pipeline_has_bubbles():
    rng = random.Random(1)
    for _ in range(60):
        profiles, links, num_seqs, act, tok = _scenario(rng, rng.randint(2, 5))
        cap = rng.choice([0, 0, 8, 16])
        n0 = max(1, -(-num_seqs // cap)) if cap else 1
        want, sim = _expected_choice(profiles, links, num_seqs, act, tok, n0, num_seqs)
        got = C.choose(profiles, links, num_seqs, act, tok, max_batch_per_microbatch=cap)
        assert got.num_microbatches == want, (got.num_microbatches, want, [round(sim[k], 3) for k in sorted(sim)])
        assert got.period_ms == pytest.approx(sim[want], rel=1e-6)
        if cap:
            assert got.batch_per_microbatch <= cap


def test_the_best_count_lies_past_a_plateau_of_equal_micro_batch_sizes():
    """96 sequences over slow links: from 10 micro-batches on, consecutive counts share a micro-batch size
    (ceil(96/10) == ceil(96/11) == 9 ... ) and with it the round trip, while the stages still idle.  A search
    that compared N + 1 with N alone would stop at the first such pair; the shortest iteration of the whole
    simulated range lies beyond it and is what the controller returns."""
    num_seqs = 96
    profiles = [[(b, 3.0 + 0.05 * b) for b in range(1, num_seqs + 1)]] * 4
    links = [(40.0, 1.25e6)] * 4
    act, tok = 16384.0, 4.0
    sim = {k: _simulated(profiles, links, num_seqs, act, tok, k) for k in range(1, num_seqs + 1)}
    best = min(sim.values())
    first_best = min(k for k, v in sim.items() if v <= best * (1 + 1e-9))
    plateau = next(k for k in range(1, num_seqs) if -(-num_seqs // k) == -(-num_seqs // (k + 1)))
    assert first_best > plateau + 1, (first_best, plateau)
    assert sim[plateau + 1] >= sim[plateau] * (1 - 1e-9)            # the step a pairwise search would stop at
    got = C.choose(profiles, links, num_seqs, act, tok)
    assert got.num_microbatches == first_best, (got.num_microbatches, first_best)
    assert got.period_ms == pytest.approx(best, rel=1e-6)
    assert got.period_ms < sim[plateau] * (1 - 1e-3)             # and it is shorter than where that search stops


def test_interpolation_in_the_profile():
    prof = [[(1, 10.0), (8, 17.0), (32, 41.0)]]
    links = [(0.0, 1e9)]
    at = lambda b: C.evaluate(prof, links, b, 0.0, 0.0, 1).round_trip_ms
    assert at(1) == pytest.approx(10.0) and at(8) == pytest.approx(17.0) and at(32) == pytest.approx(41.0)
    assert at(4) == pytest.approx(13.0)        # 10 + 3/7 * 7
    assert at(20) == pytest.approx(29.0)       # 17 + 12/24 * 24
    assert at(40) == pytest.approx(49.0)       # last segment's slope beyond the last point
    assert C.evaluate([[(4, 9.0)]], links, 2, 0.0, 0.0, 1).round_trip_ms == pytest.approx(9.0)   # constant below / single point


def test_the_settings_of_the_main_table():
    """10 ms links at 10 Gbps, 1 Gbps, 100 Mbps; four stages with the latency profile measured for the
    Llama-3-70B-shaped stage (20 of 80 layers, the sweep table).  While latency dominates, more micro-batches
    than the pipeline has stages shorten the iteration, the more so the slower the link; at 100 Mbps the
    links' serialisation is the busiest resource, whose work per iteration no micro-batch count changes."""
    profile = [(52, 12.5), (103, 18.1), (206, 30.1), (411, 55.9), (820, 109.4), (1639, 221.9)]
    gains = []
    for bytes_per_ms in (1.25e6, 125e3, 12.5e3):
        links = [(10.0, bytes_per_ms)] * 4
        got = C.choose([profile] * 4, links, 256, 8192 * 2.0, 4.0, max_batch_per_microbatch=128, max_microbatches=64)
        degree = C.evaluate([profile] * 4, links, 256, 8192 * 2.0, 4.0, 4)
        assert got.num_microbatches > 4 and got.period_ms <= degree.period_ms
        gains.append(degree.period_ms / got.period_ms)
        if bytes_per_ms == 12.5e3:
            assert got.period_ms == got.busiest_ms and got.busiest_ms == pytest.approx(256 * 16384.0 / 12.5e3, rel=0.02)
    assert gains[1] > gains[0] > 1.0 and gains[2] < gains[1]


def test_invalid_arguments():
    prof, links = [[(1, 1.0)]], [(0.0, 1.0)]
    for bad in (dict(profiles=[[(2, 1.0), (1, 2.0)]]), dict(profiles=[[(1, 0.0)]]), dict(links=[(0.0, 0.0)]),
                dict(links=[(-1.0, 1.0)]), dict(num_seqs=0)):
        args = dict(profiles=prof, links=links, num_seqs=4)
        args.update(bad)
        with pytest.raises(C.ControllerError):
            C.choose(args["profiles"], args["links"], args["num_seqs"], 1.0, 1.0)
    with pytest.raises(C.ControllerError):
        C.evaluate(prof, links, 4, 1.0, 1.0, 5)
    with pytest.raises(C.ControllerError):
        C.choose(prof, links, 100, 1.0, 1.0, max_batch_per_microbatch=10, max_microbatches=5)
