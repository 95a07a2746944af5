"""The library's request scheduler (Eq. 3, Algorithm 1; Section 3.5) against the scheduler oracle.
Host-only entry points: no GPU is needed."""
import os

import numpy as np
import pytest

import paper_2503_06823_amd as P
from oracle import scheduling as sch
from test_oracle_scheduling_pins import random_queues, read_example


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(P.LIB_PATH):
        from paper_2503_06823_amd.build import build_library
        build_library(force=False)
    return P.lib()


def to_lib(r: sch.Request) -> P.EmoeRequest:
    return P.make_request(r.input_tokens, r.slo, r.first_token_slo, r.run_time, r.g_remaining, r.g_initial, r.delta_e)


def test_hand_worked_example():
    ex = read_example()
    run = [to_lib(r) for r in ex["running"]]
    wait = [to_lib(r) for r in ex["waiting"]]
    assert np.allclose([P.emoe_expected_latency(run, i, ex["c"]) for i in range(len(run))], ex["now"], rtol=1e-12)
    assert np.isclose(P.emoe_expected_latency(run, 1, ex["c"], wait[1]), 4.9, rtol=1e-12)
    assert P.emoe_schedule(wait, run, ex["t_max"], ex["c"]) == ex["admitted"]


@pytest.mark.parametrize("seed", range(5))
def test_schedules_match_the_oracle(seed):
    rng = np.random.default_rng(300 + seed)
    for _ in range(100):
        run, wait = random_queues(rng, int(rng.integers(0, 7)), int(rng.integers(0, 9)))
        t_max, c = int(rng.integers(300, 3000)), float(rng.uniform(0.001, 0.02))
        assert P.emoe_schedule([to_lib(r) for r in wait], [to_lib(r) for r in run], t_max, c) == sch.schedule(wait, run, t_max, c)
        for i in range(len(run)):
            for new in [None] + wait[:1]:
                got = P.emoe_expected_latency([to_lib(r) for r in run], i, c, to_lib(new) if new else None)
                assert np.isclose(got, sch.expected_latency(run, i, c, new), rtol=1e-13)


def test_generation_tick_matches_the_oracle():
    rng = np.random.default_rng(7)
    for _ in range(300):
        r = sch.Request(10, 1.0, 1.0, g_remaining=int(rng.integers(0, 4)), g_initial=int(rng.integers(0, 400)))
        done = bool(rng.integers(0, 2))
        frac = float(rng.choice([0.05, 0.1, 0.0]))
        lr = to_lib(r)
        P.emoe_generation_tick(lr, done, frac)
        assert lr.g_remaining == sch.generation_tick(r, done, frac).g_remaining


def test_argument_errors():
    r = P.make_request(10, 1.0, 1.0)
    assert P.emoe_expected_latency([r], 1, 0.01, check=False) == P.EMOE_ERR_SHAPE
    assert P.lib().emoe_schedule(1, None, 0, None, 10, 0, None, None) == P.EMOE_ERR_NULL
    assert P.lib().emoe_generation_tick(None, 0, 0) == P.EMOE_ERR_NULL
    assert P.emoe_generation_tick(r, False, -1.0, check=False) == P.EMOE_ERR_SHAPE
