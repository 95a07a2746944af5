"""Pins of the scheduler oracle (oracle/scheduling.py): the hand-worked example of Eq. 3 and
Algorithm 1, and properties that hold for any input.  CPU only."""
import os

import numpy as np

from oracle import scheduling as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scheduler_example.txt")


def read_example():
    ex = {"running": [], "waiting": []}
    for line in open(GOLDEN):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] == "c": ex["c"] = float(p[1])
        elif p[0] == "t_max": ex["t_max"] = int(p[1])
        elif p[0] == "running":
            ex["running"].append(sch.Request(int(p[1]), float(p[2]), 0.0, run_time=float(p[3]), g_remaining=int(p[4]),
                                             g_initial=int(p[4])))
        elif p[0] == "waiting":
            ex["waiting"].append(sch.Request(int(p[1]), float(p[2]), float(p[3]), g_remaining=int(p[4]),
                                             g_initial=int(p[4]), delta_e=float(p[5])))
        elif p[0] == "n": ex["n"] = [int(v) for v in p[1:]]
        elif p[0] == "now": ex["now"] = [float(v) for v in p[1:]]
        elif p[0] == "admitted": ex["admitted"] = [int(v) for v in p[1:]]
    return ex


def test_hand_worked_example():
    ex = read_example()
    run = ex["running"]
    assert [sch.finishes_after(run, i) for i in range(len(run))] == ex["n"]
    assert np.allclose([sch.expected_latency(run, i, ex["c"]) for i in range(len(run))], ex["now"], rtol=1e-12)
    y = ex["waiting"][1]
    assert np.isclose(sch.expected_latency(run, 1, ex["c"], y), 4.9, rtol=1e-12)
    assert sch.schedule(ex["waiting"], run, ex["t_max"], ex["c"]) == ex["admitted"]


def random_queues(rng, n_run, n_wait):
    run = [sch.Request(int(rng.integers(10, 400)), float(rng.uniform(2, 12)), 0.0, run_time=float(rng.uniform(0, 3)),
                       g_remaining=int(rng.integers(1, 200)), g_initial=200) for _ in range(n_run)]
    wait = [sch.Request(int(rng.integers(10, 400)), float(rng.uniform(2, 12)), float(rng.integers(1, 6)) * 0.5,
                        g_remaining=int(rng.integers(20, 200)), g_initial=200, delta_e=float(rng.uniform(0, 1.5)))
            for _ in range(n_wait)]
    return run, wait


def test_properties_of_any_schedule():
    rng = np.random.default_rng(3)
    for _ in range(200):
        run, wait = random_queues(rng, int(rng.integers(0, 6)), int(rng.integers(0, 8)))
        t_max, c = int(rng.integers(300, 3000)), float(rng.uniform(0.001, 0.02))
        adm = sch.schedule(wait, run, t_max, c)
        assert len(set(adm)) == len(adm)
        keys = [(wait[i].first_token_slo, i) for i in adm]
        assert keys == sorted(keys)                                    # tried, hence admitted, in order of stringency
        if adm:                                                        # the token limit holds (strictly, as in the listing)
            assert sum(s.input_tokens for s in run) + sum(wait[i].input_tokens for i in adm) < t_max
        # replay: at each admission no running request that met its SLO misses it through the new request
        cur = list(run)
        for i in adm:
            for j, s in enumerate(cur):
                if sch.expected_latency(cur, j, c) < s.slo:
                    assert sch.expected_latency(cur, j, c, wait[i]) < s.slo
            cur.append(wait[i])


def test_special_cases():
    w = [sch.Request(100, 5.0, 1.0, g_remaining=10, g_initial=10)]
    assert sch.schedule(w, [], 1000, 0.01) == [0]                       # nothing running: only the token limit counts
    assert sch.schedule(w, [], 100, 0.01) == []                         # 100 + 0 < 100 is false
    late = [sch.Request(50, 1.0, 0.0, run_time=3.0, g_remaining=5, g_initial=5)]   # already past its SLO: no veto
    assert sch.schedule(w, late, 1000, 0.01) == [0]
    # with c = 0 and dE = 0 a new request changes nobody's latency
    rng = np.random.default_rng(4)
    run, wait = random_queues(rng, 4, 5)
    wait = [sch.Request(r.input_tokens, r.slo, r.first_token_slo, g_remaining=r.g_remaining, g_initial=200) for r in wait]
    adm = sch.schedule(wait, run, 10 ** 9, 0.0)
    assert sorted(adm) == list(range(5))


def test_generation_length_bookkeeping():
    r = sch.Request(10, 1.0, 1.0, g_remaining=3, g_initial=200)
    r = sch.generation_tick(r, completed=False); assert r.g_remaining == 2
    r = sch.generation_tick(r, completed=False); assert r.g_remaining == 1
    r = sch.generation_tick(r, completed=False); assert r.g_remaining == 10      # 5 % of 200
    r2 = sch.generation_tick(sch.Request(10, 1.0, 1.0, g_remaining=1, g_initial=200), completed=True)
    assert r2.g_remaining == 0
    r3 = sch.generation_tick(sch.Request(10, 1.0, 1.0, g_remaining=1, g_initial=8), completed=False)
    assert r3.g_remaining == 1                                                   # never reset to nothing
