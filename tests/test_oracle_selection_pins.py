"""Pins of the resident-set selection oracle (oracle/selection.py) against what the paper and the
mathematics fix: the hand-worked Eq. 2 example, linearity and the s = 0 case, sums, a library sort,
and brute-force replay of the load list.  CPU only."""
import os

import numpy as np
import pytest

import emoe_inputs as gen
import oracle
from oracle import selection as sel

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "expected_tokens_example.txt")


def read_example():
    ex = {"freq": {}, "req_task": [], "req_tokens": [], "top": {}}
    for line in open(GOLDEN):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] == "E": ex["E"] = int(p[1])
        elif p[0] == "tasks": ex["tasks"] = int(p[1])
        elif p[0] == "freq": ex["freq"][int(p[1])] = [float(v) for v in p[2:]]
        elif p[0] == "w_out": ex["w_out"] = [float(v) for v in p[1:]]
        elif p[0] == "sensitive": ex["sensitive"] = [int(v) for v in p[1:]]
        elif p[0] == "request":
            ex["req_task"].append(int(p[1])); ex["req_tokens"].append(int(p[2]))
        elif p[0] == "expected": ex["expected"] = [float(v) for v in p[1:]]
        elif p[0] == "top": ex["top"][int(p[1])] = [int(v) for v in p[2:]]
    ex["freq"] = np.array([ex["freq"][t] for t in range(ex["tasks"])])
    return ex


def test_hand_worked_example_of_eq2():
    ex = read_example()
    n = sel.expected_tokens(ex["freq"], ex["req_task"], ex["req_tokens"], ex["w_out"], ex["sensitive"])
    assert np.array_equal(n, np.array(ex["expected"]))          # all values are exact in binary
    for L, want in ex["top"].items():
        assert sel.select_top(n, L).tolist() == want


def random_case(rng, n_tasks=5, E=16, n_req=12):
    freq = rng.dirichlet(np.ones(E), size=n_tasks)
    task = rng.integers(0, n_tasks, n_req)
    tokens = rng.integers(1, 2000, n_req)
    w_out = rng.uniform(10, 400, n_tasks)
    s = rng.integers(0, 2, n_tasks)
    return freq, task, tokens, w_out, s


def test_eq2_is_linear_in_the_token_counts_and_ignores_insensitive_tasks():
    rng = np.random.default_rng(5)
    freq, task, tokens, w_out, s = random_case(rng)
    n = sel.expected_tokens(freq, task, tokens, w_out, s)
    assert np.allclose(sel.expected_tokens(freq, task, 2 * tokens, 2 * w_out, s), 2 * n, rtol=1e-14)
    assert not sel.expected_tokens(freq, task, tokens, w_out, np.zeros_like(s)).any()
    # an insensitive task's frequencies do not matter
    f2 = freq.copy()
    for t in range(len(s)):
        if not s[t]:
            f2[t] = rng.dirichlet(np.ones(freq.shape[1]))
    assert np.array_equal(sel.expected_tokens(f2, task, tokens, w_out, s), n)
    # a task type without running requests (T = 0) contributes nothing
    lonely = task.copy(); lonely[:] = 0
    n0 = sel.expected_tokens(freq, lonely, tokens, w_out, np.ones_like(s))
    assert np.allclose(n0, (tokens.sum() + len(tokens) * w_out[0]) * freq[0], rtol=1e-14)


def test_eq2_total_equals_the_expected_token_count_of_the_sensitive_tasks():
    rng = np.random.default_rng(6)
    freq, task, tokens, w_out, s = random_case(rng)
    n = sel.expected_tokens(freq, task, tokens, w_out, s)
    want = sum((tokens[task == t].sum() + (task == t).sum() * w_out[t]) * s[t] for t in range(len(s)))
    assert np.isclose(n.sum(), want, rtol=1e-12)          # every f sums to one


def test_top_L_against_a_stable_library_sort_and_ties_go_to_the_lower_index():
    rng = np.random.default_rng(7)
    for _ in range(20):
        v = rng.integers(0, 6, 24).astype(np.float64)       # many ties
        for L in (1, 5, 24):
            assert sel.select_top(v, L).tolist() == np.argsort(-v, kind="stable")[:L].tolist()
    assert sel.select_top(np.array([1.0, 3.0, 3.0, 2.0]), 2).tolist() == [1, 2]


def replay(expert_of_slot, experts, slots):
    eos = list(expert_of_slot)
    for e, s in zip(experts, slots):
        eos[s] = e
    return eos


def test_load_list_brings_exactly_the_selected_experts_onto_the_gpu():
    rng = np.random.default_rng(8)
    for trial in range(200):
        E = int(rng.integers(2, 20)); S = int(rng.integers(1, E + 1)); L = int(rng.integers(1, S + 1))
        resident = rng.permutation(E)[: rng.integers(0, S + 1)]
        eos = np.full(S, -1); eos[rng.permutation(S)[: len(resident)]] = resident
        selected = rng.permutation(E)[:L]
        experts, slots, after = sel.plan_load(eos, selected)
        assert replay(eos, experts, slots) == after.tolist()                       # the list, applied in order
        assert sorted(e for e in after if e >= 0) == sorted(selected.tolist())      # exactly the selection is resident
        assert len(set(slots)) == len(slots)                                       # a slot is written once
        new = [e for e in selected if e not in eos]
        assert [e for e in experts if e >= 0] == new                               # only new experts, higher workload first
        for s in range(S):                                                         # resident and selected: not moved
            if eos[s] >= 0 and eos[s] in selected:
                assert after[s] == eos[s]


def test_load_list_refuses_more_experts_than_slots():
    with pytest.raises(ValueError):
        sel.plan_load([-1, -1], [0, 1, 2])


def test_observed_workload_counts_tokens_per_expert():
    rng = np.random.default_rng(9)
    topk = np.stack([rng.permutation(8)[:2] for _ in range(300)])
    w = sel.observed_workload(topk, 8)
    assert np.array_equal(w, np.bincount(topk.ravel(), minlength=8))
    assert w.sum() == 300 * 2


def test_with_every_expert_resident_the_workload_is_the_permutation_s_row_count():
    """Ties step W1 to the layer: with all experts on the GPU restricted routing is ordinary routing,
    so the workload of expert e is the number of rows of its slot."""
    c = gen.LayerConfig(name="workload", index=70, T=257, d_model=64, d_ff=64, E=8, k=2, R=8, dtype="bf16", act="swiglu")
    inp = gen.make_routing_inputs(c)
    res = oracle.layer_forward(inp, with_ffn=False)
    w = sel.observed_workload(oracle.route_unrestricted(res.logits, c.k), c.E)
    assert np.array_equal(w, res.permutation.slot_counts[inp.slot_of_expert])


def test_period_rule_of_section_3_3():
    """First request: all experts; then the predictor once per p requests (p = 40 in the paper's overhead study)."""
    acts = [sel.prompt_action(i, 40) for i in range(121)]
    assert acts[0] == sel.LOAD_ALL
    assert [i for i, a in enumerate(acts) if a == sel.PREDICT] == [40, 80, 120]
    assert all(a == sel.REUSE for i, a in enumerate(acts) if i % 40)
    for p in (1, 2, 7):
        n = 50
        assert sum(sel.prompt_action(i, p) == sel.PREDICT for i in range(n)) == (n - 1) // p
    assert sel.prompt_action(0, 5, all_experts_fit=False) == sel.PREDICT
