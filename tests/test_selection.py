"""The library's host-side choice of resident experts (Eq. 2, top-L, load list; Sections 3.4 and
3.2.2) against the selection oracle.  No GPU is needed: these entry points take host memory only."""
import os

import numpy as np
import pytest

import paper_2503_06823_amd as P
from oracle import selection as sel
from test_oracle_selection_pins import random_case, read_example


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(P.LIB_PATH):
        from paper_2503_06823_amd.build import build_library
        build_library(force=False)
    return P.lib()


def test_hand_worked_example():
    ex = read_example()
    n = P.emoe_expected_tokens(ex["freq"], ex["req_task"], ex["req_tokens"], ex["w_out"], ex["sensitive"])
    assert n == ex["expected"]
    for L, want in ex["top"].items():
        assert P.emoe_select_experts(n, L) == want


@pytest.mark.parametrize("seed", range(6))
def test_expected_tokens_and_selection_match_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    E = int(rng.choice([4, 8, 16, 64]))
    freq, task, tokens, w_out, s = random_case(rng, n_tasks=int(rng.integers(1, 6)), E=E, n_req=int(rng.integers(0, 30)))
    want = sel.expected_tokens(freq, task, tokens, w_out, s)
    got = np.array(P.emoe_expected_tokens(freq, task, tokens, w_out, s))
    # the same fp64 operations in the same order; a fused multiply-add on one side may differ in the last bit
    assert np.allclose(got, want, rtol=1e-14, atol=0.0)
    for L in {1, E // 2, E}:
        assert P.emoe_select_experts(want, L) == sel.select_top(want, L).tolist()   # same numbers in: same decision


def test_ties_in_the_selection_go_to_the_lower_index():
    v = [3.0, 7.0, 7.0, 1.0, 7.0, 3.0]
    assert P.emoe_select_experts(v, 4) == [1, 2, 4, 0] == sel.select_top(np.array(v), 4).tolist()


@pytest.mark.parametrize("seed", range(4))
def test_load_list_matches_the_oracle(seed):
    rng = np.random.default_rng(200 + seed)
    for _ in range(100):
        E = int(rng.integers(2, 65)); S = int(rng.integers(1, E + 1)); L = int(rng.integers(1, S + 1))
        k = int(rng.integers(1, L + 1))
        resident = rng.permutation(E)[: rng.integers(0, S + 1)]
        eos = np.full(S, -1, dtype=np.int32); eos[rng.permutation(S)[: len(resident)]] = resident
        selected = rng.permutation(E)[:L]
        experts, slots, _ = sel.plan_load(eos, selected)
        assert P.emoe_plan_load(E, S, k, eos, selected) == (experts, slots)


def test_load_list_feeds_load_experts_validation():
    """The list must pass emoe_load_experts' own checks (ids in range, no slot twice, at least k resident after)."""
    eos = [5, -1, 2, 7]
    experts, slots = P.emoe_plan_load(8, 4, 2, eos, [2, 0, 6])
    assert (experts, slots) == ([0, 6, -1], [0, 1, 3])


def test_selection_argument_errors():
    assert P.emoe_select_experts([1.0, 2.0], 3, check=False) == P.EMOE_ERR_SHAPE
    assert P.emoe_select_experts([1.0, 2.0], 0, check=False) == P.EMOE_ERR_SHAPE
    assert P.emoe_expected_tokens([[1.0]], [1], [5], [1.0], [1], check=False) == P.EMOE_ERR_SHAPE      # task id out of range
    assert P.emoe_expected_tokens([[1.0]], [0], [-5], [1.0], [1], check=False) == P.EMOE_ERR_SHAPE     # negative tokens
    assert P.emoe_plan_load(8, 4, 2, [0, 1, 2, 3], [0, 1, 2, 3, 4], check=False) == P.EMOE_ERR_RESIDENT  # L > S
    assert P.emoe_plan_load(8, 4, 2, [0, 1, 2, 3], [4], check=False) == P.EMOE_ERR_RESIDENT              # L < k
    assert P.emoe_plan_load(8, 4, 2, [0, 1, 2, 3], [4, 4], check=False) == P.EMOE_ERR_RESIDENT           # repeated
    assert P.emoe_plan_load(8, 4, 2, [0, 0, 2, 3], [4, 5], check=False) == P.EMOE_ERR_RESIDENT           # bad map
    assert P.lib().emoe_select_experts(2, None, 1, None) == P.EMOE_ERR_NULL


def test_period_rule_matches_the_oracle():
    for period in (1, 2, 3, 40, 57):
        for fit in (True, False):
            for i in range(0, 200):
                assert P.emoe_prompt_action(i, period, fit) == sel.prompt_action(i, period, fit)
    assert P.emoe_prompt_action(-1, 3, True) == P.EMOE_ERR_SHAPE
    assert P.emoe_prompt_action(5, 0, True) == P.EMOE_ERR_SHAPE


def test_loader_rejects_bad_arguments_before_touching_the_device():
    lib = P.lib()
    import ctypes
    h = ctypes.c_void_p(0)
    assert lib.emoe_loader_create(1, None, 3, ctypes.byref(h)) == P.EMOE_ERR_NULL
    d = P.make_desc(0, 64, 64, 4, 2, 4, "bf16", "swiglu")
    w = [np.zeros(8, np.uint16) for _ in range(4)]
    good = dict(desc=d, host_w1=w, host_w3=w, host_w2=w, w1_slots=4096, w3_slots=4096, w2_slots=4096,
                slot_of_expert=4096, expert_of_slot=4096)
    for bad, code in ((dict(good, w3_slots=None), P.EMOE_ERR_NULL), (dict(good, slot_of_expert=None), P.EMOE_ERR_NULL),
                      (dict(good, desc=P.make_desc(0, 60, 64, 4, 2, 4, "bf16", "swiglu")), P.EMOE_ERR_UNSUPPORTED)):
        with pytest.raises(P.EmoeError) as ei:
            P.Loader([bad], 3)
        assert ei.value.status == code
    with pytest.raises(P.EmoeError) as ei:
        P.Loader([good], 0)
    assert ei.value.status == P.EMOE_ERR_SHAPE
    assert lib.emoe_loader_destroy(None) == P.EMOE_ERR_NULL
    assert lib.emoe_loader_layer_begin(None, 0, None) == P.EMOE_ERR_NULL
