"""Pins for the fp64 oracle: each test ties one part of it to something other than
itself -- a closed form, an invariant, a special case that is a textbook / numpy
routine, brute force, or the hand-worked fixture under tests/golden/.

The layer definition and the fallback rule come from eMoE Section 3.2.2 (last
paragraph) and Section 1 (gate + experts); Section 3.3 (the first prompt has every
expert resident) gives the all-resident special case.
"""
import math
import os
from dataclasses import replace

import numpy as np
import pytest

import emoe_inputs as gen
import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def tiny_cfg(**kw):
    base = dict(name="pin", index=17, T=24, d_model=20, d_ff=28, E=8, k=2, R=4, dtype="f32", act="swiglu")
    base.update(kw)
    return gen.LayerConfig(**base)


def f64(a, dtype):
    return gen.storage_to_f64(a, dtype)


def silu(g):
    return g / (1.0 + np.exp(-g))


def dense_ffn(x64, w1, w3, w2, act):
    """Independent dense FFN by numpy matmul (float64)."""
    g = x64 @ w1.T
    h = silu(g) * (x64 @ w3.T) if act == "swiglu" else np.maximum(g, 0.0)
    return h @ w2.T


# ---------------------------------------------------------------- golden fixture (fallback rule)
def _read_golden():
    cases = []
    with open(os.path.join(HERE, "golden", "fallback_example.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, lg, ex, w = [p.strip() for p in line.split(";")]
            cases.append((int(k), [float(v) for v in lg.split()], [int(v) for v in ex.split()],
                          [float(v) for v in w.split()]))
    return cases


@pytest.mark.parametrize("formulation", ["mask_then_topk", "rank_then_skip"])
def test_golden_fallback_example(formulation):
    soe = np.array([-1, 0, -1, 1], dtype=np.int32)  # resident = {1, 3}
    cases = _read_golden()
    assert len(cases) == 4
    for k, lg, experts, weights in cases:
        idx, w = oracle.route(np.array([lg]), soe, k, formulation)
        assert idx[0].tolist() == experts
        np.testing.assert_allclose(w[0], weights, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- O1 against a library matmul
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gate_logits_match_numpy_matmul(dtype):
    cfg = tiny_cfg(dtype=dtype, zipf_s=1.1, d_model=33, E=7, R=3)
    inp = gen.make_routing_inputs(cfg)
    lg = oracle.gate_logits(inp.x, inp.w_gate, inp.gate_bias, dtype)
    ref = f64(inp.x, dtype) @ f64(inp.w_gate, dtype).T + inp.gate_bias.astype(np.float64)[None, :]
    np.testing.assert_allclose(lg, ref, rtol=0, atol=1e-12)
    assert np.abs(inp.gate_bias).max() > 0.5  # the bias term is really there


# ---------------------------------------------------------------- P1, P2
@pytest.mark.parametrize("cfg", [tiny_cfg(), tiny_cfg(E=16, k=3, R=5, zipf_s=1.2), tiny_cfg(k=1, R=2, act="relu")])
def test_weights_sum_to_one_and_only_resident_experts(cfg):
    inp = gen.make_routing_inputs(cfg, shuffle_slots=True)
    res = oracle.layer_forward(inp, with_ffn=False)
    w, idx = res.topk_weight, res.topk_expert
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    assert (w > 0).all()
    assert (np.diff(w, axis=1) <= 0).all()                     # non-increasing in j
    assert (inp.slot_of_expert[idx] >= 0).all()                # masked-out experts never get a token
    for t in range(cfg.T):                                     # k distinct experts, descending logit
        assert len(set(idx[t])) == cfg.k
        assert (np.diff(res.logits[t, idx[t]]) < 0).all()
    pm = res.permutation
    assert pm.slot_counts.sum() == cfg.T * cfg.k
    empty = np.flatnonzero(inp.expert_of_slot < 0)
    assert (pm.slot_counts[empty] == 0).all()
    # the k chosen are the k largest resident logits
    for t in range(cfg.T):
        resident = np.flatnonzero(inp.slot_of_expert >= 0)
        best = resident[np.argsort(-res.logits[t, resident], kind="stable")[:cfg.k]]
        assert idx[t].tolist() == best.tolist()


# ---------------------------------------------------------------- P3: all resident == textbook gate
def test_all_resident_is_textbook_softmax_topk_renormalise():
    cfg = tiny_cfg(E=8, k=2, R=8)
    inp = gen.make_routing_inputs(cfg)
    lg = oracle.gate_logits(inp.x, inp.w_gate, inp.gate_bias, cfg.dtype)
    idx, w = oracle.route(lg, inp.slot_of_expert, cfg.k)
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)                          # softmax over all E
    top = np.argsort(-p, axis=1, kind="stable")[:, :cfg.k]     # top-k of the probabilities
    pk = np.take_along_axis(p, top, axis=1)
    assert np.array_equal(idx, top.astype(np.int32))
    np.testing.assert_allclose(w, pk / pk.sum(axis=1, keepdims=True), rtol=0, atol=1e-13)
    assert np.array_equal(idx, oracle.route_unrestricted(lg, cfg.k))


# ---------------------------------------------------------------- P4: E = 1 is a dense FFN
@pytest.mark.parametrize("act", ["swiglu", "relu"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_expert_is_dense_ffn(act, dtype):
    cfg = tiny_cfg(E=1, k=1, R=1, act=act, dtype=dtype, T=9, d_model=12, d_ff=21)
    inp = gen.make_layer_inputs(cfg)
    res = oracle.layer_forward(inp)
    w3 = f64(inp.w3_slots[0], dtype) if act == "swiglu" else None
    ref = dense_ffn(f64(inp.x, dtype), f64(inp.w1_slots[0], dtype), w3, f64(inp.w2_slots[0], dtype), act)
    np.testing.assert_allclose(res.out, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(res.topk_weight, 1.0, rtol=0, atol=0)


# ---------------------------------------------------------------- P5: k = R is a dense mixture
def test_k_equals_resident_count_is_dense_mixture():
    cfg = tiny_cfg(E=6, k=3, R=3, T=10)
    inp = gen.make_layer_inputs(cfg, shuffle_slots=True)
    res = oracle.layer_forward(inp)
    x64 = f64(inp.x, cfg.dtype)
    resident = np.flatnonzero(inp.slot_of_expert >= 0)
    lg = res.logits[:, resident]
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    ref = np.zeros((cfg.T, cfg.d_model))
    for c, e in enumerate(resident):
        s = inp.slot_of_expert[e]
        ref += p[:, c:c + 1] * dense_ffn(x64, f64(inp.w1_slots[s], cfg.dtype), f64(inp.w3_slots[s], cfg.dtype),
                                         f64(inp.w2_slots[s], cfg.dtype), cfg.act)
    np.testing.assert_allclose(res.out, ref, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- general case against a numpy loop
def test_layer_matches_independent_numpy_composition():
    cfg = tiny_cfg(E=8, k=2, R=4, T=12, zipf_s=1.1)
    inp = gen.make_layer_inputs(cfg, shuffle_slots=True)
    res = oracle.layer_forward(inp)
    x64 = f64(inp.x, cfg.dtype)
    lg = x64 @ f64(inp.w_gate, cfg.dtype).T + inp.gate_bias.astype(np.float64)
    ref = np.zeros((cfg.T, cfg.d_model))
    for t in range(cfg.T):
        masked = np.where(inp.slot_of_expert >= 0, lg[t], -np.inf)
        top = np.argsort(-masked, kind="stable")[:cfg.k]
        wk = np.exp(masked[top] - masked[top].max())
        wk /= wk.sum()
        for e, wj in zip(top, wk):
            s = inp.slot_of_expert[e]
            ref[t] += wj * dense_ffn(x64[t:t + 1], f64(inp.w1_slots[s], cfg.dtype), f64(inp.w3_slots[s], cfg.dtype),
                                     f64(inp.w2_slots[s], cfg.dtype), cfg.act)[0]
    np.testing.assert_allclose(res.out, ref, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- P6: two formulations agree
def test_two_formulations_of_the_fallback_rule_agree():
    rng = np.random.default_rng(5)
    for E, k, R in [(8, 2, 4), (64, 6, 24), (64, 1, 16), (5, 5, 5), (3, 1, 1)]:
        lg = rng.standard_normal((50, E))
        lg[::7, 1:3] = lg[::7, :1]          # plant exact ties: lower index must win in both
        soe = np.full(E, -1, dtype=np.int32)
        soe[rng.choice(E, R, replace=False)] = np.arange(R)
        a = oracle.route(lg, soe, k, "mask_then_topk")
        b = oracle.route(lg, soe, k, "rank_then_skip")
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_tie_goes_to_lower_index():
    lg = np.array([[1.0, 2.0, 2.0, 2.0]])
    soe = np.array([0, -1, 1, 2], dtype=np.int32)
    idx, w = oracle.route(lg, soe, 2)
    assert idx[0].tolist() == [2, 3]
    np.testing.assert_allclose(w[0], [0.5, 0.5])


def test_fewer_than_k_resident_is_an_error():
    lg = np.zeros((2, 4))
    soe = np.array([-1, 0, -1, -1], dtype=np.int32)
    for form in ("mask_then_topk", "rank_then_skip"):
        with pytest.raises(oracle.OracleError) as ei:
            oracle.route(lg, soe, 2, form)
        assert ei.value.code == oracle.ERR_RESIDENT


# ---------------------------------------------------------------- P7: permutation vs brute force
@pytest.mark.parametrize("seed", range(4))
def test_permutation_matches_brute_force(seed):
    rng = np.random.default_rng(seed)
    T, k, E, S = 16, 2, 8, 6
    soe = np.full(E, -1, dtype=np.int32)
    soe[rng.choice(E, 4, replace=False)] = rng.permutation(S)[:4]
    resident = np.flatnonzero(soe >= 0)
    idx = np.stack([rng.choice(resident, k, replace=False) for _ in range(T)]).astype(np.int32)
    pm = oracle.permute(idx, soe, S)
    lists = [[] for _ in range(S)]
    for a in range(T * k):                                     # scan assignments in order, append to slot list
        lists[soe[idx[a // k, a % k]]].append(a)
    flat = [a for lst in lists for a in lst]
    assert pm.perm.tolist() == flat
    assert pm.slot_counts.tolist() == [len(lst) for lst in lists]
    assert pm.slot_offsets.tolist() == np.concatenate([[0], np.cumsum([len(lst) for lst in lists])]).tolist()
    assert (pm.inv_perm[pm.perm] == np.arange(T * k)).all()
    assert (np.diff(pm.slot_offsets) >= 0).all()
    # gather is a pure copy of the token rows
    x = rng.standard_normal((T, 5)).astype(np.float32)
    xp = oracle.gather_rows(x, pm.perm, k, "f32")
    assert np.array_equal(xp, x[np.array(flat) // k])


# ---------------------------------------------------------------- P8: token-permutation equivariance
def test_token_permutation_equivariance():
    cfg = tiny_cfg(T=14)
    inp = gen.make_layer_inputs(cfg)
    base = oracle.layer_forward(inp).out
    sigma = np.random.default_rng(3).permutation(cfg.T)
    inp.x = np.ascontiguousarray(inp.x[sigma])
    np.testing.assert_allclose(oracle.layer_forward(inp).out, base[sigma], rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P9: slot-relabel invariance
def test_slot_relabel_invariance():
    cfg = tiny_cfg(S=6)
    a = gen.make_layer_inputs(cfg, shuffle_slots=False)
    b = gen.make_layer_inputs(cfg, shuffle_slots=True)
    assert not np.array_equal(a.slot_of_expert, b.slot_of_expert)
    ra, rb = oracle.layer_forward(a), oracle.layer_forward(b)
    assert np.array_equal(ra.topk_expert, rb.topk_expert)
    np.testing.assert_allclose(ra.out, rb.out, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P10: scalar closed forms
def test_scalar_closed_forms():
    one = lambda v: np.array([[[v]]], dtype=np.float32)
    x = np.array([[1.0]], dtype=np.float32)
    y = oracle.expert_ffn_rows([0], [0], x, one(1.0), one(2.0), one(3.0), "swiglu", "f32")
    assert y[0, 0] == pytest.approx(6.0 / (1.0 + math.exp(-1.0)), abs=1e-14)
    assert y[0, 0] == pytest.approx(4.386351, abs=1e-6)
    y = oracle.expert_ffn_rows([0], [0], x, one(1.0), None, one(3.0), "relu", "f32")
    assert y[0, 0] == 3.0
    y = oracle.expert_ffn_rows([0], [0], x, one(-1.0), None, one(3.0), "relu", "f32")
    assert y[0, 0] == 0.0
    # negative gate pre-activation: silu(-2) * 5 * 7 with silu(-2) = -2 / (1 + e^2)
    y = oracle.expert_ffn_rows([0], [0], x, one(-2.0), one(5.0), one(7.0), "swiglu", "f32")
    assert y[0, 0] == pytest.approx(-2.0 / (1.0 + math.exp(2.0)) * 35.0, abs=1e-13)


def test_ffn_operand_orientation_two_by_three():
    # d = 2, f = 3, hand-computed: distinguishes W[f,d] from its transpose and W1 from W3
    x = np.array([[1.0, 2.0]], dtype=np.float32)
    w1 = np.array([[[1, 0], [0, 1], [1, 1]]], dtype=np.float32)          # g = (1, 2, 3)
    w3 = np.array([[[2, 0], [0, 0.5], [1, -1]]], dtype=np.float32)       # u = (2, 1, -1)
    w2 = np.array([[[1, 0, 0], [0, 1, 1]]], dtype=np.float32)            # y = (h0, h1 + h2)
    y, h = oracle.expert_ffn_rows([0], [0], x, w1, w3, w2, "swiglu", "f32", return_h=True)
    s = lambda g: g / (1 + math.exp(-g))
    np.testing.assert_allclose(h[0], [2 * s(1), s(2), -s(3)], atol=1e-14)
    np.testing.assert_allclose(y[0], [2 * s(1), s(2) - s(3)], atol=1e-14)


# ---------------------------------------------------------------- P11: homogeneity / degenerate experts
def test_homogeneity_in_w2_and_identical_experts():
    cfg = tiny_cfg(T=8)
    inp = gen.make_layer_inputs(cfg)
    base = oracle.layer_forward(inp).out
    keep = inp.w2_slots.copy()
    inp.w2_slots = keep * np.float32(-2.0)
    np.testing.assert_allclose(oracle.layer_forward(inp).out, -2.0 * base, rtol=1e-13, atol=1e-13)
    inp.w2_slots = np.zeros_like(keep)
    assert not oracle.layer_forward(inp).out.any()
    # two identical resident experts, k = 2, E = 2: same as that expert alone with weight 1
    cfg2 = tiny_cfg(E=2, k=2, R=2, T=8)
    two = gen.make_layer_inputs(cfg2)
    two.w1_slots[1], two.w3_slots[1], two.w2_slots[1] = two.w1_slots[0], two.w3_slots[0], two.w2_slots[0]
    ref = dense_ffn(f64(two.x, "f32"), f64(two.w1_slots[0], "f32"), f64(two.w3_slots[0], "f32"),
                    f64(two.w2_slots[0], "f32"), "swiglu")
    np.testing.assert_allclose(oracle.layer_forward(two).out, ref, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- P12: miss accounting
def test_miss_accounting():
    cfg = tiny_cfg(E=16, k=2, R=5, T=64, zipf_s=1.1)
    inp = gen.make_routing_inputs(cfg)
    res = oracle.layer_forward(inp, with_ffn=False)
    free = oracle.route_unrestricted(res.logits, cfg.k)
    absent_choices = int((inp.slot_of_expert[free] < 0).sum())
    replaced = sum(len(set(res.topk_expert[t]) - set(free[t])) for t in range(cfg.T))
    assert absent_choices == replaced
    assert absent_choices > 0  # the case really exercises the fallback
    # tokens with no miss are routed exactly as the unrestricted gate would
    ok = (inp.slot_of_expert[free] >= 0).all(axis=1)
    assert np.array_equal(res.topk_expert[ok], free[ok])


# ---------------------------------------------------------------- sampled tokens == full run
def test_sampled_tokens_equal_full_layer():
    cfg = tiny_cfg(T=20, act="relu", k=1, R=3, dtype="bf16")
    inp = gen.make_layer_inputs(cfg)
    full = oracle.layer_forward(inp)
    some = oracle.layer_forward(inp, tokens=[3, 19, 0])
    assert np.array_equal(some.out, full.out[[3, 19, 0]])
    for r, y in some.y_rows.items():
        assert np.array_equal(y, full.y_rows[r])
