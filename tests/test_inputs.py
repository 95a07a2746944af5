"""The seeded input generator: determinism, storage rounding, structure, and the logit margin
(checked with the oracle's logits, not the generator's own filter)."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle


def test_bf16_rounding_is_round_to_nearest_even_like_torch():
    a = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]   # two exact ties, a negative tie, a subnormal
    bits = gen.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = gen.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_generator_is_deterministic_and_expert_streams_independent():
    a = gen.make_layer_inputs(gen.C1)
    b = gen.make_layer_inputs(gen.C1)
    for name in ("x", "w_gate", "slot_of_expert", "w1_slots", "w3_slots", "w2_slots"):
        assert np.array_equal(getattr(a, name), getattr(b, name))
    e = int(a.expert_of_slot[2])
    w1, w3, w2 = gen.expert_weights(gen.C1, e)
    assert np.array_equal(a.w1_slots[2], w1) and np.array_equal(a.w3_slots[2], w3) and np.array_equal(a.w2_slots[2], w2)
    c = gen.make_layer_inputs(gen.C1, seed=1)
    assert not np.array_equal(a.x, c.x)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_structure_and_margin_at_full_size(name):
    cfg = gen.CONFIGS[name]
    inp = gen.make_routing_inputs(cfg)
    assert inp.x.shape == (cfg.T, cfg.d_model) and inp.w_gate.shape == (cfg.E, cfg.d_model)
    assert (inp.slot_of_expert >= 0).sum() == cfg.R
    res = inp.resident_experts
    assert np.array_equal(inp.expert_of_slot[inp.slot_of_expert[res]], res)
    assert (inp.gate_bias is not None) == (cfg.zipf_s > 0)
    if cfg.resident == "popular":   # the R best-ranked (largest-bias) experts are the resident ones
        assert set(res) == set(np.argsort(-inp.gate_bias, kind="stable")[:cfg.R])
    lg = oracle.gate_logits(inp.x, inp.w_gate, inp.gate_bias, cfg.dtype)[:, res]
    top = -np.sort(-lg, axis=1)[:, :min(cfg.k + 1, cfg.R)]
    assert (top[:, :-1] - top[:, 1:]).min() >= gen.MARGIN
    # value distributions: x ~ N(0,1), gate weights std 1/sqrt(d)
    x64 = gen.storage_to_f64(inp.x, cfg.dtype)
    assert abs(x64.std() - 1.0) < 0.02 and abs(x64.mean()) < 0.02
    assert abs(gen.storage_to_f64(inp.w_gate, cfg.dtype).std() * np.sqrt(cfg.d_model) - 1.0) < 0.1


def test_zipf_bias_skews_the_routing():
    inp = gen.make_routing_inputs(gen.C2)
    r = oracle.layer_forward(inp, with_ffn=False)
    counts = np.sort(r.permutation.slot_counts)[::-1]
    assert counts.sum() == gen.C2.T and counts[0] > 4 * max(1, counts[-1])


def test_expert_weight_scales():
    cfg = gen.small_variant(gen.C3, T=8, d_model=256, d_ff=512)
    w1, w3, w2 = gen.expert_weights(cfg, 3)
    assert w1.shape == (512, 256) and w3.shape == (512, 256) and w2.shape == (256, 512)
    assert abs(gen.storage_to_f64(w1, "bf16").std() * 16 - 1) < 0.05
    assert abs(gen.storage_to_f64(w2, "bf16").std() * np.sqrt(512) - 1) < 0.05
    assert not np.array_equal(w1, w3)
