"""Workload observation on the GPU (emoe_route_observe) and the loop the paper describes in
Sections 3.2.2 and 3.4: observe which experts the tokens ask for, pick the L with the highest
expected number of tokens, load them, and serve with those."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P
from gpu_util import desc_of, to_dev
from oracle import selection as sel
from test_gpu_load import Host, oracle_inputs

pytestmark = pytest.mark.gpu


def all_resident_cfg(name, index, **kw):
    base = dict(name=name, index=index, T=500, d_model=256, d_ff=64, E=8, k=2, dtype="bf16", act="swiglu")
    base.update(kw)
    base["R"] = base["E"]      # margins then hold between ALL experts' logits, which ordinary routing needs
    return gen.LayerConfig(**base)


CASES = [
    all_resident_cfg("observe_mixtral_like", 80),
    all_resident_cfg("observe_64_experts", 81, T=777, d_model=200, E=64, k=6, zipf_s=1.2),
    all_resident_cfg("observe_32_experts_top1", 82, T=300, E=32, k=1, zipf_s=1.1),
    all_resident_cfg("observe_few_tokens_long_rows", 85, T=70, d_model=2048, E=16, k=2, zipf_s=1.1),
    all_resident_cfg("observe_f32", 83, T=150, d_model=72, E=16, k=2, dtype="f32"),
    all_resident_cfg("observe_f32_many_tokens", 84, T=2500, d_model=64, E=8, k=2, dtype="f32"),
]


@pytest.mark.parametrize("c", CASES, ids=lambda c: c.name)
def test_observed_workload_matches_the_oracle_and_routing_is_unchanged(gpu_device, c):
    inp = gen.make_routing_inputs(c)
    logits = oracle.gate_logits(inp.x, inp.w_gate, inp.gate_bias, c.dtype)
    want = sel.observed_workload(oracle.route_unrestricted(logits, c.k), c.E)
    # serve with only some experts resident: the observation must not depend on that
    rng = np.random.default_rng(c.index)
    R = max(c.k, c.E // 2)
    soe_host = np.full(c.E, -1, dtype=np.int32)
    soe_host[rng.permutation(c.E)[:R]] = np.arange(R)
    d = P.make_desc(c.T, c.d_model, c.d_ff, c.E, c.k, R, c.dtype, c.act)
    x, wg, bias = to_dev(inp.x, c.dtype), to_dev(inp.w_gate, c.dtype), to_dev(inp.gate_bias, "f32")
    soe = torch.from_numpy(soe_host).cuda()
    te0 = torch.empty((c.T, c.k), dtype=torch.int32, device="cuda"); tw0 = torch.empty((c.T, c.k), device="cuda")
    te1, tw1 = torch.empty_like(te0), torch.empty_like(tw0)
    hist = torch.zeros(c.E, dtype=torch.int64, device="cuda")
    P.emoe_route(d, x, wg, bias, soe, te0, tw0)
    P.emoe_route_observe(d, x, wg, bias, soe, te1, tw1, hist)
    torch.cuda.synchronize()
    assert torch.equal(te0, te1) and torch.equal(tw0, tw1)
    assert np.array_equal(hist.cpu().numpy(), want)
    assert int(hist.sum()) == c.T * c.k
    P.emoe_route_observe(d, x, wg, bias, soe, te1, tw1, hist)      # counts accumulate across calls
    torch.cuda.synchronize()
    assert np.array_equal(hist.cpu().numpy(), 2 * want)


def test_observe_select_load_serve(gpu_device):
    """Section 3.3 / 3.4 in small: the first batch runs with every expert resident while the workload is
    observed; Eq. 2 and the top-L rule pick the residents; the load list is applied; the next batch is
    served by exactly those experts and matches the oracle for that resident set."""
    cfg = gen.LayerConfig(name="loop", index=85, T=600, d_model=256, d_ff=384, E=8, k=2, R=8, dtype="bf16",
                          act="swiglu", zipf_s=1.0)
    base = gen.make_routing_inputs(cfg)
    host = Host(cfg)
    E, S, L, f, dm = cfg.E, cfg.E, 4, cfg.d_ff, cfg.d_model
    d = P.make_desc(cfg.T, dm, f, E, cfg.k, S, cfg.dtype, cfg.act)
    w1s = torch.zeros((S, f, dm), dtype=torch.bfloat16, device="cuda")
    w3s, w2s = torch.zeros_like(w1s), torch.zeros((S, dm, f), dtype=torch.bfloat16, device="cuda")
    soe = torch.full((E,), -1, dtype=torch.int32, device="cuda")
    eos = torch.full((S,), -1, dtype=torch.int32, device="cuda")
    mirror = np.full(S, -1, dtype=np.int32)
    side, compute = torch.cuda.Stream(), torch.cuda.current_stream()
    loaded, done = P.make_event(), P.make_event()     # events the library records and waits on: their handles must exist
    x, wg, bias = to_dev(base.x, "bf16"), to_dev(base.w_gate, "bf16"), to_dev(base.gate_bias, "f32")
    buf = P.LayerBuffers.allocate(d)
    hist = torch.zeros(E, dtype=torch.int64, device="cuda")
    side.wait_stream(compute)

    # first prompt: every expert is loaded (Section 3.3)
    P.emoe_load_experts(d, list(range(E)), list(range(S)), host.w1, host.w3, host.w2, w1s, w3s, w2s, soe, eos, mirror,
                        side, done_event=loaded)
    compute.wait_event(loaded)
    P.emoe_route_observe(d, x, wg, bias, soe, buf.topk_expert, buf.topk_weight, hist)
    done.record(compute)
    torch.cuda.synchronize()
    workload = hist.cpu().numpy()
    logits = oracle.gate_logits(base.x, base.w_gate, base.gate_bias, cfg.dtype)
    assert np.array_equal(workload, sel.observed_workload(oracle.route_unrestricted(logits, cfg.k), E))

    # the predictor's stand-in: the observed relative frequencies; one sensitive task type, three running requests
    freq = [workload / workload.sum()]
    req_task, req_tokens, w_out, sens = [0, 0, 0], [120, 64, 300], [200.0], [1]
    expected = P.emoe_expected_tokens(freq, req_task, req_tokens, w_out, sens)
    assert np.allclose(expected, sel.expected_tokens(np.array(freq), req_task, req_tokens, w_out, sens), rtol=1e-14)
    selected = P.emoe_select_experts(expected, L)
    assert selected == sel.select_top(np.array(expected), L).tolist()
    experts, slots = P.emoe_plan_load(E, S, cfg.k, mirror, selected)
    want_experts, want_slots, want_map = sel.plan_load(mirror, selected)
    assert (experts, slots) == (want_experts, want_slots)
    assert sorted(e for e in want_map if e >= 0) == sorted(selected) and len(experts) == E - L   # evictions only

    P.emoe_load_experts(d, experts, slots, host.w1, host.w3, host.w2, w1s, w3s, w2s, soe, eos, mirror, side,
                        wait_event=done, done_event=loaded)
    compute.wait_event(loaded)
    P.layer_forward(buf, x, wg, bias, soe, w1s, w3s, w2s)
    torch.cuda.synchronize()
    assert np.array_equal(mirror, want_map) and np.array_equal(eos.cpu().numpy(), want_map)

    ref = oracle.layer_forward(oracle_inputs(cfg, base, host, want_map))
    lg = ref.logits[:, want_map[want_map >= 0]]
    top = -np.sort(-lg, axis=1)[:, :cfg.k + 1]
    safe = np.flatnonzero((top[:, :-1] - top[:, 1:]).min(axis=1) > 1e-3)   # margins were drawn for the full set
    assert safe.size > cfg.T * 0.8
    assert np.array_equal(buf.topk_expert.cpu().numpy()[safe], ref.topk_expert[safe])
    assert set(np.unique(buf.topk_expert.cpu().numpy())) <= set(selected)
    out = buf.out.double().cpu().numpy()[safe]
    assert np.linalg.norm(out - ref.out[safe]) / np.linalg.norm(ref.out[safe]) < 1e-2
