"""Helpers for the GPU parity tests: move seeded inputs to the device, run the layer through the
C-ABI binding, bring results back as numpy, and compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P

# tolerances of the parity contract
TOL_WEIGHT = 1e-5
TOL_OUT = {"bf16": 1e-2, "f32": 1e-5}


def to_dev(a, dtype: str, device="cuda:0"):
    """numpy storage array -> device tensor (bf16 bit patterns become torch.bfloat16)."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def raw_bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def desc_of(cfg: gen.LayerConfig):
    return P.make_desc(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.slots, cfg.dtype, cfg.act)


class DeviceLayer:
    """Inputs of one layer resident on the device plus its output buffers."""

    def __init__(self, inp: gen.LayerInputs, device="cuda:0"):
        cfg = inp.cfg
        self.inp, self.cfg = inp, cfg
        self.desc = desc_of(cfg)
        self.x = to_dev(inp.x, cfg.dtype, device)
        self.w_gate = to_dev(inp.w_gate, cfg.dtype, device)
        self.gate_bias = to_dev(inp.gate_bias, "f32", device)
        self.slot_of_expert = to_dev(inp.slot_of_expert, "i32", device)
        self.w1 = to_dev(inp.w1_slots, cfg.dtype, device)
        self.w3 = to_dev(inp.w3_slots, cfg.dtype, device)
        self.w2 = to_dev(inp.w2_slots, cfg.dtype, device)
        self.buf = P.LayerBuffers.allocate(self.desc, device)

    def forward(self, stream=None, gather_in_ffn=False):
        """gather_in_ffn=False also fills buf.x_perm (which the permutation checks compare)."""
        return P.layer_forward(self.buf, self.x, self.w_gate, self.gate_bias, self.slot_of_expert, self.w1, self.w3,
                               self.w2, stream, gather_in_ffn=gather_in_ffn)

    def check_gather_path_is_identical(self):
        """The FFN that reads token rows through perm must reproduce y_perm and out bit for bit."""
        b = self.buf
        y0, o0, h0 = b.y_perm.clone(), b.out.clone(), b.ffn_ws.clone()
        b.y_perm.fill_(0); b.out.fill_(0); b.x_perm.fill_(0)
        self.forward(gather_in_ffn=True)
        torch.cuda.synchronize()
        assert torch.equal(b.y_perm, y0) and torch.equal(b.out, o0)
        assert not b.x_perm.any(), "the gather path must not touch x_perm"


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def check_routing_and_permutation(dl: DeviceLayer, ref: oracle.LayerResult):
    """Bit-exact index work, gate weights within 1e-5, x_perm a bit copy."""
    b, cfg = dl.buf, dl.cfg
    A = cfg.T * cfg.k
    assert np.array_equal(b.topk_expert.cpu().numpy(), ref.topk_expert), "topk_expert differs"
    dw = np.abs(b.topk_weight.cpu().numpy().astype(np.float64) - ref.topk_weight).max() if cfg.T else 0.0
    assert dw <= TOL_WEIGHT, f"topk_weight off by {dw}"
    pm = ref.permutation
    assert np.array_equal(b.slot_counts.cpu().numpy(), pm.slot_counts), "slot_counts differ"
    assert np.array_equal(b.slot_offsets.cpu().numpy(), pm.slot_offsets), "slot_offsets differ"
    assert np.array_equal(b.perm.cpu().numpy()[:A], pm.perm), "perm differs"
    assert np.array_equal(b.inv_perm.cpu().numpy()[:A], pm.inv_perm), "inv_perm differs"
    xp_ref = oracle.gather_rows(dl.inp.x, pm.perm, cfg.k, cfg.dtype)
    assert np.array_equal(raw_bits(b.x_perm)[:A], xp_ref), "x_perm is not a bit copy"


def check_outputs(dl: DeviceLayer, ref: oracle.LayerResult):
    """y_perm rows and out against the oracle for the tokens the oracle computed."""
    b, cfg = dl.buf, dl.cfg
    tol = TOL_OUT[cfg.dtype]
    out = to_f64(b.out)[ref.tokens]
    err = rel_l2(out, ref.out)
    assert err <= tol, f"out rel-L2 {err:.3e} > {tol}"
    rows = np.array(sorted(ref.y_rows))
    y_ref = np.stack([ref.y_rows[int(r)] for r in rows])
    y_err = rel_l2(to_f64(b.y_perm)[rows], y_ref)
    assert y_err <= tol, f"y_perm rel-L2 {y_err:.3e} > {tol}"
    # worst single token, reported (looser bound: one token has fewer terms to average over)
    per_tok = np.linalg.norm(out - ref.out, axis=1) / np.maximum(np.linalg.norm(ref.out, axis=1), 1e-30)
    assert per_tok.max() <= 4 * tol, f"worst token rel-L2 {per_tok.max():.3e}"
    return err
