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
# Element-wise bounds |got - ref| <= REL * |ref| + ABS * rms(ref row).
# bf16: a value is rounded once to 8 significant bits, at most 2^-8 of itself (2^-7 if the fp32 value sat next
# to a rounding boundary on the other side of it than the exact value).  h: that rounding plus the fp32
# accumulation error of the two products (2^-12 of the row's rms is a generous cover).  y_perm and out: the
# rounding of y plus the roundings of the f values of h carried through the second product, a sum of f
# independent errors whose standard deviation is about 2^-9.3 of the row's rms; 2^-6 is ten of them.
# fp32: accumulation error only.
TOL_ELEM = {"bf16": {"h": (2.0 ** -7, 2.0 ** -12), "y": (2.0 ** -7, 2.0 ** -6)},
            "f32": {"h": (1e-5, 1e-5), "y": (1e-5, 1e-5)}}


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
        y0, o0 = b.y_perm.clone(), b.out.clone()
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
    rel, abs_rms = TOL_ELEM[cfg.dtype]["y"]
    check_elementwise(to_f64(b.y_perm)[rows], y_ref, rel, abs_rms, "y_perm")
    # out: the bounds of its k rows of y carried through the combine, plus its own rounding
    bound = rel * np.abs(ref.out)
    for j in range(cfg.k):
        yj = np.stack([ref.y_rows[int(r)] for r in ref.permutation.inv_perm[ref.tokens.astype(np.int64) * cfg.k + j]])
        wj = ref.topk_weight[ref.tokens, j][:, None]
        bound += wj * (rel * np.abs(yj) + abs_rms * np.sqrt((yj * yj).mean(axis=1, keepdims=True)))
    excess = np.abs(out - ref.out) - bound
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, f"out: element {worst} got {out[worst]!r} ref {ref.out[worst]!r}"
    return err


def check_elementwise(got: np.ndarray, ref: np.ndarray, rel: float, abs_rms: float, what: str):
    """|got - ref| <= rel * |ref| + abs_rms * rms(ref row), for every element."""
    rms = np.sqrt((ref * ref).mean(axis=1, keepdims=True))
    excess = np.abs(got - ref) - (rel * np.abs(ref) + abs_rms * rms)
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (f"{what}: element {worst} got {got[worst]!r} ref {ref[worst]!r}, "
                                f"row rms {rms[worst[0], 0]:.4g}")


def stratified_rows(slot_offsets: np.ndarray, seed: int, block: int = 32) -> np.ndarray:
    """Grouped rows to compare at full size: of every slot its first and last row and one seeded row
    of every `block`-row block counted from the slot's start.  Every kernel here cuts a slot's rows
    into tiles at multiples of 32 rows from the slot's start and multiplies them in blocks of 32, so
    this puts a row into every block of every m-tile; a row is compared over all its columns, which
    covers every n-tile, whole or cut along K."""
    rng = np.random.default_rng(seed)
    rows = []
    for s in range(len(slot_offsets) - 1):
        b, e = int(slot_offsets[s]), int(slot_offsets[s + 1])
        if e <= b:
            continue
        rows += [b, e - 1]
        for lo in range(b, e, block):
            rows.append(int(rng.integers(lo, min(lo + block, e))))
    return np.unique(np.asarray(rows, dtype=np.int64))


def h_rows(dl: DeviceLayer, rows: np.ndarray) -> np.ndarray:
    """Rows of the intermediate h [A, f], which the FFN leaves at the start of its workspace."""
    cfg = dl.cfg
    A, f = cfg.T * cfg.k, cfg.d_ff
    el = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    h = dl.buf.ffn_ws[:A * f * cfg.elem_bytes].view(el).view(A, f)
    return to_f64(h[torch.from_numpy(rows).to(h.device)])


def check_ffn_rows(dl: DeviceLayer, pm: oracle.Permutation, rows: np.ndarray):
    """h and y_perm of the given grouped rows against the oracle's FFN of the same (token, slot)
    pairs: relative L2 over the block and the element-wise bound.  Returns both relative errors."""
    cfg, inp = dl.cfg, dl.inp
    row_token = (pm.perm[rows] // cfg.k).astype(np.int32)
    row_slot = (np.searchsorted(pm.slot_offsets, rows, side="right") - 1).astype(np.int32)
    y_ref, h_ref = oracle.expert_ffn_rows(row_token, row_slot, inp.x, inp.w1_slots, inp.w3_slots, inp.w2_slots,
                                          cfg.act, cfg.dtype, return_h=True)
    tol, el = TOL_OUT[cfg.dtype], TOL_ELEM[cfg.dtype]
    h_got = h_rows(dl, rows)
    y_got = to_f64(dl.buf.y_perm[torch.from_numpy(rows).to(dl.buf.y_perm.device)])
    h_err, y_err = rel_l2(h_got, h_ref), rel_l2(y_got, y_ref)
    assert h_err <= tol, f"h rel-L2 {h_err:.3e} > {tol}"
    assert y_err <= tol, f"y_perm rel-L2 {y_err:.3e} > {tol}"
    check_elementwise(h_got, h_ref, *el["h"], "h")
    check_elementwise(y_got, y_ref, *el["y"], "y_perm")
    return h_err, y_err
