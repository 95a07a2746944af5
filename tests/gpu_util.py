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
# Element-wise bounds.
# h: |got - ref| <= REL * |ref| + ABS * rms(ref row).  bf16: a value is rounded once to 8 significant bits, at
# most 2^-8 of itself (2^-7 if the fp32 value sat next to a rounding boundary on the other side of it than the
# exact value); 2^-12 of the row's rms is a generous cover of the fp32 accumulation error of the two products.
# y_perm: see y_bound().  fp32: accumulation error only.
TOL_ELEM = {"bf16": {"h": (2.0 ** -7, 2.0 ** -12)}, "f32": {"h": (1e-5, 1e-5)}}

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


def y_bound(dl: DeviceLayer, row_slot: np.ndarray, h_ref: np.ndarray, y_ref: np.ndarray) -> np.ndarray:
    """Element-wise bound on |y_perm - y_ref| for rows with the oracle's h_ref [n, f], y_ref [n, d], slots row_slot.
    y[n] = sum_i h[i] W2[n, i].  bf16: the GPU multiplies h rounded to bf16, every h[i] off by at most 2^-8 |h[i]|
    (1.05 covers an h next to a rounding boundary); carried through the product these errors add up to at most
    1.05 * 2^-8 * T1, T1 = sum_i |h[i] W2[n, i]|, whatever their signs.  Being independent and bounded they also stay,
    by Hoeffding's inequality, within 2^-5 * sqrt(T2), T2 = sum_i (h[i] W2[n, i])^2, except with a probability
    below 1e-12 per element: the tighter of the two is taken (the second is, once a row of h has a few
    hundred entries; a K tile of 64 left out of 14336 terms moves an element by about 2^-3.9 * sqrt(T2)).
    Then y is rounded itself: 2^-7 |y| (2^-8, or the neighbour across a boundary).  1e-6 * T1 covers the fp32
    accumulation of this product, and 2e-6 * sum_i |W2[n, i]| the fp32 accumulation behind h itself, which is an
    absolute error of h (the pre-activations are O(1) by the input recipe), not one relative to h.
    fp32 layers: accumulation errors only, 1e-5 |y| + 2e-6 * T1 + 2e-6 * sum_i |W2[n, i]|."""
    cfg, inp = dl.cfg, dl.inp
    to_f32 = gen.bf16_bits_to_f32 if cfg.dtype == "bf16" else (lambda a: a)
    t1 = np.empty_like(y_ref, dtype=np.float64)
    t2 = np.empty_like(y_ref, dtype=np.float64)
    wsum = np.empty_like(y_ref, dtype=np.float64)
    habs = np.abs(h_ref).astype(np.float32)
    for s in np.unique(row_slot):
        sel = np.flatnonzero(row_slot == s)
        w = np.abs(to_f32(inp.w2_slots[int(s)]))                 # [d, f]
        t1[sel] = habs[sel] @ w.T
        t2[sel] = (habs[sel] * habs[sel]) @ (w * w).T
        wsum[sel] = w.sum(axis=1, dtype=np.float64)[None, :]
    if cfg.dtype == "f32":
        return 1e-5 * np.abs(y_ref) + 2e-6 * t1 + 2e-6 * wsum
    return (2.0 ** -7 * np.abs(y_ref) + np.minimum(1.05 * 2.0 ** -8 * t1, 2.0 ** -5 * np.sqrt(t2)) + 1e-6 * t1
            + 2e-6 * wsum)


def check_within(got: np.ndarray, ref: np.ndarray, bound: np.ndarray, what: str):
    excess = np.abs(got - ref) - bound
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (f"{what}: element {worst} got {got[worst]!r} ref {ref[worst]!r}, "
                                f"bound {bound[worst]:.4g}")


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
    # element by element: y_perm within y_bound(), out within the bounds of its k rows of y carried through the
    # combine plus its own rounding
    h_ref = np.stack([ref.h_rows[int(r)] for r in rows])
    row_slot = (np.searchsorted(ref.permutation.slot_offsets, rows, side="right") - 1).astype(np.int32)
    yb = y_bound(dl, row_slot, h_ref, y_ref)
    check_within(to_f64(b.y_perm)[rows], y_ref, yb, "y_perm")
    where = {int(r): i for i, r in enumerate(rows)}
    bound = (2.0 ** -7 if cfg.dtype == "bf16" else 1e-5) * np.abs(ref.out)
    for j in range(cfg.k):
        at = [where[int(r)] for r in ref.permutation.inv_perm[ref.tokens.astype(np.int64) * cfg.k + j]]
        bound += ref.topk_weight[ref.tokens, j][:, None] * yb[at]
    check_within(out, ref.out, bound, "out")
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
    check_within(y_got, y_ref, y_bound(dl, row_slot, h_ref, y_ref), "y_perm")
    return h_err, y_err
