"""Device buffers for one layer and the four-call forward (route -> permute -> expert FFN ->
combine).  Only allocation and call order live here; all arithmetic is in libemoe."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as B


@dataclass
class LayerBuffers:
    """Every output and workspace buffer of one layer forward, allocated once with torch."""
    desc: B.EmoeLayerDesc
    topk_expert: torch.Tensor
    topk_weight: torch.Tensor
    slot_counts: torch.Tensor
    slot_offsets: torch.Tensor
    perm: torch.Tensor
    inv_perm: torch.Tensor
    x_perm: torch.Tensor
    y_perm: torch.Tensor
    out: torch.Tensor
    permute_ws: torch.Tensor
    ffn_ws: torch.Tensor

    @staticmethod
    def allocate(desc: B.EmoeLayerDesc, device="cuda:0") -> "LayerBuffers":
        T, k, S, d = desc.T, desc.k, desc.S, desc.d_model
        A = T * k
        el = torch.float32 if desc.dtype == B.EMOE_F32 else torch.bfloat16
        pws, fws = B.emoe_workspace_bytes(desc)
        i32 = dict(dtype=torch.int32, device=device)
        return LayerBuffers(
            desc=desc,
            topk_expert=torch.empty((max(T, 1), k), **i32),
            topk_weight=torch.empty((max(T, 1), k), dtype=torch.float32, device=device),
            slot_counts=torch.empty(S, **i32), slot_offsets=torch.empty(S + 1, **i32),
            perm=torch.empty(max(A, 1), **i32), inv_perm=torch.empty(max(A, 1), **i32),
            x_perm=torch.empty((max(A, 1), d), dtype=el, device=device),
            y_perm=torch.empty((max(A, 1), d), dtype=el, device=device),
            out=torch.empty((max(T, 1), d), dtype=el, device=device),
            permute_ws=torch.empty(pws, dtype=torch.uint8, device=device),
            ffn_ws=torch.empty(fws, dtype=torch.uint8, device=device))


def _to_device(a, device):
    """numpy storage array -> device tensor; uint16 arrays are bf16 bit patterns."""
    if a is None:
        return None
    import numpy as np
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


@dataclass
class DeviceInputs:
    """One layer's inputs resident in HBM (a plain upload of host arrays, no arithmetic)."""
    x: torch.Tensor
    w_gate: torch.Tensor
    gate_bias: Optional[torch.Tensor]
    slot_of_expert: torch.Tensor
    w1_slots: torch.Tensor
    w3_slots: Optional[torch.Tensor]
    w2_slots: torch.Tensor

    @staticmethod
    def upload(host, device="cuda:0") -> "DeviceInputs":
        """`host` has numpy fields x, w_gate, gate_bias, slot_of_expert, w1_slots, w3_slots, w2_slots."""
        return DeviceInputs(*[_to_device(getattr(host, n), device) for n in
                              ("x", "w_gate", "gate_bias", "slot_of_expert", "w1_slots", "w3_slots", "w2_slots")])


def layer_forward(buf: LayerBuffers, x, w_gate, gate_bias, slot_of_expert, w1_slots, w3_slots, w2_slots,
                  stream=None, gather_in_ffn: bool = True, one_call: bool = False) -> torch.Tensor:
    """Enqueue the four calls on one stream; returns buf.out (no host synchronisation).
    `gather_in_ffn`: the FFN reads the token rows through perm (buf.x_perm stays unwritten); otherwise
    emoe_permute copies them into buf.x_perm first.  `one_call`: the same four steps through the
    library's emoe_layer_forward (implies gather_in_ffn)."""
    d = buf.desc
    if one_call:
        B.emoe_layer_forward(d, x, w_gate, gate_bias, slot_of_expert, w1_slots, w3_slots, w2_slots, buf.topk_expert,
                             buf.topk_weight, buf.slot_counts, buf.slot_offsets, buf.perm, buf.inv_perm, buf.y_perm,
                             buf.out, buf.permute_ws, buf.permute_ws.numel(), buf.ffn_ws, buf.ffn_ws.numel(), stream)
        return buf.out
    B.emoe_route(d, x, w_gate, gate_bias, slot_of_expert, buf.topk_expert, buf.topk_weight, stream)
    B.emoe_permute(d, x, buf.topk_expert, slot_of_expert, buf.slot_counts, buf.slot_offsets, buf.perm, buf.inv_perm,
                   None if gather_in_ffn else buf.x_perm, buf.permute_ws, buf.permute_ws.numel(), stream)
    if gather_in_ffn:
        B.emoe_expert_ffn_gather(d, x, buf.perm, buf.slot_offsets, w1_slots, w3_slots, w2_slots, buf.y_perm,
                                 buf.ffn_ws, buf.ffn_ws.numel(), stream)
    else:
        B.emoe_expert_ffn(d, buf.x_perm, buf.slot_offsets, w1_slots, w3_slots, w2_slots, buf.y_perm, buf.ffn_ws,
                          buf.ffn_ws.numel(), stream)
    B.emoe_combine(d, buf.y_perm, buf.inv_perm, buf.topk_weight, buf.out, stream)
    return buf.out
