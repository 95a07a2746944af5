"""emoe_permute_static, the entry point for callers that cannot allocate, against emoe_permute: the
same permutation bit for bit, on two calls in a row that share the library's static scratch, the
second with a smaller input (what the first call left in the scratch must not matter), then a third
that fits one workgroup.  Collected last on purpose: see the file name."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P
from gpu_util import desc_of, to_dev

pytestmark = pytest.mark.gpu


def _case(name, index, T, E, k, R, S, d_model=64):
    return gen.LayerConfig(name=name, index=index, T=T, d_model=d_model, d_ff=64, E=E, k=k, R=R, S=S, dtype="bf16",
                           act="swiglu", zipf_s=1.1)


def _both(c, with_rows):
    """Runs emoe_permute and emoe_permute_static on the oracle's routing of a seeded case; returns the outputs."""
    inp = gen.make_routing_inputs(c, shuffle_slots=True)
    ref = oracle.layer_forward(inp, with_ffn=False)
    d = desc_of(c)
    A = c.T * c.k
    x = to_dev(inp.x, c.dtype)
    te = torch.from_numpy(ref.topk_expert).cuda()
    soe = torch.from_numpy(inp.slot_of_expert).cuda()
    res = []
    for static in (False, True):
        i32 = dict(dtype=torch.int32, device="cuda")
        counts, offsets = torch.full((c.slots,), -3, **i32), torch.full((c.slots + 1,), -3, **i32)
        perm, inv = torch.full((A,), -3, **i32), torch.full((A,), -3, **i32)
        xp = torch.zeros((A, c.d_model), dtype=torch.bfloat16, device="cuda") if with_rows else None
        if static:
            P.emoe_permute_static(d, x, te, soe, counts, offsets, perm, inv, xp)
        else:
            pws, _ = P.emoe_workspace_bytes(d)
            ws = torch.empty(pws, dtype=torch.uint8, device="cuda")
            P.emoe_permute(d, x, te, soe, counts, offsets, perm, inv, xp, ws, pws)
        torch.cuda.synchronize()
        res.append((counts, offsets, perm, inv, xp))
    # and the existing entry point is itself the oracle's permutation
    pm = ref.permutation
    assert np.array_equal(res[0][2].cpu().numpy(), pm.perm) and np.array_equal(res[0][3].cpu().numpy(), pm.inv_perm)
    return res


def test_static_scratch_permute_equals_the_workspace_one(gpu_device):
    for c, with_rows in ((_case("static_largest", 304, T=40000, E=32, k=2, R=11, S=16, d_model=16), False),  # 79 x 16: three launches
                         (_case("static_large", 300, T=9000, E=64, k=6, R=24, S=40), True),     # 53 workgroups x 40 slots
                         (_case("static_smaller", 301, T=2500, E=16, k=2, R=7, S=9), False),    # 5 workgroups x 9 slots
                         (_case("static_one_workgroup", 302, T=300, E=8, k=2, R=4, S=4), True)):
        plain, static = _both(c, with_rows)
        for a, b, what in zip(plain, static, ("slot_counts", "slot_offsets", "perm", "inv_perm", "x_perm")):
            assert (a is None and b is None) or torch.equal(a, b), f"{c.name}: {what} differs"


def test_static_scratch_permute_rejects_what_does_not_fit(gpu_device):
    c = _case("static_too_large", 303, T=1 << 20, E=64, k=2, R=64, S=64, d_model=8)       # 2048 workgroups x 64 slots
    d = desc_of(c)
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = P.emoe_permute_static(d, None, one, one, one, one, one, one, None, check=False)
    assert rc == P.EMOE_ERR_WORKSPACE
    assert "workspace" in P.status_string(rc)
