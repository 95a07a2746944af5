"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.
Routing and the permutation are compared in full (bit-exact).  The expert FFN is compared on a
stratified sample of grouped rows that the oracle computes one by one: of every slot the first and the
last row and a seeded row of every 32-row block, so that every output tile of every round of the
persistent launch, every tile cut along K and every ragged last tile holds compared rows; both the
intermediate h and y_perm, by relative L2 and element by element.  The combine is compared on a seeded
sample of tokens."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
import paper_2503_06823_amd as P
from gpu_util import DeviceLayer, check_ffn_rows, check_outputs, check_routing_and_permutation, stratified_rows

pytestmark = pytest.mark.gpu

# tokens whose `out` the oracle computes (each costs k FFN rows); None = all
TOKEN_SAMPLE = {"C1": None, "C2": 256, "C3": 16, "C4": None, "C5": 96, "X1": 8, "X2": 48, "X3": 16, "X4": 16, "X5": 16}


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5", "X1", "X2", "X3", "X4", "X5"])
def test_full_size_workload(gpu_device, name):
    cfg = gen.CONFIGS.get(name) or gen.EXTRA_CONFIGS[name]
    print(f"full-size {cfg.name}: generating", flush=True)
    inp = gen.make_layer_inputs(cfg)
    n = TOKEN_SAMPLE[name]
    tokens = None if n is None else np.sort(np.random.default_rng(cfg.seed).choice(cfg.T, n, replace=False))
    print(f"full-size {cfg.name}: oracle on {n or cfg.T} tokens", flush=True)
    ref = oracle.layer_forward(inp, tokens=tokens)
    print(f"full-size {cfg.name}: GPU", flush=True)
    dl = DeviceLayer(inp)
    dl.forward()
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    err = check_outputs(dl, ref)
    counts = ref.permutation.slot_counts
    print(f"full-size {cfg.name}: out rel-L2 {err:.3e}; rows per slot min {counts.min()} max {counts.max()}", flush=True)
    rows = stratified_rows(ref.permutation.slot_offsets, cfg.seed)
    print(f"full-size {cfg.name}: oracle FFN on {rows.size} stratified rows of {cfg.T * cfg.k}", flush=True)
    h_err, y_err = check_ffn_rows(dl, ref.permutation, rows)
    print(f"full-size {cfg.name}: h rel-L2 {h_err:.3e}, y_perm rel-L2 {y_err:.3e}", flush=True)
    # properties that hold for every token, not only the sample
    out = dl.buf.out.float()
    assert torch.isfinite(out).all()
    assert int(dl.buf.slot_offsets[-1]) == cfg.T * cfg.k
    tw = dl.buf.topk_weight
    assert torch.allclose(tw.sum(dim=1), torch.ones(cfg.T, device=tw.device), atol=1e-5)
    dl.check_gather_path_is_identical()       # the configuration bench.py times reads x through perm
    if cfg.k == 1:                             # ... and, with one expert per token, folds the combine into the second product
        b = dl.buf
        separate = b.out.clone()
        b.out.zero_()
        P.emoe_expert_ffn_gather_combine(dl.desc, dl.x, b.perm, b.inv_perm, b.slot_offsets, dl.w1, dl.w3, dl.w2,
                                         b.topk_weight, None, b.out, b.ffn_ws, b.ffn_ws.numel())
        torch.cuda.synchronize()
        assert torch.equal(b.out, separate)
