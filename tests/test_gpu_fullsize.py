"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.
Routing and the permutation are compared in full (bit-exact); the FFN and the combine on a seeded
sample of tokens that the oracle computes one by one."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
from gpu_util import DeviceLayer, check_outputs, check_routing_and_permutation

pytestmark = pytest.mark.gpu

SAMPLE = {"C1": None, "C2": 256, "C3": 16, "C4": 16, "C5": 96, "X1": 8, "X2": 48, "X3": 16, "X4": 16, "X5": 16}


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5", "X1", "X2", "X3", "X4", "X5"])
def test_full_size_workload(gpu_device, name):
    cfg = gen.CONFIGS.get(name) or gen.EXTRA_CONFIGS[name]
    print(f"full-size {cfg.name}: generating", flush=True)
    inp = gen.make_layer_inputs(cfg)
    n = SAMPLE[name]
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
    # properties that hold for every token, not only the sample
    out = dl.buf.out.float()
    assert torch.isfinite(out).all()
    assert int(dl.buf.slot_offsets[-1]) == cfg.T * cfg.k
    tw = dl.buf.topk_weight
    assert torch.allclose(tw.sum(dim=1), torch.ones(cfg.T, device=tw.device), atol=1e-5)
    dl.check_gather_path_is_identical()       # the configuration bench.py times reads x through perm
