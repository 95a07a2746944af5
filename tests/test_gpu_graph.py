"""The layer's calls only enqueue kernels (no allocation, no memset, no host synchronisation), so a
decode step can be captured once into a HIP graph and replayed.  Replays are checked against the
eager result several times, with eager work and synchronisations between them."""
import numpy as np
import pytest
import torch

import emoe_inputs as gen
import oracle
from gpu_util import DeviceLayer, check_outputs, check_routing_and_permutation

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw", [
    ("graph_decode", dict(T=64, d_model=512, d_ff=1088, E=8, k=2, R=6)),          # streaming FFN path
    ("graph_prefill", dict(T=700, d_model=328, d_ff=456, E=8, k=2, R=4)),         # tiled FFN path with split tiles
    ("graph_one_prompt", dict(T=190, d_model=328, d_ff=456, E=8, k=2, R=4)),      # 128-row-tile FFN path
])
def test_graph_replays_match_eager(gpu_device, name, kw):
    c = gen.LayerConfig(name=name, index=110, dtype="bf16", act="swiglu", **kw)
    inp = gen.make_layer_inputs(c)
    ref = oracle.layer_forward(inp)
    dl = DeviceLayer(inp)
    b = dl.buf
    outputs = lambda: [t.clone() for t in (b.topk_expert, b.topk_weight, b.perm, b.inv_perm, b.slot_offsets, b.y_perm, b.out)]

    dl.forward(gather_in_ffn=True)                      # eager: also sets the kernels' launch attributes
    torch.cuda.synchronize()
    eager = outputs()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            dl.forward(gather_in_ffn=True)
    torch.cuda.synchronize()

    x0 = dl.x.clone()
    for replay in range(4):
        for t in (b.topk_expert, b.perm, b.inv_perm, b.slot_offsets):
            t.fill_(-7)
        b.y_perm.fill_(0); b.out.fill_(0); b.topk_weight.fill_(0)
        if replay == 2:                                   # other inputs in the same buffers: the graph reads them
            dl.x.copy_(torch.roll(x0, 1, dims=0))
        elif replay == 3:
            dl.x.copy_(x0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = outputs()
        if replay == 2:
            dl.forward(gather_in_ffn=True)                # eager on the rolled inputs
            torch.cuda.synchronize()
            want = outputs()
        else:
            want = eager
        for g, w in zip(got, want):
            assert torch.equal(g, w), f"replay {replay}"
    dl.forward(gather_in_ffn=False)                       # x_perm for the permutation check
    torch.cuda.synchronize()
    check_routing_and_permutation(dl, ref)
    check_outputs(dl, ref)
