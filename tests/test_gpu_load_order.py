"""The orderings of Section 4 observed through event times, with a hazard that is real: the load is
issued while forwards of several milliseconds still read the slots it overwrites, and copies of
about a millisecond per expert make the order of completion visible.

  - a load waits for the forward that still reads its slots (the paper's per-layer lock): the whole
    copy lies after the event the forward records when it is done;
  - loads of consecutive layers run one after the other on the loader's stream (the paper: the
    next layer's load starts when the previous one has finished), and a layer's forward waits for
    its own load only."""
import numpy as np
import pytest
import torch

import paper_2503_06823_amd as P

pytestmark = pytest.mark.gpu

D, F, E, S, K, T = 2048, 4096, 4, 2, 2, 4096        # 50 MB per expert: about 0.9 ms on the host link


def pinned_experts(n, seed):
    g = torch.Generator().manual_seed(seed)
    mk = lambda *shape: (torch.randn(*shape, generator=g) * 0.02).bfloat16().pin_memory()
    return [mk(F, D) for _ in range(n)], [mk(F, D) for _ in range(n)], [mk(D, F) for _ in range(n)]


def slot_buffers():
    z = lambda *shape: torch.zeros(*shape, dtype=torch.bfloat16, device="cuda")
    return z(S, F, D), z(S, F, D), z(S, D, F)


def timed():
    return P.make_event(timing=True)


def test_a_load_waits_for_the_forward_that_reads_its_slots(gpu_device):
    desc = P.make_desc(T, D, F, E, K, S, "bf16", "swiglu")
    h1, h3, h2 = pinned_experts(E, 1)
    w1, w3, w2 = slot_buffers()
    soe = torch.full((E,), -1, dtype=torch.int32, device="cuda")
    eos = torch.full((S,), -1, dtype=torch.int32, device="cuda")
    mirror = np.full(S, -1, dtype=np.int32)
    g = torch.Generator(device="cuda").manual_seed(2)
    x = torch.randn(T, D, generator=g, device="cuda").bfloat16()
    wg = (torch.randn(E, D, generator=g, device="cuda") / D ** 0.5).bfloat16()
    buf = P.LayerBuffers.allocate(desc)
    compute, side = torch.cuda.current_stream(), torch.cuda.Stream()
    side.wait_stream(compute)

    def load(experts, wait=None, done=None):
        P.emoe_load_experts(desc, experts, [0, 1], h1, h3, h2, w1, w3, w2, soe, eos, mirror, side, wait_event=wait,
                            done_event=done)

    load([0, 1]); side.synchronize()                      # first touch of the pinned pages, untimed
    a, b = timed(), timed()
    a.record(side); load([2, 3]); b.record(side); side.synchronize()
    copy_alone_ms = a.elapsed_time(b)                     # two experts with nothing else running
    load([0, 1]); side.synchronize()

    def forward():
        return P.layer_forward(buf, x, wg, None, soe, w1, w3, w2)

    forward(); torch.cuda.synchronize()
    first = buf.out.clone()
    n_forwards = 10
    started, released, issued, loaded = timed(), timed(), timed(), timed()
    started.record(compute)
    for _ in range(n_forwards):
        forward()
    released.record(compute)                              # after this point the slots may be overwritten
    issued.record(side)                                   # the side stream is idle: it reaches this at once
    load([2, 3], wait=released, done=loaded)              # overwrites both slots the forwards are reading
    torch.cuda.synchronize()
    forward_ms = started.elapsed_time(released)
    assert forward_ms > 2.0, f"the forwards took only {forward_ms:.2f} ms: no window for the hazard"
    # the hazard was real: the load sat on its stream while the forwards still had most of their time to run
    assert issued.elapsed_time(released) > 0.5 * forward_ms, "the load was not issued while the forwards ran"
    # and it was honoured: the whole copy lies after `released`
    assert released.elapsed_time(loaded) >= 0.9 * copy_alone_ms, (
        f"the copy ({copy_alone_ms:.2f} ms alone) ended {released.elapsed_time(loaded):.2f} ms after the forward's "
        "release: part of it ran while the forward still read the slots")
    assert torch.equal(buf.out, first), "a forward saw weights change under it"
    assert mirror.tolist() == [2, 3]


def test_layers_load_one_after_the_other_and_each_forward_waits_for_its_own(gpu_device):
    n_layers = 3
    desc = P.make_desc(64, D, F, E, K, S, "bf16", "swiglu")
    h1, h3, h2 = pinned_experts(E, 3)
    layers = []
    for _ in range(n_layers):
        w1, w3, w2 = slot_buffers()
        layers.append(dict(desc=desc, host_w1=h1, host_w3=h3, host_w2=h2, w1_slots=w1, w3_slots=w3, w2_slots=w2,
                           slot_of_expert=torch.full((E,), -1, dtype=torch.int32, device="cuda"),
                           expert_of_slot=torch.full((S,), -1, dtype=torch.int32, device="cuda")))
    torch.cuda.synchronize()
    loader = P.Loader(layers, 40)
    _, action = loader.next_prompt()
    assert action == P.EMOE_PROMPT_PREDICT                # two slots for four experts: the first prompt needs a selection
    loader.update([[0, 1]] * n_layers); loader.synchronize()      # first touch of the pinned pages, untimed
    t0, t1 = timed(), timed()
    t0.record()
    loader.update([[2, 3]] * n_layers); loader.synchronize()
    t1.record(); torch.cuda.synchronize()
    per_layer_ms = t0.elapsed_time(t1) / n_layers         # one layer's two experts

    begin, ready = timed(), [timed() for _ in range(n_layers)]
    begin.record()
    loader.update([[0, 1]] * n_layers)                    # every layer changes both experts
    for i in range(n_layers):
        loader.layer_begin(i)                             # the compute stream waits for layer i's load only
        ready[i].record()                                 # ... so this is when that load was done
        loader.layer_end(i)
    torch.cuda.synchronize()
    loader.close()
    at = [begin.elapsed_time(e) for e in ready]
    # layer 0 is usable after one layer's copy, long before the whole chain is done
    assert at[0] < 1.6 * per_layer_ms, f"layer 0 waited {at[0]:.2f} ms, one layer's load takes {per_layer_ms:.2f} ms"
    # and the loads do not overlap: each finishes a whole copy time after the one before
    for i in range(1, n_layers):
        assert at[i] - at[i - 1] >= 0.8 * per_layer_ms, (
            f"layer {i}'s load finished {at[i] - at[i - 1]:.2f} ms after layer {i - 1}'s; alone it takes {per_layer_ms:.2f} ms")
