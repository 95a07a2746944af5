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


def stream_beside(compute):
    """A stream whose work really runs beside `compute`'s: a process has a handful of hardware queues and two
    streams may share one, in which case their work runs in the order it was submitted and there is no overlap
    to observe.  Tries new streams until an event recorded on one completes while a 2 ms kernel (the library's
    matrix-instruction loop) still runs on `compute`; None if none does."""
    a = torch.ones(256 * 64, dtype=torch.bfloat16, device="cuda")
    sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    for _ in range(8):
        cand = torch.cuda.Stream()
        torch.cuda.synchronize()
        P.emoe_measure_mfma_loop(a, a, False, 256, 1800, sink, stream=compute)
        busy = P.make_event(stream=compute)
        probe = P.make_event(stream=cand)
        probe.synchronize()
        beside = not busy.query()          # the probe is done and the long kernel is not
        torch.cuda.synchronize()
        if beside:
            return cand
    return None


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
    compute = torch.cuda.current_stream()
    side = stream_beside(compute)
    if side is None:
        pytest.skip("no stream runs beside the compute stream here (they share a hardware queue): no hazard to observe")
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


def test_layers_load_one_after_the_other(gpu_device):
    """Watched from the host with the loader's non-blocking query, so that no second stream's place in a
    hardware queue can blur the picture: layer i becomes ready a whole copy time after layer i - 1."""
    import time
    n_layers = 6
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
    assert all(loader.layer_ready(i) for i in range(n_layers))            # nothing enqueued yet
    _, action = loader.next_prompt()
    assert action == P.EMOE_PROMPT_PREDICT                # two slots for four experts: the first prompt needs a selection
    loader.update([[0, 1]] * n_layers); loader.synchronize()      # first touch of the pinned pages, untimed
    loader.update([[2, 3]] * n_layers); loader.synchronize()
    # one layer's two experts cannot cross the host link faster than this (64 GB/s is the link's raw rate)
    floor_ms = 2 * 3 * D * F * 2 / 64e9 * 1e3

    t0 = time.perf_counter()
    loader.update([[0, 1]] * n_layers)                    # every layer changes both experts
    watched_from = (time.perf_counter() - t0) * 1e3       # enqueueing takes the host a few ms: the first loads may be done by now
    at = [None] * n_layers
    while any(a is None for a in at) and time.perf_counter() - t0 < 5.0:
        for i in range(n_layers):
            if at[i] is None and loader.layer_ready(i):
                at[i] = (time.perf_counter() - t0) * 1e3
    loader.synchronize()
    loader.close()
    assert all(a is not None for a in at), "a load did not finish within 5 s"
    assert at == sorted(at), f"layers became ready out of order: {at}"
    # Loads that ran side by side would share the link and all end near the end.  Every load that ended while
    # the host was watching must end a whole copy time after the one before it.
    seen = [i for i in range(1, n_layers) if at[i - 1] > watched_from + 0.2]
    if len(seen) < 2:
        pytest.skip(f"only {len(seen)} loads ended while the host watched (enqueued in {watched_from:.2f} ms, ready at {at})")
    for i in seen:
        assert at[i] - at[i - 1] >= 0.8 * floor_ms, (
            f"layer {i}'s load finished {at[i] - at[i - 1]:.2f} ms after layer {i - 1}'s; two experts need at least {floor_ms:.2f} ms "
            f"(ready at {at})")
