#!/usr/bin/env python3
"""Benchmark of the resident-expert MoE layer on one MI355X.

A step is one pass of the whole hot path (route -> permute -> expert FFN, which gathers the token
rows itself -> combine) over one
batch of synthetic input that is already resident in HBM.  The headline workload is the
Mixtral-8x7B-shaped prefill layer (4096 tokens, 4 of 8 experts resident); the decode step
(64 tokens, 6 of 8 resident) is measured in the same run and reported under "decode".
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
# HBM bytes per launch of the dominant kernels come from two hardware-counter runs of this command
# (FETCH_SIZE, then WRITE_SIZE; each scaled by what the same counter reads for a 1 GiB device copy).
# Counters cannot be read from inside the process: `python -m paper_2503_06823_amd.profile_tools traffic`
# turns the two runs into this tracked summary, whose machine-readable block is read back here.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "ffn_hbm_traffic_c3_prefill_c4_decode.md")


def measured_traffic(kernel_prefix):
    """HBM bytes per launch (fetched + written, scaled) of the kernel whose name starts with
    `kernel_prefix`, from the tracked counter summary; None if the summary does not hold it."""
    try:
        text = open(TRAFFIC_SUMMARY).read()
        block = text.split("```json", 1)[1].split("```", 1)[0]
        for k in json.loads(block)["kernels"]:
            if k["kernel"].startswith(kernel_prefix):
                return k["hbm_bytes_per_launch"]
    except (OSError, IndexError, KeyError, ValueError):
        pass
    return None


def host_cpu():
    """CPU model name and the number of physical cores of the machine, from /proc/cpuinfo."""
    model, cores = "unknown", set()
    try:
        phys = core = None
        for line in open("/proc/cpuinfo"):
            key, _, val = line.partition(":")
            key, val = key.strip(), val.strip()
            if key == "model name":
                model = val
            elif key == "physical id":
                phys = val
            elif key == "core id":
                core = val
            elif not key and phys is not None:
                cores.add((phys, core))
                phys = core = None
        if phys is not None:
            cores.add((phys, core))
    except OSError:
        pass
    return model, len(cores) or None


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


SETTLE_SECONDS = 0.3   # untimed steps before the warm-up of every workload but the headline, see settle()


def settle(torch, step, seconds=SETTLE_SECONDS):
    """Untimed steps for `seconds` of wall time.  After an idle spell (generating the next workload's inputs on
    the host takes seconds) the GPU's clocks take some tens of milliseconds of load to come back up; a
    workload whose whole measurement lasts 20 ms would be timed during that ramp (the fine-grained layer:
    0.94 ms per step straight after idle, 0.85 ms after 0.3 s of load).  The headline workload is not
    settled this way: it gets exactly the W warm-up steps the command line asks for."""
    t0, i = time.perf_counter(), 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            step(i); i += 1
        torch.cuda.synchronize()
    return i


def timed_steps(torch, P, dev, buf, steps, warmup, weight_sets, settle_first=False):
    """Runs warmup + steps layer forwards; the FFN is issued as its two passes with events between
    them so each grouped product's launch duration is measured inside the timed region."""
    d = buf.desc
    ws_n = buf.ffn_ws.numel()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]

    folded = d.k == 1     # one expert per token: the library folds the combine into the second product (one launch fewer)

    def step(i, events=None):
        w1, w3, w2 = weight_sets[i % len(weight_sets)]
        if events: events[0].record()
        P.emoe_route(d, dev.x, dev.w_gate, dev.gate_bias, dev.slot_of_expert, buf.topk_expert, buf.topk_weight)
        P.emoe_permute(d, dev.x, buf.topk_expert, dev.slot_of_expert, buf.slot_counts, buf.slot_offsets, buf.perm,
                       buf.inv_perm, None, buf.permute_ws, buf.permute_ws.numel())     # indices only
        if events: events[1].record()
        if folded:
            P.emoe_expert_ffn_gather_combine(d, dev.x, buf.perm, buf.inv_perm, buf.slot_offsets, w1, w3, w2, buf.topk_weight,
                                             None, buf.out, buf.ffn_ws, ws_n)
            if events:
                for e in events[2:]: e.record()
            return
        # the FFN reads the token rows through perm (no x_perm copy)
        P.emoe_expert_ffn_gather_pass(d, 1, dev.x, buf.perm, buf.slot_offsets, w1, w3, w2, buf.y_perm, buf.ffn_ws, ws_n)
        if events: events[2].record()
        P.emoe_expert_ffn_gather_pass(d, 2, dev.x, buf.perm, buf.slot_offsets, w1, w3, w2, buf.y_perm, buf.ffn_ws, ws_n)
        if events: events[3].record()
        P.emoe_combine(d, buf.y_perm, buf.inv_perm, buf.topk_weight, buf.out)
        if events: events[4].record()

    if settle_first:
        settle(torch, step)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i, ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    names = ["route_permute", "ffn_and_combine_folded", "-", "-"] if folded else ["route_permute", "ffn_pass1", "ffn_pass2", "combine"]
    ms = {n: sum(e[j].elapsed_time(e[j + 1]) for e in ev) / steps for j, n in enumerate(names)}
    for j, n in enumerate(names):     # median and minimum over the timed steps, per call
        v = sorted(e[j].elapsed_time(e[j + 1]) for e in ev)
        ms[n + "_median"], ms[n + "_min"] = v[len(v) // 2], v[0]
    for key in [k for k in ms if k.startswith("-")]:
        del ms[key]
    v = sorted(e[0].elapsed_time(e[4]) for e in ev)
    ms["step_median"], ms["step_min"] = v[len(v) // 2], v[0]
    return wall, ms


def run_workload(torch, P, gen, cfg, steps, warmup, copies, graph=False, settle_first=True):
    log(f"generating {cfg.name} on the host ...")
    t = time.perf_counter()
    inp = gen.make_layer_inputs(cfg)
    log(f"  done in {time.perf_counter() - t:.1f}s; uploading")
    dev = P.DeviceInputs.upload(inp)
    desc = P.make_desc(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.slots, cfg.dtype, cfg.act)
    buf = P.LayerBuffers.allocate(desc)
    sets = [(dev.w1_slots, dev.w3_slots, dev.w2_slots)]
    for _ in range(copies - 1):   # independent copies of the slot buffers, rotated so no step finds its weights cached
        sets.append(tuple(None if w is None else w.clone() for w in sets[0]))
    wall, ms = timed_steps(torch, P, dev, buf, steps, warmup, sets, settle_first)
    torch.cuda.synchronize()
    counts = buf.slot_counts.cpu().numpy()
    if graph:
        ms["graph_wall_s"] = graph_steps(torch, P, dev, buf, steps, warmup, sets)
    return inp, wall, ms, counts, dev, buf


def graph_steps(torch, P, dev, buf, steps, warmup, weight_sets):
    """The same step captured once per weight set into a HIP graph (the calls only enqueue kernels) and
    replayed: what a serving loop does with a launch-bound step.  Returns seconds for `steps` replays."""
    d = buf.desc
    ws_n = buf.ffn_ws.numel()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs = []
    for w1, w3, w2 in weight_sets:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                P.emoe_route(d, dev.x, dev.w_gate, dev.gate_bias, dev.slot_of_expert, buf.topk_expert, buf.topk_weight)
                P.emoe_permute(d, dev.x, buf.topk_expert, dev.slot_of_expert, buf.slot_counts, buf.slot_offsets,
                               buf.perm, buf.inv_perm, None, buf.permute_ws, buf.permute_ws.numel())
                P.emoe_expert_ffn_gather_combine(d, dev.x, buf.perm, buf.inv_perm, buf.slot_offsets, w1, w3, w2,
                                                 buf.topk_weight, buf.y_perm, buf.out, buf.ffn_ws, ws_n)
        graphs.append(g)
    torch.cuda.synchronize()
    settle(torch, lambda i: graphs[i % len(graphs)].replay())
    for i in range(warmup):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        graphs[(warmup + i) % len(graphs)].replay()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def miss_rate(torch, P, dev, buf):
    """Fraction of the (token, rank) pairs whose expert under ordinary top-k routing is not resident, so
    that the fallback rule of Section 3.2.2 reroutes the token: the layer's routing is run once more
    with every expert marked resident and its choices are looked up in the real slot map (all on the
    device, from the library's results)."""
    d = buf.desc
    everyone = torch.arange(d.E, dtype=torch.int32, device=dev.x.device)
    free = torch.empty_like(buf.topk_expert)
    w = torch.empty_like(buf.topk_weight)
    P.emoe_route(d, dev.x, dev.w_gate, dev.gate_bias, everyone, free, w)
    torch.cuda.synchronize()
    return float((dev.slot_of_expert[free.long()] < 0).float().mean())


def combine_by_scatter(torch, P, buf):
    """Section 5.1 argues with global-memory reads, and folding the combine into the second product would spare
    the y_perm round trip; with several experts per token that needs atomics.  Times the combine kernel against
    the same combine done that way (clear an fp32 image, add every grouped row into it with atomics, convert):
    a lower bound of what the fold costs, since the second product's own work is not even included."""
    d = buf.desc
    image = torch.empty((d.T, d.d_model), dtype=torch.float32, device="cuda")
    out2 = torch.empty_like(buf.out)
    def timed(fn, n=12):
        for _ in range(3): fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record()
        for i in range(n):
            fn(); ev[i + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))[n // 2] * 1e3
    t_combine = timed(lambda: P.emoe_combine(d, buf.y_perm, buf.inv_perm, buf.topk_weight, buf.out))
    t_scatter = timed(lambda: P.emoe_measure_scatter_combine(d, buf.y_perm, buf.perm, buf.topk_weight, image, out2))
    diff = float((out2.float() - buf.out.float()).abs().max())
    el = 2
    return {"combine_kernel_us": t_combine, "clear_scatter_add_convert_us": t_scatter, "max_abs_difference": diff,
            "combine_bytes": (d.T * d.k + d.T) * d.d_model * el,
            "scatter_bytes_beside_the_second_product": d.T * d.d_model * (4 + 4 * d.k + 4 + el),
            "y_perm_bytes_the_fold_would_spare": 2 * d.T * d.k * d.d_model * el}


def measure_ceilings(torch, P, x, w, read_buffers):
    """What this GPU sustains on the two resources that bound the FFN, with kernels that do nothing else:
    the matrix-instruction loop on the workload's own operand values (no global traffic) and a plain
    read stream over weight buffers (rotated so no launch finds its data cached)."""
    res = {}
    sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    iters = 896     # 256 workgroups x 896 rounds = 1.924 TFLOP, one launch of the prefill layer's first product
    for key, lds in (("mfma_loop_with_lds_reads", True), ("mfma_loop_registers_only", False)):
        for _ in range(3):
            P.emoe_measure_mfma_loop(x, w, lds, 256, iters, sink)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(21)]
        ev[0].record()
        for i in range(20):
            flop = P.emoe_measure_mfma_loop(x, w, lds, 256, iters, sink)
            ev[i + 1].record()
        torch.cuda.synchronize()
        t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(20))
        res[key] = {"tflops_mean": flop / (sum(t) / 20 * 1e-3) / 1e12, "tflops_best": flop / (t[0] * 1e-3) / 1e12,
                    "launch_ms_mean": sum(t) / 20, "launches": 20, "flop_per_launch": flop}
    sink16 = torch.empty(4, dtype=torch.int32, device="cuda")
    best = None
    for wgs in (2048, 4096, 8192, 16384):
        nbytes = [b.numel() * b.element_size() // 32768 * 32768 for b in read_buffers]
        for i in range(len(read_buffers)):
            P.emoe_measure_read_stream(read_buffers[i], nbytes[i], wgs, sink16)
        n = 12
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record()
        for i in range(n):
            P.emoe_measure_read_stream(read_buffers[i % len(read_buffers)], nbytes[i % len(read_buffers)], wgs, sink16)
            ev[i + 1].record()
        torch.cuda.synchronize()
        gbs = sum(nbytes[i % len(read_buffers)] for i in range(n)) / (ev[0].elapsed_time(ev[n]) * 1e-3) / 1e9
        if best is None or gbs > best["gbs"]:
            best = {"gbs": gbs, "workgroups": wgs, "bytes_per_launch": nbytes[0], "launches": n}
    res["read_stream"] = best
    log(f"ceilings: {res}")
    return res


def layer_work(cfg, counts):
    """Algorithmic work of one layer forward: flop of the routed rows, weight bytes of the non-empty slots."""
    A = cfg.T * cfg.k
    mats = 3 if cfg.act == "swiglu" else 2
    occupied = int((counts > 0).sum())
    return 2.0 * A * mats * cfg.d_model * cfg.d_ff, occupied * mats * cfg.d_model * cfg.d_ff * cfg.elem_bytes


def other_config(torch, P, gen, cfg, steps, warmup, copies, label, graph=False):
    _, wall, ms, counts, dev, buf = run_workload(torch, P, gen, cfg, steps, warmup, copies, graph=graph)
    missed = miss_rate(torch, P, dev, buf)
    fold = combine_by_scatter(torch, P, buf) if (cfg.k > 1 and cfg.dtype == "bf16") else None
    del dev, buf
    torch.cuda.empty_cache()
    flop, wbytes = layer_work(cfg, counts)
    extra = {}
    if graph:       # a launch-bound layer is timed as a replayed HIP graph, like the decode step
        extra = {"launch": "one HIP graph per weight copy, replayed", "ms_per_step_eager": wall / steps * 1e3}
        wall = ms.pop("graph_wall_s")
    t = wall / steps
    log(f"{cfg.name}: {t * 1e3:.3f} ms/step, miss rate {missed:.3f}, breakdown {ms}")
    return {"config": {"workload": label, "rows_per_slot_max": int(counts.max()), "slots_with_rows": int((counts > 0).sum())},
            "value": cfg.T / t, "unit": "tokens/s", "ms_per_step": t * 1e3, "steps": steps, "breakdown_ms": ms,
            "miss_rate": missed, **extra, **({"combine_fold_measurement": fold} if fold else {}),
            "layer_tflops": flop / t / 1e12, "layer_mfma_frac": flop / t / 1e12 / PEAK_BF16_MFMA_TFLOPS,
            "layer_weight_gbs": wbytes / t / 1e9, "layer_hbm_frac": wbytes / t / 1e9 / PEAK_HBM_GBS}


def bench_load(torch, P, gen, c3, dev3, buf3):
    """Section 4's upload: experts from pinned host memory into slots on a side stream.  Times one
    Mixtral-sized expert, a list of four, and the list of four while the prefill layer runs on the
    compute stream out of other slot buffers."""
    import numpy as np
    f, d, E = c3.d_ff, c3.d_model, c3.E
    S = 4
    desc = P.make_desc(c3.T, d, f, E, c3.k, S, c3.dtype, c3.act)
    def pin(src):   # pinned host copy of a device matrix (real weight values: zeros would flatter the clock)
        t = torch.empty(src.shape, dtype=src.dtype).pin_memory()
        t.copy_(src)
        return t
    h1 = [pin(dev3.w1_slots[i % 4]) for i in range(5)] + [None] * (E - 5)
    h3 = [pin(dev3.w3_slots[i % 4]) for i in range(5)] + [None] * (E - 5)
    h2 = [pin(dev3.w2_slots[i % 4]) for i in range(5)] + [None] * (E - 5)
    w1 = torch.empty((S, f, d), dtype=torch.bfloat16, device="cuda")
    w3, w2 = torch.empty_like(w1), torch.empty((S, d, f), dtype=torch.bfloat16, device="cuda")
    soe = torch.full((E,), -1, dtype=torch.int32, device="cuda")
    eos = torch.full((S,), -1, dtype=torch.int32, device="cuda")
    mirror = np.full(S, -1, dtype=np.int32)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    expert_bytes = 3 * f * d * 2

    def timed_load(experts, slots):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        P.emoe_load_experts(desc, experts, slots, h1, h3, h2, w1, w3, w2, soe, eos, mirror, side)
        e1.record(side)
        return e0, e1

    timed_load([0, 1, 2, 3], [0, 1, 2, 3]); side.synchronize()          # untimed: first touch of the pinned pages
    e0, e1 = timed_load([0, 1, 2, 3], [0, 1, 2, 3]); side.synchronize()
    four_ms = e0.elapsed_time(e1)
    e0, e1 = timed_load([4], [0]); side.synchronize()
    one_ms = e0.elapsed_time(e1)
    # overlapped with the prefill layer
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_fwd = 40
    e0, e1 = timed_load([0, 1, 2, 3], [0, 1, 2, 3])
    c0.record()
    for _ in range(n_fwd):
        P.layer_forward(buf3, dev3.x, dev3.w_gate, dev3.gate_bias, dev3.slot_of_expert, dev3.w1_slots, dev3.w3_slots,
                        dev3.w2_slots)
    c1.record()
    torch.cuda.synchronize()
    ov_ms, fwd_ms = e0.elapsed_time(e1), c0.elapsed_time(c1) / n_fwd
    res = {"one_expert": {"bytes": expert_bytes, "ms": one_ms, "gbs": expert_bytes / one_ms / 1e6},
           "four_experts": {"bytes": 4 * expert_bytes, "ms": four_ms, "gbs": 4 * expert_bytes / four_ms / 1e6},
           "four_experts_during_prefill": {"ms": ov_ms, "gbs": 4 * expert_bytes / ov_ms / 1e6,
                                           "layer_ms_per_step_meanwhile": fwd_ms},
           "note": "pinned host -> HBM through emoe_load_experts on a side stream; not part of tokens/s"}
    log(f"load: {res}")
    del w1, w3, w2
    torch.cuda.empty_cache()
    res["stack_of_4_layers"] = bench_loader(torch, P, c3, dev3, buf3, h1, h3, h2)
    return res


def bench_loader(torch, P, c3, dev3, buf3, h1, h3, h2):
    """Sections 3.3 / 4 on four Mixtral-shaped layers (4 slots each): the prompt that changes the residents
    (two of four experts per layer, 2.8 GB in all) with the loads exposed (wait for all of them, then compute)
    and hidden (compute starts at once; each layer waits for its own load only)."""
    n_layers, S, E = 4, 4, c3.E
    f, d = c3.d_ff, c3.d_model
    desc = P.make_desc(c3.T, d, f, E, c3.k, S, c3.dtype, c3.act)
    full = lambda h: [h[i % 5] for i in range(E)]     # every expert has host weights (five distinct buffers)
    layers = []
    for _ in range(n_layers):
        w1 = torch.empty((S, f, d), dtype=torch.bfloat16, device="cuda")
        layers.append(dict(desc=desc, host_w1=full(h1), host_w3=full(h3), host_w2=full(h2), w1_slots=w1,
                           w3_slots=torch.empty_like(w1), w2_slots=torch.empty((S, d, f), dtype=torch.bfloat16, device="cuda"),
                           slot_of_expert=torch.full((E,), -1, dtype=torch.int32, device="cuda"),
                           expert_of_slot=torch.full((S,), -1, dtype=torch.int32, device="cuda")))
    torch.cuda.synchronize()
    loader = P.Loader(layers, 40)
    index, action = loader.next_prompt()              # 4 of 8 experts fit: the first prompt needs a selection
    assert action == P.EMOE_PROMPT_PREDICT
    loader.update([[0, 1, 2, 3]] * n_layers)
    loader.synchronize()

    def prompt(exposed, selection):
        t0 = time.perf_counter()
        if selection is not None:
            loader.update([selection] * n_layers)
            if exposed:
                loader.synchronize()
        for i, l in enumerate(layers):
            loader.layer_begin(i)
            P.layer_forward(buf3, dev3.x, dev3.w_gate, dev3.gate_bias, l["slot_of_expert"], l["w1_slots"], l["w3_slots"],
                            l["w2_slots"])
            loader.layer_end(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    prompt(False, None)
    plain = min(prompt(False, None) for _ in range(3))
    exposed = prompt(True, [0, 1, 4, 5])
    hidden = prompt(False, [0, 1, 2, 3])
    exposed2 = prompt(True, [0, 1, 4, 5])
    hidden2 = prompt(False, [0, 1, 2, 3])
    loader.close()
    res = {"layers": n_layers, "bytes_loaded_per_change": n_layers * 2 * 3 * f * d * 2,
           "prompt_ms_no_load": plain, "prompt_ms_loads_exposed": min(exposed, exposed2),
           "prompt_ms_loads_hidden": min(hidden, hidden2)}
    log(f"loader: {res}")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the matrix-loop and read-stream ceiling measurements")
    ap.add_argument("--no-extras", action="store_true", help="skip the upload measurement and the C5 / C2 workloads")
    ap.add_argument("--more-shapes", action="store_true",
                    help="also time a Mixtral-8x22B-shaped prefill layer, an OpenMoE-shaped layer and one short prompt at the Mixtral-8x7B shape")
    ap.add_argument("--only", default="", help="time just this workload (C2, C5, X1 .. X5) and print its record: for profiler "
                                               "runs of a workload that is not the headline")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = size the sample for about 15 s")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run the library's plain copy kernel on 1 GiB, so that a hardware-counter run of this "
                         "command also holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards by tokens with no "
              "exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import emoe_inputs as gen
    import paper_2503_06823_amd as P
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    P.lib()  # fails loudly if libemoe.so has not been built

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            P.emoe_measure_copy_stream(src, dst, 1 << 30, 8192)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.only:
        cfg = gen.CONFIGS.get(args.only) or gen.EXTRA_CONFIGS[args.only]
        copies = {"C2": 4, "C4": 3, "X3": 3, "X5": 2}.get(args.only, 1)
        print(json.dumps(other_config(torch, P, gen, cfg, args.steps, args.warmup, copies, cfg.name,
                                      graph=args.only in ("C2", "C4", "X3", "X5"))), flush=True)
        return

    # ---------------- prefill (headline) ----------------
    c3 = gen.C3
    inp3, wall, ms, counts, dev3, buf3 = run_workload(torch, P, gen, c3, args.steps, args.warmup, copies=1,
                                                      settle_first=False)    # exactly W warm-up steps, then K timed
    ms_step = wall / args.steps * 1e3
    tokens_s = c3.T * args.steps / wall
    A = c3.T * c3.k
    flop_pass1 = 2.0 * A * 2 * c3.d_model * c3.d_ff       # gate and up products of the routed rows
    flop_pass2 = 2.0 * A * c3.d_model * c3.d_ff
    tf1 = flop_pass1 / (ms["ffn_pass1"] * 1e-3) / 1e12
    result = {
        "metric": "MoE-layer tokens/s at Mixtral-8x7B shape (prefill, decode); % MFMA / HBM roofline",
        "value": tokens_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C3 Mixtral-8x7B-shaped prefill layer: T=4096 d_model=4096 d_ff=14336 E=8 top-2 SwiGLU, "
                               "4 of 8 experts resident, bf16", "rows_per_slot": [int(c) for c in counts]},
        "roofline": {"bound": "mfma", "kernel": "grouped_gemm_bf16<SwiGLU> + splitk_fixup (FFN pass 1)", "achieved": tf1,
                     "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tf1 / PEAK_BF16_MFMA_TFLOPS,
                     "traffic": measured_traffic("grouped_gemm_bf16<1"), "traffic_unit": "bytes per launch",
                     "launch_ms": ms["ffn_pass1"]},
        "prefill_breakdown_ms": ms,
        "prefill_layer_mfma_frac": (flop_pass1 + flop_pass2) / (ms_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "prefill_pass2_tflops": flop_pass2 / (ms["ffn_pass2"] * 1e-3) / 1e12,
    }
    log(f"prefill: {ms_step:.3f} ms/step, {tokens_s:,.0f} tokens/s, pass1 {tf1:.0f} TFLOP/s, breakdown {ms}")

    result["prefill_miss_rate"] = miss_rate(torch, P, dev3, buf3)
    result["combine_fold_measurement"] = combine_by_scatter(torch, P, buf3)
    ceilings = None
    if not args.no_ceilings:
        # measured ceilings beside the datasheet peaks: the matrix-instruction loop on this layer's own token rows
        # and weights, a read stream over its three weight buffers (470 MB each, rotated)
        ceilings = measure_ceilings(torch, P, dev3.x, dev3.w1_slots, [dev3.w1_slots, dev3.w3_slots, dev3.w2_slots])
        result["ceilings"] = ceilings
        ach = ceilings["mfma_loop_with_lds_reads"]["tflops_mean"]
        result["roofline"].update({"achievable": ach, "frac_of_achievable": tf1 / ach,
                                   "achievable_kernel": "matrix-instruction loop with the GEMM's LDS fragment reads on this "
                                                        "layer's operand values, no global traffic, same flop per launch"})
    if not args.no_extras:
        result["load_experts"] = bench_load(torch, P, gen, c3, dev3, buf3)
    del inp3, dev3, buf3
    torch.cuda.empty_cache()

    # ---------------- decode ----------------
    if not args.no_decode:
        c4 = gen.C4
        dsteps, dwarm = max(args.steps, 30), max(args.warmup, 6)
        _, dwall_eager, dms, dcounts, ddev, dbuf = run_workload(torch, P, gen, c4, dsteps, dwarm, copies=3, graph=True)
        dwall = dms.pop("graph_wall_s")     # the step as a replayed HIP graph; the eager run gives the per-call times
        dmiss = miss_rate(torch, P, ddev, dbuf)
        del ddev, dbuf
        torch.cuda.empty_cache()
        el = c4.elem_bytes
        occupied = int((dcounts > 0).sum())
        bytes_pass1 = occupied * 2 * c4.d_model * c4.d_ff * el      # W1 and W3 of the non-empty slots
        bytes_pass2 = occupied * c4.d_model * c4.d_ff * el
        d_ms = dwall / dsteps * 1e3
        gbs1 = bytes_pass1 / (dms["ffn_pass1"] * 1e-3) / 1e9
        result["decode"] = {
            "value": c4.T * dsteps / dwall, "unit": "tokens/s", "ms_per_step": d_ms, "steps": dsteps,
            "launch": "one HIP graph per weight copy, replayed", "ms_per_step_eager": dwall_eager / dsteps * 1e3,
            "config": {"workload": "C4 Mixtral-8x7B-shaped decode step: 64 tokens, top-2, 6 of 8 experts resident, "
                                   "bf16; 3 rotating copies of the slot buffers", "rows_per_slot": [int(c) for c in dcounts]},
            "roofline": {"bound": "hbm", "kernel": "stream_gemm_bf16<SwiGLU> (FFN pass 1)", "achieved": gbs1,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs1 / PEAK_HBM_GBS,
                         "traffic": measured_traffic("stream_gemm_bf16<1"), "traffic_unit": "bytes per launch",
                         "algorithmic_bytes": bytes_pass1, "launch_ms": dms["ffn_pass1"]},
            "breakdown_ms": dms, "miss_rate": dmiss,
            "pass2_gbs": bytes_pass2 / (dms["ffn_pass2"] * 1e-3) / 1e9,
            "layer_hbm_frac": (bytes_pass1 + bytes_pass2) / (d_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        }
        if ceilings:
            ach = ceilings["read_stream"]["gbs"]
            result["decode"]["roofline"].update({"achievable": ach, "frac_of_achievable": gbs1 / ach,
                                                 "achievable_kernel": "plain read stream over 470 MB weight buffers"})
        log(f"decode: {d_ms:.3f} ms/step as a graph ({dwall_eager / dsteps * 1e3:.3f} eager), pass1 {gbs1:.0f} GB/s, breakdown {dms}")

    # ---------------- the other workloads (reported, not the headline) ----------------
    if not args.no_extras:
        result["c5"] = other_config(torch, P, gen, gen.C5, 20, 5, 1,
                                    "C5 fine-grained layer: T=8192 d_model=2048 d_ff=1408 E=64 top-6 SwiGLU, 24 of 64 "
                                    "resident (the most popular), Zipf(1.2) gate bias, bf16")
        result["c2"] = other_config(torch, P, gen, gen.C2, 40, 8, 4,
                                    "C2 Switch-style layer: T=1024 d_model=768 d_ff=3072 E=64 top-1 ReLU, 16 of 64 resident, "
                                    "Zipf(1.1) gate bias, bf16; 4 rotating copies of the slot buffers", graph=True)

    if args.more_shapes:
        result["x1"] = other_config(torch, P, gen, gen.X1, 10, 3, 1,
                                    "X1 Mixtral-8x22B-shaped prefill layer: T=4096 d_model=6144 d_ff=16384 E=8 top-2 "
                                    "SwiGLU, 4 of 8 resident, bf16")
        result["x2"] = other_config(torch, P, gen, gen.X2, 20, 5, 1,
                                    "X2 OpenMoE-shaped layer: T=2048 d_model=2048 d_ff=8192 E=32 top-2 SwiGLU, 16 of 32 "
                                    "resident, Zipf(1.1) gate bias, bf16")

        result["x3"] = other_config(torch, P, gen, gen.X3, 30, 5, 3,
                                    "X3 one short prompt at the Mixtral-8x7B shape: T=256 d_model=4096 d_ff=14336 E=8 "
                                    "top-2 SwiGLU, 6 of 8 resident, bf16; 3 rotating copies of the slot buffers")

        result["x4"] = other_config(torch, P, gen, gen.X4, 20, 5, 1,
                                    "X4 two prompts of 512 tokens at the Mixtral-8x7B shape, every expert resident: T=1024 "
                                    "d_model=4096 d_ff=14336 E=8 top-2 SwiGLU, bf16")

        result["x5"] = other_config(torch, P, gen, gen.X5, 30, 5, 2,
                                    "X5 decode step of 128 tokens at the Mixtral-8x7B shape, every expert resident: T=128 "
                                    "d_model=4096 d_ff=14336 E=8 top-2 SwiGLU, bf16; 2 rotating copies of the slot buffers")

    # ---------------- the oracle on the host cores, on a bounded sample of the prefill workload ------------
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        inp = gen.make_layer_inputs(c3)
        rng = np.random.default_rng(0)
        n = args.cpu_sample_tokens
        if n <= 0:
            t = time.perf_counter()
            oracle.layer_forward(inp, tokens=rng.choice(c3.T, 4, replace=False))
            probe = time.perf_counter() - t           # includes routing all T tokens
            t = time.perf_counter()
            oracle.layer_forward(inp, tokens=rng.choice(c3.T, 12, replace=False))
            per_tok = max((time.perf_counter() - t - probe) / 8, 1e-3)
            n = int(max(16, min(2048, 15.0 / per_tok)))
        toks = np.sort(rng.choice(c3.T, n, replace=False))
        t = time.perf_counter()
        oracle.layer_forward(inp, tokens=toks)
        cpu_s = time.perf_counter() - t
        model, physical = host_cpu()
        result["cpu_baseline"] = {
            "value": n / cpu_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of the {c3.T} prefill tokens through the fp64 oracle (routing and permutation of all "
                      f"tokens, FFN and combine of the sample), {cpu_s:.1f} s",
            "cpu_model": model, "physical_cores_of_the_machine": physical,
            "threads_note": "cores = OpenMP threads the oracle ran on (the share of the machine this process may use)"}
        log(f"cpu baseline: {n} tokens in {cpu_s:.1f}s on {oracle.num_threads()} threads")
        del inp
        # the small workloads whole, best of three (decode step and Switch-style layer)
        others = {}
        all_threads = oracle.num_threads()
        for key, cfg, threads in (("c4_decode", gen.C4, all_threads), ("c2_switch", gen.C2, all_threads),
                                  ("c2_switch_one_thread", gen.C2, 1), ("c1_tiny", gen.C1, all_threads),
                                  ("c1_tiny_one_thread", gen.C1, 1)):
            cin = gen.make_layer_inputs(cfg)
            oracle.set_num_threads(threads)
            ts = []
            for _ in range(3 if threads > 1 else 1):      # one thread takes seconds: a single run
                t = time.perf_counter()
                oracle.layer_forward(cin)
                ts.append(time.perf_counter() - t)
            others[key] = {"value": cfg.T / min(ts), "unit": "tokens/s", "threads": threads, "best_of": len(ts),
                           "seconds": sorted(ts), "sample": f"all {cfg.T} tokens"}
        oracle.set_num_threads(all_threads)
        result["cpu_baseline"]["other_workloads"] = others
        log(f"cpu baseline, small workloads whole: {others}")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
