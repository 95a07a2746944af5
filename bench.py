#!/usr/bin/env python3
"""Benchmark of the resident-expert MoE layer on one MI355X.

A step is one pass of the whole hot path (route -> permute -> expert FFN -> combine) over one
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
# HBM bytes per launch of the dominant kernels, from two hardware-counter runs of this command
# (FETCH_SIZE, then WRITE_SIZE; each scaled by what the same counter reads for a 1 GiB device copy:
# x2.00 and x1.00).  Counters cannot be read from inside the process, so the figures are carried here.
TRAFFIC_BYTES_PREFILL_PASS1 = (2040888.5 * 2.00 + 335429.8 * 1.00) * 1024   # 4.52 GB: operands re-read through L2
TRAFFIC_BYTES_DECODE_PASS1 = (701657.9 * 2.00 + 3665.8 * 1.00) * 1024       # 1.44 GB: 1.02x the weight bytes


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def timed_steps(torch, P, dev, buf, steps, warmup, weight_sets):
    """Runs warmup + steps layer forwards; the FFN is issued as its two passes with events between
    them so each grouped product's launch duration is measured inside the timed region."""
    d = buf.desc
    ws_n = buf.ffn_ws.numel()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]

    def step(i, events=None):
        w1, w3, w2 = weight_sets[i % len(weight_sets)]
        if events: events[0].record()
        P.emoe_route(d, dev.x, dev.w_gate, dev.gate_bias, dev.slot_of_expert, buf.topk_expert, buf.topk_weight)
        P.emoe_permute(d, dev.x, buf.topk_expert, dev.slot_of_expert, buf.slot_counts, buf.slot_offsets, buf.perm,
                       buf.inv_perm, buf.x_perm, buf.permute_ws, buf.permute_ws.numel())
        if events: events[1].record()
        P.emoe_expert_ffn_pass(d, 1, buf.x_perm, buf.slot_offsets, w1, w3, w2, buf.y_perm, buf.ffn_ws, ws_n)
        if events: events[2].record()
        P.emoe_expert_ffn_pass(d, 2, buf.x_perm, buf.slot_offsets, w1, w3, w2, buf.y_perm, buf.ffn_ws, ws_n)
        if events: events[3].record()
        P.emoe_combine(d, buf.y_perm, buf.inv_perm, buf.topk_weight, buf.out)
        if events: events[4].record()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i, ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    names = ["route_permute", "ffn_pass1", "ffn_pass2", "combine"]
    ms = {n: sum(e[j].elapsed_time(e[j + 1]) for e in ev) / steps for j, n in enumerate(names)}
    return wall, ms


def run_workload(torch, P, gen, cfg, steps, warmup, copies):
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
    wall, ms = timed_steps(torch, P, dev, buf, steps, warmup, sets)
    torch.cuda.synchronize()
    counts = buf.slot_counts.cpu().numpy()
    return inp, wall, ms, counts


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = size the sample for about 15 s")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device-to-device copy, so that a hardware-counter run of this "
                         "command also holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards by tokens with no "
              "exchange; see DESIGN.md). Run with --gpus 1.", file=sys.stderr)
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
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ---------------- prefill (headline) ----------------
    c3 = gen.C3
    inp3, wall, ms, counts = run_workload(torch, P, gen, c3, args.steps, args.warmup, copies=1)
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
                     "traffic": TRAFFIC_BYTES_PREFILL_PASS1, "traffic_unit": "bytes per launch",
                     "launch_ms": ms["ffn_pass1"]},
        "prefill_breakdown_ms": ms,
        "prefill_layer_mfma_frac": (flop_pass1 + flop_pass2) / (ms_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "prefill_pass2_tflops": flop_pass2 / (ms["ffn_pass2"] * 1e-3) / 1e12,
    }
    log(f"prefill: {ms_step:.3f} ms/step, {tokens_s:,.0f} tokens/s, pass1 {tf1:.0f} TFLOP/s, breakdown {ms}")

    # ---------------- decode ----------------
    if not args.no_decode:
        del inp3
        torch.cuda.empty_cache()
        c4 = gen.C4
        dsteps, dwarm = max(args.steps, 30), max(args.warmup, 6)
        _, dwall, dms, dcounts = run_workload(torch, P, gen, c4, dsteps, dwarm, copies=3)
        el = c4.elem_bytes
        occupied = int((dcounts > 0).sum())
        bytes_pass1 = occupied * 2 * c4.d_model * c4.d_ff * el      # W1 and W3 of the non-empty slots
        bytes_pass2 = occupied * c4.d_model * c4.d_ff * el
        d_ms = dwall / dsteps * 1e3
        gbs1 = bytes_pass1 / (dms["ffn_pass1"] * 1e-3) / 1e9
        result["decode"] = {
            "value": c4.T * dsteps / dwall, "unit": "tokens/s", "ms_per_step": d_ms, "steps": dsteps,
            "config": {"workload": "C4 Mixtral-8x7B-shaped decode step: 64 tokens, top-2, 6 of 8 experts resident, "
                                   "bf16; 3 rotating copies of the slot buffers", "rows_per_slot": [int(c) for c in dcounts]},
            "roofline": {"bound": "hbm", "kernel": "stream_gemm_bf16<SwiGLU> (FFN pass 1)", "achieved": gbs1,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs1 / PEAK_HBM_GBS,
                         "traffic": TRAFFIC_BYTES_DECODE_PASS1, "traffic_unit": "bytes per launch",
                         "algorithmic_bytes": bytes_pass1, "launch_ms": dms["ffn_pass1"]},
            "breakdown_ms": dms,
            "pass2_gbs": bytes_pass2 / (dms["ffn_pass2"] * 1e-3) / 1e9,
            "layer_hbm_frac": (bytes_pass1 + bytes_pass2) / (d_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        }
        log(f"decode: {d_ms:.3f} ms/step, pass1 {gbs1:.0f} GB/s, breakdown {dms}")

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
        result["cpu_baseline"] = {
            "value": n / cpu_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of the {c3.T} prefill tokens through the fp64 oracle (routing and permutation of all "
                      f"tokens, FFN and combine of the sample), {cpu_s:.1f} s"}
        log(f"cpu baseline: {n} tokens in {cpu_s:.1f}s on {oracle.num_threads()} threads")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
