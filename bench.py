#!/usr/bin/env python3
"""Benchmark of the SwiftPrune layer path on one MI355X.

Workload (default): a Llama-3-8B-shaped stack, 32 decoder blocks x 7 linear layers, bf16 random
weights, 128 x 2048 synthetic calibration tokens per layer input, 50 % unstructured (la = 0.5).
One step = pruning the whole stack in place: per linear layer, calibration statistics
(swiftprune_layer_stats) then score + EWMA selection with the apply fused in
(swiftprune_score_select | SP_APPLY_INPLACE).  Everything is resident in HBM before timing starts;
between steps the weights are restored from a pristine copy outside the timed region.

Prints ONE JSON line: weights-pruned GB/s, ms per step, HBM-roofline numbers of the dominant kernel
(measured with events on the launch stream inside the timed steps) and the CPU oracle's rate on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--blocks", type=int, default=32, help="decoder blocks in the stack (32 = the 8B shape)")
    ap.add_argument("--model", default="llama3-8b",
                    choices=["llama3-8b", "llama2-7b", "llama2-13b", "llama2-70b", "pythia-2.8b"],
                    help="block shape; llama2-70b has 80 blocks of 1.7 GB: pass --blocks <= 32 so that the "
                         "weights, their pristine copy and the activations fit in HBM (llama2-13b has 40 blocks)")
    ap.add_argument("--la", type=float, default=0.5, help="threshold multiplier of the unstructured mode")
    ap.add_argument("--mode", default="unstructured", choices=["unstructured", "2:4", "4:8"])
    ap.add_argument("--tokens", type=int, default=128 * 2048)
    ap.add_argument("--storage", default="bf16", choices=["bf16", "f16"],
                    help="16-bit storage type of W and X (same bytes either way)")
    ap.add_argument("--shared-stats", action="store_true",
                    help="compute statistics once per distinct layer input (q/k/v and gate/up share)")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2],
                    help="2 = statistics on one stream, selection+apply on another (double-buffered factors), "
                         "so a layer's selection overlaps the next layer's statistics")
    ap.add_argument("--layer-sweep", action="store_true",
                    help="also time every distinct layer shape of the block on its own (statistics + "
                         "selection/apply) and add the per-layer HBM fractions to the JSON line")
    ap.add_argument("--prime", type=int, default=4,
                    help="untimed passes at the end of set-up, before the W warm-up steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket the statistics launches with events")
    ap.add_argument("--event-stride", type=int, default=4,
                    help="bracket the statistics launches of every N-th decoder block with events (each "
                         "pair of event records costs a few microseconds of stream time; all blocks "
                         "have the same shapes, so every N-th block samples the same launch mix)")
    return ap.parse_args()


# which activation feeds which layer of a block
INPUT_OF = {"q": "attn_in", "k": "attn_in", "v": "attn_in", "o": "attn_out",
            "gate": "mlp_in", "up": "mlp_in", "down": "mlp_mid",
            "qkv": "attn_in", "dense": "attn_out", "h_to_4h": "mlp_in", "4h_to_h": "mlp_mid"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_16376_amd import binding as sp, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    sp.load_library()

    block = synth.MODEL_BLOCKS[args.model][0]
    T = args.tokens
    nm = None if args.mode == "unstructured" else tuple(int(x) for x in args.mode.split(":"))
    la = args.la

    # ---- resident data: activations per distinct layer input, weights per (block, layer)
    t_setup = time.time()
    widths = {INPUT_OF[name]: n for name, _, n in block}
    X = {key: synth.device_activations(T, n, seed=1000 + i, device=dev, dtype=args.storage)
         for i, (key, n) in enumerate(sorted(widths.items()))}
    weights, pristine = [], []
    for bi in range(args.blocks):
        for li, (name, out, n) in enumerate(block):
            W = synth.device_weights(out, n, seed=10_000 + 16 * bi + li, device=dev, dtype=args.storage)
            pristine.append(W)
            weights.append(W.clone())
    layers = [(name, out, n) for _ in range(args.blocks) for (name, out, n) in block]
    bufs = {}
    for name, out, n in block:
        if (out, n) not in bufs:
            bufs[(out, n)] = sp.LayerBuffers(out, n, T, dev)
    # one plain copy of known size for calibrating the HBM byte counters of a profiler run: the apply
    # kernel with an all-ones keep mask reads and rewrites an 8192 x 8192 bf16 matrix (128 MiB each way,
    # plus 8 MiB of mask) with the same 16-byte non-temporal loads as the timed kernels
    cal_W = torch.zeros((8192, 8192), dtype=torch.bfloat16, device=dev)
    cal_mask = torch.full((8192, 256), -1, dtype=torch.int32, device=dev)
    sp.swiftprune_apply(cal_W, cal_mask)
    torch.cuda.synchronize()
    del cal_W, cal_mask
    setup_s = time.time() - t_setup

    w_bytes = sum(out * n * 2 for _, out, n in layers)
    n_weights = sum(out * n for _, out, n in layers)
    if args.shared_stats:
        stats_bytes = args.blocks * sum(T * n * 2 for n in widths.values())
    else:
        stats_bytes = sum(T * n * 2 for _, _, n in layers)
    # select + apply fused: W read, W written, mask written, factor read
    select_bytes = sum(out * n * 2 * 2 + out * n // 8 + n * 4 for _, out, n in layers)
    algo_bytes = stats_bytes + select_bytes

    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream(device=dev) if args.streams == 2 else None
    ev_pairs = []       # (start, stop, bytes) around statistics launches of timed steps
    # with two streams every layer shape has two sets of (xsq, S, hr, workspace, mask) used alternately
    bufs2 = {k: sp.LayerBuffers(k[0], k[1], T, dev) for k in bufs} if side is not None else None

    def step(record):
        idx = 0
        use = {}            # (out, n) -> parity of the buffer set to use next
        sel_done = {}       # buffer set id -> event recorded after the selection that last read it
        for bi in range(args.blocks):
            done_inputs = set()
            for name, out, n in block:
                W = weights[idx]
                idx += 1
                par = use.get((out, n), 0)
                b = bufs[(out, n)] if (side is None or par == 0) else bufs2[(out, n)]
                if side is not None:
                    use[(out, n)] = par ^ 1
                    if id(b) in sel_done:              # statistics may not overwrite hr while it is read
                        stream.wait_event(sel_done[id(b)])
                key = INPUT_OF[name]
                if not (args.shared_stats and key in done_inputs):
                    timed = record and bi % max(1, args.event_stride) == 0
                    if timed:
                        e0 = torch.cuda.Event(enable_timing=True)
                        e1 = torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                    sp.swiftprune_layer_stats(X[key], b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream)
                    if timed:
                        e1.record(stream)
                        ev_pairs.append((e0, e1, T * n * 2))
                    done_inputs.add(key)
                    if args.shared_stats:
                        # keep the factor of this input for the layers that share it
                        with torch.cuda.stream(stream):
                            shared_hr[key].copy_(b.hr)
                hr = shared_hr[key] if args.shared_stats else b.hr
                sel_stream = stream
                if side is not None:
                    ready = torch.cuda.Event()
                    ready.record(stream)
                    side.wait_event(ready)
                    sel_stream = side
                if nm is None:
                    sp.swiftprune_score_select(W, hr, b.keep_mask, la=la, row_pruned=b.row_pruned,
                                               flags=sp.SP_APPLY_INPLACE, stream=sel_stream)
                else:
                    sp.swiftprune_nm_select(W, hr, nm[0], nm[1], b.keep_mask, flags=sp.SP_APPLY_INPLACE,
                                            stream=sel_stream)
                if side is not None:
                    done = torch.cuda.Event()
                    done.record(side)
                    sel_done[id(b)] = done
        if side is not None:
            stream.wait_stream(side)                   # the step ends when both streams have drained

    shared_hr = {key: torch.empty(n, dtype=torch.float32, device=dev) for key, n in widths.items()}

    def restore():
        for W, P in zip(weights, pristine):
            W.copy_(P)

    # Set-up ends with a few untimed passes: the first three or four passes of a process run 1-8 % slower
    # (clocks, address translation), more so in a process that starts right after another one has released
    # tens of GB.  They are not part of the W warm-up steps so that a small W does not time them.
    for _ in range(args.prime):
        restore()
        step(False)
    torch.cuda.synchronize()

    # The host must not pause while it feeds the GPU: a full collection of Python's garbage collector
    # (tens of ms with torch loaded) that falls right after a synchronisation shows up as GPU idle time
    # inside one step.  Collect now, then keep the collector off until the timed steps are done.
    import gc
    gc.collect()
    gc.disable()

    for _ in range(args.warmup):          # identical to a timed step, instrumentation included
        restore()
        torch.cuda.synchronize()
        step(not args.no_kernel_events)
    torch.cuda.synchronize()
    ev_pairs.clear()

    step_events = []
    t_wall0 = time.time()
    for _ in range(args.steps):
        restore()
        torch.cuda.synchronize()
        s0 = torch.cuda.Event(enable_timing=True)
        s1 = torch.cuda.Event(enable_timing=True)
        s0.record(stream)
        step(not args.no_kernel_events)
        s1.record(stream)
        step_events.append((s0, s1))
    torch.cuda.synchronize()
    wall_s = time.time() - t_wall0
    gc.enable()
    step_ms = [a.elapsed_time(b) for a, b in step_events]
    ms_per_step = sum(step_ms) / len(step_ms)

    # achieved sparsity of the last step (from the per-row counts of the last layer of each shape)
    pruned_frac = None
    if nm is None:
        b = bufs[(block[-1][1], block[-1][2])]
        pruned_frac = float(b.row_pruned.sum().item()) / (block[-1][1] * block[-1][2])

    roofline = {"bound": "hbm",
                "kernel": "stats_partial_kernel (events bracket swiftprune_layer_stats = it + the 4 us combine kernel)",
                "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                # the committed counters were taken on the default workload (bf16 instantiation)
                "traffic": committed_traffic() if (args.storage == "bf16" and args.model == "llama3-8b"
                                                   and T == 128 * 2048 and not args.shared_stats) else None}
    if ev_pairs:
        tot_ms = sum(a.elapsed_time(b) for a, b, _ in ev_pairs)
        tot_bytes = sum(nb for _, _, nb in ev_pairs)
        ach = tot_bytes / (tot_ms * 1e-3) / 1e9
        roofline.update(achieved=round(ach, 1), frac=round(ach / HBM_PEAK_GBS, 4),
                        launches=len(ev_pairs), event_stride_blocks=max(1, args.event_stride), avg_launch_us=round(tot_ms * 1e3 / len(ev_pairs), 2),
                        bytes_per_launch_avg=int(tot_bytes / len(ev_pairs)))

    value = w_bytes / (ms_per_step * 1e-3) / 1e9
    result = {
        "metric": "GB/s of weights pruned (% of HBM peak); seconds to prune 8B-shaped model",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.model}-shaped stack, {args.blocks} blocks x {len(block)} linear layers, {args.storage} W, "
                               f"{T} calibration tokens per layer, "
                               + (f"unstructured (la={la:g})" if nm is None else f"{args.mode} structured"),
                   "storage": args.storage, "tokens": T, "blocks": args.blocks, "mode": args.mode,
                   "stats_calls_per_block": len(widths) if args.shared_stats else len(block), "streams": args.streams,
                   "weights": n_weights},
        "seconds_per_model": round(ms_per_step * 1e-3, 5),
        "step_ms_min_max": [round(min(step_ms), 3), round(max(step_ms), 3)],
        "step_ms": [round(x, 2) for x in step_ms],
        "algorithmic_bytes_per_step": int(algo_bytes),
        "hbm_frac_whole_step": round(algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "achieved_sparsity_last_layer": pruned_frac,
        "setup_s": round(setup_s, 1), "setup_prime_passes": args.prime,
        "timed_wall_s_incl_restore": round(wall_s, 3),
        "roofline": roofline,
        "paper_context": "LLaMA3.1-8B pruned in 9.49 s (50%) / 9.28 s (2:4) on 8x RTX 4090 (Table 3 of the paper); "
                         "not the same machine, weights or calibration set",
    }

    if args.layer_sweep:
        result["layer_sweep"] = layer_sweep(sp, torch, block, X, weights, pristine, bufs, T, nm, la, stream)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(block, X, pristine, T, nm, la)

    print(json.dumps(result))


def layer_sweep(sp, torch, block, X, weights, pristine, bufs, T, nm, la, stream, reps=20):
    """Each distinct layer shape of the block on its own: statistics, then selection + apply, timed with
    events over `reps` layers drawn from different blocks of the stack (different weight buffers, so no
    launch re-reads a cached matrix); algorithmic bytes / time / 8 TB/s per layer."""
    n_layers = len(block)
    n_blocks = len(weights) // n_layers
    out_rows = []
    seen = set()
    for li, (name, out, n) in enumerate(block):
        if (out, n) in seen:
            continue
        seen.add((out, n))
        b = bufs[(out, n)]
        idxs = [((r % n_blocks) * n_layers + li) for r in range(reps)]
        for i in set(idxs):
            weights[i].copy_(pristine[i])
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * reps)]
        for r, i in enumerate(idxs):
            ev[3 * r].record(stream)
            sp.swiftprune_layer_stats(X[INPUT_OF[name]], b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream)
            ev[3 * r + 1].record(stream)
            if nm is None:
                sp.swiftprune_score_select(weights[i], b.hr, b.keep_mask, la=la, row_pruned=b.row_pruned,
                                           flags=sp.SP_APPLY_INPLACE, stream=stream)
            else:
                sp.swiftprune_nm_select(weights[i], b.hr, nm[0], nm[1], b.keep_mask,
                                        flags=sp.SP_APPLY_INPLACE, stream=stream)
            ev[3 * r + 2].record(stream)
        torch.cuda.synchronize()
        t_stats = sum(ev[3 * r].elapsed_time(ev[3 * r + 1]) for r in range(reps)) / reps * 1e3
        t_sel = sum(ev[3 * r + 1].elapsed_time(ev[3 * r + 2]) for r in range(reps)) / reps * 1e3
        stats_b = T * n * 2
        sel_b = out * n * 4 + out * n // 8 + n * 4
        out_rows.append({"layer": f"{name} {out}x{n}", "stats_us": round(t_stats, 1), "select_apply_us": round(t_sel, 1),
                         "stats_hbm_frac": round(stats_b / t_stats / 1e6 / HBM_PEAK_GBS * 1e3, 4),
                         "select_apply_hbm_frac": round(sel_b / t_sel / 1e6 / HBM_PEAK_GBS * 1e3, 4),
                         "layer_hbm_frac": round((stats_b + sel_b) / (t_stats + t_sel) / 1e6 / HBM_PEAK_GBS * 1e3, 4)})
    return out_rows


def stats_kernel_fingerprint():
    """sha256 of the statistics kernel's source with comments and white space removed, so that only a
    change of the code (not of its commentary) invalidates the committed counters."""
    import hashlib
    import re
    text = open(os.path.join(ROOT, "paper_2501_16376_amd", "csrc", "stats.hip")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    text = re.sub(r"\s+", "", text)
    return hashlib.sha256(text.encode()).hexdigest()


def committed_traffic():
    """HBM bytes per launch of the statistics kernel from the committed counter runs
    (profiles/stats_partial_kernel_llama3_8b_pmc.txt); None when the kernel source has changed since."""
    path = os.path.join(ROOT, "profiles", "stats_partial_kernel_llama3_8b_pmc.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    if kv.get("kernel_source_sha256") != stats_kernel_fingerprint():
        return None
    try:
        return int(float(kv["traffic_bytes_per_launch_avg"]))
    except (KeyError, ValueError):
        return None


def cpu_baseline(block, X, pristine, T, nm, la, sample_blocks=2):
    """The CPU oracle, as it stands, single-threaded, on a bounded sample of the workload: the first
    `sample_blocks` decoder blocks of the stack (7 layers each, at the full calibration token count)."""
    import oracle
    from paper_2501_16376_amd import synth

    oracle.lib()
    t_stats = 0.0
    t_sel = 0.0
    w_bytes = 0
    chunk = 32768                      # tokens per host copy: bounds the host memory to ~1 GB
    sample_blocks = max(1, min(sample_blocks, len(pristine) // len(block)))
    for li_all in range(sample_blocks * len(block)):
        name, out, n = block[li_all % len(block)]
        Xd = X[INPUT_OF[name]]
        Wh = synth.torch_to_host_bits(pristine[li_all])
        acc = None
        for t0 in range(0, T, chunk):
            Xh = synth.torch_to_host_bits(Xd[t0:t0 + chunk])
            t_a = time.perf_counter()
            acc = oracle.stats_accumulate(Xh, acc)
            t_stats += time.perf_counter() - t_a
        t0_ = time.perf_counter()
        xsq, S = oracle.stats_finalize(acc)
        hr = oracle.channel_factor_f32(xsq, S)
        t1 = time.perf_counter()
        if nm is None:
            mask, _, _ = oracle.ewma_select(Wh, hr, 0.125, 0.125, la)
        else:
            mask, _ = oracle.nm_select(Wh, hr, nm[0], nm[1])
        oracle.apply(Wh, mask)
        t2 = time.perf_counter()
        t_stats += t1 - t0_
        t_sel += t2 - t1
        w_bytes += out * n * 2
    total = t_stats + t_sel
    return {"value": round(w_bytes / total / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample_blocks} decoder blocks of the stack ({sample_blocks * len(block)} layers, "
                      f"{w_bytes / 1e9:.3f} GB of weights) at the full {T} calibration tokens per layer; "
                      f"host copies are not timed",
            "cpu_seconds": round(total, 2), "cpu_seconds_statistics": round(t_stats, 2),
            "cpu_seconds_select_apply": round(t_sel, 2)}


if __name__ == "__main__":
    main()
