#!/usr/bin/env python3
"""Benchmark of the SwiftPrune layer path on one MI355X.

Workload (default): a Llama-3-8B-shaped stack, 32 decoder blocks x 7 linear layers, bf16 random
weights, 128 x 2048 synthetic calibration tokens per layer input, 50 % unstructured (la = 0.5).
One step = pruning the whole stack in place: per linear layer, calibration statistics
(swiftprune_layer_stats) then score + EWMA selection with the apply fused in
(swiftprune_score_select | SP_APPLY_INPLACE).  Everything is resident in HBM before timing starts;
between steps the weights are restored from a pristine copy outside the timed region.

Prints ONE JSON line: weights-pruned GB/s, ms per step, HBM-roofline numbers of the dominant kernel
(measured with events on the launch stream inside the timed steps), the CPU oracle's rate on a
bounded sample of the same workload, and a few bounded side measurements (`shared_stats`,
`secondary`): the same stack with one statistics pass per distinct layer input and grouped
selection, the same stack in 2:4, and a sample of Llama-2-70B-shaped blocks at three unstructured
ratios and 2:4.
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
PMC_SUMMARY = os.path.join("profiles", "stats_partial_kernel_llama3_8b_pmc.txt")


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
                    help="make the shared-statistics variant the main measurement: statistics once per distinct "
                         "layer input and one grouped selection launch for the matrices that share it")
    ap.add_argument("--layer-sweep", action="store_true",
                    help="also time every distinct layer shape of the block on its own (statistics + "
                         "selection/apply) and add the per-layer HBM fractions to the JSON line")
    ap.add_argument("--tuning-sweep", action="store_true",
                    help="instead of the benchmark: time the kernels of the 8B layer shapes under the library's "
                         "launch-shape overrides (SWIFTPRUNE_STATS_PLAN, SWIFTPRUNE_SELECT_TEAM, "
                         "SWIFTPRUNE_BAND_GROUPS) and print one line per setting")
    ap.add_argument("--prime", type=int, default=4,
                    help="untimed passes at the end of set-up, before the W warm-up steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the side measurements (shared statistics, 2:4, the 70B-shaped sample)")
    ap.add_argument("--secondary-steps", type=int, default=3)
    ap.add_argument("--sample-blocks-70b", type=int, default=8)
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


class Stack:
    """A stack of decoder blocks resident in HBM: activations per distinct layer input (reused by every
    block; each is far larger than the 256 MB Infinity Cache), fresh weights per (block, layer), their
    pristine copy, and the per-shape buffers of the library calls."""

    def __init__(self, sp, synth, torch, dev, model, blocks, tokens, storage):
        self.sp, self.torch, self.dev = sp, torch, dev
        self.block = synth.MODEL_BLOCKS[model][0]
        self.model, self.blocks, self.T, self.storage = model, blocks, tokens, storage
        self.widths = {INPUT_OF[name]: n for name, _, n in self.block}
        self.X = {key: synth.device_activations(tokens, n, seed=1000 + i, device=dev, dtype=storage)
                  for i, (key, n) in enumerate(sorted(self.widths.items()))}
        self.weights, self.pristine = [], []
        for bi in range(blocks):
            for li, (name, out, n) in enumerate(self.block):
                W = synth.device_weights(out, n, seed=10_000 + 16 * bi + li, device=dev, dtype=storage)
                self.pristine.append(W)
                self.weights.append(W.clone())
        # one buffer set per layer of the block (masks and counts are per matrix; a grouped launch writes
        # the masks of all its matrices at once)
        self.bufs = [sp.LayerBuffers(out, n, tokens, dev) for _, out, n in self.block]
        # layers of a block grouped by the input they share, in block order
        self.groups = []
        for li, (name, _, _) in enumerate(self.block):
            key = INPUT_OF[name]
            if self.groups and self.groups[-1][0] == key:
                self.groups[-1][1].append(li)
            else:
                self.groups.append((key, [li]))
        self.layers = [(name, out, n) for _ in range(blocks) for (name, out, n) in self.block]
        self.w_bytes = sum(out * n * 2 for _, out, n in self.layers)
        self.n_weights = sum(out * n for _, out, n in self.layers)
        # select + apply fused: W read, W written, mask written, factor read
        self.select_bytes = sum(out * n * 2 * 2 + out * n // 8 + n * 4 for _, out, n in self.layers)
        self.stats_bytes_per_layer = sum(tokens * n * 2 for _, _, n in self.layers)
        self.stats_bytes_shared = blocks * sum(tokens * n * 2 for n in self.widths.values())

    def algo_bytes(self, shared):
        return (self.stats_bytes_shared if shared else self.stats_bytes_per_layer) + self.select_bytes

    def restore(self):
        for W, P in zip(self.weights, self.pristine):
            W.copy_(P)

    def step(self, stream, nm=None, la=0.5, shared=False, ev_pairs=None, event_stride=4):
        """One pass over the whole stack.  shared=False: statistics + selection per linear layer.
        shared=True: statistics once per distinct input, one grouped selection for the layers sharing it."""
        sp, torch = self.sp, self.torch
        nl = len(self.block)
        for bi in range(self.blocks):
            timed = ev_pairs is not None and bi % max(1, event_stride) == 0
            for key, lis in self.groups:
                units = [lis] if shared else [[li] for li in lis]
                for unit in units:
                    b0 = self.bufs[unit[0]]
                    n = self.block[unit[0]][2]
                    if timed:
                        e0 = torch.cuda.Event(enable_timing=True)
                        e1 = torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                    sp.swiftprune_layer_stats(self.X[key], b0.xsq, b0.S, b0.hr, workspace=b0.workspace, stream=stream)
                    if timed:
                        e1.record(stream)
                        ev_pairs.append((e0, e1, self.T * n * 2))
                    Ws = [self.weights[bi * nl + li] for li in unit]
                    if len(unit) == 1:
                        b = self.bufs[unit[0]]
                        if nm is None:
                            sp.swiftprune_score_select(Ws[0], b0.hr, b.keep_mask, la=la, row_pruned=b.row_pruned,
                                                       flags=sp.SP_APPLY_INPLACE, stream=stream)
                        else:
                            sp.swiftprune_nm_select(Ws[0], b0.hr, nm[0], nm[1], b.keep_mask,
                                                    flags=sp.SP_APPLY_INPLACE, stream=stream)
                    else:
                        masks = [self.bufs[li].keep_mask for li in unit]
                        if nm is None:
                            sp.swiftprune_score_select_group(Ws, b0.hr, masks, la=la,
                                                             row_pruned=[self.bufs[li].row_pruned for li in unit],
                                                             flags=sp.SP_APPLY_INPLACE, stream=stream)
                        else:
                            sp.swiftprune_nm_select_group(Ws, b0.hr, nm[0], nm[1], masks,
                                                          flags=sp.SP_APPLY_INPLACE, stream=stream)

    def time_steps(self, stream, steps, warmup, **kw):
        """Per-step HIP-event times (ms) of `steps` passes after `warmup` identical ones; weights restored
        from the pristine copy before every pass, outside the event bracket."""
        torch = self.torch
        ev_pairs = kw.get("ev_pairs")
        for _ in range(warmup):
            self.restore()
            torch.cuda.synchronize()
            self.step(stream, **kw)
        torch.cuda.synchronize()
        if ev_pairs is not None:
            ev_pairs.clear()
        brackets = []
        t0 = time.time()
        for _ in range(steps):
            self.restore()
            torch.cuda.synchronize()
            s0 = torch.cuda.Event(enable_timing=True)
            s1 = torch.cuda.Event(enable_timing=True)
            s0.record(stream)
            self.step(stream, **kw)
            s1.record(stream)
            brackets.append((s0, s1))
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in brackets], time.time() - t0

    def pruned_fraction(self):
        """Pruned fraction over the last block of the stack, from the per-row counts its calls left."""
        tot = sum(int(self.bufs[li].row_pruned.sum().item()) for li in range(len(self.block)))
        return tot / sum(out * n for _, out, n in self.block)

    def release(self):
        self.X.clear()
        self.weights.clear()
        self.pristine.clear()
        self.bufs.clear()
        self.torch.cuda.empty_cache()


def side_entry(stack, stream, steps, label, nm=None, la=0.5, shared=False, extrapolate_to=None):
    ms, _ = stack.time_steps(stream, steps, 1, nm=nm, la=la, shared=shared)
    mean = sum(ms) / len(ms)
    algo = stack.algo_bytes(shared)
    e = {"workload": label, "steps": steps, "ms_per_step": round(mean, 3),
         "weights_GBps": round(stack.w_bytes / mean / 1e6, 2),
         "algorithmic_bytes": int(algo), "hbm_frac": round(algo / mean / 1e6 / HBM_PEAK_GBS, 4)}
    if nm is None:
        e["la"] = round(float(la), 4)
        e["achieved_sparsity_last_block"] = round(stack.pruned_fraction(), 4)
    if extrapolate_to is not None:
        e["seconds_per_model_extrapolated"] = round(mean * 1e-3 * extrapolate_to / stack.blocks, 4)
        e["extrapolated_from_blocks"] = stack.blocks
        e["model_blocks"] = extrapolate_to
    return e


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

    T = args.tokens
    nm = None if args.mode == "unstructured" else tuple(int(x) for x in args.mode.split(":"))
    la = args.la
    if args.tuning_sweep:
        tuning_sweep(sp, synth, torch, dev, T, args.storage)
        return

    t_setup = time.time()
    stack = Stack(sp, synth, torch, dev, args.model, args.blocks, T, args.storage)
    block = stack.block
    # one plain copy of known size for calibrating the HBM byte counters of a profiler run: the apply
    # kernel with an all-ones keep mask reads and rewrites an 8192 x 8192 bf16 matrix (128 MiB each way,
    # plus 8 MiB of mask) with the same 16-byte non-temporal loads as the timed kernels
    cal_W = torch.zeros((8192, 8192), dtype=torch.bfloat16, device=dev)
    cal_mask = torch.full((8192, 256), -1, dtype=torch.int32, device=dev)
    sp.swiftprune_apply(cal_W, cal_mask)
    torch.cuda.synchronize()
    del cal_W, cal_mask
    setup_s = time.time() - t_setup

    stream = torch.cuda.current_stream()
    shared = bool(args.shared_stats)
    algo_bytes = stack.algo_bytes(shared)

    # Set-up ends with a few untimed passes: the first three or four passes of a process run 1-8 % slower
    # (clocks, address translation), more so in a process that starts right after another one has released
    # tens of GB.  They are not part of the W warm-up steps so that a small W does not time them.
    for _ in range(args.prime):
        stack.restore()
        stack.step(stream, nm=nm, la=la, shared=shared)
    torch.cuda.synchronize()

    # The host must not pause while it feeds the GPU: a full collection of Python's garbage collector
    # (tens of ms with torch loaded) that falls right after a synchronisation shows up as GPU idle time
    # inside one step.  Collect now, then keep the collector off until the timed steps are done.
    import gc
    gc.collect()
    gc.disable()

    ev_pairs = None if args.no_kernel_events else []   # (start, stop, bytes) around statistics launches
    step_ms, wall_s = stack.time_steps(stream, args.steps, args.warmup, nm=nm, la=la, shared=shared,
                                       ev_pairs=ev_pairs, event_stride=args.event_stride)
    ms_per_step = sum(step_ms) / len(step_ms)
    pruned_frac = stack.pruned_fraction() if nm is None else None

    default_workload = (args.storage == "bf16" and args.model == "llama3-8b" and T == 128 * 2048)
    traffic = committed_traffic() if default_workload else None
    roofline = {"bound": "hbm",
                "kernel": "stats_partial_kernel (events bracket swiftprune_layer_stats = it + the 4 us combine kernel)",
                "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                # HBM counters cannot be read from inside this process: the figure comes from the committed
                # rocprofv3 --pmc summary of this command and is dropped when the kernel source has changed
                "traffic": traffic, "traffic_source": PMC_SUMMARY if traffic is not None else None}
    if ev_pairs:
        tot_ms = sum(a.elapsed_time(b) for a, b, _ in ev_pairs)
        tot_bytes = sum(nb for _, _, nb in ev_pairs)
        ach = tot_bytes / (tot_ms * 1e-3) / 1e9
        roofline.update(achieved=round(ach, 1), frac=round(ach / HBM_PEAK_GBS, 4),
                        launches=len(ev_pairs), event_stride_blocks=max(1, args.event_stride),
                        avg_launch_us=round(tot_ms * 1e3 / len(ev_pairs), 2),
                        bytes_per_launch_avg=int(tot_bytes / len(ev_pairs)))

    value = stack.w_bytes / (ms_per_step * 1e-3) / 1e9
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
                   "stats_calls_per_block": len(stack.groups) if shared else len(block),
                   "weights": stack.n_weights},
        "seconds_per_model": round(ms_per_step * 1e-3, 5),
        "step_ms_min_max": [round(min(step_ms), 3), round(max(step_ms), 3)],
        "step_ms": [round(x, 2) for x in step_ms],
        "algorithmic_bytes_per_step": int(algo_bytes),
        "hbm_frac_whole_step": round(algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "achieved_sparsity_last_block": pruned_frac,
        "setup_s": round(setup_s, 1), "setup_prime_passes": args.prime,
        "timed_wall_s_incl_restore": round(wall_s, 3),
        "roofline": roofline,
        "paper_context": "LLaMA3.1-8B pruned in 9.49 s (50%) / 9.28 s (2:4) on 8x RTX 4090 (Table 3 of the paper); "
                         "not the same machine, weights or calibration set",
    }

    if args.layer_sweep:
        result["layer_sweep"] = layer_sweep(sp, torch, stack, nm, la, stream)

    if not args.no_secondary:
        k = max(1, args.secondary_steps)
        name = f"{args.model}-shaped stack, {args.blocks} blocks"
        if not shared:
            e = side_entry(stack, stream, k, f"{name}, shared statistics ({len(stack.groups)} statistics passes and grouped "
                           f"selection launches per block instead of {len(block)}), "
                           + ("unstructured" if nm is None else args.mode), nm=nm, la=la, shared=True)
            result["shared_stats"] = e
        secondary = []
        if nm is None:
            secondary.append(side_entry(stack, stream, k, f"{name}, 2:4 structured", nm=(2, 4)))
        else:
            secondary.append(side_entry(stack, stream, k, f"{name}, unstructured (la={la:g})", la=la))
        result["secondary"] = secondary
        result["chunked_stats"] = chunked_stats(sp, torch, stack, stream)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(block, stack.X, stack.pristine, T, nm, la, model_blocks=args.blocks)

    if not args.no_secondary and args.model != "llama2-70b":
        # Llama-2-70B-shaped blocks streamed block by block: only a sample of blocks is resident and timed,
        # the 80-block figure is that sample scaled up (every block has the same shapes)
        stack.release()
        del stack
        gc.collect()
        result["secondary"] += sample_70b(sp, synth, torch, dev, stream, T, args.storage,
                                          args.sample_blocks_70b, max(1, args.secondary_steps))
    gc.enable()

    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


def tuning_sweep(sp, synth, torch, dev, T, storage, reps=6):
    """The evidence behind the built-in launch shapes: every kernel of the path on the 8B layer shapes under
    the library's environment overrides, HIP events over `reps` launches on rotating buffers."""
    stream = torch.cuda.current_stream()

    def timed(fn, n):
        fn(0)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record(stream)
        for i in range(n):
            fn(i)
        ev[1].record(stream)
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / n * 1e3            # microseconds per launch

    def say(kind, shape, setting, us, nbytes):
        print(json.dumps({"kernel": kind, "shape": shape, "setting": setting, "us": round(us, 1),
                          "TBps": round(nbytes / us / 1e6, 3), "hbm_frac": round(nbytes / us / 1e6 / 8.0, 4)}), flush=True)

    for k in ("SWIFTPRUNE_STATS_PLAN", "SWIFTPRUNE_SELECT_TEAM", "SWIFTPRUNE_BAND_GROUPS"):
        os.environ.pop(k, None)
    # ---- statistics kernel: rows in flight x workgroups x load kind
    for n in (4096, 14336):
        X = synth.device_activations(T, n, seed=1, device=dev, dtype=storage)
        settings = [None] + [f"{r},{g}{p}" for p in ("", ",plain") for r in (4, 8, 16) for g in (192, 224, 256, 384, 512, 1024)
                             if not (p and g not in (224, 256, 384))] + [None]
        warm = sp.LayerBuffers(8, n, T, dev)
        for _ in range(40):                                   # clocks and address translation settle first
            sp.swiftprune_layer_stats(X, warm.xsq, warm.S, warm.hr, workspace=warm.workspace, stream=stream)
        torch.cuda.synchronize()
        for st in settings:
            if st is None:
                os.environ.pop("SWIFTPRUNE_STATS_PLAN", None)
            else:
                os.environ["SWIFTPRUNE_STATS_PLAN"] = st
            b = sp.LayerBuffers(8, n, T, dev)
            us = timed(lambda i: sp.swiftprune_layer_stats(X, b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream), reps)
            say("layer_stats", f"{T}x{n}", st or "built-in", us, T * n * 2)
        os.environ.pop("SWIFTPRUNE_STATS_PLAN", None)
        del X
        torch.cuda.empty_cache()
    # ---- per-weight kernels: rotating matrices so that no launch re-reads a cached one
    for out, n in ((1024, 4096), (4096, 4096), (14336, 4096), (4096, 14336)):
        nbuf = max(2, min(24, (3 << 30) // (out * n * 2)))
        Ws = [synth.device_weights(out, n, seed=50 + i, device=dev, dtype=storage) for i in range(nbuf)]
        b = sp.LayerBuffers(out, n, 8, dev)
        hr = torch.full((n,), 0.5, dtype=torch.float32, device=dev)
        algo = out * n * 4.125
        for team in (None, "1", "2", "4", "1,direct", "2,direct", "4,direct"):
            if team is None:
                os.environ.pop("SWIFTPRUNE_SELECT_TEAM", None)
            else:
                os.environ["SWIFTPRUNE_SELECT_TEAM"] = team
            us = timed(lambda i: sp.swiftprune_score_select(Ws[i % nbuf], hr, b.keep_mask, la=0.5, row_pruned=b.row_pruned,
                                                            flags=sp.SP_APPLY_INPLACE, stream=stream), 2 * nbuf)
            say("score_select+apply", f"{out}x{n}", f"team {team or 'built-in'}", us, algo)
        os.environ.pop("SWIFTPRUNE_SELECT_TEAM", None)
        for g in (None, 256, 384, 512, 768, 1024, 2048):
            if g is None:
                os.environ.pop("SWIFTPRUNE_BAND_GROUPS", None)
            else:
                os.environ["SWIFTPRUNE_BAND_GROUPS"] = f"{g},{g}"
            us = timed(lambda i: sp.swiftprune_nm_select(Ws[i % nbuf], hr, 2, 4, b.keep_mask, flags=sp.SP_APPLY_INPLACE,
                                                         stream=stream), 2 * nbuf)
            say("nm_select 2:4+apply", f"{out}x{n}", f"groups {g or 'built-in'}", us, algo)
            us = timed(lambda i: sp.swiftprune_apply(Ws[i % nbuf], b.keep_mask, stream=stream), 2 * nbuf)
            say("apply", f"{out}x{n}", f"groups {g or 'built-in'}", us, algo)
        os.environ.pop("SWIFTPRUNE_BAND_GROUPS", None)
        del Ws
        torch.cuda.empty_cache()
    # ---- time against the number of rows at one width: the slope is the streaming rate of the kernel, the
    # intercept what a launch costs before and after it streams (start-up, per-wavefront set-up, drain)
    n = 4096
    arena = synth.device_weights(3 * 24576, n, seed=77, device=dev, dtype=storage)     # 604 MB, three windows of the largest
    hr = torch.full((n,), 0.5, dtype=torch.float32, device=dev)
    b = sp.LayerBuffers(24576, n, 8, dev)
    calls = {
        "score_select+apply": lambda W: sp.swiftprune_score_select(W, hr, b.keep_mask, la=0.5, row_pruned=b.row_pruned,
                                                                   flags=sp.SP_APPLY_INPLACE, stream=stream),
        "nm_select 2:4+apply": lambda W: sp.swiftprune_nm_select(W, hr, 2, 4, b.keep_mask, flags=sp.SP_APPLY_INPLACE,
                                                                 stream=stream),
        "apply": lambda W: sp.swiftprune_apply(W, b.keep_mask, stream=stream),
    }
    for kind, call in calls.items():
        pts = []
        for out in (4096, 6144, 8192, 10240, 12288, 14336, 16384, 20480, 24576):
            nwin = arena.shape[0] // out
            us = timed(lambda i: call(arena[(i % nwin) * out:(i % nwin + 1) * out]), 24)
            say(kind, f"{out}x{n}", "rows sweep", us, out * n * 4.125)
            pts.append((out, us))
        mx = sum(p[0] for p in pts) / len(pts)
        my = sum(p[1] for p in pts) / len(pts)
        slope = sum((p[0] - mx) * (p[1] - my) for p in pts) / sum((p[0] - mx) ** 2 for p in pts)
        print(json.dumps({"kernel": kind, "width": n, "fit": "us = intercept + slope * rows / 1024",
                          "slope_us_per_1024_rows": round(slope * 1024, 3), "intercept_us": round(my - slope * mx, 2),
                          "streaming_TBps": round(1024 * n * 4.125 / (slope * 1024) / 1e6, 3)}), flush=True)


def chunked_stats(sp, torch, stack, stream, chunks=8, reps=10):
    """Statistics of one layer input arriving in token chunks (as a producer of X would hand them over):
    `chunks` accumulate calls, the last one finalising, against the single call on the whole X."""
    key, n = next(iter(sorted(stack.widths.items())))
    X, T = stack.X[key], stack.T
    b = stack.bufs[0] if stack.block[0][2] == n else sp.LayerBuffers(8, n, T, stack.dev)
    per = T // chunks

    def chunked():
        for c in range(chunks):
            sp.swiftprune_layer_stats(X[c * per:(c + 1) * per if c < chunks - 1 else T], b.xsq, b.S, b.hr,
                                      accumulate=c > 0, finalize=c == chunks - 1, workspace=b.workspace, stream=stream)

    def whole():
        sp.swiftprune_layer_stats(X, b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream)

    # the producer has summed the squares of its own 256 pieces of the tokens: nothing of X is read
    parts = 256
    P = torch.rand((parts, n), dtype=torch.float32, device=stack.dev) * (T / parts)

    def from_partials():
        sp.swiftprune_layer_stats_from_partials(P, b.xsq, b.S, b.hr, stream=stream)

    out = {}
    for name, fn in (("from_partials", from_partials), ("whole", whole), ("chunked", chunked)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / reps * 1e3
    nbytes = T * n * 2
    return {"workload": f"statistics of one {T} x {n} layer input in {chunks} token chunks (accumulate mode)",
            "chunks": chunks, "us_chunked": round(out["chunked"], 1), "us_single_call": round(out["whole"], 1),
            "hbm_frac_chunked": round(nbytes / out["chunked"] / 1e3 / HBM_PEAK_GBS, 4),
            "hbm_frac_single_call": round(nbytes / out["whole"] / 1e3 / HBM_PEAK_GBS, 4),
            "us_from_256_producer_partials": round(out["from_partials"], 1),
            "from_partials_note": "swiftprune_layer_stats_from_partials on 256 per-piece sums of squares (random values "
                                  "here): what remains of step 1 when the kernel that writes X also sums its squares"}


def sample_70b(sp, synth, torch, dev, stream, T, storage, blocks, steps):
    n_model = synth.MODEL_BLOCKS["llama2-70b"][1]
    st = Stack(sp, synth, torch, dev, "llama2-70b", blocks, T, storage)
    out = []
    # la for a 30 % ratio is not in the paper's table: calibrated on the first q matrix of the sample
    W0 = st.pristine[0]
    b0 = st.bufs[0]
    sp.swiftprune_layer_stats(st.X["attn_in"], b0.xsq, b0.S, b0.hr, workspace=b0.workspace, stream=stream)
    la_dev = torch.empty(1, dtype=torch.float32, device=dev)
    status_dev = torch.empty(1, dtype=torch.int32, device=dev)
    sp.swiftprune_calibrate_la_device(W0, b0.hr, 0.30, la_dev, status_out=status_dev, stream=stream)
    la30, ok30 = float(la_dev.item()), int(status_dev.item()) == 0      # read back once, for the report
    label = f"llama2-70b-shaped sample, {blocks} of {n_model} blocks x 7 linear layers"
    for tag, kw in ((f"unstructured, la calibrated on the device for 30 % on one matrix ({'exact rank' if ok30 else 'clamped'})",
                     {"la": la30}),
                    ("unstructured, la=0.5 (table: 50 %)", {"la": 0.5}),
                    ("unstructured, la=-0.2 (table: 70 %)", {"la": -0.2}),
                    ("2:4 structured", {"nm": (2, 4)})):
        out.append(side_entry(st, stream, steps, f"{label}, {tag}", extrapolate_to=n_model, **kw))
    st.release()
    return out


def layer_sweep(sp, torch, stack, nm, la, stream, reps=20):
    """Each distinct layer shape of the block on its own: statistics, then selection + apply, timed with
    events over `reps` layers drawn from different blocks of the stack (different weight buffers, so no
    launch re-reads a cached matrix); algorithmic bytes / time / 8 TB/s per layer."""
    block, weights, pristine, T = stack.block, stack.weights, stack.pristine, stack.T
    n_layers = len(block)
    n_blocks = len(weights) // n_layers
    out_rows = []
    seen = set()
    for li, (name, out, n) in enumerate(block):
        if (out, n) in seen:
            continue
        seen.add((out, n))
        b = stack.bufs[li]
        idxs = [((r % n_blocks) * n_layers + li) for r in range(reps)]
        for i in set(idxs):
            weights[i].copy_(pristine[i])
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * reps)]
        for r, i in enumerate(idxs):
            ev[3 * r].record(stream)
            sp.swiftprune_layer_stats(stack.X[INPUT_OF[name]], b.xsq, b.S, b.hr, workspace=b.workspace, stream=stream)
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
    path = os.path.join(ROOT, PMC_SUMMARY)
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


def host_cpu():
    """(model name, logical CPUs the process may use) of the machine the oracle is timed on."""
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        n = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        n = os.cpu_count() or 1
    return model, n


def cpu_baseline(block, X, pristine, T, nm, la, sample_blocks=2, model_blocks=32):
    """The CPU oracle, as it stands, single-threaded, on a bounded sample of the workload: the first
    `sample_blocks` decoder blocks of the stack (7 layers each, at the full calibration token count),
    every step timed on its own; plus the median over repeated runs of the small single-layer case."""
    import statistics

    import numpy as np

    import oracle
    from paper_2501_16376_amd import synth

    oracle.lib()
    t = {"statistics": 0.0, "factor": 0.0, "score_select": 0.0, "apply": 0.0}
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
            t["statistics"] += time.perf_counter() - t_a
        t0_ = time.perf_counter()
        xsq, S = oracle.stats_finalize(acc)
        hr = oracle.channel_factor_f32(xsq, S)
        t1 = time.perf_counter()
        if nm is None:
            mask, _, _ = oracle.ewma_select(Wh, hr, 0.125, 0.125, la)
        else:
            mask, _ = oracle.nm_select(Wh, hr, nm[0], nm[1])
        t2 = time.perf_counter()
        oracle.apply(Wh, mask)
        t3 = time.perf_counter()
        t["factor"] += t1 - t0_
        t["score_select"] += t2 - t1
        t["apply"] += t3 - t2
        w_bytes += out * n * 2
    total = sum(t.values())

    # the small single-layer case (W 256 x 256 fp32, X 128 x 256 fp32, la 0.5): whole path, median of 31 runs
    W1, X1 = synth.config1()
    runs = []
    for _ in range(31):
        Wc = W1.copy()
        a = time.perf_counter()
        xsq, S, hr = oracle.layer_stats(X1)
        mask, _, _ = oracle.ewma_select(Wc, hr, 0.125, 0.125, 0.5)
        oracle.apply(Wc, mask)
        runs.append(time.perf_counter() - a)
    cpu_model, ncpu = host_cpu()
    return {"value": round(w_bytes / total / 1e9, 5), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample_blocks} decoder blocks of the stack ({sample_blocks * len(block)} layers, "
                      f"{w_bytes / 1e9:.3f} GB of weights) at the full {T} calibration tokens per layer; "
                      f"host copies are not timed",
            "cpu_model": cpu_model, "host_logical_cpus": ncpu, "threads_used": 1,
            "cpu_seconds": round(total, 2),
            "cpu_seconds_by_step": {k: round(v, 3) for k, v in t.items()},
            "seconds_per_model_extrapolated": round(total * model_blocks / sample_blocks, 1),
            "extrapolated_from_blocks": sample_blocks,
            "single_layer_256x256_fp32_median_ms": round(statistics.median(runs) * 1e3, 3),
            "single_layer_runs": len(runs)}


if __name__ == "__main__":
    main()
