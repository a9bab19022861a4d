#!/usr/bin/env python3
"""Benchmark of the hierarchical-attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: hdt_build_layout (level/parent ids ->
tile schedule), hdt_attn_fwd and hdt_attn_bwd, all through the C ABI, inputs resident in HBM, everything on
one stream.  Every step builds its own layout (a deferred build: the call only enqueues, so the host never
waits inside the loop) and destroys it again.
Workload = the training step at 8192 positions (batch 4, 12 heads, head_dim 64, bf16), the configuration
the headline metric is quoted on.  Prints ONE JSON line.

Timing: W warm-up steps, then R regions of exactly K steps each, every region bracketed by a device
synchronisation on both sides with nothing but the path's own calls in between; `ms_per_step` and `value` are
the MEDIAN over the regions (p10 / p90 and the single regions are reported as well).  Beside that: the
distribution of single steps (an event between steps), the same loop with the layout builds on a second
stream, a pass with every kernel bracketed by events (per-kernel times, roofline), the dense masked-attention
baseline on the same inputs, a copy kernel as the practical HBM peak, and the CPU oracle.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--repeats R] [--config 2|3|4|5] [--windowed]
                    [--tile 64x32] [--edges E] [--no-cpu-baseline] [--no-extras] [--no-dense]
"""
from __future__ import annotations

import argparse
import collections
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def algorithmic_bytes_per_unit(kernel: str, d: int) -> int:
    """Compulsory HBM bytes per (position, head) of one launch of `kernel` (bf16 tensors, fp32 row scalars):
    forward reads Q,K,V and writes O,LSE; the D pass reads O,dO,LSE and writes the pair (-D, -LSE/scale); the
    backward kernel reads Q,K,V,dO,LSE and that pair and writes dQ,dK,dV."""
    row = 2 * d
    if kernel.startswith("hdt_fwd"):
        return 4 * row + 4
    if kernel.startswith("hdt_bwd_delta"):
        return 2 * row + 12
    if kernel.startswith("hdt_bwd_bf16"):
        return 7 * row + 12
    raise KeyError(kernel)


def mfma_flop_per_subblock(kernel: str, d: int) -> int:
    """MFMA work a kernel executes per 32x32 sub-block it does not skip: the forward two contractions
    (S = K Q^T, O += V^T P), the backward kernel seven at head size 64 (the dQ role S, dP, dQ; the dK/dV role S, dP,
    dK, dV) and eight at head size 128, where the dK/dV role is split into a dV role (S, dV) and a dK role (S, dP, dK)."""
    per_gemm = 2 * 32 * 32 * d
    return (2 if kernel.startswith("hdt_fwd") else (7 if d == 64 else 8)) * per_gemm


def kernel_source_hash() -> str:
    """Identifies the kernels a profile was taken on: sha256 over the library's sources."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2407_08330_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def pct(xs, q):
    import numpy as np
    return float(np.percentile(np.asarray(xs, dtype=np.float64), q))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="steps per timed region")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=7, help="timed regions of --steps steps each (median reported)")
    ap.add_argument("--config", type=int, default=4, choices=[2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--windowed", action="store_true",
                    help="key tiles = fixed windows of the level-sorted key order (Alg. 1 as printed) instead of "
                         "the default per-query-tile key lists")
    ap.add_argument("--tile", default="", help="tile shape of the layout, 64x32 or 128x64 (default: 64x32 for a step with a backward pass, "
                                               "else the library's 128x64)")
    ap.add_argument("--edges", type=int, default=0,
                    help="edge kinds of the mask (1 parent, 2 siblings, 4 children, OR-ed; 0 = all): the thinned "
                         "patterns of the paper's ListOps study applied to the workload's documents")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="only the timed regions: no event-bracketed passes, no baselines (for external profilers)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements beside the path (positional encoding, cross-attention)")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense masked-attention baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy 3 times (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--source-hash", action="store_true", help="print the hash that ties a profile to the kernel sources")
    args = ap.parse_args()
    if args.source_hash:
        print(kernel_source_hash())
        return 0
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (batch and heads shard without any exchange; "
              "no multi-GPU path is part of it). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2407_08330_amd as hdt
    from paper_2407_08330_amd import inputs

    wl = inputs.make_workload(args.config)
    B, H, N, D = wl.batch, wl.heads, wl.n_pos, wl.head_dim
    scale = wl.softmax_scale
    do_bwd = wl.backward
    dev = torch.device("cuda:0")
    level = torch.from_numpy(wl.level).to(dev)
    parent = torch.from_numpy(wl.parent).to(dev)
    K, R = args.steps, max(1, args.repeats)

    # several independent buffer sets so that successive steps do not find their inputs in the
    # 256 MB last-level cache
    n_sets = 3
    sets = []
    for i in range(n_sets):
        xs = inputs.make_qkv(B, H, N, D, inputs.sample_seed(args.config, 70 + i), 4 if do_bwd else 3)
        t = [torch.from_numpy(inputs.bf16_bits(inputs.round_to_bf16(x)).view(np.int16)).to(dev).view(torch.bfloat16)
             for x in xs]
        outs = dict(o=torch.empty_like(t[0]), lse=torch.empty((B, H, N), dtype=torch.float32, device=dev))
        if do_bwd:
            outs.update(dq=torch.empty_like(t[0]), dk=torch.empty_like(t[0]), dv=torch.empty_like(t[0]))
        sets.append((t, outs))
    del xs
    # Tile shape: a step with a backward pass runs on 64 x 32 tiles (the backward kernel is the faster one on them,
    # by more than their layout and forward cost), a forward-only step on the library's default (128 x 64)
    if args.tile:
        tile_m, tile_n = (int(x) for x in args.tile.split("x"))
    else:
        tile_m, tile_n = (64, 32) if do_bwd else (0, 0)
    lay_opts = dict(tile_m=tile_m, tile_n=tile_n, windowed=args.windowed, edges=args.edges)
    probe = hdt.hdt_build_layout(level, parent, **lay_opts)
    info = probe.info()
    # 32x32 sub-blocks the attention kernels execute (the others are skipped): bits 0..15 of every entry's summary
    executed_subblocks = 0
    for b in range(B):
        qs = probe.export(b)["q_sub"]
        executed_subblocks += int(sum(bin(int(x) & 0xffff).count("1") for x in qs))
    ws_bytes = hdt.hdt_attn_bwd_workspace_bytes(probe, H, D, 0)
    workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    probe.destroy()

    def attention(lay, i):
        t, outs = sets[i % n_sets]
        hdt.hdt_attn_fwd(lay, t[0], t[1], t[2], scale, o=outs["o"], lse=outs["lse"])
        if do_bwd:
            hdt.hdt_attn_bwd(lay, t[0], t[1], t[2], outs["o"], outs["lse"], t[3], scale, dq=outs["dq"],
                             dk=outs["dk"], dv=outs["dv"], workspace=workspace)

    def build(stream=None):
        # deferred: the call only enqueues the build (a windowed layout is built by a call that waits)
        return hdt.hdt_build_layout(level, parent, deferred=True, stream=stream, **lay_opts)

    def run_serial(k0, k1, between=None):
        """Steps k0..k1-1, everything on one stream: build, forward, backward, destroy."""
        last = None
        for i in range(k0, k1):
            if between is not None:
                between(i)
            lay = build()
            attention(lay, i)
            if last is not None:
                last.destroy()   # buffers go back to the library's cache; a later build reuses them in stream order
            last = lay
        if last is not None:
            last.status()        # the last build's report stands for the loop: valid ids, enough room
            last.destroy()

    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream()   # default priority

    def run_pipelined(k0, k1):
        """The same steps with the layouts built on a second stream, two steps ahead (a build depends only on
        the ids).  Every step still does its own build; the main stream waits for a layout's event before the
        forward that uses it.  A layout is destroyed once the attention calls that use it have finished (the host
        waits for an event recorded behind them, three steps late), which is what hdt_layout_destroy_completed is
        for: the library then has nothing to order when a later build takes the buffers."""
        n = k1 - k0
        if n <= 0:
            return
        coming = collections.deque()   # layouts of the steps not yet enqueued, with their "built" events
        live = collections.deque()     # layouts of enqueued steps, with their "attention done" events

        def start_build():
            lay = build(side_stream)
            ev = torch.cuda.Event()
            ev.record(side_stream)
            coming.append((lay, ev))

        def enqueue(i):
            lay, ready = coming.popleft()
            main_stream.wait_event(ready)
            attention(lay, i)
            done = torch.cuda.Event()
            done.record(main_stream)
            live.append((lay, done))

        start_build()
        if n > 1:
            start_build()
        for i in range(k0, k1):
            enqueue(i)
            if i + 2 < k1:
                start_build()
            while len(live) > 3:
                old_lay, old_done = live.popleft()
                old_done.synchronize()
                old_lay.destroy(completed=True)
        while live:
            old_lay, old_done = live.popleft()
            old_done.synchronize()
            old_lay.destroy(completed=True)

    def timed_regions(run):
        """R regions of exactly K steps, each between two device synchronisations; ms per step of each."""
        out = []
        for _ in range(R):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(0, K)
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) * 1e3 / K)
        return out

    if args.calibrate_copy:
        # a copy kernel of known size: 256 MiB read + 256 MiB written per launch
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Warm-up: the W steps asked for, and as many more as it takes to have the device busy for about 60 ms: after
    # an idle phase its clocks need some tens of milliseconds of work to settle, which a short run (W = 5, K = 20)
    # would otherwise spend inside its timed regions.
    # (Not under an external profiler: --no-kernel-timing runs exactly the steps asked for.)
    warm_steps = args.warmup if args.no_kernel_timing else max(args.warmup, 300)
    run_serial(0, warm_steps)
    torch.cuda.synchronize()
    regions = timed_regions(run_serial)
    ms_per_step = pct(regions, 50)

    tokens = B * N
    value = tokens / (ms_per_step * 1e-3)
    nnz, n_tiles = info["nnz"], info["n_tiles"]
    useful_flop = (4 + (10 if do_bwd else 0)) * nnz * D * H
    out = {
        "metric": "hier-attn fwd+bwd tokens/s at 8192 tok (layout build + forward + backward per step)"
        if do_bwd else "hier-attn fwd tokens/s (layout build + forward per step)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "warmup_steps_run": warm_steps,
        "ms_per_step": round(ms_per_step, 4),
        "timing": {"statistic": f"median over {R} regions of {K} steps, one stream, a device synchronisation on both sides",
                   "regions_ms_per_step": [round(x, 4) for x in regions],
                   "p10_ms_per_step": round(pct(regions, 10), 4), "p90_ms_per_step": round(pct(regions, 90), 4)},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config{args.config}:{wl.name}", "batch": B, "heads": H, "head_dim": D,
                   "n_pos": N, "real_positions": wl.n_real, "tile": f"{info['tile_m']}x{info['tile_n']}",
                   "schedule": "windowed" if args.windowed else "key-lists", "edges": info["edges"],
                   "n_tiles": n_tiles, "nnz": nnz, "executed_subblocks_32x32": executed_subblocks},
        "useful_tflops": round(useful_flop / (ms_per_step * 1e-3) / 1e12, 3),
    }
    if args.no_kernel_timing:
        print(json.dumps(out))
        return 0

    # single steps: an event between consecutive steps of one more serial run (the events cost a little)
    n_single = max(100, K)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_single + 1)]
    run_serial(0, n_single, between=lambda i: evs[i].record())
    evs[n_single].record()
    torch.cuda.synchronize()
    single = [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n_single)]
    out["timing"]["single_steps_us"] = {"n": n_single, "median": round(pct(single, 50), 2), "p10": round(pct(single, 10), 2),
                                        "p90": round(pct(single, 90), 2)}

    # the same steps with the layout builds on a second stream, beside the attention kernels
    if do_bwd:
        run_pipelined(0, max(args.warmup, 50))
        torch.cuda.synchronize()
        pr = timed_regions(run_pipelined)
        out["layouts_on_a_second_stream"] = {
            "ms_per_step": round(pct(pr, 50), 4), "p10_ms_per_step": round(pct(pr, 10), 4),
            "p90_ms_per_step": round(pct(pr, 90), 4), "tokens_per_s": round(tokens / (pct(pr, 50) * 1e-3), 1),
            "note": "every step still builds its own layout, two steps ahead on a second stream (not `value`)"}

    # the same K steps once more with every kernel launch bracketed by HIP events on its stream (the events
    # cost a few percent of a step, so they stay out of the regions `value` is taken from)
    hdt.hdt_timing_enable(True)
    hdt.hdt_timing_reset()
    torch.cuda.synchronize()
    e0 = time.perf_counter()
    run_serial(0, K)
    torch.cuda.synchronize()
    out["ms_per_step_with_kernel_events"] = round((time.perf_counter() - e0) * 1e3 / K, 4)
    kernels = hdt.hdt_timing_read()
    hdt.hdt_timing_enable(False)

    per_kernel = {name: {"launches": c, "avg_us": 1e3 * ms / c} for name, (c, ms) in kernels.items() if c}
    phase_us = {"layout": 0.0, "fwd": 0.0, "bwd": 0.0}
    for name, kv in per_kernel.items():
        per_step = kv["avg_us"] * kv["launches"] / K
        if name.startswith("hdt_layout"):
            phase_us["layout"] += per_step
        elif name.startswith("hdt_fwd"):
            phase_us["fwd"] += per_step
        else:
            phase_us["bwd"] += per_step
    out["phase_us_per_step"] = {k: round(v, 2) for k, v in phase_us.items()}
    out["kernel_sum_us_per_step"] = round(sum(phase_us.values()), 2)
    out["kernels"] = {n: {"launches": kv["launches"], "avg_us": round(kv["avg_us"], 2)} for n, kv in per_kernel.items()}

    # practical HBM peak: a plain device copy (256 MiB read + 256 MiB written), event-timed
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    c_ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
    for i in range(10):
        c_ev[i].record()
        dst.copy_(src)
    c_ev[10].record()
    torch.cuda.synchronize()
    copy_ms = [c_ev[i].elapsed_time(c_ev[i + 1]) for i in range(10)]
    copy_gbs = 2 * (256 << 20) / (pct(copy_ms, 50) * 1e-3) / 1e9
    del src, dst
    # practical MFMA peak: the library's measuring kernel (nothing but bf16 32x32x16 contraction instructions, four
    # waves on every SIMD of the chip), event-timed on this stream; launches of ~0.5 ms each
    sink = torch.zeros(16, dtype=torch.float32, device=dev)
    m_ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
    flop = hdt.hdt_probe_mfma_bf16(1024, 2000, sink)   # warm-up (clocks settle under the load)
    for i in range(6):
        m_ev[i].record()
        flop = hdt.hdt_probe_mfma_bf16(1024, 2000, sink)
    m_ev[6].record()
    torch.cuda.synchronize()
    mfma_ms = [m_ev[i].elapsed_time(m_ev[i + 1]) for i in range(6)]
    mfma_tflops = flop / (pct(mfma_ms, 50) * 1e-3) / 1e12
    out["practical_peak"] = {"hbm_copy_gbs": round(copy_gbs, 1),
                             "what": "median of 10 device copies of 256 MiB, bytes read + bytes written over time",
                             "mfma_bf16_tflops": round(mfma_tflops, 1),
                             "mfma_what": "median of 6 launches of the library's MFMA-only kernel (1024 workgroups x 4 "
                                          "waves x 64 000 instructions v_mfma_f32_32x32x16_bf16)"}

    units = B * H * N
    attn = {n: kv for n, kv in per_kernel.items() if not n.startswith("hdt_layout")}
    if attn:
        dom = max(attn, key=lambda n: attn[n]["avg_us"] * attn[n]["launches"])
        alg_bytes = algorithmic_bytes_per_unit(dom, D) * units
        achieved = alg_bytes / (attn[dom]["avg_us"] * 1e-6) / 1e9
        # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a copy kernel of
        # known size).  Counters cannot be read from inside this process: the figure of the last profiled run of
        # this workload is kept under profiles/, stamped with the hash of the kernel sources it was taken on, and
        # reported only while the sources are still those.
        traffic, traffic_note = None, "no counter run on record for this workload"
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                rec = json.load(f)
            if rec.get("kernel_source_hash") != kernel_source_hash():
                traffic_note = "profiles/hbm_traffic.json was measured on other kernel sources: not reported"
            elif args.tile or args.windowed or args.edges:
                traffic_note = "the counter run on record is of this workload's default options: not reported"
            else:
                traffic = rec.get(f"config{args.config}", {}).get(dom)
                if traffic is not None:
                    traffic_note = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on these kernel sources (profiles/)"
        except (OSError, ValueError):
            pass
        out["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                           "traffic_note": traffic_note,
                           "frac_of_practical_peak": round(achieved / copy_gbs, 4),
                           "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": round(attn[dom]["avg_us"], 2)}
    for phase, prefix in (("fwd", "hdt_fwd"), ("bwd_kernel", "hdt_bwd_bf16")):
        name = next((n for n in per_kernel if n.startswith(prefix)), None)
        if not name:
            continue
        us = per_kernel[name]["avg_us"]
        gemms = 2 if phase == "fwd" else (7 if D == 64 else 8)
        executed = executed_subblocks * H * mfma_flop_per_subblock(name, D)
        issued = n_tiles * info["tile_m"] * info["tile_n"] * H * gemms * 2 * D
        out[phase] = {
            "avg_us": round(us, 2),
            "tokens_per_s": round(tokens / (us * 1e-6), 1),
            "useful_tflops": round((4 if phase == "fwd" else 10) * nnz * D * H / (us * 1e-6) / 1e12, 3),
            # MFMA work the kernel executes: the sub-blocks it does not skip (the layout's summaries give the
            # count exactly; profiles/ holds the cross-check against SQ_INSTS_VALU_MFMA_MOPS_BF16)
            "executed_mfma_tflops": round(executed / (us * 1e-6) / 1e12, 2),
            "mfma_frac": round(executed / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "mfma_frac_of_practical_peak": round(executed / (us * 1e-6) / 1e12 / mfma_tflops, 4),
            # every sub-block of every issued tile, skipped or not
            "whole_tile_tflops_incl_skipped_subblocks": round(issued / (us * 1e-6) / 1e12, 2),
            "hbm_gbs_algorithmic": round(algorithmic_bytes_per_unit(name, D) * units / (us * 1e-6) / 1e9, 1),
            "hbm_frac": round(algorithmic_bytes_per_unit(name, D) * units / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        }

    if do_bwd and not args.no_dense and N <= 8192:
        # The dense masked-attention baseline on the same inputs: the same kernels on a layout that issues and
        # computes every tile of the N x N score matrix (force_dense), the mask applied per element.  Layout built
        # once, outside the timed calls, with 128 x 64 tiles: the faster shape when every tile is issued.
        dense = hdt.hdt_build_layout(level, parent, tile_m=128, tile_n=64, force_dense=True, edges=args.edges)
        dinfo = dense.info()
        dense_ws = torch.empty(max(hdt.hdt_attn_bwd_workspace_bytes(dense, H, D, 0), 16), dtype=torch.uint8, device=dev)
        t, outs = sets[0]
        n_rep = 3

        def dense_step():
            hdt.hdt_attn_fwd(dense, t[0], t[1], t[2], scale, o=outs["o"], lse=outs["lse"])
            hdt.hdt_attn_bwd(dense, t[0], t[1], t[2], outs["o"], outs["lse"], t[3], scale, dq=outs["dq"],
                             dk=outs["dk"], dv=outs["dv"], workspace=dense_ws)
        dense_step()
        torch.cuda.synchronize()
        hdt.hdt_timing_enable(True)
        hdt.hdt_timing_reset()
        d0 = time.perf_counter()
        for _ in range(n_rep):
            dense_step()
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - d0) * 1e3 / n_rep
        dk_ = {n: 1e3 * ms / c for n, (c, ms) in hdt.hdt_timing_read().items() if c}
        hdt.hdt_timing_enable(False)
        dense_sub = dinfo["n_tiles"] * (dinfo["tile_m"] // 32) * (dinfo["tile_n"] // 32)
        f_us = dk_.get(f"hdt_fwd_bf16_d{D}")
        b_us = dk_.get(f"hdt_bwd_bf16_d{D}")
        sparse_attn_ms = (phase_us["fwd"] + phase_us["bwd"]) * 1e-3
        out["dense_baseline"] = {
            "what": f"dense {N}x{N} masked attention, forward + backward, same inputs and kernels, every tile issued",
            "tile": f"{dinfo['tile_m']}x{dinfo['tile_n']}", "n_tiles": dinfo["n_tiles"], "ms_fwd_bwd": round(dense_ms, 3),
            "tokens_per_s": round(tokens / (dense_ms * 1e-3), 1),
            "kernels_us": {n: round(v, 1) for n, v in dk_.items()},
            "fwd_mfma_tflops": None if not f_us else round(dense_sub * H * mfma_flop_per_subblock("hdt_fwd", D) / (f_us * 1e-6) / 1e12, 1),
            "fwd_mfma_frac": None if not f_us else round(dense_sub * H * mfma_flop_per_subblock("hdt_fwd", D) / (f_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "bwd_mfma_tflops": None if not b_us else round(dense_sub * H * mfma_flop_per_subblock("hdt_bwd_bf16", D) / (b_us * 1e-6) / 1e12, 1),
            "bwd_mfma_frac": None if not b_us else round(dense_sub * H * mfma_flop_per_subblock("hdt_bwd_bf16", D) / (b_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "sparse_fwd_bwd_ms": round(sparse_attn_ms, 4),
            "speedup_of_the_sparse_schedule": round(dense_ms / sparse_attn_ms, 1) if sparse_attn_ms > 0 else None,
        }
        dense.destroy()

    if not args.no_extras:
        # the step before the path (not part of `value`): hierarchical positional encoding of the same batch,
        # index vectors from the ids and the fused add into bf16 embeddings of d_model = heads * head_dim
        d_model, n_lev = H * D, 3
        emb = torch.zeros((B, N, d_model), dtype=torch.bfloat16, device=dev)
        table = hdt.hdt_hpe_table(1024, d_model)
        pvec = hdt.hdt_index_vectors(level, parent, n_lev)
        hdt.hdt_hpe_add(pvec, table, emb)
        torch.cuda.synchronize()
        hdt.hdt_timing_enable(True)
        hdt.hdt_timing_reset()
        for _ in range(20):
            hdt.hdt_index_vectors(level, parent, n_lev, out=pvec)
            hdt.hdt_hpe_add(pvec, table, emb)
        torch.cuda.synchronize()
        tk = {n: round(1e3 * ms / c, 2) for n, (c, ms) in hdt.hdt_timing_read().items() if n.startswith("hdt_hpe")}
        hdt.hdt_timing_enable(False)
        add_us = tk.get("hdt_hpe_add_bf16")
        add_bytes = B * N * (2 * 2 * d_model + 4 * n_lev)   # x read + written, index vector read
        out["hpe"] = {"d_model": d_model, "levels": n_lev, "kernels_us": tk,
                      "add_algorithmic_bytes": add_bytes,
                      "add_gbs": None if not add_us else round(add_bytes / (add_us * 1e-6) / 1e9, 1),
                      "add_frac_of_hbm_peak": None if not add_us else round(add_bytes / (add_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}

        # decoder cross-attention over level subsets of the same encoder batch (not part of `value`): 512
        # decoder rows per sample attending to the [SEC] anchors, + [SENT] anchors, + tokens
        n_dec = 512
        qd = torch.randn((B, H, n_dec, D), device=dev).to(torch.bfloat16)
        dod = torch.randn((B, H, n_dec, D), device=dev).to(torch.bfloat16)
        kt, vt = sets[0][0][1], sets[0][0][2]
        dkc, dvc = torch.empty_like(kt), torch.empty_like(kt)
        cross = {}
        for name, mask in (("sec", 2), ("sec+sent", 6), ("sec+sent+tokens", 14)):
            lay_c = hdt.hdt_build_cross_layout(level, n_dec, mask)
            ws_c = torch.empty(max(16, hdt.hdt_attn_bwd_workspace_bytes(lay_c, H, D, 0)), dtype=torch.uint8, device=dev)
            wf_bytes = hdt.hdt_attn_fwd_workspace_bytes(lay_c, H, D, 0)   # > 0: long key lists, walked in pieces
            ws_f = torch.empty(wf_bytes, dtype=torch.uint8, device=dev) if wf_bytes else None
            oc, lc = hdt.hdt_attn_fwd(lay_c, qd, kt, vt, scale, workspace=ws_f)
            dqc = torch.empty_like(qd)
            hdt.hdt_attn_bwd(lay_c, qd, kt, vt, oc, lc, dod, scale, dq=dqc, dk=dkc, dv=dvc, workspace=ws_c)
            torch.cuda.synchronize()
            hdt.hdt_timing_enable(True)
            hdt.hdt_timing_reset()
            for _ in range(20):
                tmp = hdt.hdt_build_cross_layout(level, n_dec, mask)
                tmp.destroy()
                hdt.hdt_attn_fwd(lay_c, qd, kt, vt, scale, o=oc, lse=lc, workspace=ws_f)
                hdt.hdt_attn_bwd(lay_c, qd, kt, vt, oc, lc, dod, scale, dq=dqc, dk=dkc, dv=dvc, workspace=ws_c)
            torch.cuda.synchronize()
            tk = {n: round(1e3 * ms / c, 2) for n, (c, ms) in hdt.hdt_timing_read().items()}
            hdt.hdt_timing_enable(False)
            visible = lay_c.info()["nnz"] // n_dec
            row = 2 * D
            fwd_bytes = H * (B * n_dec * (2 * row + 4) + visible * 2 * row)          # Q, O, LSE; visible K, V rows
            bwd_bytes = H * (B * n_dec * (3 * row + 8) + visible * 2 * row + B * N * 2 * row)  # Q, dO, dQ; K, V; all of dK, dV
            # the whole forward call: the kernel, plus the kernel that combines the pieces of cut key lists
            fwd_us = tk.get(f"hdt_fwd_bf16_d{D}")
            if fwd_us and tk.get("hdt_cross_combine_fwd"):
                fwd_us += tk["hdt_cross_combine_fwd"]
            # the whole backward call: D pass and kernel, plus the copies of a compact layout or the sum of dQ's parts
            bwd_parts = [tk.get(k) for k in (f"hdt_bwd_delta_d{D}", f"hdt_bwd_bf16_d{D}", "hdt_cross_gather", "hdt_cross_scatter",
                                             "hdt_cross_sum_dq")]
            bwd_us = sum(x for x in bwd_parts if x) if tk.get(f"hdt_bwd_bf16_d{D}") else None
            cross[name] = {"visible_positions": int(visible), "compact_rows": int(lay_c.info()["compact_rows"]), "kernels_us": tk,
                           "fwd_us": None if not fwd_us else round(fwd_us, 2),
                           "bwd_us": None if not bwd_us else round(bwd_us, 2),
                           "forward_workspace_bytes": int(wf_bytes),
                           "fwd_algorithmic_bytes": fwd_bytes, "bwd_algorithmic_bytes": bwd_bytes,
                           "fwd_gbs": None if not fwd_us else round(fwd_bytes / (fwd_us * 1e-6) / 1e9, 1),
                           "bwd_gbs": None if not bwd_us else round(bwd_bytes / (bwd_us * 1e-6) / 1e9, 1),
                           "fwd_useful_tflops": None if not fwd_us else round(4 * visible * n_dec * D * H / (fwd_us * 1e-6) / 1e12, 1)}
            lay_c.destroy()
        out["cross_attention"] = {"n_dec": n_dec, "n_enc": N, "cases": cross}

    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host cores: pairwise mask enumeration + fp64 forward (+ backward) with
        # fresh seeded inputs.  All threads: the whole batch once.  One thread: the first sample only (the same
        # work per position; the thread count is set through the OpenMP runtime the oracle uses).
        import ctypes
        from oracle import oracle
        xs = [inputs.round_to_bf16(x) for x in inputs.make_qkv(B, H, N, D, inputs.sample_seed(args.config, 70),
                                                               4 if do_bwd else 3)]

        def oracle_pass(nb):
            c0 = time.perf_counter()
            with oracle.edges(args.edges or oracle.EDGE_ALL):
                oracle.attn_fwd(xs[0][:nb], xs[1][:nb], xs[2][:nb], wl.level[:nb], wl.parent[:nb], scale)
                if do_bwd:
                    oracle.attn_bwd(xs[0][:nb], xs[1][:nb], xs[2][:nb], xs[3][:nb], wl.level[:nb], wl.parent[:nb], scale)
            return time.perf_counter() - c0

        threads = oracle.num_threads()
        wall = oracle_pass(B)
        what = f"pairwise mask enumeration + fp64 forward{' + backward' if do_bwd else ''}"
        out["cpu_baseline"] = {"value": round(tokens / wall, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
                               "sample": f"the whole batch once ({tokens} positions, {H} heads): {what}, {wall:.2f} s wall"}
        try:
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            wall1 = oracle_pass(1)
            gomp.omp_set_num_threads(threads)
            out["cpu_baseline"]["single_thread"] = {
                "value": round(N / wall1, 1), "unit": "tokens/s", "cores": 1,
                "sample": f"the first sample once ({N} positions, {H} heads): {what}, {wall1:.2f} s wall"}
        except OSError:
            pass
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
