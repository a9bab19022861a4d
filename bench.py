#!/usr/bin/env python3
"""Benchmark of the hierarchical-attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: hdt_build_layout (level/parent ids ->
tile schedule), hdt_attn_fwd and hdt_attn_bwd, all through the C ABI, inputs resident in HBM.  Every
step builds its own layout; by default the build of the next step's layout runs on a second stream
while the current step's attention kernels run (it depends only on the ids), --serial keeps everything
on one stream.  Per-kernel times always come from a serial, event-bracketed pass.
Workload = the training step at 8192 positions (batch 4, 12 heads, head_dim 64, bf16), the
configuration the headline metric is quoted on.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--serial] [--windowed] [--edges E]
                    [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import collections
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def algorithmic_bytes_per_unit(kernel: str, d: int) -> int:
    """Compulsory HBM bytes per (position, head) of one launch of `kernel` (bf16 tensors, fp32 LSE/D):
    forward reads Q,K,V and writes O,LSE; the D pass reads O,dO and writes D; the backward kernel reads
    Q,K,V,dO,LSE,D and writes dQ,dK,dV."""
    row = 2 * d
    if kernel.startswith("hdt_fwd"):
        return 4 * row + 4
    if kernel.startswith("hdt_bwd_delta"):
        return 2 * row + 4
    if kernel.startswith("hdt_bwd_bf16"):
        return 7 * row + 8
    raise KeyError(kernel)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, choices=[2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--windowed", action="store_true",
                    help="key tiles = fixed windows of the level-sorted key order (Alg. 1 as printed) instead of "
                         "the default per-query-tile key lists")
    ap.add_argument("--tile", default="", help="tile shape of the layout, 64x32 or 128x64 (default: the library's)")
    ap.add_argument("--serial", action="store_true",
                    help="one stream, strictly build -> forward -> backward per step (default for the forward-only "
                         "configurations, whose steps are too short to hide a build that reports back to the host)")
    ap.add_argument("--pipelined", action="store_true",
                    help="the next step's layout is built on a second stream while this step's attention kernels "
                         "run (default for configurations with a backward pass)")
    ap.add_argument("--edges", type=int, default=0,
                    help="edge kinds of the mask (1 parent, 2 siblings, 4 children, OR-ed; 0 = all): the thinned "
                         "patterns of the paper's ListOps study applied to the workload's documents")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="do not bracket kernels with events (for external profilers)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements beside the path (positional encoding, cross-attention)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy 3 times (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
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
    tile_m, tile_n = (int(x) for x in args.tile.split("x")) if args.tile else (0, 0)
    probe = hdt.hdt_build_layout(level, parent, tile_m=tile_m, tile_n=tile_n, windowed=args.windowed, edges=args.edges)
    info = probe.info()
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
        return hdt.hdt_build_layout(level, parent, tile_m=tile_m, tile_n=tile_n, windowed=args.windowed,
                                    edges=args.edges, stream=stream)

    def run_serial(k0, k1):
        """Steps k0..k1-1, everything on one stream: build, forward, backward, destroy."""
        for i in range(k0, k1):
            lay = build()
            attention(lay, i)
            lay.destroy()   # buffers go back to the library's cache; the next build reuses them in stream order

    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream()   # default priority

    def run_pipelined(k0, k1):
        """The same steps, with the layouts built on a second stream two steps ahead (a build depends only
        on the ids): the host call of a build waits for the layout kernel's report, so the attention
        kernels of the next step are enqueued before it, and the GPU always has a step's work in its queue
        while the host waits.  Every step still does its own build; a layout is destroyed only after the
        attention calls that use it have finished."""
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
        enqueue(k0)
        for i in range(k0, k1):   # step i is in the queue
            if i + 1 < k1:
                enqueue(i + 1)
            if i + 2 < k1:
                start_build()
            while len(live) > 3:
                old_lay, old_done = live.popleft()
                old_done.synchronize()
                old_lay.destroy()
        while live:
            old_lay, old_done = live.popleft()
            old_done.synchronize()
            old_lay.destroy()

    if args.serial and args.pipelined:
        ap.error("--serial and --pipelined exclude each other")
    serial = args.serial or (not args.pipelined and not do_bwd)
    run = run_serial if serial else run_pipelined

    if args.calibrate_copy:
        # a copy kernel of known size: 256 MiB read + 256 MiB written per launch
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    run(0, args.warmup)
    torch.cuda.synchronize()

    # timed region: exactly K steps, nothing but the path's own calls between the two synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(0, args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # for reference: the same K steps strictly one after the other on a single stream
    ms_per_step_serial = ms_per_step
    if not serial:
        run_serial(0, args.warmup)
        torch.cuda.synchronize()
        s0 = time.perf_counter()
        run_serial(0, args.steps)
        torch.cuda.synchronize()
        ms_per_step_serial = (time.perf_counter() - s0) * 1e3 / args.steps

    # the same K steps once more with every kernel launch bracketed by HIP events on its stream (the
    # events themselves cost ~10 % of a step, so they stay out of the region `value` is taken from)
    kernels, ms_per_step_events = {}, None
    if not args.no_kernel_timing:
        hdt.hdt_timing_enable(True)
        hdt.hdt_timing_reset()
        torch.cuda.synchronize()
        e0 = time.perf_counter()
        run_serial(0, args.steps)
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - e0) * 1e3 / args.steps
        kernels = hdt.hdt_timing_read()
        hdt.hdt_timing_enable(False)

    tokens = B * N
    value = tokens / (ms_per_step * 1e-3)
    nnz, n_tiles = info["nnz"], info["n_tiles"]
    useful_flop = (4 + (10 if do_bwd else 0)) * nnz * D * H
    issued_fwd_flop = 4 * n_tiles * info["tile_m"] * info["tile_n"] * D * H

    per_kernel = {name: {"launches": c, "avg_us": 1e3 * ms / c} for name, (c, ms) in kernels.items() if c}
    phase_us = {"layout": 0.0, "fwd": 0.0, "bwd": 0.0}
    for name, kv in per_kernel.items():
        per_step = kv["avg_us"] * kv["launches"] / args.steps
        if name.startswith("hdt_layout"):
            phase_us["layout"] += per_step
        elif name.startswith("hdt_fwd"):
            phase_us["fwd"] += per_step
        else:
            phase_us["bwd"] += per_step

    roofline = None
    attn = {n: kv for n, kv in per_kernel.items() if not n.startswith("hdt_layout")}
    if attn:
        dom = max(attn, key=lambda n: attn[n]["avg_us"] * attn[n]["launches"])
        units = B * H * N
        alg_bytes = algorithmic_bytes_per_unit(dom, D) * units
        achieved = alg_bytes / (attn[dom]["avg_us"] * 1e-6) / 1e9
        # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a copy
        # kernel of known size); counters cannot be read from inside this process, so the figure of the
        # last profiled run of this workload is kept under profiles/
        traffic = None
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                traffic = json.load(f).get(f"config{args.config}", {}).get(dom)
        except (OSError, ValueError):
            pass
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": round(attn[dom]["avg_us"], 2)}

    out = {
        "metric": "hier-attn fwd+bwd tokens/s at 8192 tok (layout build + forward + backward per step)"
        if do_bwd else "hier-attn fwd tokens/s (layout build + forward per step)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_serial": round(ms_per_step_serial, 4),
        "pipelining": "none" if serial else "layouts built two steps ahead on a second stream, beside the attention kernels",
        "ms_per_step_with_kernel_events": None if ms_per_step_events is None else round(ms_per_step_events, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config{args.config}:{wl.name}", "batch": B, "heads": H, "head_dim": D,
                   "n_pos": N, "real_positions": wl.n_real, "tile": f"{info['tile_m']}x{info['tile_n']}",
                   "schedule": "windowed" if args.windowed else "key-lists", "edges": info["edges"],
                   "n_tiles": n_tiles, "nnz": nnz},
        "useful_tflops": round(useful_flop / (ms_per_step * 1e-3) / 1e12, 3),
        "phase_us_per_step": {k: round(v, 2) for k, v in phase_us.items()},
        "kernels": {n: {"launches": kv["launches"], "avg_us": round(kv["avg_us"], 2)} for n, kv in per_kernel.items()},
        "roofline": roofline,
    }
    fwd_name = next((n for n in per_kernel if n.startswith("hdt_fwd")), None)
    if fwd_name:
        fwd_us = per_kernel[fwd_name]["avg_us"]
        out["fwd"] = {
            "tokens_per_s": round(tokens / (fwd_us * 1e-6), 1),
            "useful_tflops": round(4 * nnz * D * H / (fwd_us * 1e-6) / 1e12, 3),
            "issued_tile_tflops": round(issued_fwd_flop / (fwd_us * 1e-6) / 1e12, 2),
            "mfma_frac_on_issued_tiles": round(issued_fwd_flop / (fwd_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "hbm_gbs_algorithmic": round(algorithmic_bytes_per_unit(fwd_name, D) * B * H * N / (fwd_us * 1e-6) / 1e9, 1),
        }

    if not args.no_kernel_timing and not args.no_extras:
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

    if not args.no_kernel_timing and not args.no_extras:
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
            oc, lc = hdt.hdt_attn_fwd(lay_c, qd, kt, vt, scale)
            dqc = torch.empty_like(qd)
            hdt.hdt_attn_bwd(lay_c, qd, kt, vt, oc, lc, dod, scale, dq=dqc, dk=dkc, dv=dvc, workspace=ws_c)
            torch.cuda.synchronize()
            hdt.hdt_timing_enable(True)
            hdt.hdt_timing_reset()
            for _ in range(20):
                tmp = hdt.hdt_build_cross_layout(level, n_dec, mask)
                tmp.destroy()
                hdt.hdt_attn_fwd(lay_c, qd, kt, vt, scale, o=oc, lse=lc)
                hdt.hdt_attn_bwd(lay_c, qd, kt, vt, oc, lc, dod, scale, dq=dqc, dk=dkc, dv=dvc, workspace=ws_c)
            torch.cuda.synchronize()
            tk = {n: round(1e3 * ms / c, 2) for n, (c, ms) in hdt.hdt_timing_read().items()}
            hdt.hdt_timing_enable(False)
            visible = lay_c.info()["nnz"] // n_dec
            row = 2 * D
            fwd_bytes = H * (B * n_dec * (2 * row + 4) + visible * 2 * row)          # Q, O, LSE; visible K, V rows
            bwd_bytes = H * (B * n_dec * (3 * row + 8) + visible * 2 * row + B * N * 2 * row)  # Q, dO, dQ; K, V; all of dK, dV
            fwd_us = tk.get(f"hdt_fwd_bf16_d{D}")
            # the whole backward call: D pass and kernel, plus the copies of a compact layout
            bwd_parts = [tk.get(k) for k in (f"hdt_bwd_delta_d{D}", f"hdt_bwd_bf16_d{D}", "hdt_cross_gather", "hdt_cross_scatter")]
            bwd_us = sum(x for x in bwd_parts if x) if tk.get(f"hdt_bwd_bf16_d{D}") else None
            cross[name] = {"visible_positions": int(visible), "compact_rows": int(lay_c.info()["compact_rows"]), "kernels_us": tk,
                           "bwd_us": None if not bwd_us else round(bwd_us, 2),
                           "fwd_algorithmic_bytes": fwd_bytes, "bwd_algorithmic_bytes": bwd_bytes,
                           "fwd_gbs": None if not fwd_us else round(fwd_bytes / (fwd_us * 1e-6) / 1e9, 1),
                           "bwd_gbs": None if not bwd_us else round(bwd_bytes / (bwd_us * 1e-6) / 1e9, 1)}
            lay_c.destroy()
        out["cross_attention"] = {"n_dec": n_dec, "n_enc": N, "cases": cross}

    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores: mask enumeration + forward (+ backward) of the
        # same batch with fresh seeded inputs, once
        from oracle import oracle
        xs = [inputs.round_to_bf16(x) for x in inputs.make_qkv(B, H, N, D, inputs.sample_seed(args.config, 70),
                                                               4 if do_bwd else 3)]
        c0 = time.perf_counter()
        with oracle.edges(args.edges or oracle.EDGE_ALL):
            oracle.attn_fwd(xs[0], xs[1], xs[2], wl.level, wl.parent, scale)
            if do_bwd:
                oracle.attn_bwd(xs[0], xs[1], xs[2], xs[3], wl.level, wl.parent, scale)
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": round(tokens / (c1 - c0), 1), "unit": "tokens/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"the whole batch once ({tokens} positions, {H} heads): pairwise mask "
                                         f"enumeration + fp64 forward{' + backward' if do_bwd else ''}, "
                                         f"{c1 - c0:.2f} s wall"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
