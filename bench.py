#!/usr/bin/env python3
"""Benchmark of the CASK compression event on one MI355X.

A step is one whole compression event (score -> prefix eviction -> core/scratch partition ->
consolidation -> fold -> compaction) over every (layer, KV head) unit of a synthetic cache
that is already resident in HBM.  The default workload is the Qwen2.5-7B-shaped cache at
budget 384 (28 layers x 4 KV heads, 256 prefix + 8192 decode tokens, 128-query window).

Prints ONE JSON line: whole-event throughput in KV tokens/s (one KV token = one
(token, layer, KV head) K/V row pair), the roofline position of the dominant kernel measured
with HIP events recorded between the kernels inside the timed region, and the CPU oracle
timed on a bounded sample of the same units.
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

METRIC = "KV tokens compressed/s per layer x head at budget 384; % HBM/MFMA roofline"
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel (the first scoring sweep) as read by
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in separate runs of this file, each counter scaled by
# what it reads for the copy probe of known size in the same run.  These are constants taken
# from the named summaries under profiles/, not measured by the run that prints them; a workload
# without a summary, or a cut-down run (--layers / --seqs), reports null.
PROFILED_TRAFFIC = {
    "cfg2": {"bytes": (130983.6 * 2.0 + 6272.0) * 1024, "source": "profiles/cfg2_kernels_and_hbm_traffic.md (score_mfma_kernel<0, 4, false>)"},
    "cfg3": {"bytes": (475940.1 * 2.0 + 6272.0) * 1024, "source": "profiles/cfg3_kernels_and_hbm_traffic.md (score_mfma_kernel<0, 4, false>)"},
    "cfg4": {"bytes": (270769.8 * 2.0 + 6272.0) * 1024, "source": "profiles/cfg4_kernels_and_hbm_traffic.md (score_mfma_kernel<0, 4, false>)"},
    "cfg4v": {"bytes": (959114.4 * 2.0 + 6272.0) * 1024, "source": "profiles/cfg4v_kernels_and_hbm_traffic.md (score_mfma_kernel<0, 4, false>)"},
    # (the slower of the two sweeps on this workload is the second one)
    "cfg5": {"bytes": (42022467.9 * 2.0 + 1282985.8) * 1024, "source": "profiles/cfg5_kernels_and_hbm_traffic.md (score_mfma_kernel<1, 4, true>)"},
    "cfg2ss": {"bytes": (22075.3 * 2.0 + 3136.0) * 1024, "source": "profiles/cfg2ss_kernels_and_hbm_traffic.md (score_mfma_kernel<2, 2, false>)"},
}


def sample_sclk(fn, seconds=4.0):
    """Median and range of the shader clock `rocm-smi --showclocks --json` reports (MHz) while fn is
    called in a loop for `seconds`; None where rocm-smi is missing or prints no clock."""
    import re
    import subprocess
    import threading

    import torch
    vals, stop = [], threading.Event()

    def sampler():
        while not stop.is_set():
            try:
                out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True,
                                     timeout=10).stdout
                card = json.loads(out)
                for k, v in card[sorted(card)[0]].items():
                    m = re.search(r"(\d+)\s*mhz", str(v).lower())
                    if k.lower().startswith("sclk clock speed") and m:
                        vals.append(int(m.group(1)))
            except Exception:
                return

    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.time()
    while time.time() - t0 < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    stop.set()
    th.join()
    vals = vals[1:]  # the first sample may predate the load
    if not vals:
        return None
    return {"median": int(sorted(vals)[len(vals) // 2]), "min": int(min(vals)), "max": int(max(vals)), "samples": len(vals)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed events first; the clocks settle within about 20")
    ap.add_argument("--workload", default="cfg2",
                    help="cfg2 (default) | cfg3 | cfg4 | cfg4v | cfg5; cfg2ss / cfg3ss = the steady state of a "
                         "decode loop on that shape: every event compresses budget + window rows back to the "
                         "budget (cask_compress_step with token counts), also timed as a replayed HIP graph")
    ap.add_argument("--sample-clocks", action="store_true",
                    help="with --probe-only: also report the shader clock rocm-smi shows while cask_score and "
                         "the probe loops run (is the part at its power limit?)")
    ap.add_argument("--layers", type=int, default=0, help="use only the first L layers (0 = all)")
    ap.add_argument("--seqs", type=int, default=0, help="cfg5: use only the first S sequences")
    ap.add_argument("--copies", type=int, default=0,
                    help="input copies alternated between steps (0 = 2 when they fit in 2 GB)")
    ap.add_argument("--cpu-units", type=int, default=48, help="units the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--pmc-copy-mib", type=int, default=0,
                    help="also run the copy probe once on a buffer of this many MiB (a kernel of known "
                         "traffic, N MiB read and N MiB written, for scaling rocprofv3 FETCH_SIZE / "
                         "WRITE_SIZE readings)")
    ap.add_argument("--sim-threshold", type=float, default=0.9,
                    help="cask_params.sim_threshold; the headline is quoted at the default 0.9, -1 makes "
                         "every donor fold (the merge-heavy variant that loads the fold path)")
    ap.add_argument("--probe-only", action="store_true",
                    help="run only the library's probe loops (every instruction mix at 1-3 waves per SIMD, the "
                         "copy and the read stream), print them as one JSON object and exit")
    ap.add_argument("--no-pinned-peaks", action="store_true",
                    help="skip the two probe loops (MFMA chain, streaming copy) that pin this box's ceilings")
    ap.add_argument("--no-stage-events", action="store_true",
                    help="record no HIP events inside the timed region (no roofline object then)")
    ap.add_argument("--graph-steps", type=int, default=50,
                    help="replays of the extra HIP-graph measurement (0 = skip)")
    ap.add_argument("--overlap-steps", type=int, default=50,
                    help="events of the extra two-stream measurement (0 = skip)")
    ap.add_argument("--seed-dedup", type=int, default=0,
                    help="cask_params.seed_dedup for the event (0 = the default seeding rule; the headline "
                         "figure is quoted with 0)")
    ap.add_argument("--attend-steps", type=int, default=50,
                    help="after the timed region: time the consumer side, one decode step's attention "
                         "(cask_attend) over the compressed caches the event wrote (0 = skip)")
    ap.add_argument("--breakdown-steps", type=int, default=20,
                    help="extra untimed steps with an event after every kernel for config.stage_ms (0 = skip)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; the compression event shards over units "
              "with no exchange, so N > 1 is not run here (use --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2604_10900_amd as cask
    from paper_2604_10900_amd import binding
    from synth import caches

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    cask.load()
    dev = torch.device("cuda:0")
    if args.probe_only:
        names = {0: "mfma alone", 1: "mfma + softmax epilogue of two logits (fma, fma, exp2, exp2, add, add)",
                 2: "the six vector instructions alone", 3: "as 1, first operand read from LDS at the sweeps' rate",
                 4: "as 1, epilogue in dependent order with one running sum"}
        rows = []
        for kind in (0, 1, 2, 3, 4):
            for wps in (1, 2, 3):
                r = binding.probe_issue(kind, waves_per_simd=wps, blocks=256, iters=24000 // wps)
                rows.append({"kind": kind, "what": names[kind], "waves_per_simd": wps,
                             **{k: round(v, 3) for k, v in r.items()}})
        mem = {"copy_1GiB": binding.probe_copy(1 << 30), "copy_4GiB": binding.probe_copy(4 << 30),
               "read_1GiB": binding.probe_read(1 << 30), "read_4GiB": binding.probe_read(4 << 30)}
        clocks = None
        if args.sample_clocks:
            # the shader clock rocm-smi reports while one kernel loops: the sweeps and the MFMA loops
            # hold the part at its power limit, the vector-only loop does not
            w3 = caches.WORKLOADS["cfg3"]
            c3 = caches.make(w3, device=dev)
            p3 = cask.Params(dtype=cask.BF16, head_dim=w3.head_dim, q_per_kv=w3.q_per_kv, window=w3.window,
                             budget=w3.budget)
            b3 = cask.Batch(p3, c3["row_off"], c3["prefix_len"], c3["K"], c3["V"], c3["Q"])
            clocks = {"idle": sample_sclk(lambda: None, 2.0),
                      "cask_score cfg3": sample_sclk(lambda: cask.score(b3)),
                      "probe kind 0, two waves": sample_sclk(lambda: binding.probe_issue(0, 2, 256, 20000)),
                      "probe kind 1, two waves": sample_sclk(lambda: binding.probe_issue(1, 2, 256, 20000)),
                      "probe kind 3, two waves": sample_sclk(lambda: binding.probe_issue(3, 2, 256, 20000)),
                      "probe kind 3, three waves": sample_sclk(lambda: binding.probe_issue(3, 3, 256, 20000)),
                      "probe kind 2, two waves": sample_sclk(lambda: binding.probe_issue(2, 2, 256, 20000))}
        print(json.dumps({"probe_issue": rows, "probe_memory": mem, "sclk_MHz_under_load": clocks,
                          "note": "256 workgroups (one per compute unit); TFLOP/s counts the MFMA flop; cycles per unit "
                                  "and SIMD = time x shader clock / units; copy GB/s counts bytes read plus written"}))
        return
    steady = args.workload.endswith("ss")
    w = caches.WORKLOADS[args.workload[:-2] if steady else args.workload]
    if steady:
        # B + delta rows per unit, delta = the window; the prefix has shrunk to its steady p_keep
        p0 = cask.Params(dtype=cask.BF16, head_dim=w.head_dim, q_per_kv=w.q_per_kv, window=w.window,
                         recent=w.recent, budget=w.budget, core=w.core)
        keep = cask.plan(p0, w.prefix, w.prefix + w.decode)["p_keep"]
        w = caches.scaled(w, prefix=keep, decode=w.budget + w.window - keep)
    layers = range(args.layers) if args.layers > 0 else None
    seqs = range(args.seqs) if args.seqs > 0 else None
    n_layers = args.layers if args.layers > 0 else w.n_layers
    p = cask.Params(dtype=cask.F32 if w.dtype == "f32" else cask.BF16, head_dim=w.head_dim,
                    q_per_kv=w.q_per_kv, window=w.window, recent=w.recent, budget=w.budget,
                    core=w.core, seed_dedup=args.seed_dedup, sim_threshold=args.sim_threshold)

    # ---- inputs, resident in HBM; alternate copies so the 256 MB last-level cache cannot
    # stand in for HBM between steps
    first = caches.make(w, seed=caches.BASE_SEED, device=dev, layers=layers, seqs=seqs)
    in_bytes = first["K"].numel() * first["K"].element_size() * 2
    copies = args.copies if args.copies > 0 else (2 if in_bytes <= (2 << 30) else 1)
    batches = []
    for i in range(copies):
        c = first if i == 0 else caches.make(w, seed=caches.BASE_SEED + i, device=dev, layers=layers, seqs=seqs)
        b = cask.Batch(p, c["row_off"], c["prefix_len"], c["K"], c["V"], c["Q"])
        batches.append((c, b))
    b0 = batches[0][1]
    outs = cask.Outputs(b0)
    ws = b0.workspace()
    for _, b in batches[1:]:
        b._ws = ws
    kv_tokens = b0.total_rows
    n_units = b0.n_units

    if steady:
        stride = w.budget + w.window
        dt = torch.float32 if w.dtype == "f32" else torch.bfloat16
        K_next = torch.zeros(n_units, stride, w.head_dim, dtype=dt, device=dev)
        V_next = torch.zeros_like(K_next)
        counts = torch.ones(kv_tokens, dtype=torch.int32, device=dev)
        out_count = torch.zeros(n_units, w.budget, dtype=torch.int32, device=dev)

    def step(i):
        if steady:
            cask.compress_step(batches[i % copies][1], K_next, V_next, outs, in_count=counts, out_count=out_count)
        else:
            cask.compress(batches[i % copies][1], outs)

    if args.pmc_copy_mib > 0:
        src = torch.empty(args.pmc_copy_mib << 20, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        rc = cask.load().cask_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(),
                                         torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        torch.cuda.synchronize()
        del src, dst
    # ---- this box's ceilings, pinned by two plain loops of the library (a chain of bf16 MFMA on
    # random register operands, two waves per SIMD on every compute unit; a 1 GiB streaming copy)
    pinned = None
    if not args.no_pinned_peaks:
        pm = binding.probe_issue(0, waves_per_simd=2, blocks=256, iters=20000)
        pv = binding.probe_issue(1, waves_per_simd=2, blocks=256, iters=20000)
        pc = binding.probe_copy(1 << 30)
        pr = binding.probe_read(1 << 30)
        pinned = {"mfma_bf16_TFLOP/s": round(pm["tflops"], 1), "mfma_loop_clock_GHz": round(pm["ghz"], 3),
                  "mfma_loop_cycles_per_mfma": round(pm["cycles_per_unit"], 2),
                  "mfma_with_softmax_epilogue_TFLOP/s": round(pv["tflops"], 1),
                  "mfma_with_softmax_epilogue_clock_GHz": round(pv["ghz"], 3),
                  "mfma_with_softmax_epilogue_cycles_per_mfma": round(pv["cycles_per_unit"], 2),
                  "copy_GB/s": round(pc["gbs"], 1), "read_GB/s": round(pr["gbs"], 1),
                  "note": "cask_probe_issue kinds 0 and 1 (256 workgroups x 8 waves: two waves per SIMD on every "
                          "compute unit), cask_probe_copy (1 GiB, bytes read + written), cask_probe_read (1 GiB)"}
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # timed region: K whole events; the library brackets the two scoring sweeps (the dominant
    # kernels) with three HIP events per step on the stream they run on
    use_events = not args.no_stage_events
    if use_events:
        binding.timing_enable(args.steps, 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sweep_ms = None
    if use_events:
        sweep_ms, n_rec = binding.timing_read()
        binding.timing_enable(0)
        assert n_rec == args.steps
    # per-kernel breakdown and per-event spread: a separate, untimed pass with an event after
    # every kernel (the events cost about 2 us each, so they stay out of the timed region)
    stage_ms = None
    spread = None
    if args.breakdown_steps > 0:
        binding.timing_enable(args.breakdown_steps)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.breakdown_steps + 1)]
        marks[0].record()
        for i in range(args.breakdown_steps):
            step(i)
            marks[i + 1].record()
        torch.cuda.synchronize()
        stage_ms, _ = binding.timing_read()
        binding.timing_enable(0)
        per = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(args.breakdown_steps)])
        spread = {"median": round(float(np.median(per)), 4), "p10": round(float(np.percentile(per, 10)), 4),
                  "p90": round(float(np.percentile(per, 90)), 4), "steps": args.breakdown_steps,
                  "note": "separate pass with an event after every kernel"}
    # two independent batches in flight on two streams (own workspace and outputs each): the
    # latency-bound kernels behind the sweeps overlap the next batch's sweeps.  Reported beside
    # the serial figure, never as `value`.
    overlap_ms = None
    if not steady and copies >= 2 and args.overlap_steps > 0:
        b1 = batches[1][1]
        b1._ws = torch.empty_like(ws)
        outs1 = cask.Outputs(b1)
        lanes = [(torch.cuda.Stream(), b0, outs), (torch.cuda.Stream(), b1, outs1)]
        for n in (args.warmup, args.overlap_steps):
            torch.cuda.synchronize()
            to0 = time.perf_counter()
            for i in range(n):
                st, bb, oo = lanes[i % 2]
                with torch.cuda.stream(st):
                    cask.compress(bb, oo)
            torch.cuda.synchronize()
            overlap_ms = (time.perf_counter() - to0) * 1e3 / max(n, 1)
        b1._ws = ws
        del outs1, lanes
    graph_ms = None
    if args.graph_steps > 0:
        # the same event as one replayed HIP graph: the launch gaps between its kernels go away
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(0)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(args.graph_steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg0) * 1e3 / args.graph_steps
    step(0)   # leave the outputs of an eager event on the first input copy behind for the checks below
    torch.cuda.synchronize()
    status = outs.status.cpu().numpy()
    out_len = outs.out_len.cpu().numpy()

    # ---- consumer side (not part of the event, reported beside it): one decode step's attention
    # of the G query heads of every unit over the cache the event wrote; HBM-bound, its bytes are
    # the kept key and value rows
    consumer = None
    if args.attend_steps > 0:
        gen = torch.Generator(device=dev).manual_seed(7)
        qd = torch.randn(n_units, p.q_per_kv, p.head_dim, device=dev, generator=gen).to(outs.K_out.dtype)
        od = torch.empty_like(qd)
        cnt = torch.ones(n_units, p.budget, dtype=torch.int32, device=dev)
        for _ in range(5):
            cask.attend(p, qd, outs.K_out, outs.V_out, outs.out_len, count=cnt, out=od)
        # the kernel takes about 10 us: the timed loop calls the C entry point with arguments
        # marshalled once, so that the Python side of the binding does not set the pace
        import ctypes as C
        cp = p.c()
        call = (C.byref(cp), n_units, qd.data_ptr(), outs.K_out.data_ptr(), outs.V_out.data_ptr(),
                outs.K_out.shape[1], outs.out_len.data_ptr(), cnt.data_ptr(), cnt.shape[1], od.data_ptr(),
                torch.cuda.current_stream().cuda_stream)
        lib = cask.load()
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea.record()
        for _ in range(args.attend_steps):
            rc = lib.cask_attend(*call)
        eb.record()
        assert rc == 0
        torch.cuda.synchronize()
        att_us = ea.elapsed_time(eb) * 1e3 / args.attend_steps
        att_bytes = float(out_len.sum()) * p.head_dim * outs.K_out.element_size() * 2
        consumer = {"kernel": "cask_attend", "us": round(att_us, 2), "row_bytes": att_bytes,
                    "GB/s": round(att_bytes / att_us * 1e-3, 1),
                    "frac_of_hbm_peak": round(att_bytes / att_us * 1e-3 / PEAK_HBM_GBS, 4)}
    lens = (b0.row_off_host[1:] - b0.row_off_host[:-1]).numpy()
    saved = 1.0 - float(out_len.sum()) / float(lens.sum())
    # how much the fold path had to do: donors folded into representatives by the last event
    n_assigned = int((outs.assign >= 0).sum().item())
    folded_donors = n_assigned - int(out_len.sum())
    fold_path = {"folded_donors_per_event": folded_donors, "sim_threshold": args.sim_threshold}
    if stage_ms:
        esz = outs.K_out.element_size()
        # The grouping launch also copies K and V of every kept row; emit reads K and V of the
        # seeds that fold and of their donors and writes the folded rows: together every kept row
        # and folded donor is read and every kept row is written, over the two stages.
        moved = 2.0 * p.head_dim * esz * (n_assigned + float(out_len.sum()))
        both = stage_ms["gather"] + stage_ms["emit"]
        fold_path.update({"gather_ms": round(stage_ms["gather"], 4), "emit_ms": round(stage_ms["emit"], 4),
                          "copy_fold_row_bytes": moved,
                          "copy_fold_GB/s": round(moved / (both * 1e-3) / 1e9, 1) if both > 0 else None})

    # ---- roofline of the dominant kernel: one scoring sweep is one Q.K^T pass of
    # 2 * (W*G) * N * d flops per unit on the matrix cores
    Mq = p.q_per_kv * p.window
    flops_pass = 2.0 * Mq * float(kv_tokens) * p.head_dim
    roof = None
    if sweep_ms is not None:
        # Both sweeps are the same kernel with the same flops; sweep A's bracket holds that
        # kernel alone (sweep B's also holds the small kernel that combines the key splits),
        # so A is the one reported unless B is clearly the slower one (few window rows per
        # workgroup: the Llama-shaped batch); `both_sweeps_frac` covers the pair.
        dom = "score_cols" if sweep_ms["score_cols"] > 1.05 * sweep_ms["score_rows"] else "score_rows"
        t_dom = sweep_ms[dom] * 1e-3
        # Both sweeps as ONE launch, bracketed as the first stage (the second bracket is then
        # empty): short units (score_mfma_kernel<2>, with the one-launch tail), and many long units
        # with W*G <= 256 (score_mfma_kernel<3>).  Told from the brackets themselves.
        one_launch = w.dtype != "f32" and p.head_dim == 128 and sweep_ms["score_cols"] < 0.25 * sweep_ms["score_rows"]
        fused_name = ("score_mfma_kernel<2> (both sweeps in one launch, short units)" if int(lens.max()) <= 1024
                      else "score_mfma_kernel<3> (both sweeps in one launch)")
        passes = 2.0 if one_launch else 1.0
        achieved = passes * flops_pass / t_dom / 1e12
        # (second template argument: resident 32-row tiles per wave, 4 in the wide form the library
        # takes for these shapes, 2 in the narrow one)
        two_name = ("score_mfma_kernel<0, CT> (score_rows)" if dom == "score_rows" else
                    "score_mfma_kernel<1, CT> (score_cols; its bracket also holds the kernel that combines the key splits)")
        roof = {"bound": "mfma", "kernel": (fused_name if one_launch else two_name),
                "achieved": round(achieved, 2), "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_MFMA_BF16_TFLOPS, 4),
                "traffic": (PROFILED_TRAFFIC.get(args.workload, {}).get("bytes")
                            if args.layers == 0 and args.seqs == 0 and args.seed_dedup == 0 else None),
                "traffic_source": (PROFILED_TRAFFIC.get(args.workload, {}).get("source")
                                   if args.layers == 0 and args.seqs == 0 and args.seed_dedup == 0 else None),
                "traffic_note": "profile constant (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), not measured by this run",
                "kernel_ms": round(sweep_ms[dom], 4),
                "flops_per_launch": passes * flops_pass,
                "both_sweeps_frac": round(2 * flops_pass / ((sweep_ms["score_rows"] + sweep_ms["score_cols"]) * 1e-3)
                                          / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4),
                # whole event against its own bound: one algorithmic Q.K^T pass at MFMA peak
                "event_frac_of_one_pass_at_peak": round(flops_pass / (ms_per_step * 1e-3) / 1e12
                                                        / PEAK_MFMA_BF16_TFLOPS, 4)}
        if pinned is not None:
            roof["pinned_peaks"] = pinned
            roof["frac_of_pinned_mfma"] = round(achieved / pinned["mfma_bf16_TFLOP/s"], 4)
            roof["frac_of_pinned_mfma_with_epilogue"] = round(achieved / pinned["mfma_with_softmax_epilogue_TFLOP/s"], 4)

    # ---- CPU oracle on a bounded sample of the same units (rank 0, N = 1 only)
    cpu = None
    if args.cpu_units > 0:
        from oracle import ref
        rng = np.random.default_rng(0)
        take = min(args.cpu_units, n_units)
        pick = np.sort(rng.choice(n_units, size=take, replace=False))
        c0 = batches[0][0]
        ro = b0.row_off_host.numpy()
        Ks, Vs, Qs, sub_lens = [], [], [], []
        for u in pick:
            sl = slice(int(ro[u]), int(ro[u + 1]))
            Ks.append(c0["K"][sl].cpu())
            Vs.append(c0["V"][sl].cpu())
            Qs.append(c0["Q"][u:u + 1].cpu())
            sub_lens.append(sl.stop - sl.start)
        Kh, Vh, Qh = (caches.host_bits(torch.cat(x)) for x in (Ks, Vs, Qs))
        sub_ro = np.concatenate([[0], np.cumsum(sub_lens)]).astype(np.int64)
        sub_pl = b0.prefix_len_host.numpy()[pick]
        rp = ref.Params(dtype=p.dtype, head_dim=p.head_dim, q_per_kv=p.q_per_kv, window=p.window,
                        recent=p.recent, budget=p.budget, core=p.core, seed_dedup=p.seed_dedup,
                        sim_threshold=p.sim_threshold)
        threads = min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1, take)
        tc0 = time.perf_counter()
        want = ref.compress(rp, sub_ro, sub_pl, Kh, Vh, Qh, n_threads=threads)
        tc1 = time.perf_counter()
        cpu = {"value": round(float(sum(sub_lens)) / (tc1 - tc0), 1), "unit": "KV tokens/s",
               "cores": threads, "kind": "oracle",
               "sample": "%d of %d units of %s (%d KV tokens), %.1f s" % (take, n_units, args.workload,
                                                                          sum(sub_lens), tc1 - tc0)}
        # the sampled units double as a live parity check of this very run
        # outs holds the last step's result: recompute on copy 0 for the comparison
        cask.compress(b0, outs)
        torch.cuda.synchronize()
        got_src = outs.out_src.cpu().numpy()[pick]
        got_scores = outs.scores.cpu().numpy()
        worst = 0.0
        for k, u in enumerate(pick):
            sl = slice(int(ro[u]), int(ro[u + 1]))
            ssl = slice(int(sub_ro[k]), int(sub_ro[k + 1]))
            worst = max(worst, float(np.abs(got_scores[sl] - want["scores"][ssl]).max() / want["scores"][ssl].max()))
        cpu["parity"] = {"score_rel_err_max": worst,
                         "keep_set_equal_units": int(sum(np.array_equal(got_src[k], want["out_src"][k]) for k in range(take)))}

    value = kv_tokens / (ms_per_step * 1e-3)
    line = {
        "metric": METRIC, "value": round(value, 1), "unit": "KV tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %d layers x %d KV heads x %d seqs, G=%d, d=%d, prefix %d, decode %s, window %d, budget %d"
                   % (args.workload, n_layers, w.n_kv_heads, (args.seqs or w.n_seqs), w.q_per_kv, w.head_dim, w.prefix,
                      (str(w.decode) if w.decode_hi is None else "%d..%d" % (w.decode, w.decode_hi)), w.window, w.budget),
                   "units": n_units, "kv_tokens_per_event": kv_tokens,
                   "seq_tokens_per_s": round(value / (n_layers * w.n_kv_heads), 1),
                   "input_copies": copies, "saved_ratio": round(saved, 4), "seed_dedup": args.seed_dedup,
                   "status_counts": {str(k): int(v) for k, v in zip(*np.unique(status, return_counts=True))},
                   "stage_ms": ({k: round(v, 4) for k, v in stage_ms.items()} if stage_ms else None),
                   "event_ms_spread": spread,
                   # an event fires once per `window` decoded tokens of a sequence
                   "ms_per_decode_step_amortised": round(ms_per_step / w.window, 6),
                   "graph_ms_per_step": (round(graph_ms, 4) if graph_ms is not None else None),
                   "two_stream_ms_per_step": (round(overlap_ms, 4) if overlap_ms is not None else None),
                   "fold_path": fold_path,
                   "consumer_attend": consumer},
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
