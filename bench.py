#!/usr/bin/env python3
"""Benchmark of the OSP synchronization step on one MI355X.

One "step" is the whole hot path over one batch of synthetic gradients, in the
paper's order (Sec. 3.1; Eq. 5 ordering):
    osp_ps_aggregate_update(1) -> osp_apply_stage(1) -> osp_lgp_correct ->
    osp_ps_aggregate_update(2) -> osp_apply_stage(2) -> osp_split
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

Two byte counts appear side by side.

`value` (the metric) is computed on the ALGORITHMIC bytes of a step as the metric defines
them, the traffic of the six calls each taken on its own (E1 + E2 = M parameters, E2 =
stage-2 elements in effect during the step, N workers):
    aggregate+update  4 (N + 4) E_s     per stage  (N grads + P + V read, P + V written)
    apply_stage       4 (N + 1) E_s     per stage  (P read once, N replicas written)
    lgp_correct       12 N E2                      (P_w and g_w read, P_w written)
    split (layer)     0                            (a few hundred KB of partials)
    split (element)   4 M + M/8  (+ 4 M key writes inside aggregate+update)
It is a throughput in units of that work, not a bandwidth: the implementation moves fewer
bytes than the six calls taken one by one would (LGP reads the stale stage-2 values once from
the PS arena instead of once per replica and leaves the aggregate of the stage-2 gradients it
reads for the stage-2 call; the element-granular windows are single passes).

`GB_moved_per_step`, `GBps_on_bytes_moved`, `pct_hbm_peak` and the per-call `GBps` use the
bytes the launches of this implementation have to move (moved_bytes below); these are the
figures to hold against the 8 TB/s of the HBM and against the copy rate of the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
BRACKET_EVERY = 4               # steps between two event-bracketed steps of the timed region

# HBM bytes per launch as rocprofv3 counted them (two --pmc runs, FETCH_SIZE and WRITE_SIZE in
# KiB per dispatch, FETCH_SIZE scaled by 2.0 and WRITE_SIZE by 1.0: what each reads for the
# 2 GiB k_stream_copy).  Taken from the committed summaries, NOT measured by this run; only
# reported for the workload and launch configuration they were taken on.
PROFILED_TRAFFIC = {
    # (workload, granularity, kernel): (bytes per launch in the timed region, summary)
    ("vgg16", "layer", "k_aggregate_update"):
        (8235800000, "profiles/sync_step_vgg16_layer.txt"),
    ("vgg16", "element", "k_rs_window_element"):
        (21136400000, "profiles/sync_step_vgg16_element.txt"),
}


def step_bytes(N, M, E2, element, gb=4):
    """The metric's algorithmic bytes per call; gb = bytes per stored gradient element (4, or
    2 for bfloat16)."""
    E1 = M - E2
    b = {
        "agg1": (gb * N + 16) * E1, "apply1": 4 * (N + 1) * E1, "lgp": (8 + gb) * N * E2,
        "agg2": (gb * N + 16) * E2, "apply2": 4 * (N + 1) * E2, "split": 0,
    }
    if element:
        b["agg1"] += 4 * E1
        b["agg2"] += 4 * E2
        b["split"] = 4 * M + M // 8
    b["rs_window"] = b["agg1"] + b["apply1"] + b["lgp"]
    b["ics_window"] = b["agg2"] + b["apply2"] + b["split"]
    b["split_gradients"] = 2 * gb * N * M   # every gradient read once, written once
    return b


def moved_bytes(N, M, E2, element, gb, lgp_shared, lgp_kept, fused_rs, fused_ics):
    """HBM bytes the launches behind each call have to move in this implementation (what a
    traffic counter sees, up to a fraction of a per cent of table and bitmap reads).
    Layer granularity: stage tables, so a call touches its stage's elements only.  LGP with
    the replicas in sync reads the stale values from the PS arena (once per 8 MB block, the
    other replicas' sweeps hit in cache); when it also keeps the stage-2 aggregate it writes
    4 E2 more and the stage-2 call reads P, V and that aggregate (20 E2 in all).
    Element granularity: a scattered half of the elements touches every 16-byte group, so
    every call is a pass over whole arenas of M elements (bitmap: M/8)."""
    E1 = M - E2
    b = {}
    if not element:
        b["agg1"] = (gb * N + 16) * E1
        b["apply1"] = 4 * (N + 1) * E1
        b["lgp"] = ((gb + 4) * N + 8) * E2 if lgp_kept else \
                   ((gb + 4) * N + 4) * E2 if lgp_shared else (8 + gb) * N * E2
        b["agg2"] = 20 * E2 if lgp_kept else (gb * N + 16) * E2
        b["apply2"] = 4 * (N + 1) * E2
        b["split"] = 0
        if fused_rs:        # one launch: aggregate workgroups write the replicas themselves
            b["rs_window"] = (gb * N + 16 + 4 * N) * E1 + ((gb + 4) * N + 4) * E2
        else:
            b["rs_window"] = b["agg1"] + b["apply1"] + b["lgp"]
        b["ics_window"] = (gb * N + 16 + 4 * N) * E2 if fused_ics else b["agg2"] + b["apply2"]
    else:
        bm = M // 8
        b["agg1"] = (gb * N + 8 + 16) * M + bm          # P, V, key and kept aggregate written
        b["apply1"] = 4 * (N + 1) * M
        b["lgp"] = ((gb + 4) * N + 4) * M + bm if lgp_shared else (8 + gb) * N * M + bm
        b["agg2"] = 20 * M + bm                          # from the kept aggregate
        b["apply2"] = 4 * (N + 1) * M
        # one histogram pass + the bitmap pass: the first pass also counts the second digit
        # under the previous split's first digit, and in a run of steps that guess holds (a
        # step whose threshold leaves that bucket reads the keys a third time)
        b["split"] = 2 * 4 * M + bm
        b["rs_window"] = ((gb * N + 8) * M + bm + (16 + 4 * N) * M if fused_rs
                          else b["agg1"] + b["apply1"] + b["lgp"])
        b["ics_window"] = (12 * M + bm + (8 + 4 * N) * M if fused_ics
                           else b["agg2"] + b["apply2"]) + b["split"]
    b["split_gradients"] = 2 * gb * N * M
    return b


def step_calls(mode, c, stride, gran, budget, dense, bf16=False):
    """One sync step as a list of (name, call(g)); names index step_bytes()."""
    if bf16 and mode == "packed":
        gi, gu, ds = dense
        return [("split_gradients", lambda g: c.osp_split_gradients_bf16(g, stride, gi, ds, gu, ds)),
                ("agg1", lambda g: c.osp_ps_aggregate_update_packed_bf16(1, gi, ds)),
                ("apply1", lambda g: c.osp_apply_stage(1)),
                ("lgp", lambda g: c.osp_lgp_correct_bf16(g, stride)),
                ("agg2", lambda g: c.osp_ps_aggregate_update_packed_bf16(2, gu, ds)),
                ("apply2", lambda g: c.osp_apply_stage(2)),
                ("split", lambda g: c.osp_split(gran, budget))]
    if bf16 and mode == "windows":
        return [("rs_window", lambda g: c.osp_rs_window_bf16(g, stride)),
                ("ics_window", lambda g: c.osp_ics_window_bf16(g, stride, gran, budget))]
    if bf16:
        return [("agg1", lambda g: c.osp_ps_aggregate_update_bf16(1, g, stride)),
                ("apply1", lambda g: c.osp_apply_stage(1)),
                ("lgp", lambda g: c.osp_lgp_correct_bf16(g, stride)),
                ("agg2", lambda g: c.osp_ps_aggregate_update_bf16(2, g, stride)),
                ("apply2", lambda g: c.osp_apply_stage(2)),
                ("split", lambda g: c.osp_split(gran, budget))]
    if mode == "windows":
        return [("rs_window", lambda g: c.osp_rs_window(g, stride)),
                ("ics_window", lambda g: c.osp_ics_window(g, stride, gran, budget))]
    six = [("agg1", lambda g: c.osp_ps_aggregate_update(1, g, stride)),
           ("apply1", lambda g: c.osp_apply_stage(1)),
           ("lgp", lambda g: c.osp_lgp_correct(g, stride)),
           ("agg2", lambda g: c.osp_ps_aggregate_update(2, g, stride)),
           ("apply2", lambda g: c.osp_apply_stage(2)),
           ("split", lambda g: c.osp_split(gran, budget))]
    if mode == "six":
        return six
    gi, gu, ds = dense                          # the PS is fed by the splitter's dense parts
    six[0] = ("agg1", lambda g: c.osp_ps_aggregate_update_packed(1, gi, ds))
    six[3] = ("agg2", lambda g: c.osp_ps_aggregate_update_packed(2, gu, ds))
    return [("split_gradients", lambda g: c.osp_split_gradients(g, stride, gi, ds, gu, ds))] + six


BRACKETED = {"six": ("agg1", "agg2"), "windows": ("rs_window",), "packed": ("split_gradients",)}


def run_leg(torch, wl, job, gsets, element, mode, K, Wm, graph, bf16, keep_on, log):
    """Warm up, time K whole steps, then a second pass with every call bracketed.  Returns the
    measurements and the list of steps run (which gradient set each used), so that the oracle
    can be taken through the same chain afterwards."""
    c = job.ctx
    N, M = wl.n_workers, wl.n_params
    stride = wl.worker_stride()
    gran = 1 if element else 0
    gb = 2 if bf16 else 4
    c.osp_set_keep_stage2_aggregate(keep_on)
    c.osp_set_gib(0, np.ones(wl.n_tensors, np.uint8))     # iteration 1 is BSP (Algorithm 1)
    dense = None
    if mode == "packed":
        ds = -(-M // 64) * 64 + 64
        dense_dtype = torch.int16 if bf16 else torch.float32
        dense = (torch.empty((N, ds), dtype=dense_dtype, device="cuda"),
                 torch.empty((N, ds), dtype=dense_dtype, device="cuda"), ds)
    calls_of_step = step_calls(mode, c, stride, gran, wl.budget, dense, bf16)
    names = [n for n, _ in calls_of_step]
    K2 = min(K, 10)
    total_steps = Wm + K + K2
    # stage-2 size in effect during each step: every split appends the size it chose to a log in
    # device memory (no stream operation per step, and no call in the loop waits for the GPU: the
    # host runs ahead of it); step 0 runs on the all-important GIB set above
    n2_log = torch.zeros(total_steps, dtype=torch.int64, device="cuda")
    c.osp_set_stage2_log(n2_log)
    history = []

    def enqueue_step(i, e=None):
        g = gsets[i % 2]
        for name, call in calls_of_step:
            if e is not None and name in e:
                e[name][0].record(); call(g); e[name][1].record()
            else:
                call(g)
        history.append(i % 2)

    for i in range(Wm):
        enqueue_step(i)
    # Timed region: K whole steps.  Inside it only the dominant kernel (six calls: the aggregate;
    # windows: the RS window; packed: the splitter) is bracketed by events, on the stream it is
    # launched on, and only in every BRACKET_EVERY-th step: an event record between two kernels
    # costs about 5 us of idle GPU.  The per-call breakdown of the other calls comes from a
    # second pass after the timed region.
    bracketed = BRACKETED[mode]
    # LGP over a layer-granular stage 2 keeps the stage-2 aggregate (the warm-up steps have shown
    # whether it does): the stage-2 call is then a short pass over the kept values and the
    # aggregate kernel is launched once per step, on stage 1
    lgp_kept = bool(mode == "six" and c.osp_lgp_kept_aggregate())
    windows = mode == "windows"
    if lgp_kept:
        bracketed = ("agg1",)
    ev = [{n: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for n in bracketed} if i % BRACKET_EVERY == 0 else None for i in range(K)]
    graphs = None
    if graph:
        torch.cuda.synchronize()
        graphs = []
        for gset in gsets:                       # one graph per gradient set; capture runs nothing
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                for _, call in calls_of_step:
                    call(gset)
            graphs.append(gr)
        ev = [None] * K                          # events cannot sit between the nodes of a graph
    torch.cuda.synchronize()

    t_start = time.perf_counter()
    for i in range(K):
        if graphs:
            graphs[(Wm + i) % 2].replay()
            history.append((Wm + i) % 2)
        else:
            enqueue_step(Wm + i, ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    lgp_shared = bool(c.osp_lgp_read_shared())
    wf = c.osp_windows_fused() if windows else 0
    fused_rs, fused_ics = bool(wf & 1), bool(wf & 2)
    if windows and not element and not fused_rs:    # the single-stage kernels ran inside the windows
        lgp_kept = bool(c.osp_lgp_kept_aggregate())
    n2_all = [0] + [int(x) for x in n2_log.cpu()]       # entry i: stage-2 size during step i
    n2 = n2_all[Wm:Wm + K]
    total_bytes = total_moved = 0
    dom_ms = 0.0
    dom_bytes = dom_moved = dom_launches = 0
    for i in range(K):
        b = step_bytes(N, M, n2[i], element, gb)
        mv = moved_bytes(N, M, n2[i], element, gb, lgp_shared, lgp_kept, fused_rs, fused_ics)
        total_bytes += sum(b[n] for n in names)
        total_moved += sum(mv[n] for n in names)
        if not ev[i]:
            continue
        for n in bracketed:
            dom_ms += ev[i][n][0].elapsed_time(ev[i][n][1])
            dom_bytes += b[n]
            dom_moved += mv[n]
            dom_launches += 1
    if mode == "packed":                          # the packed aggregate's traffic is not itemised
        total_moved = None

    # second pass (not part of `value`): every call bracketed, for the per-call breakdown
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls_of_step) + 1)]
           for _ in range(K2)]
    for i in range(K2):
        g = gsets[(Wm + K + i) % 2]
        e = ev2[i]
        for j, (_, call) in enumerate(calls_of_step):
            e[j].record(); call(g)
        e[len(calls_of_step)].record()
        history.append((Wm + K + i) % 2)
    torch.cuda.synchronize()
    n2_all = [0] + [int(x) for x in n2_log.cpu()]
    c.osp_set_stage2_log(None)
    call_ms = {n: 0.0 for n in names}
    call_bytes = {n: 0 for n in names}
    call_moved = {n: 0 for n in names}
    for i in range(K2):
        e2 = n2_all[Wm + K + i]
        b = step_bytes(N, M, e2, element, gb)
        mv = moved_bytes(N, M, e2, element, gb, lgp_shared, lgp_kept, fused_rs, fused_ics)
        for j, n in enumerate(names):
            call_ms[n] += ev2[i][j].elapsed_time(ev2[i][j + 1])
            call_bytes[n] += b[n]
            call_moved[n] += mv[n]

    # dominant kernel: the longest launch of a step
    kernel = ("k_aggregate_update" if mode == "six" else
              "k_split_gradients" if mode == "packed" else
              ("k_rs_window_element" if element else "k_window_layer") if fused_rs else
              "osp_rs_window (three single-stage kernels)")
    note = None
    if dom_launches == 0:                         # graph replay: events cannot sit inside a graph
        n0 = bracketed[0]
        dom_ms, dom_bytes, dom_moved, dom_launches = call_ms[n0], call_bytes[n0], call_moved[n0], K2
        note = "taken from the eager second pass (events cannot sit inside a graph)"
    avg_ms = dom_ms / dom_launches
    ach = dom_bytes / dom_launches / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    ach_moved = dom_moved / dom_launches / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    prof = PROFILED_TRAFFIC.get((wl.name, "element" if element else "layer", kernel))
    use_prof = (prof is not None and c.osp_chunk_elems() == 256 and not bf16 and
                (element or lgp_kept))
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                "traffic": prof[0] if use_prof else None,
                "traffic_from": (prof[1] + " (rocprofv3 --pmc; not measured by this run)"
                                 if use_prof else None),
                "launches": dom_launches, "avg_launch_ms": round(avg_ms, 5),
                "bytes_per_launch": int(dom_bytes / dom_launches),
                "bytes_moved_per_launch": int(dom_moved / dom_launches),
                "frac_on_bytes_moved": round(ach_moved / HBM_PEAK_GBPS, 4)}
    if note:
        roofline["note"] = note

    def rate(nbytes, ms):
        return round(nbytes / (ms * 1e-3) / 1e9, 1) if ms > 0 else None

    # the kernels that share the step's time with the dominant one, on the bytes they move
    others = None
    if mode == "six" and not element:
        inst_ms = call_ms["apply1"] + call_ms["apply2"]
        inst_b = call_moved["apply1"] + call_moved["apply2"]
        lgp_kernel = "k_lgp_keep" if lgp_kept else "k_lgp_sweep" if lgp_shared else "k_lgp_correct"
        others = [
            {"kernel": "k_apply_stage (two launches per step)", "achieved": rate(inst_b, inst_ms),
             "frac": round((rate(inst_b, inst_ms) or 0.0) / HBM_PEAK_GBPS, 4),
             "ms_per_step": round(inst_ms / K2, 5)},
            {"kernel": lgp_kernel, "achieved": rate(call_moved["lgp"], call_ms["lgp"]),
             "frac": round((rate(call_moved["lgp"], call_ms["lgp"]) or 0.0) / HBM_PEAK_GBPS, 4),
             "ms_per_step": round(call_ms["lgp"] / K2, 5)}]
        if lgp_kept:
            others.append(
                {"kernel": "k_update_from_stash", "achieved": rate(call_moved["agg2"], call_ms["agg2"]),
                 "frac": round((rate(call_moved["agg2"], call_ms["agg2"]) or 0.0) / HBM_PEAK_GBPS, 4),
                 "ms_per_step": round(call_ms["agg2"] / K2, 5)})
    calls = {n: {"ms": round(call_ms[n] / K2, 5),
                 "GBps": rate(call_moved[n], call_ms[n]) if mode != "packed" else None,
                 "GBps_on_metric_bytes": rate(call_bytes[n], call_ms[n])}
             for n in names}
    gbps = total_bytes / elapsed / 1e9
    moved_gbps = None if total_moved is None else total_moved / elapsed / 1e9
    return {
        "ms_per_step": elapsed * 1e3 / K, "elapsed": elapsed, "value": gbps,
        "GB_per_step": total_bytes / K / 1e9,
        "GB_moved_per_step": None if total_moved is None else total_moved / K / 1e9,
        "GBps_on_bytes_moved": moved_gbps,
        "lgp_shared": lgp_shared, "lgp_kept": lgp_kept, "fused_rs": fused_rs, "fused_ics": fused_ics,
        "stage2_elems": n2[K - 1], "calls": calls, "roofline": roofline, "others": others,
        "history": history, "n2_end": n2_all[total_steps],
    }


def reference_lines(torch, gsets, N, stride, arena, bf16):
    """Two live reference lines on the same box: the library's plain streaming copy of 2 GiB
    (also the known-size kernel the rocprofv3 traffic counters are calibrated against), and
    the traffic of the aggregate's shape without its arithmetic (N streams read, two streams
    read and written back) on this run's own gradient arenas."""
    from paper_2306_16926_amd.binding import osp_stream_copy, osp_stream_pattern
    src = torch.empty(1 << 29, dtype=torch.float32, device="cuda"); dst = torch.empty_like(src)
    src.fill_(1.0)
    osp_stream_copy(dst, src, src.numel() * 4)
    a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(); a.record()
    for _ in range(10):
        osp_stream_copy(dst, src, src.numel() * 4)
    b2.record(); torch.cuda.synchronize()
    copy_gbps = 10 * 2 * src.numel() * 4 / (a.elapsed_time(b2) * 1e-3) / 1e9
    assert bool((dst[:1024] == 1.0).all()) and bool((dst[-1024:] == 1.0).all())
    del src, dst
    pattern_gbps = None
    if not bf16:
        rw = torch.zeros((2, stride), dtype=torch.float32, device="cuda")
        osp_stream_pattern(gsets[0], N, stride, rw, 2, stride, arena)
        torch.cuda.synchronize(); a.record()
        for r in range(6):
            osp_stream_pattern(gsets[r % 2], N, stride, rw, 2, stride, arena)
        b2.record(); torch.cuda.synchronize()
        pattern_gbps = 6 * 4 * (N + 4) * arena / (a.elapsed_time(b2) * 1e-3) / 1e9
        del rw
    return copy_gbps, pattern_gbps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16",
                    choices=["tiny", "resnet18", "resnet50", "resnet152", "vgg16", "bert_base"])
    ap.add_argument("--granularity", default="layer", choices=["layer", "element"])
    ap.add_argument("--calls", default="six", choices=["six", "windows", "packed"],
                    help="six single-stage calls per step, the RS and ICS window calls, or the "
                         "gradient splitter followed by the six calls with the PS fed by its dense parts")
    ap.add_argument("--grad-dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of the gradient arenas (and of the splitter's dense parts)")
    ap.add_argument("--keep-stage2-aggregate", default="on", choices=["on", "off"],
                    help="layer granularity: LGP leaves the aggregate of the stage-2 gradients for "
                         "the stage-2 call (library default) or every call reads what it needs")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step as a captured HIP graph (six calls or windows; no call "
                         "of a step needs the host)")
    ap.add_argument("--element-leg", default="auto", choices=["auto", "on", "off"],
                    help="also measure the element-granular step (window calls) of the same workload "
                         "in this process and report it under \"element\"; auto: when the main run is "
                         "the default layer-granular one")
    ap.add_argument("--element-steps", type=int, default=6)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--chunk-elems", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the CPU oracle (baseline timing and the parity verdict)")
    ap.add_argument("--gen-threads", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: all N simulated workers' buffers are "
              "resident on one MI355X and there is no multi-GPU path; use --gpus 1",
              file=sys.stderr)
        return 2
    if args.graph and (args.calls == "packed" or args.warmup < 2):
        print("bench.py: --graph needs --calls six or windows and --warmup >= 2", file=sys.stderr)
        return 2

    import torch
    from paper_2306_16926_amd import workloads as W
    from paper_2306_16926_amd.device import DeviceJob

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    wl = W.get(args.workload)
    element = args.granularity == "element"
    N, M = wl.n_workers, wl.n_params
    arena, stride, pstride = wl.arena_elems(), wl.worker_stride(), wl.replica_stride()
    K, Wm = args.steps, args.warmup
    bf16 = args.grad_dtype == "bf16"
    keep_on = args.keep_stage2_aggregate == "on"
    element_leg = (args.element_leg == "on" or
                   (args.element_leg == "auto" and not element and args.calls == "six" and
                    not bf16 and not args.graph and keep_on and args.workload != "tiny"))

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    t0 = time.time()
    params = wl.make_params(args.seed)
    # two gradient sets, alternated, so a step never re-reads what the last one left in cache
    host_sets = [wl.make_grads(args.seed, s, stride=stride, threads=args.gen_threads) for s in (0, 1)]
    job = DeviceJob(wl.numel, wl.offsets(), arena, N, wl.lr, wl.momentum, params,
                    element_keys=element, chunk_elems=args.chunk_elems, param_stride=pstride)
    if bf16:                                    # rounded once, on the host; the oracle gets the widened values
        halves = [W.to_bf16(h) for h in host_sets]
        host_sets = [W.from_bf16(h) for h in halves]
        gsets = [job.upload_grads_bf16(h) for h in halves]
        del halves
    else:
        gsets = [job.upload_grads(h) for h in host_sets]
    if args.no_cpu_baseline:
        host_sets = None
    log(f"{wl.name}: N={N} L={wl.n_tensors} M={M} inputs ready in {time.time()-t0:.1f}s")

    leg = run_leg(torch, wl, job, gsets, element, args.calls, K, Wm, args.graph, bf16, keep_on, log)
    log(f"main leg: {leg['ms_per_step']:.4f} ms per step")
    copy_gbps, pattern_gbps = reference_lines(torch, gsets, N, stride, arena, bf16)

    cpu = parity = None
    if not args.no_cpu_baseline:
        cpu, parity = cpu_baseline(wl, params, host_sets, job, leg["history"], element, stride, log)
    chunk = job.ctx.osp_chunk_elems()

    element_out = None
    if element_leg:
        del job
        torch.cuda.empty_cache()
        job = DeviceJob(wl.numel, wl.offsets(), arena, N, wl.lr, wl.momentum, params,
                        element_keys=True, chunk_elems=args.chunk_elems, param_stride=pstride)
        eleg = run_leg(torch, wl, job, gsets, True, "windows", args.element_steps, 3, False, False,
                       True, log)
        log(f"element leg: {eleg['ms_per_step']:.4f} ms per step")
        eparity = None
        if not args.no_cpu_baseline:
            _, eparity = cpu_baseline(wl, params, host_sets, job, eleg["history"], True, stride, log,
                                      baseline=False)
        element_out = leg_summary(eleg, args.element_steps, 3)
        element_out.update({"granularity": "element", "calls": "windows", "parity": eparity,
                            "roofline": eleg["roofline"]})

    out = {
        "metric": "osp_sync_step_GBps", "value": round(leg["value"], 1), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(leg["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "f32 (gradients stored as bf16)", "data": "synthetic",
        "config": {"workload": f"{wl.name}-shaped", "n_workers": N, "n_tensors": wl.n_tensors,
                   "n_params": M, "granularity": args.granularity, "calls": args.calls,
                   "keep_stage2_aggregate": keep_on, "graph_replay": bool(args.graph),
                   "windows_fused": ({"rs": leg["fused_rs"], "ics": leg["fused_ics"]}
                                     if args.calls == "windows" else None),
                   "stage2_fraction_nominal": wl.stage2_fraction,
                   "stage2_elems_achieved": leg["stage2_elems"], "lr": wl.lr, "momentum": wl.momentum,
                   "seed": args.seed, "chunk_elems": chunk},
        "value_is": "throughput on the metric's algorithmic bytes (six calls taken one by one); "
                    "not a bandwidth, see GBps_on_bytes_moved and pct_hbm_peak",
    }
    out.update(leg_summary(leg, K, Wm))
    out.update({
        "calls_second_pass": leg["calls"],
        "copy_GBps_same_box": round(copy_gbps, 1),
        "aggregate_pattern_GBps_same_box": None if pattern_gbps is None else round(pattern_gbps, 1),
        "roofline": leg["roofline"], "roofline_other": leg["others"],
        "parity": parity, "element": element_out,
        "cpu_baseline": cpu,
        "paper_context": "paper reports up to 50% end-to-end training throughput gain on 8xT4 "
                         "workers + 1 PS over 10 Gbps Ethernet; it never times this arithmetic",
    })
    print(json.dumps(out))
    return 0


def leg_summary(leg, K, Wm):
    moved = leg["GBps_on_bytes_moved"]
    return {
        "ms_per_step": round(leg["ms_per_step"], 4), "steps": K, "warmup": Wm,
        "sync_steps_per_s": round(K / leg["elapsed"], 2),
        "GBps_on_metric_bytes": round(leg["value"], 1),
        "pct_of_8TBps_on_metric_bytes": round(100.0 * leg["value"] / HBM_PEAK_GBPS, 2),
        "GB_per_step": round(leg["GB_per_step"], 4),
        "GB_moved_per_step": None if moved is None else round(leg["GB_moved_per_step"], 4),
        "GBps_on_bytes_moved": None if moved is None else round(moved, 1),
        "pct_hbm_peak": None if moved is None else round(100.0 * moved / HBM_PEAK_GBPS, 2),
        "lgp_reads_ps_once": leg["lgp_shared"], "lgp_keeps_stage2_aggregate": leg["lgp_kept"],
        "stage2_elems_achieved": leg["stage2_elems"],
    }


def cpu_baseline(wl, params, host_sets, job, history, element, stride, log, baseline=True):
    """The CPU oracle on this machine's host cores, and the parity verdict of the run.

    Parity: the oracle (the OpenMP build of its loops, which a CPU test shows to be
    bit-identical to the serial one) starts from the same initial parameters and is taken
    through every step the GPU ran in this leg (warm-up, timed region and second pass: the
    same gradient set per step, the same budget, the GIB carried over); then P, V, every
    replica and the GIB are compared.  Nothing the GPU computed enters the oracle.  At element
    granularity the oracle cuts by selection on its own keys (its full sort takes minutes at
    these sizes; a CPU test pins the selection to the sort).
    Baseline (the metric's unit, GB/s on the metric's bytes): the serial oracle as it stands
    on the first steps of the same chain, about 10 s of work, median of the staged steps; the
    OpenMP figure is the median over the whole chain."""
    from oracle.osp_oracle import OracleOSP
    N, M = wl.n_workers, wl.n_params
    gran = 1 if element else 0
    all1 = np.ones(wl.n_tensors, np.uint8)

    def chain(omp, steps, budget_s=None):
        o = OracleOSP(wl.numel, wl.offsets(), wl.arena_elems(), N, wl.lr, wl.momentum,
                      param_stride=wl.replica_stride(), omp=omp)
        o.load_params(params)
        o.set_gib(0, all1)
        times = []
        t_all = time.perf_counter()
        for i, s in enumerate(history[:steps]):
            e2 = o.n_stage2
            t = time.perf_counter()
            o.sync_step(host_sets[s], gran, wl.budget, element_by_selection=True)
            dt = time.perf_counter() - t
            b = step_bytes(N, M, e2, element)
            six = ("agg1", "apply1", "lgp", "agg2", "apply2", "split")
            times.append((dt, sum(b[n] for n in six), e2))
            if budget_s is not None and time.perf_counter() - t_all > budget_s and i >= 2:
                break
        return o, times

    def median_rate(times):
        staged = [t for t in times if t[2] > 0] or times     # (the first step is a BSP step)
        staged.sort(key=lambda t: t[0])
        dt, nbytes, _ = staged[len(staged) // 2]
        return dt, nbytes / dt / 1e9, len(staged)

    t0 = time.time()
    o, times = chain(True, len(history))
    log(f"oracle (OpenMP) through {len(history)} steps in {time.time()-t0:.1f}s")
    P, V, Pw = job.download()
    layer, bits, n2 = job.ctx.osp_get_gib()
    arena = o.arena
    same = {"P": bool(np.array_equal(P, o.P, equal_nan=True)),
            "V": bool(np.array_equal(V, o.V, equal_nan=True)),
            "replicas": all(bool(np.array_equal(Pw[w, :arena], o.Pw[w, :arena], equal_nan=True))
                            for w in range(N))}
    worst = 0.0
    if not all(same.values()):
        for got, want in ((P, o.P), (V, o.V), (Pw[:, :arena], o.Pw[:, :arena])):
            d = np.abs(got.astype(np.float64) - want.astype(np.float64))
            worst = max(worst, float(np.nanmax(d / np.maximum(np.abs(want), 1e-30))))
    gib_equal = bool(np.array_equal(bits, o.gib_bits) if element else np.array_equal(layer, o.gib_layer))
    parity = {"against": "CPU oracle (OpenMP build of the same loops), from the same initial state "
                         "through every step of this leg",
              "steps_chained": len(history),
              "state": "bit-identical" if all(same.values()) else "differs",
              "max_rel_err": worst, "gib": "equal" if gib_equal and n2 == o.n_stage2 else "differs",
              "n_stage2": int(n2)}
    del P, V, Pw
    if not baseline:
        return None, parity
    omp_dt, omp_rate, omp_n = median_rate(times)
    o1, times1 = chain(False, len(history), budget_s=8.0)
    dt1, rate1, n1 = median_rate(times1)
    # the serial and the OpenMP build agree on the steps both ran
    o_chk, _ = chain(True, len(times1))
    serial_equals_omp = bool(np.array_equal(o1.P, o_chk.P, equal_nan=True) and
                             np.array_equal(o1.Pw, o_chk.Pw, equal_nan=True))
    try:
        cores_all = len(os.sched_getaffinity(0))
    except AttributeError:
        cores_all = os.cpu_count()
    omp_threads = int(os.environ.get("OMP_NUM_THREADS", cores_all))
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    cpu = {"value": round(rate1, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"the first {len(times1)} sync steps of this run's chain on {wl.name}-shaped "
                     f"(median of the {n1} staged ones; the element split by selection)",
           "ms_per_step": round(dt1 * 1e3, 1),
           "all_cores": {"value": round(omp_rate, 3), "cores": min(omp_threads, cores_all),
                         "ms_per_step": round(omp_dt * 1e3, 1), "steps": omp_n,
                         "bit_identical_to_serial": serial_equals_omp},
           "cpu": model}
    return cpu, parity


if __name__ == "__main__":
    sys.exit(main())
