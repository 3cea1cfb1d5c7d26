#!/usr/bin/env python3
"""Benchmark of the OSP synchronization step on one MI355X.

One "step" is the whole hot path over one batch of synthetic gradients, in the
paper's order (Sec. 3.1; Eq. 5 ordering):
    osp_ps_aggregate_update(1) -> osp_apply_stage(1) -> osp_lgp_correct ->
    osp_ps_aggregate_update(2) -> osp_apply_stage(2) -> osp_split
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

`value` is computed on the ALGORITHMIC bytes of a step as the metric defines them
(E1 + E2 = M parameters, E2 = stage-2 elements in effect during the step, N workers);
`GBps_on_bytes_moved` uses the smaller byte count the step really needs when LGP
reads the stale stage-2 values once from the PS instead of once per replica
(4 (N-1) E2 bytes less) and, with a layer-granular GIB, keeps the aggregate of the stage-2
gradients it reads anyway, so that the stage-2 call does not read the N arenas again
((8 N - 12) E2 bytes less in all, see bytes_not_moved):
    aggregate+update  4 (N + 4) E_s     per stage  (N grads + P + V read, P + V written)
    apply_stage       4 (N + 1) E_s     per stage  (P read once, N replicas written)
    lgp_correct       12 N E2                      (P_w and g_w read, P_w written)
    split (layer)     0                            (a few hundred KB of partials)
    split (element)   4 M + M/8  (+ 4 M key writes inside aggregate+update)
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

# HBM bytes per launch of k_aggregate_update on the default workload (VGG-16-shaped, layer
# granularity, chunk 256; one launch per step, on stage 1: LGP keeps the stage-2 aggregate), from
# the two rocprofv3 --pmc runs summarised in profiles/sync_step_traffic_vgg16_layer.txt:
# (7226993 + 815368) KiB, FETCH_SIZE scaled by 2.0 and WRITE_SIZE by 1.0 (what each reads for
# the 2 GiB k_stream_copy).  Algorithmic: 4 (N + 4) E1 = 8220835840.
AGG_TRAFFIC_VGG16_LAYER = (7226993 + 815368) * 1024
# HBM bytes per launch of k_rs_window_element on VGG-16-shaped, element granularity, --calls windows,
# from profiles/window_kernels_vgg16_element.txt: (9797972 + 10844502) KiB.  The launch does the work the
# metric counts as stage-1 aggregate + install + LGP (30.4 GB) in one pass over 21.2 GB.
RS_TRAFFIC_VGG16_ELEMENT = 21137893376


def step_bytes(N, M, E2, element, gb=4):
    """Algorithmic bytes per call; gb = bytes per stored gradient element (4, or 2 for bfloat16)."""
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


def bytes_not_moved(N, E2, gb, lgp_shared, lgp_kept):
    """What a layer-granular step moves less than the metric's byte count credits it with.
    LGP reading the stale values once from the PS arena instead of once per replica:
    4 (N-1) E2.  LGP that also keeps the stage-2 aggregate (reads N gradients + P, writes N
    replicas + the aggregate; the stage-2 call then reads P, V and the aggregate and writes P, V):
    the metric's (8 + gb) N E2 + (gb N + 16) E2 against (gb N + 4 + 4 N + 4) E2 + 20 E2."""
    if lgp_kept:
        return ((8 + gb) * N + gb * N + 16) * E2 - ((gb + 4) * N + 8 + 20) * E2
    if lgp_shared:
        return 4 * (N - 1) * E2
    return 0


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
                    help="replay each step as a captured HIP graph (element granularity with "
                         "--calls windows only: no call of such a step needs the host)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--chunk-elems", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-threads", type=int, default=16)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: all N simulated workers' buffers are "
              "resident on one MI355X and there is no multi-GPU path; use --gpus 1",
              file=sys.stderr)
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
    gran = 1 if element else 0
    N, M = wl.n_workers, wl.n_params
    arena, stride = wl.arena_elems(), wl.worker_stride()
    K, Wm = args.steps, args.warmup

    t0 = time.time()
    params = wl.make_params(args.seed)
    job = DeviceJob(wl.numel, wl.offsets(), arena, N, wl.lr, wl.momentum, params,
                    element_keys=element, chunk_elems=args.chunk_elems, param_stride=stride)
    # two gradient sets, alternated, so a step never re-reads what the last one left in cache
    host_g0 = wl.make_grads(args.seed, 0, stride=stride, threads=args.gen_threads)
    bf16 = args.grad_dtype == "bf16"
    gb = 2 if bf16 else 4
    if bf16:                                    # rounded once, on the host; the oracle leg gets the widened values
        h = W.to_bf16(host_g0)
        host_g0 = W.from_bf16(h)
        gsets = [job.upload_grads_bf16(h)]
        gsets.append(job.upload_grads_bf16(W.to_bf16(
            wl.make_grads(args.seed, 1, stride=stride, threads=args.gen_threads))))
        del h
    else:
        gsets = [job.upload_grads(host_g0)]
        tmp = wl.make_grads(args.seed, 1, stride=stride, threads=args.gen_threads)
        gsets.append(job.upload_grads(tmp))
        del tmp
    print(f"[bench] {wl.name}: N={N} L={wl.n_tensors} M={M} inputs ready in {time.time()-t0:.1f}s",
          file=sys.stderr, flush=True)

    c = job.ctx
    c.osp_set_keep_stage2_aggregate(args.keep_stage2_aggregate == "on")
    c.osp_set_gib(0, np.ones(wl.n_tensors, np.uint8))     # iteration 1 is BSP (Algorithm 1)
    n2_log = np.zeros(K, dtype=np.int64)
    windows = args.calls == "windows"
    mode = args.calls
    dense = None
    if mode == "packed":
        ds = -(-M // 64) * 64 + 64
        dense_dtype = torch.int16 if bf16 else torch.float32
        dense = (torch.empty((N, ds), dtype=dense_dtype, device="cuda"),
                 torch.empty((N, ds), dtype=dense_dtype, device="cuda"), ds)
    calls_of_step = step_calls(mode, c, stride, gran, wl.budget, dense, bf16)
    for i in range(Wm):
        for _, call in calls_of_step:
            call(gsets[i % 2])
    # Timed region: K whole steps.  Inside it only the dominant kernel (six calls: the aggregate,
    # launched twice per step; windows: the RS window; packed: the splitter) is bracketed by events,
    # on the stream it is launched on, and only in every BRACKET_EVERY-th step: an event record
    # between two kernels costs about 5 us of idle GPU.  The per-call breakdown of the other calls
    # comes from a second pass after the timed region.
    bracketed = BRACKETED[mode]
    # LGP over a layer-granular stage 2 keeps the stage-2 aggregate (the warm-up steps have shown
    # whether it does): the stage-2 call is then a short pass over the kept values and the
    # aggregate kernel is launched once per step, on stage 1
    lgp_kept = mode == "six" and c.osp_lgp_kept_aggregate()
    if lgp_kept:
        bracketed = ("agg1",)
    ev = [{n: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for n in bracketed} if i % BRACKET_EVERY == 0 else None for i in range(K)]
    graphs = None
    if args.graph:
        if not (element and windows) or Wm < 2:
            print("bench.py: --graph needs --granularity element --calls windows --warmup >= 2",
                  file=sys.stderr)
            return 2
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
            n2_log[i] = wl.budget                # element split: exactly the budget
            continue
        g = gsets[(Wm + i) % 2]
        e = ev[i]
        for j, (name, call) in enumerate(calls_of_step):
            if e and name in e:
                e[name][0].record(); call(g); e[name][1].record()
            else:
                call(g)
            if j == 0:
                # host-side; every step's first call has waited for the split that set this size,
                # or (fused RS window) the next call waits for it anyway
                n2_log[i] = c.osp_n_stage2()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    n2 = n2_log
    total_bytes = 0
    agg_ms_sum = 0.0
    agg_bytes_sum = 0
    agg_launches = 0
    step_names = [n for n, _ in calls_of_step]
    for i in range(K):
        b = step_bytes(N, M, int(n2[i]), element, gb)
        total_bytes += sum(b[n] for n in step_names)
        if not ev[i]:
            continue
        for n in bracketed:
            agg_ms_sum += ev[i][n][0].elapsed_time(ev[i][n][1])
            agg_bytes_sum += b[n]
            agg_launches += 1
    ms_per_step = elapsed * 1e3 / K
    gbps = total_bytes / elapsed / 1e9
    lgp_shared = c.osp_lgp_read_shared()
    moved_bytes = total_bytes - sum(bytes_not_moved(N, int(n2[i]), gb, lgp_shared and not element,
                                                    lgp_kept) for i in range(K))
    if (lgp_shared and element) or mode != "six":  # whole groups / fused passes: not itemised here
        moved_bytes = None

    # dominant kernel: the aggregate+update kernel (the longest launch of a step and the one
    # furthest from the roofline; the two install launches together take about as long, see
    # roofline_other), launched once per step when LGP keeps the stage-2 aggregate, else twice
    fused_rs = windows and (c.osp_windows_fused() & 1) != 0
    kernel = ("k_aggregate_update" if mode == "six" else
              "k_split_gradients" if mode == "packed" else
              ("k_rs_window_element" if element else "k_window_layer") if fused_rs else
              "osp_rs_window (three single-stage kernels)")
    roofline_from_second_pass = agg_launches == 0
    if roofline_from_second_pass:                # graph replay: filled in from the eager second pass
        agg_ms_sum, agg_bytes_sum, agg_launches = 1.0, 0, 1
    agg_ms = agg_ms_sum / agg_launches
    agg_bytes = agg_bytes_sum / agg_launches
    agg_gbps = agg_bytes / (agg_ms * 1e-3) / 1e9 if agg_ms > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": round(agg_gbps, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(agg_gbps / HBM_PEAK_GBPS, 4),
                "traffic": (None if wl.name != "vgg16" or c.osp_chunk_elems() != 256 else
                            AGG_TRAFFIC_VGG16_LAYER if not element and lgp_kept and not bf16 else
                            RS_TRAFFIC_VGG16_ELEMENT if element and fused_rs else None),
                "launches": agg_launches,
                "avg_launch_ms": round(agg_ms, 5), "bytes_per_launch": int(agg_bytes)}

    # second pass (not part of `value`): every call bracketed, for the per-call breakdown
    K2 = min(K, 10)
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls_of_step) + 1)]
           for _ in range(K2)]
    n2b = torch.zeros(K2 + 1, dtype=torch.int64).pin_memory()
    c.osp_read_n_stage2_async(n2b.data_ptr())
    for i in range(K2):
        g = gsets[(Wm + K + i) % 2]
        e = ev2[i]
        for j, (_, call) in enumerate(calls_of_step):
            e[j].record(); call(g)
        e[len(calls_of_step)].record()
        c.osp_read_n_stage2_async(n2b.data_ptr() + 8 * (i + 1))
    torch.cuda.synchronize()
    names = step_names
    call_ms = {n: 0.0 for n in names}
    call_bytes = {n: 0 for n in names}
    for i in range(K2):
        b = step_bytes(N, M, int(n2b[i]), element, gb)
        for j, n in enumerate(names):
            call_ms[n] += ev2[i][j].elapsed_time(ev2[i][j + 1])
            call_bytes[n] += b[n]
    if roofline_from_second_pass:
        n0 = bracketed[0]
        ms0 = call_ms[n0] / K2
        roofline.update({"achieved": round(call_bytes[n0] / K2 / (ms0 * 1e-3) / 1e9, 1),
                         "frac": round(call_bytes[n0] / K2 / (ms0 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "launches": K2, "avg_launch_ms": round(ms0, 5),
                         "bytes_per_launch": int(call_bytes[n0] / K2),
                         "note": "events cannot sit inside a graph: taken from the eager second pass"})
    # the other two kernels that share the step's time with the aggregate, on the bytes they move
    roofline_other = None
    if lgp_kept and not element:
        e2 = [int(x) for x in n2b[:K2]]
        inst_b = sum(4 * (N + 1) * M for _ in e2)                       # both installs of a step
        inst_ms = call_ms["apply1"] + call_ms["apply2"]
        keep_b = sum((gb * N + 4 + 4 * N + 4) * x for x in e2)
        roofline_other = [
            {"kernel": "k_apply_stage_sweep (two launches per step)",
             "achieved": round(inst_b / (inst_ms * 1e-3) / 1e9, 1),
             "frac": round(inst_b / (inst_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
             "ms_per_step": round(inst_ms / K2, 5)},
            {"kernel": "k_lgp_keep",
             "achieved": round(keep_b / (call_ms["lgp"] * 1e-3) / 1e9, 1),
             "frac": round(keep_b / (call_ms["lgp"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
             "ms_per_step": round(call_ms["lgp"] / K2, 5)}]
    calls = {n: {"ms": round(call_ms[n] / K2, 5),
                 "GBps": round(call_bytes[n] / (call_ms[n] * 1e-3) / 1e9, 1) if call_ms[n] > 0 else None}
             for n in names}

    # reference line: the library's plain streaming copy of 2 GiB on the same box (also the
    # known-size kernel the rocprofv3 traffic counters are calibrated against)
    from paper_2306_16926_amd.binding import osp_stream_copy
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
    # second reference line: the aggregate's traffic shape without its arithmetic (N gradient
    # streams read, two streams read and written back), on this run's own gradient arenas
    pattern_gbps = None
    if not bf16:
        from paper_2306_16926_amd.binding import osp_stream_pattern
        rw = torch.zeros((2, stride), dtype=torch.float32, device="cuda")
        osp_stream_pattern(gsets[0], N, stride, rw, 2, stride, arena)
        torch.cuda.synchronize(); a.record()
        for r in range(6):
            osp_stream_pattern(gsets[r % 2], N, stride, rw, 2, stride, arena)
        b2.record(); torch.cuda.synchronize()
        pattern_gbps = 6 * 4 * (N + 4) * arena / (a.elapsed_time(b2) * 1e-3) / 1e9
        del rw

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, args, params, host_g0, job, gran, element, stride)

    out = {
        "metric": "osp_sync_step_GBps", "value": round(gbps, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "f32 (gradients stored as bf16)", "data": "synthetic",
        "config": {"workload": f"{wl.name}-shaped", "n_workers": N, "n_tensors": wl.n_tensors,
                   "n_params": M, "granularity": args.granularity, "calls": args.calls, "keep_stage2_aggregate": args.keep_stage2_aggregate == "on",
                   "graph_replay": bool(args.graph),
                   "windows_fused": ({"rs": bool(c.osp_windows_fused() & 1),
                                      "ics": bool(c.osp_windows_fused() & 2)} if windows else None),
                   "stage2_fraction_nominal": wl.stage2_fraction,
                   "stage2_elems_achieved": int(n2[K - 1]), "lr": wl.lr, "momentum": wl.momentum,
                   "seed": args.seed, "chunk_elems": c.osp_chunk_elems()},
        "sync_steps_per_s": round(K / elapsed, 2),
        "pct_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "GB_per_step": round(total_bytes / K / 1e9, 4),
        "lgp_reads_ps_once": bool(lgp_shared), "lgp_keeps_stage2_aggregate": bool(lgp_kept),
        "GB_moved_per_step": None if moved_bytes is None else round(moved_bytes / K / 1e9, 4),
        "GBps_on_bytes_moved": None if moved_bytes is None else round(moved_bytes / elapsed / 1e9, 1),
        "calls_second_pass": calls,
        "copy_GBps_same_box": round(copy_gbps, 1),
        "aggregate_pattern_GBps_same_box": None if pattern_gbps is None else round(pattern_gbps, 1),
        "roofline": roofline, "roofline_other": roofline_other,
        "cpu_baseline": cpu,
        "paper_context": "paper reports up to 50% end-to-end training throughput gain on 8xT4 "
                         "workers + 1 PS over 10 Gbps Ethernet; it never times this arithmetic",
    }
    print(json.dumps(out))
    return 0


def cpu_baseline(wl, args, params, host_g, job, gran, element, stride):
    """The CPU oracle, as it stands, on this machine's host cores: one sync step of
    the same workload from the same GIB the GPU is at, single-threaded (the
    reference of record) and the same loops under OpenMP."""
    from oracle.osp_oracle import OracleOSP
    N, M = wl.n_workers, wl.n_params
    layer, bits, n2 = job.ctx.osp_get_gib()
    res = {}
    for omp in (False, True):
        o = OracleOSP(wl.numel, wl.offsets(), wl.arena_elems(), N, wl.lr, wl.momentum,
                      param_stride=stride, omp=omp)
        o.load_params(params)
        o.set_gib(gran, bits if element else layer)
        t = time.perf_counter()
        o.ps_aggregate_update(1, host_g); o.apply_stage(1); o.lgp_correct(host_g)
        o.ps_aggregate_update(2, host_g); o.apply_stage(2)
        if not element or M <= 30_000_000:       # the oracle's element split is a full sort
            o.split(gran, wl.budget)
            sample = "1 full sync step"
        else:
            sample = "1 sync step without the element split (a full sort of M keys)"
        dt = time.perf_counter() - t
        b = step_bytes(N, M, n2, element)
        six = ("agg1", "apply1", "lgp", "agg2", "apply2", "split")
        res[omp] = (dt, sum(b[n] for n in six) / dt / 1e9, sample)
        del o
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
    return {"value": round(res[False][1], 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": res[False][2] + f" of {wl.name}-shaped, same GIB as the GPU run",
            "ms_per_step": round(res[False][0] * 1e3, 1),
            "all_cores": {"value": round(res[True][1], 3), "cores": min(omp_threads, cores_all),
                          "ms_per_step": round(res[True][0] * 1e3, 1)},
            "cpu": model}


if __name__ == "__main__":
    sys.exit(main())
