"""The RS and ICS window calls against the oracle's six calls; the caller's stream schedule;
random legal call sequences over every state-changing entry point."""
import numpy as np
import pytest

from oracle.osp_oracle import GRAN_ELEMENT, GRAN_LAYER
from paper_2306_16926_amd import workloads as W
from tests import brute
from tests.gpu_common import F, compare_gib, compare_state, device_job, run_steps, say
from tests.helpers import make_oracle, random_bits, random_layer_gib

pytestmark = pytest.mark.gpu

# --------------------------------------------------------------------------
# the two windows (one call each) against the oracle's six calls
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("weighted", [False, True])
def test_windows_tiny_three_chained_steps(gran, weighted):
    say("windows tiny", gran, weighted)
    wl = W.get("tiny")
    wts = np.array([0.4, 0.1, 0.3, 0.2], F) if weighted else None
    sizes = run_steps(wl, gran, 3, weights=wts, windows=True)
    assert sizes[0] > 0
    run_steps(wl, gran, 2, align=64, chunk_elems=1024, windows=True)


@pytest.mark.parametrize("n_workers", [1, 2, 3, 4, 5, 8, 9, 16, 17, 35])
def test_windows_worker_counts(n_workers):
    """Fused kernels up to 8 (layer) / 16 (element, RS) workers, single-stage kernels above."""
    say("windows workers", n_workers)
    wl = W.custom([5000, 3, 1029, 64, 2048, 1], n_workers, 0.4, align=4, config_id=140 + n_workers)
    run_steps(wl, GRAN_LAYER, 3, windows=True)
    run_steps(wl, GRAN_ELEMENT, 3, windows=True)
    wts = np.random.default_rng(n_workers).random(n_workers).astype(F)
    wts /= wts.sum()
    run_steps(wl, GRAN_ELEMENT, 2, weights=wts, windows=True)
    run_steps(wl, GRAN_LAYER, 2, weights=wts, windows=True)


@pytest.mark.parametrize("name,gran", [("resnet18", GRAN_LAYER), ("resnet18", GRAN_ELEMENT)])
def test_windows_cnn_shaped(name, gran):
    say("windows", name, gran)
    sizes = run_steps(W.get(name), gran, 3, threads=8, windows=True)
    assert sizes[-1] > 0


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("in_sync", [True, False])
def test_windows_mixed_with_single_calls(gran, in_sync):
    """Windows and single calls in one run, starting from replicas that are or are not declared
    equal to the PS, over iterations that do and do not restore consistency; stage 2 from
    another gradient buffer on some steps."""
    say("windows mixed", gran, in_sync)
    wl = W.custom([5000, 3, 1029, 64, 2048, 70000, 2], 6, 0.5, align=4, config_id=170)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True, declare_in_sync=in_sync)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    plans = ["ww", "ws", "sw", "ww", "w-", "ww", "s-", "ww", "wW", "ww"]
    for step, plan in enumerate(plans):
        g = wl.make_grads(0, step); gd = job.upload_grads(g); s_ = g.shape[1]
        g2, gd2 = g, gd
        if plan[1] == "W":                      # ICS window from a different gradient buffer
            g2 = wl.make_grads(3, step); gd2 = job.upload_grads(g2)
        o.ps_aggregate_update(1, g)
        if plan[0] == "w":
            o.apply_stage(1); o.lgp_correct(g)
            c.osp_rs_window(gd, s_)
        else:                                   # single calls, stage 1 never installed
            o.lgp_correct(g)
            c.osp_ps_aggregate_update(1, gd, s_); c.osp_lgp_correct(gd, s_)
        compare_state(job, o, f"step {step} {plan} RS")
        o.ps_aggregate_update(2, g2)
        if plan[1] in "wW":
            o.apply_stage(2); o.split(gran, wl.budget)
            c.osp_ics_window(gd2, s_, gran, wl.budget)
        elif plan[1] == "s":
            o.apply_stage(2); o.split(gran, wl.budget)
            c.osp_ps_aggregate_update(2, gd2, s_); c.osp_apply_stage(2); c.osp_split(gran, wl.budget)
        else:                                   # stage 2 aggregated but not installed, old GIB stays
            c.osp_ps_aggregate_update(2, gd2, s_)
        compare_state(job, o, f"step {step} {plan} ICS")
        compare_gib(job, o, f"step {step} {plan}")


def test_windows_reject_bad_arguments_before_launching():
    say("windows errors")
    from paper_2306_16926_amd.binding import OspError
    wl = W.get("tiny")
    o = make_oracle(wl)
    job = device_job(wl)                        # no element keys
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    g = wl.make_grads(0, 0); gd = job.upload_grads(g); s_ = g.shape[1]
    with pytest.raises(OspError):
        c.osp_ics_window(gd, s_, GRAN_LAYER, wl.budget)        # no stage 1 yet
    c.osp_rs_window(gd, s_)
    o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
    with pytest.raises(OspError):
        c.osp_rs_window(gd, s_)                                # stage 2 pending
    with pytest.raises(OspError):
        c.osp_ics_window(gd, s_, GRAN_ELEMENT, wl.budget)      # needs element keys
    with pytest.raises(OspError):
        c.osp_ics_window(gd, s_, GRAN_LAYER, wl.n_params + 1)
    compare_state(job, o, "after rejected calls")              # nothing was touched
    c.osp_ics_window(gd, s_, GRAN_LAYER, wl.budget)
    o.ps_aggregate_update(2, g); o.apply_stage(2); o.split(GRAN_LAYER, wl.budget)
    compare_state(job, o, "after ICS")
    compare_gib(job, o, "after ICS")


# --------------------------------------------------------------------------
# the caller's stream schedule: RS on one stream, ICS on another, ordered by events
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_two_streams_with_events(gran):
    """What OSP overlaps is the ICS window with the next iteration's compute: the RS calls go to
    one stream, the ICS calls to a second one behind an event, while the first stream carries
    other work (here a copy standing in for the forward/backward pass); the next RS waits for
    the ICS through another event.  Default priorities, no host synchronization in the loop."""
    import torch
    say("two streams", gran)
    wl = W.get("resnet18")
    o = make_oracle(wl)
    job = device_job(wl, element_keys=(gran == GRAN_ELEMENT))
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    rs, ics = torch.cuda.Stream(), torch.cuda.Stream()
    busy_src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
    busy_dst = torch.empty_like(busy_src)
    grads = [wl.make_grads(0, step, threads=8) for step in range(3)]
    dev = [job.upload_grads(g) for g in grads]
    torch.cuda.synchronize()
    ics_done = torch.cuda.Event()
    ics_done.record(ics)
    for step in range(3):
        gd = dev[step]; s_ = gd.shape[1]
        rs.wait_event(ics_done)                         # stage 2 of the previous iteration is complete
        if step % 2 == 0:
            c.osp_rs_window(gd, s_, stream=rs)
        else:
            c.osp_ps_aggregate_update(1, gd, s_, stream=rs)
            c.osp_apply_stage(1, stream=rs)
            c.osp_lgp_correct(gd, s_, stream=rs)
        rs_done = torch.cuda.Event(); rs_done.record(rs)
        with torch.cuda.stream(rs):                     # "compute" of the next iteration
            busy_dst.copy_(busy_src, non_blocking=True)
        ics.wait_event(rs_done)
        if step % 2 == 0:
            c.osp_ics_window(gd, s_, gran, wl.budget, stream=ics)
        else:
            c.osp_ps_aggregate_update(2, gd, s_, stream=ics)
            c.osp_apply_stage(2, stream=ics)
            c.osp_split(gran, wl.budget, stream=ics)
        ics_done = torch.cuda.Event(); ics_done.record(ics)
        o.sync_step(grads[step], gran, wl.budget)
    torch.cuda.synchronize()
    compare_state(job, o, "two streams")
    compare_gib(job, o, "two streams")
    assert bool((busy_dst[:1024] == 1.0).all())


# --------------------------------------------------------------------------
# no staged call waits for the GPU: whole layer-granular iterations are enqueued while the
# stream is still busy with earlier work (Sec. 3.1: the ICS of iteration t runs under the
# compute of iteration t+1, so the host must be able to enqueue RS(t+1) behind it)
# --------------------------------------------------------------------------

def scaled_grads(wl, step, scales_seed, align=None):
    """The workload's gradients with every tensor multiplied by its own power of two, redrawn
    per step: the layer ranking, hence the lengths of the two stage tables, changes from one
    iteration to the next."""
    g = wl.make_grads(0, step, align, threads=8)
    rng = np.random.default_rng([scales_seed, step])
    for a, n in zip(wl.offsets(align), wl.numel):
        g[:, int(a):int(a) + int(n)] *= F(2.0) ** int(rng.integers(-6, 7))
    return g


def busy_kernel_ms(torch, ms):
    """Enqueue about `ms` milliseconds of GPU work on the current stream; returns an event
    recorded behind it."""
    cycles = 2_000_000
    torch.cuda._sleep(cycles)                          # warm-up and calibration
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record(); torch.cuda._sleep(cycles); b.record()
    torch.cuda.synchronize()
    per_ms = cycles / max(a.elapsed_time(b), 1e-3)
    torch.cuda._sleep(int(per_ms * ms))
    done = torch.cuda.Event()
    done.record()
    return done


@pytest.mark.parametrize("calls", ["six", "windows"])
@pytest.mark.parametrize("shape", ["tiny", "n16", "n8_many_tensors"])
def test_layer_steps_are_enqueued_without_waiting(calls, shape):
    import torch
    say("no host wait", calls, shape)
    if shape == "tiny":
        wl = W.get("tiny")
    elif shape == "n16":
        wl = W.custom([70000, 33, 5000, 131072, 4099, 64, 20000, 90001], 16, 0.5, align=4,
                      config_id=71)
    else:
        rng = np.random.default_rng(5)
        wl = W.custom([int(x) for x in rng.integers(1, 40000, 150)], 8, 0.5, align=4, config_id=72)
    o = make_oracle(wl)
    job = device_job(wl)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    steps = 4
    budgets = [int(f * wl.n_params) for f in (0.2, 0.7, 0.4, 0.5)]
    grads = [scaled_grads(wl, step, 11) for step in range(steps)]
    dev = [job.upload_grads(g) for g in grads]
    log = torch.zeros(steps, dtype=torch.int64, device="cuda")
    c.osp_set_stage2_log(log)
    busy = busy_kernel_ms(torch, 400.0)
    for step in range(steps):
        gd = dev[step]; s_ = gd.shape[1]
        if calls == "six":
            job.sync_step(gd, GRAN_LAYER, budgets[step])
        else:
            job.sync_step_windows(gd, GRAN_LAYER, budgets[step])
    still_busy = not busy.query()
    torch.cuda.synchronize()
    assert still_busy, "a call waited for the GPU (or the busy kernel was too short)"
    sizes = []
    for step in range(steps):
        o.sync_step(grads[step], GRAN_LAYER, budgets[step])
        sizes.append(o.n_stage2)
    assert len(set(sizes)) > 1, sizes                  # the table lengths did change
    assert [int(x) for x in log.cpu()] == sizes        # every iteration cut the layers as the oracle did
    compare_state(job, o, "no host wait")
    compare_gib(job, o, "no host wait")
    assert c.osp_n_stage2() == o.n_stage2


@pytest.mark.parametrize("calls", ["six", "windows"])
@pytest.mark.parametrize("shape", ["tiny", "n16"])
def test_layer_steps_replay_as_a_graph(calls, shape):
    """A layer-granular iteration captured once and replayed: the launches read the lengths of
    the stage tables on the device, so the captured grids stay valid when the split of one
    replay cuts the layers differently from the one the graph was captured under."""
    import torch
    say("layer graph replay", calls, shape)
    wl = (W.get("tiny") if shape == "tiny" else
          W.custom([70000, 33, 5000, 131072, 4099, 64, 20000, 90001], 16, 0.5, align=4, config_id=71))
    o = make_oracle(wl)
    job = device_job(wl)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    g = scaled_grads(wl, 0, 13)
    static = job.upload_grads(g); s_ = static.shape[1]
    step_fn = job.sync_step if calls == "six" else job.sync_step_windows
    for step in range(2):                               # eager: reach a staged GIB
        g = scaled_grads(wl, step, 13)
        static.copy_(torch.from_numpy(g))
        o.sync_step(g, GRAN_LAYER, wl.budget)
        step_fn(static, GRAN_LAYER, wl.budget)
    torch.cuda.synchronize()
    compare_state(job, o, "before capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                       # capture runs nothing
        step_fn(static, GRAN_LAYER, wl.budget)
    sizes = []
    for step in range(2, 7):
        g = scaled_grads(wl, step, 13)
        static.copy_(torch.from_numpy(g))               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        o.sync_step(g, GRAN_LAYER, wl.budget)
        sizes.append(o.n_stage2)
        compare_state(job, o, f"replay of step {step}")
        compare_gib(job, o, f"replay of step {step}")
    assert len(set(sizes)) > 1, sizes
    # and eager again on top of the replays
    g = scaled_grads(wl, 7, 13)
    static.copy_(torch.from_numpy(g))
    o.sync_step(g, GRAN_LAYER, wl.budget)
    step_fn(static, GRAN_LAYER, wl.budget)
    compare_state(job, o, "eager after replays")
    compare_gib(job, o, "eager after replays")


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_read_n_stage2_async_into_pinned_and_pageable_memory(gran):
    """osp_read_n_stage2_async: the stage-2 size arrives in the caller's host memory once the
    stream has passed the call, whether that memory is pinned (written by a small kernel) or
    pageable (a copy)."""
    import torch
    say("async stage-2 size", gran)
    wl = W.get("tiny")
    o = make_oracle(wl)
    job = device_job(wl, element_keys=(gran == GRAN_ELEMENT))
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    pinned = torch.full((3,), -1, dtype=torch.int64).pin_memory()
    pageable = np.full(3, -1, np.int64)
    want = []
    for step in range(3):
        g = wl.make_grads(0, step)
        gd = job.upload_grads(g)
        want.append(o.sync_step(g, gran, wl.budget))
        job.sync_step(gd, gran, wl.budget)
        c.osp_read_n_stage2_async(pinned.data_ptr() + 8 * step)
        c.osp_read_n_stage2_async(pageable.ctypes.data + 8 * step)
    torch.cuda.synchronize()
    assert [int(x) for x in pinned] == want
    assert pageable.tolist() == want
    assert c.osp_n_stage2() == want[-1]


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_stage2_log_round_robin(gran):
    """osp_set_stage2_log: every split stores the size of the stage 2 it chose, round robin in
    the caller's buffer, counted from the call; taking the log away stops it."""
    import torch
    say("stage-2 log", gran)
    wl = W.get("tiny")
    o = make_oracle(wl)
    job = device_job(wl, element_keys=(gran == GRAN_ELEMENT))
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    budgets = [int(f * wl.n_params) for f in (0.3, 0.0, 0.6, 0.1, 0.45)]
    log = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    sizes = []
    for step, b in enumerate(budgets):
        if step == 1:
            c.osp_set_stage2_log(log)                   # counting starts here
        if step == 4:
            c.osp_set_stage2_log(None)
        g = scaled_grads(wl, step, 17)
        gd = job.upload_grads(g)
        sizes.append(o.sync_step(g, gran, b))
        if step % 2:
            job.sync_step_windows(gd, gran, b)
        else:
            job.sync_step(gd, gran, b)
    torch.cuda.synchronize()
    compare_gib(job, o, "log")
    # splits 1, 2, 3 were logged at slots 0, 1, 2; split 4 was not
    assert [int(x) for x in log.cpu()] == sizes[1:4]
    # capacity 2: slot = count % 2
    log2 = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    c.osp_set_stage2_log(log2)
    for step in range(5, 8):
        g = scaled_grads(wl, step, 17)
        gd = job.upload_grads(g)
        sizes.append(o.sync_step(g, gran, budgets[step - 4]))
        job.sync_step(gd, gran, budgets[step - 4])
    torch.cuda.synchronize()
    assert [int(x) for x in log2.cpu()] == [sizes[7], sizes[6]]
    with pytest.raises(Exception):
        c.osp_set_stage2_log(log2, capacity=0)


# --------------------------------------------------------------------------
# random legal call sequences over every entry point that touches the state
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", list(range(16)))
def test_random_call_sequences(seed):
    """Iterations assembled at random from the single-stage calls (fp32, bfloat16 and dense
    gradient inputs), the two windows, optional installs and LGP in any legal order, splits of
    either granularity or an injected GIB: the state is compared with the oracle after every
    call.  Gradients are bfloat16-representable so that every input form carries the same values."""
    import torch
    say("random sequences", seed)
    rng = np.random.default_rng(1000 + seed)
    n_workers = int(rng.choice([2, 5, 8, 11]))
    wl = W.custom([5000, 3, 1029, 64, 2048, 30000, 2], n_workers, 0.5, align=4, config_id=300 + seed)
    arena = wl.arena_elems()
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    wts = None
    if seed % 2:
        wts = rng.random(n_workers).astype(F); wts /= wts.sum()
    o = make_oracle(wl, weights=wts)
    job = device_job(wl, weights=wts, element_keys=True, declare_in_sync=bool(seed % 3))
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    M = wl.n_params
    dense_i = torch.zeros((n_workers, M + 4), dtype=torch.float32, device="cuda")
    dense_u = torch.zeros((n_workers, M + 4), dtype=torch.float32, device="cuda")
    log = []

    def check(what):
        log.append(what)
        try:
            compare_state(job, o, what)
        except AssertionError:
            print("[case] calls so far:", " | ".join(log), flush=True)
            raise

    for it in range(10):
        h = W.to_bf16(wl.make_grads(seed, it)); g = W.from_bf16(h)
        gd = job.upload_grads(g); hd = job.upload_grads_bf16(h); s_ = g.shape[1]
        packed = None

        def get_packed():
            og_i, og_u = o.split_gradients(g)
            c.osp_split_gradients(gd, s_, dense_i, M + 4, dense_u, M + 4)
            return og_i, og_u

        def agg(stage):
            nonlocal packed
            form = rng.choice(["f32", "bf16", "packed"])
            if form == "packed":
                if packed is None:
                    packed = get_packed()
                part = packed[stage - 1]
                if part.shape[1]:
                    o.ps_aggregate_update_packed(stage, part)
                else:
                    o.ps_aggregate_update(stage, g)
                c.osp_ps_aggregate_update_packed(stage, dense_i if stage == 1 else dense_u, M + 4)
            elif form == "bf16":
                o.ps_aggregate_update(stage, g); c.osp_ps_aggregate_update_bf16(stage, hd, s_)
            else:
                o.ps_aggregate_update(stage, g); c.osp_ps_aggregate_update(stage, gd, s_)
            check(f"it{it} agg{stage}:{form}")

        def lgp():
            if rng.random() < 0.5:
                o.lgp_correct(g); c.osp_lgp_correct(gd, s_)
            else:
                o.lgp_correct(g); c.osp_lgp_correct_bf16(hd, s_)
            check(f"it{it} lgp")

        lgp_done = False
        if rng.random() < 0.4:
            o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
            if rng.random() < 0.5:
                c.osp_rs_window(gd, s_)
            else:
                c.osp_rs_window_bf16(hd, s_)
            lgp_done = True
            check(f"it{it} rs_window")
        else:
            agg(1)
            todo = []
            if rng.random() < 0.8:
                todo.append("apply1")
            if rng.random() < 0.7:
                todo.append("lgp")
            rng.shuffle(todo)
            for t in todo:
                if t == "apply1":
                    o.apply_stage(1); c.osp_apply_stage(1); check(f"it{it} apply1")
                else:
                    lgp(); lgp_done = True
        split_gran = int(rng.choice([GRAN_LAYER, GRAN_ELEMENT]))
        budget = int(rng.choice([0, wl.budget // 3, wl.budget, M]))
        if rng.random() < 0.4:
            o.ps_aggregate_update(2, g); o.apply_stage(2); o.split(split_gran, budget)
            if rng.random() < 0.5:
                c.osp_ics_window(gd, s_, split_gran, budget)
            else:
                c.osp_ics_window_bf16(hd, s_, split_gran, budget)
            check(f"it{it} ics_window gran{split_gran} budget{budget}")
        else:
            agg(2)
            if not lgp_done and rng.random() < 0.3:
                lgp()
            if rng.random() < 0.85:
                o.apply_stage(2); c.osp_apply_stage(2); check(f"it{it} apply2")
            r = rng.random()
            if r < 0.6:
                o.split(split_gran, budget); c.osp_split(split_gran, budget)
                log.append(f"it{it} split gran{split_gran} budget{budget}")
            elif r < 0.8:
                gib = (random_layer_gib(rng, wl.n_tensors) if split_gran == GRAN_LAYER
                       else random_bits(rng, arena, real))
                o.set_gib(split_gran, gib); c.osp_set_gib(split_gran, gib)
                log.append(f"it{it} set_gib gran{split_gran}")
        compare_gib(job, o, f"it{it} gib")
        assert c.osp_n_stage2() == o.n_stage2


# --------------------------------------------------------------------------
# an element-granular iteration as a captured graph
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "resnet18"])
def test_element_windows_replay_as_a_graph(name):
    """With an element-granular GIB no call of the iteration needs anything from the host (no
    table lengths), and the library clears its scratch with fill kernels, not memsets: the two
    window calls can be captured once and replayed.  Each replay, with eager copies and a
    synchronization in between, is compared with the oracle."""
    import torch
    say("graph replay", name)
    wl = W.get(name)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    g = wl.make_grads(0, 0, threads=8)
    static = job.upload_grads(g); s_ = static.shape[1]
    for step in range(2):                               # eager: reach an element-granular GIB
        g = wl.make_grads(0, step, threads=8)
        static.copy_(torch.from_numpy(g))
        o.sync_step(g, GRAN_ELEMENT, wl.budget)
        job.sync_step_windows(static, GRAN_ELEMENT, wl.budget)
    torch.cuda.synchronize()
    compare_state(job, o, "before capture")
    graph = torch.cuda.CUDAGraph()
    g = wl.make_grads(0, 2, threads=8)
    static.copy_(torch.from_numpy(g))
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):                       # capture runs nothing
        c.osp_rs_window(static, s_)
        c.osp_ics_window(static, s_, GRAN_ELEMENT, wl.budget)
    for step in range(2, 6):
        g = wl.make_grads(0, step, threads=8)
        static.copy_(torch.from_numpy(g))               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        o.sync_step(g, GRAN_ELEMENT, wl.budget)
        compare_state(job, o, f"replay of step {step}")
        compare_gib(job, o, f"replay of step {step}")


# --------------------------------------------------------------------------
# Algorithm 1 driving the budget of the split over several "epochs"
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_tuned_budget_over_epochs(gran):
    """S(G^u) from Eq. 5 and Algorithm 1 (library) sets the budget of each epoch's splits:
    0 in the first epoch (BSP), growing as the synthetic loss falls, capped at 80 % of the
    model; the stage-2 sizes follow the oracle's."""
    from oracle.osp_oracle import ics_upper_bound, tune_budget
    from paper_2306_16926_amd.binding import osp_ics_upper_bound, osp_tune_budget
    say("tuned budget", gran)
    wl = W.custom([5000, 3, 1029, 64, 2048, 30000, 700], 4, 0.5, align=4, config_id=410)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    M = wl.n_params
    u_lib = osp_ics_upper_bound(2.0e5, 0.01, 0.9, wl.n_workers)      # elements per compute window
    assert u_lib == ics_upper_bound(2.0e5, 0.01, 0.9, wl.n_workers)
    losses = [2.3, 1.7, 1.1, 0.6, 0.2, 0.01]
    sizes, step = [], 0
    for epoch, loss in enumerate(losses, start=1):
        budget = osp_tune_budget(epoch, loss, losses[0], u_lib, M)
        assert budget == tune_budget(epoch, loss, losses[0], u_lib, M)
        assert 0 <= budget <= int(0.8 * M)
        for _ in range(2):                                   # two iterations per epoch
            g = wl.make_grads(0, step); gd = job.upload_grads(g); step += 1
            o.sync_step(g, gran, budget)
            job.sync_step_windows(gd, gran, budget)
            compare_state(job, o, f"epoch {epoch}")
            compare_gib(job, o, f"epoch {epoch}")
        sizes.append(o.n_stage2)
    assert sizes[0] == 0 and sizes[-1] > 0
    assert sizes == sorted(sizes)                            # the loss only falls here


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_sync_step_is_both_windows(gran):
    from paper_2306_16926_amd.binding import OspError
    say("osp_sync_step", gran)
    wl = W.custom([5000, 3, 1029, 64, 2048, 30000], 6, 0.5, align=4, config_id=420)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    for step in range(3):
        g = wl.make_grads(0, step); gd = job.upload_grads(g)
        with pytest.raises(OspError):
            c.osp_sync_step(gd, g.shape[1], gran, wl.n_params + 1)     # nothing may have run
        compare_state(job, o, f"after a refused call, step {step}")
        o.sync_step(g, gran, wl.budget)
        c.osp_sync_step(gd, g.shape[1], gran, wl.budget)
        compare_state(job, o, f"step {step}")
        compare_gib(job, o, f"step {step}")


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_two_contexts_interleaved_and_rebind_resume(gran):
    """Two jobs alive at once with their calls interleaved on one stream do not disturb each
    other; and a job whose state is moved into new buffers mid-run (osp_bind again, the GIB read
    back and installed again: a resume) continues exactly where the oracle does."""
    import torch
    say("two contexts / rebind", gran)
    wl_a = W.custom([5000, 3, 1029, 64, 70000], 5, 0.5, align=4, config_id=260)
    wl_b = W.custom([300, 40000, 17, 2048], 3, 0.3, align=64, config_id=261)
    oa, ob = make_oracle(wl_a), make_oracle(wl_b, align=64)
    ja = device_job(wl_a, element_keys=True)
    jb = device_job(wl_b, align=64, element_keys=True, chunk_elems=1024)
    for o, j, wl in ((oa, ja, wl_a), (ob, jb, wl_b)):
        all1 = np.ones(wl.n_tensors, np.uint8)
        o.set_gib(GRAN_LAYER, all1); j.ctx.osp_set_gib(GRAN_LAYER, all1)
    for step in range(3):
        ga, gb = wl_a.make_grads(0, step), wl_b.make_grads(0, step, 64)
        da, db = ja.upload_grads(ga), jb.upload_grads(gb)
        oa.sync_step(ga, gran, wl_a.budget); ob.sync_step(gb, gran, wl_b.budget)
        ca, cb, sa, sb = ja.ctx, jb.ctx, ga.shape[1], gb.shape[1]
        ca.osp_ps_aggregate_update(1, da, sa); cb.osp_rs_window(db, sb)
        ca.osp_apply_stage(1); ca.osp_lgp_correct(da, sa)
        cb.osp_ps_aggregate_update(2, db, sb)
        ca.osp_ps_aggregate_update(2, da, sa); cb.osp_apply_stage(2)
        ca.osp_apply_stage(2); cb.osp_split(gran, wl_b.budget); ca.osp_split(gran, wl_a.budget)
        compare_state(ja, oa, f"job a step {step}"); compare_gib(ja, oa, f"job a step {step}")
        compare_state(jb, ob, f"job b step {step}"); compare_gib(jb, ob, f"job b step {step}")

    # resume job a in new buffers: same values, other addresses, a fresh workspace
    layer, bits, n2 = ja.ctx.osp_get_gib()
    P2, V2 = ja.P.clone(), ja.V.clone()
    stride2 = ja.arena + 260
    Pw2 = torch.full((ja.N, stride2), 9.0, dtype=torch.float32, device="cuda")
    Pw2[:, :ja.arena] = ja.Pw[:, :ja.arena]
    nbytes = ja.ctx.osp_workspace_bytes()
    ws2 = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ja.ctx.osp_bind(P2, V2, Pw2, stride2, ws2, nbytes, replicas_in_sync=True)
    from paper_2306_16926_amd.binding import OspError
    with pytest.raises(OspError):
        ja.ctx.osp_rs_window(ja.upload_grads(wl_a.make_grads(0, 3)), wl_a.make_grads(0, 3).shape[1])  # no GIB after a bind
    ja.ctx.osp_set_gib(gran, layer if gran == GRAN_LAYER else bits)
    ja.P, ja.V, ja.Pw, ja.param_stride, ja.workspace = P2, V2, Pw2, stride2, ws2
    assert ja.ctx.osp_n_stage2() == n2 == oa.n_stage2
    for step in range(3, 6):
        ga = wl_a.make_grads(0, step); da = ja.upload_grads(ga)
        oa.sync_step(ga, gran, wl_a.budget)
        if step % 2:
            ja.sync_step_windows(da, gran, wl_a.budget)
        else:
            ja.sync_step(da, gran, wl_a.budget)
        compare_state(ja, oa, f"resumed job a step {step}"); compare_gib(ja, oa, f"resumed step {step}")
    assert (Pw2[:, ja.arena:] == 9.0).all()
    # job b was not disturbed by any of it
    compare_state(jb, ob, "job b at the end")
