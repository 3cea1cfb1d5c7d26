"""Parity of the HIP library against the CPU oracle, through the C ABI: chained sync steps,
full sizes in the benchmark's launch configuration, each call on its own, the splits, the
order-of-calls state machine."""
import numpy as np
import pytest

from oracle.osp_oracle import GRAN_ELEMENT, GRAN_LAYER, OracleOSP
from paper_2306_16926_amd import workloads as W
from tests import brute
from tests.gpu_common import (F, close_enough, compare_gib, compare_state, device_job, run_steps,
                              say)
from tests.helpers import make_oracle, random_bits, random_layer_gib

pytestmark = pytest.mark.gpu

# --------------------------------------------------------------------------
# whole sync steps, chained
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("weighted", [False, True])
def test_tiny_three_chained_steps(gran, weighted):
    say("tiny", gran, weighted)
    wl = W.get("tiny")
    wts = np.array([0.4, 0.1, 0.3, 0.2], F) if weighted else None
    sizes = run_steps(wl, gran, 3, weights=wts)
    assert sizes[0] > 0


@pytest.mark.parametrize("seed", [1, 2])
def test_tiny_other_seeds(seed):
    say("tiny seed", seed)
    run_steps(W.get("tiny"), GRAN_LAYER, 2, seed=seed)
    run_steps(W.get("tiny"), GRAN_ELEMENT, 2, seed=seed)


@pytest.mark.parametrize("chunk", [256, 512, 1024, 16384])
@pytest.mark.parametrize("align", [4, 64])
def test_tiny_chunk_sizes_and_alignment(chunk, align):
    say("tiny chunk", chunk, "align", align)
    run_steps(W.get("tiny"), GRAN_LAYER, 2, align=align, chunk_elems=chunk)
    run_steps(W.get("tiny"), GRAN_ELEMENT, 2, align=align, chunk_elems=chunk)


@pytest.mark.parametrize("n_workers", [1, 2, 3, 7, 8, 9, 16, 17, 33, 40])
def test_worker_counts(n_workers):
    """Crosses the kernel's blocks of 8 (aggregate) and 4 (LGP) worker streams."""
    say("workers", n_workers)
    wl = W.custom([5000, 3, 1029, 64, 2048], n_workers, 0.4, align=4, config_id=40 + n_workers)
    run_steps(wl, GRAN_LAYER, 2)
    run_steps(wl, GRAN_ELEMENT, 2)
    wts = np.random.default_rng(n_workers).random(n_workers).astype(F)
    wts /= wts.sum()
    run_steps(wl, GRAN_ELEMENT, 2, weights=wts)


@pytest.mark.parametrize("name,gran", [("resnet18", GRAN_LAYER), ("resnet18", GRAN_ELEMENT),
                                       ("resnet50", GRAN_LAYER), ("resnet50", GRAN_ELEMENT)])
def test_cnn_shaped_three_steps(name, gran):
    """Three chained iterations: the GIB of iteration t is the one iteration t-1 produced
    (Sec. 4.1.1), so the third step runs on a GIB that itself came from a staged step."""
    say(name, gran)
    sizes = run_steps(W.get(name), gran, 3, threads=8)
    assert sizes[-1] > 0


@pytest.mark.parametrize("seed", [1, 2])
@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_resnet18_shaped_other_seeds(seed, gran):
    say("resnet18 seed", seed, gran)
    sizes = run_steps(W.get("resnet18"), gran, 3, seed=seed, threads=8)
    assert sizes[-1] > 0


# --------------------------------------------------------------------------
# full sizes, in the launch configuration the benchmark times (same worker
# stride, default chunk): every output element against the oracle (its loops
# run under OpenMP here, which a CPU test shows to be bit-identical)
# --------------------------------------------------------------------------

def full_size_steps(name, steps, windows=False):
    from paper_2306_16926_amd.device import DeviceJob
    wl = W.get(name)
    stride, pstride = wl.worker_stride(), wl.replica_stride()     # as bench.py lays them out
    arena = wl.arena_elems()
    o = make_oracle(wl, omp=True, param_stride=pstride)
    job = DeviceJob(wl.numel, wl.offsets(), arena, wl.n_workers, wl.lr, wl.momentum,
                    wl.make_params(0), param_stride=pstride)
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); job.ctx.osp_set_gib(GRAN_LAYER, all1)
    sizes = []
    g = None
    for step in range(steps):
        say(" ", name, "step", step, "generate")
        g = wl.make_grads(0, step, stride=stride, threads=16, out=g)
        gd = job.upload_grads(g)
        say(" ", name, "step", step, "oracle")
        o.sync_step(g, GRAN_LAYER, wl.budget)
        say(" ", name, "step", step, "gpu")
        if windows:
            job.sync_step_windows(gd, GRAN_LAYER, wl.budget)
        else:
            job.sync_step(gd, GRAN_LAYER, wl.budget)
        compare_gib(job, o, f"{name} step {step}")
        imp = job.ctx.osp_get_importance()
        rel = np.abs(imp - o.importance) / np.maximum(np.abs(o.importance), 1e-300)
        assert rel.max() <= 1e-12
        # smallest relative gap between neighbours in the ranking: far above the 1e-12 the
        # two summation orders can differ by, so the ranking cannot flip
        ranked = np.sort(o.importance)
        gap = np.min(np.diff(ranked) / ranked[1:])
        assert gap > 1e-9, gap
        sizes.append(o.n_stage2)
        del gd
    say(" ", name, "compare state")
    P, V, Pw = job.download()
    close_enough(P, o.P, name + " P")
    close_enough(V, o.V, name + " V")
    for w in range(wl.n_workers):                  # row by row: bounded temporaries
        close_enough(Pw[w, :arena], o.Pw[w, :arena], f"{name} Pw[{w}]")
    return sizes


def test_full_size_resnet152_layer():
    say("full size resnet152")
    sizes = full_size_steps("resnet152", 3)
    assert sizes[-1] > 0


def test_full_size_resnet152_layer_windows():
    say("full size resnet152, windows")
    sizes = full_size_steps("resnet152", 3, windows=True)
    assert sizes[-1] > 0


def test_full_size_bert_base_layer():
    say("full size bert_base")
    sizes = full_size_steps("bert_base", 3)
    assert sizes[-1] > 0


def test_full_size_vgg16_layer():
    say("full size vgg16")
    sizes = full_size_steps("vgg16", 3)
    assert sizes[-1] == 35_597_096                 # everything but the 102.76 M-element fc tensor


def full_size_element(name):
    """Element granularity at full size, in the benchmark's launch configuration: three
    chained iterations (a BSP step, the six single calls, the two windows), each on the
    bitmap the iteration before produced.  After every iteration: P, V and every replica
    element by element, the keys bit-exact, the bitmap bit-exact.  The expected bitmap of the
    first iteration is the oracle's own split (a full sort); the later ones are built from the
    oracle's keys by selection (OracleOSP.split_element_by_selection), which a CPU test pins to
    that sort."""
    from paper_2306_16926_amd.device import DeviceJob
    wl = W.get(name)
    stride, pstride, arena = wl.worker_stride(), wl.replica_stride(), wl.arena_elems()
    o = make_oracle(wl, omp=True, param_stride=pstride)
    job = DeviceJob(wl.numel, wl.offsets(), arena, wl.n_workers, wl.lr, wl.momentum,
                    wl.make_params(0), element_keys=True, param_stride=pstride)
    c = job.ctx
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    k = wl.budget

    def compare(tag, full_sort):
        P, V, Pw = job.download()
        close_enough(P, o.P, tag + " P"); close_enough(V, o.V, tag + " V")
        for w in range(wl.n_workers):              # row by row: bounded temporaries
            close_enough(Pw[w, :arena], o.Pw[w, :arena], f"{tag} Pw[{w}]")
        del P, V, Pw
        okeys = o.keys()
        assert np.array_equal(c.osp_get_keys()[real], okeys[real]), tag + " keys"
        if full_sort:
            say("   ", tag, "oracle split (full sort)")
            o.split(GRAN_ELEMENT, k)
        else:
            o.split_element_by_selection(k)
        _, bits, n2 = c.osp_get_gib()
        assert n2 == k == o.n_stage2
        assert np.array_equal(bits, o.gib_bits), tag + " element bitmap"

    say(" ", name, "step 0: BSP pass + element split")
    g = wl.make_grads(0, 0, stride=stride, threads=16)
    gd = job.upload_grads(g)
    o.ps_aggregate_update(0, g); o.apply_stage(0)
    c.osp_ps_aggregate_update(0, gd, stride); c.osp_apply_stage(0); c.osp_split(GRAN_ELEMENT, k)
    compare("step 0", True)
    say(" ", name, "step 1: six calls on the element bitmap")
    g = wl.make_grads(0, 1, stride=stride, threads=16, out=g)
    gd = job.upload_grads(g)
    o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
    o.ps_aggregate_update(2, g); o.apply_stage(2)
    job.sync_step(gd, GRAN_ELEMENT, k)
    compare("step 1", False)
    say(" ", name, "step 2: the two windows")
    g = wl.make_grads(0, 2, stride=stride, threads=16, out=g)
    gd = job.upload_grads(g)
    o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
    o.ps_aggregate_update(2, g); o.apply_stage(2)
    c.osp_rs_window(gd, stride); c.osp_ics_window(gd, stride, GRAN_ELEMENT, k)
    assert c.osp_windows_fused() & 1, "the RS window is expected to run fused at this size"
    compare("step 2", False)


def test_full_size_resnet152_element():
    say("full size resnet152 element")
    full_size_element("resnet152")


def test_full_size_vgg16_element():
    say("full size vgg16 element")
    full_size_element("vgg16")


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_calls_one_by_one_with_injected_gib(gran):
    say("one by one", gran)
    wl = W.custom([37, 1, 128, 5, 9000, 64, 3, 4096, 4097], 5, 0.5, align=4, config_id=21)
    rng = np.random.default_rng(8)
    arena = wl.arena_elems()
    stride = arena + 12                     # worker strides that differ from the arena
    o = make_oracle(wl, param_stride=stride)
    job = device_job(wl, element_keys=True, param_stride=stride, pad_fill=123.0)
    o.Pw[:, arena:] = 123.0
    # padding inside the arena carries a sentinel that nothing may overwrite
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    gib = random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER else random_bits(rng, arena, real)
    o.set_gib(gran, gib); job.ctx.osp_set_gib(gran, gib)
    compare_gib(job, o, "set_gib")
    g = np.zeros((5, stride), F)
    wl.make_grads(0, 0, stride=stride, out=g)
    g[:, ~np.pad(real, (0, 12))] = 7.0      # garbage in the gradient padding must not leak
    gd = job.upload_grads(g)
    o.ps_aggregate_update(1, g); job.ctx.osp_ps_aggregate_update(1, gd, stride)
    compare_state(job, o, "agg1")
    o.apply_stage(1); job.ctx.osp_apply_stage(1)
    compare_state(job, o, "apply1")
    o.lgp_correct(g); job.ctx.osp_lgp_correct(gd, stride)
    compare_state(job, o, "lgp")
    o.ps_aggregate_update(2, g); job.ctx.osp_ps_aggregate_update(2, gd, stride)
    compare_state(job, o, "agg2")
    o.apply_stage(2); job.ctx.osp_apply_stage(2)
    compare_state(job, o, "apply2")
    P, V, Pw = job.download()
    assert (Pw[:, arena:] == 123.0).all()
    for w in range(5):
        assert np.array_equal(Pw[w, :arena][real], P[real])
    o.split(GRAN_LAYER, wl.budget); job.ctx.osp_split(GRAN_LAYER, wl.budget)
    compare_gib(job, o, "split layer after staged " + str(gran))
    imp = job.ctx.osp_get_importance()
    assert np.allclose(imp, o.importance, rtol=1e-12, atol=0)


@pytest.mark.parametrize("stage2_input", ["same_buffer", "copy_elsewhere", "other_values", "other_stride"])
def test_element_stage2_gradient_sources(stage2_input):
    """Element-granular stage 1 keeps the aggregate of the stage-2 elements, and stage 2
    uses it only when it is handed the very gradient arenas of stage 1.  Any other
    buffer (equal values or not) must be aggregated afresh; keys and importance of the
    stage-2 elements then follow the stage-2 gradients, as in the oracle."""
    say("stage-2 gradient source", stage2_input)
    wl = W.custom([37, 1, 128, 5, 9000, 64, 3, 4096, 4097, 30001], 6, 0.5, align=4, config_id=23)
    rng = np.random.default_rng(11)
    arena = wl.arena_elems()
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    for step in range(3):
        gib = random_bits(rng, arena, real)
        o.set_gib(GRAN_ELEMENT, gib); c.osp_set_gib(GRAN_ELEMENT, gib)
        g1 = wl.make_grads(0, step)
        stride1 = g1.shape[1]
        if stage2_input == "other_values":
            g2 = wl.make_grads(1, step)
        elif stage2_input == "other_stride":
            g2 = np.zeros((wl.n_workers, stride1 + 8), F)
            g2[:, :stride1] = g1
        else:
            g2 = g1
        gd1 = job.upload_grads(g1)
        gd2 = gd1 if stage2_input == "same_buffer" else job.upload_grads(g2)
        o.ps_aggregate_update(1, g1); c.osp_ps_aggregate_update(1, gd1, stride1)
        compare_state(job, o, "agg1")
        o.apply_stage(1); c.osp_apply_stage(1)
        o.lgp_correct(g1); c.osp_lgp_correct(gd1, stride1)
        compare_state(job, o, "lgp")
        o.ps_aggregate_update(2, g2); c.osp_ps_aggregate_update(2, gd2, g2.shape[1])
        compare_state(job, o, "agg2")
        o.apply_stage(2); c.osp_apply_stage(2)
        compare_state(job, o, "apply2")
        keys = c.osp_get_keys()
        assert np.array_equal(keys[real], o.keys()[real]), "element keys"
        if step % 2 == 0:
            o.split(GRAN_LAYER, wl.budget); c.osp_split(GRAN_LAYER, wl.budget)
            imp = c.osp_get_importance()
            assert np.allclose(imp, o.importance, rtol=1e-12, atol=0)
            compare_gib(job, o, f"layer split after element stages, step {step}")
        else:
            o.split(GRAN_ELEMENT, wl.budget); c.osp_split(GRAN_ELEMENT, wl.budget)
            compare_gib(job, o, f"element split, step {step}")


@pytest.mark.parametrize("stage2_input", ["same_buffer", "other_values", "other_stride"])
@pytest.mark.parametrize("n_workers,keep", [(6, True), (6, False), (3, True), (19, True)])
def test_layer_lgp_keeps_stage2_aggregate(stage2_input, n_workers, keep):
    """Layer-granular GIB, replicas in sync, N >= 4: LGP leaves the aggregate of the stage-2
    gradients (with importance and keys) for the stage-2 call, which uses it only when it is
    handed the very arenas LGP read; any other buffer is aggregated afresh.  The option
    switches it off; below 4 workers it is not used.  Results equal the oracle's either way."""
    say("layer kept aggregate", stage2_input, n_workers, keep)
    wl = W.custom([37, 1, 128, 5, 9000, 64, 3, 4096, 4097, 30001], n_workers, 0.5, align=4,
                  config_id=24)
    rng = np.random.default_rng(12)
    arena = wl.arena_elems()
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    wts = None
    if n_workers == 19:
        wts = rng.random(n_workers).astype(F); wts /= wts.sum()
    o = make_oracle(wl, weights=wts)
    job = device_job(wl, weights=wts, element_keys=True)
    c = job.ctx
    c.osp_set_keep_stage2_aggregate(keep)
    for step in range(4):
        gib = random_layer_gib(rng, wl.n_tensors)
        if step == 3:
            gib[:] = 0                                  # everything in stage 2
        o.set_gib(GRAN_LAYER, gib); c.osp_set_gib(GRAN_LAYER, gib)
        g1 = wl.make_grads(0, step)
        stride1 = g1.shape[1]
        if stage2_input == "other_values":
            g2 = wl.make_grads(1, step)
        elif stage2_input == "other_stride":
            g2 = np.zeros((wl.n_workers, stride1 + 8), F)
            g2[:, :stride1] = g1
        else:
            g2 = g1
        gd1 = job.upload_grads(g1)
        gd2 = gd1 if stage2_input == "same_buffer" else job.upload_grads(g2)
        o.ps_aggregate_update(1, g1); c.osp_ps_aggregate_update(1, gd1, stride1)
        if step != 1:                                   # LGP before or after the install
            o.apply_stage(1); c.osp_apply_stage(1)
        o.lgp_correct(g1); c.osp_lgp_correct(gd1, stride1)
        assert c.osp_lgp_read_shared()
        assert c.osp_lgp_kept_aggregate() == (keep and n_workers >= 4)
        compare_state(job, o, "lgp")
        if step == 1:
            o.apply_stage(1); c.osp_apply_stage(1)
        if step == 2:
            with pytest.raises(Exception):
                c.osp_set_keep_stage2_aggregate(not keep)   # not between the two stages
        o.ps_aggregate_update(2, g2); c.osp_ps_aggregate_update(2, gd2, g2.shape[1])
        compare_state(job, o, "agg2")
        o.apply_stage(2); c.osp_apply_stage(2)
        compare_state(job, o, "apply2")
        keys = c.osp_get_keys()
        assert np.array_equal(keys[real], o.keys()[real]), "element keys"
        if step % 2 == 0:
            o.split(GRAN_LAYER, wl.budget); c.osp_split(GRAN_LAYER, wl.budget)
            imp = c.osp_get_importance()
            assert np.allclose(imp, o.importance, rtol=1e-12, atol=0)
            compare_gib(job, o, f"layer split, step {step}")
        else:
            o.split(GRAN_ELEMENT, wl.budget); c.osp_split(GRAN_ELEMENT, wl.budget)
            compare_gib(job, o, f"element split after layer stages, step {step}")


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_arena_refilled_between_the_stages(gran):
    """The same gradient buffer with NEW values at stage 2: the library reuses the kept
    aggregate by pointer, so the caller says that the arenas changed (osp_drop_kept_aggregate)
    and stage 2 aggregates afresh; results equal the oracle's with the new values."""
    say("arena refilled", gran)
    import torch
    wl = W.custom([37, 1, 128, 5, 9000, 64, 3, 4096, 4097, 30001], 6, 0.5, align=4, config_id=25)
    rng = np.random.default_rng(3)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    gib = (random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER
           else random_bits(rng, wl.arena_elems(), real))
    o.set_gib(gran, gib); c.osp_set_gib(gran, gib)
    g1, g2 = wl.make_grads(0, 0), wl.make_grads(1, 0)
    gd = job.upload_grads(g1); s_ = gd.shape[1]
    o.ps_aggregate_update(1, g1); o.apply_stage(1); o.lgp_correct(g1)
    c.osp_ps_aggregate_update(1, gd, s_); c.osp_apply_stage(1); c.osp_lgp_correct(gd, s_)
    gd.copy_(torch.from_numpy(g2))                      # the caller overwrites the arenas ...
    c.osp_drop_kept_aggregate()                         # ... and says so
    o.ps_aggregate_update(2, g2); o.apply_stage(2)
    c.osp_ps_aggregate_update(2, gd, s_); c.osp_apply_stage(2)
    compare_state(job, o, "refilled arena")
    assert np.array_equal(c.osp_get_keys()[real], o.keys()[real])


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("order", ["rs_lgp_last", "lgp_before_install", "lgp_after_stage2", "no_install1"])
@pytest.mark.parametrize("n_workers", [3, 12])
def test_lgp_paths_and_call_orders(gran, order, n_workers):
    """LGP has two implementations (per-replica values, or the PS values read once when the
    replicas are known to be in sync); every legal order of calls must give the oracle's
    result whichever one runs, over iterations that do and do not restore consistency."""
    say("lgp paths", gran, order, n_workers)
    wl = W.custom([5000, 3, 1029, 64, 2048, 70000], n_workers, 0.5, align=4, config_id=60 + n_workers)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True, declare_in_sync=(order != "lgp_before_install"))
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    for step in range(4):
        g = wl.make_grads(0, step); gd = job.upload_grads(g); s_ = g.shape[1]
        if order == "rs_lgp_last":
            seq = ["agg1", "apply1", "lgp", "agg2", "apply2"]
        elif order == "lgp_before_install":
            seq = ["agg1", "lgp", "apply1", "agg2", "apply2"]
        elif order == "lgp_after_stage2":
            seq = ["agg1", "apply1", "agg2", "lgp", "apply2"]
        else:                                   # stage 1 never installed on odd steps: replicas drift
            seq = ["agg1", "lgp", "agg2", "apply2"] if step % 2 else ["agg1", "apply1", "lgp", "agg2", "apply2"]
        for call in seq:
            if call == "agg1":
                o.ps_aggregate_update(1, g); c.osp_ps_aggregate_update(1, gd, s_)
            elif call == "agg2":
                o.ps_aggregate_update(2, g); c.osp_ps_aggregate_update(2, gd, s_)
            elif call == "apply1":
                o.apply_stage(1); c.osp_apply_stage(1)
            elif call == "apply2":
                o.apply_stage(2); c.osp_apply_stage(2)
            else:
                o.lgp_correct(g); c.osp_lgp_correct(gd, s_)
            compare_state(job, o, f"{order} step {step} after {call}")
        o.split(gran, wl.budget); c.osp_split(gran, wl.budget)
        compare_gib(job, o, f"{order} step {step}")


def test_single_pass_equals_two_stages():
    say("stage 0")
    wl = W.get("tiny")
    o = make_oracle(wl); job = device_job(wl, element_keys=True)
    g = wl.make_grads(0, 0); gd = job.upload_grads(g)
    o.ps_aggregate_update(0, g); o.apply_stage(0)
    job.ctx.osp_ps_aggregate_update(0, gd, g.shape[1]); job.ctx.osp_apply_stage(0)
    compare_state(job, o, "stage0")
    o.split(GRAN_ELEMENT, wl.budget); job.ctx.osp_split(GRAN_ELEMENT, wl.budget)
    compare_gib(job, o, "split after stage 0")


# --------------------------------------------------------------------------
# edge cases of the split
# --------------------------------------------------------------------------

@pytest.mark.parametrize("frac", [0.0, 1.0, 0.999])
@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("windows", [False, True])
def test_degenerate_budgets(gran, frac, windows):
    """Budget 0: every iteration is a BSP step; budget M: nothing is synchronized in the RS
    window and every worker runs on its own estimate (Sec. 4.3); one stage is empty either way."""
    say("budget", gran, frac, windows)
    wl = W.get("tiny")
    budget = int(frac * wl.n_params)
    sizes = run_steps(wl, gran, 3, budget=budget, windows=windows)
    if frac == 0.0:
        assert sizes == [0, 0, 0]
    if frac == 1.0:
        assert sizes == [wl.n_params] * 3


def _split_from_keys(keys_f32, budget, numel=None):
    """Drive both sides to a state whose element keys are |keys_f32| (P = 1,
    one worker, gradient = keys) and split at element granularity."""
    n = len(keys_f32)
    wl = W.custom(numel or [n], 1, align=4, config_id=31)
    arena = wl.arena_elems()
    off = wl.offsets()
    real = brute.real_mask(wl.numel, off, arena)
    P = np.zeros(arena, F); P[real] = 1.0
    g = np.zeros((1, arena), F); g[0, real] = keys_f32
    o = OracleOSP(wl.numel, off, arena, 1, 0.1, 0.0); o.load_params(P)
    job = device_job(wl, element_keys=True, mu=0.0, params=P)
    gd = job.upload_grads(g)
    with np.errstate(all="ignore"):
        o.ps_aggregate_update(0, g)
    job.ctx.osp_ps_aggregate_update(0, gd, arena)
    o.split(GRAN_ELEMENT, budget); job.ctx.osp_split(GRAN_ELEMENT, budget)
    compare_gib(job, o, "adversarial split")
    compare_state(job, o, "adversarial state")
    keys = job.ctx.osp_get_keys()
    assert np.array_equal(keys[real], o.keys()[real])
    return o


@pytest.mark.parametrize("case", ["all_equal", "all_zero", "inside_ties", "ties_across_tiles",
                                  "nan_inf", "neg_zero", "denormal", "two_values_multi_tensor",
                                  "nan_payloads", "few_ties", "ties_2048", "ties_2049",
                                  "ties_in_a_crowded_bucket", "big_bucket_few_ties", "all_equal_200k"])
def test_split_element_adversarial(case):
    say("adversarial", case)
    rng = np.random.default_rng(4)
    n = 50_000                                  # several 8192-key tiles and a ragged tail
    numel = None
    if case in ("few_ties", "ties_2048", "ties_2049"):
        # distinct keys except for t copies of one value, scattered over the arena; the budget
        # ends inside them (t <= 2048: cut through the listed candidates; above: per-tile counts)
        t = {"few_ties": 7, "ties_2048": 2048, "ties_2049": 2049}[case]
        keys = (1.0 + rng.permutation(n) / n).astype(F)          # distinct, one binade
        keys[keys == F(1.5)] = F(1.99999)
        where = np.sort(rng.choice(n, t, replace=False))
        keys[where] = F(1.5)
        assert int((keys == F(1.5)).sum()) == t
        k = int((keys < F(1.5)).sum()) + t // 2 + 1
    elif case == "ties_in_a_crowded_bucket":
        # 30 000 keys share the threshold's upper 22 bits (all listed), 40 of them equal it
        keys = (1.0 + rng.permutation(n) / n).astype(F)
        base = np.float32(1.25).view(np.uint32)
        low = rng.integers(0, 1024, 30_000).astype(np.uint32)
        idx = rng.choice(n, 30_000, replace=False)
        keys.view(np.uint32)[idx] = (base & np.uint32(0xFFFFFC00)) | low
        ties = idx[:40]
        keys.view(np.uint32)[ties] = (base & np.uint32(0xFFFFFC00)) | np.uint32(512)
        T = keys[ties[0]]
        k = int((keys < T).sum()) + 13
    elif case == "big_bucket_few_ties":
        # more keys in the threshold's bucket than the candidate list holds: not listed
        n = 200_000
        keys = (1.0 + rng.permutation(n) / n).astype(F)
        base = np.float32(1.25).view(np.uint32)
        idx = rng.choice(n, 90_000, replace=False)
        keys.view(np.uint32)[idx] = (base & np.uint32(0xFFFFFC00)) | rng.integers(0, 1024, 90_000).astype(np.uint32)
        T = keys[idx[0]]
        k = int((keys < T).sum()) + max(1, int((keys == T).sum()) // 2)
    elif case == "all_equal_200k":
        n = 200_000
        keys, k = np.full(n, 3.0, F), 123_457
    elif case == "all_equal":
        keys, k = np.full(n, 3.0, F), 23_456
    elif case == "all_zero":
        keys, k = np.zeros(n, F), 8192 * 3      # boundary exactly on a tile edge
    elif case == "inside_ties":
        keys, k = rng.integers(0, 4, n).astype(F), 30_001
    elif case == "ties_across_tiles":
        keys = np.ones(n, F); keys[:100] = 0.5; keys[40_000:] = 2.0; k = 100 + 8192 * 2 + 17
    elif case == "nan_inf":
        keys = rng.standard_normal(n).astype(F)
        keys[[5, 20_000]] = np.nan; keys[100] = np.inf; keys[49_999] = -np.inf
        k = n - 3
    elif case == "neg_zero":
        keys = np.zeros(n, F); keys[::2] = -0.0; keys[7] = 1.0; k = 25_000
    elif case == "nan_payloads":
        keys = rng.standard_normal(n).astype(F)
        bits = keys.view(np.uint32)
        bits[10] = 0x7FFFFFFF; bits[9000] = 0x7FC00001; bits[30_000] = 0xFFC12345; bits[30_001] = 0x7F800001
        k = n - 2                               # two of the four NaNs stay in stage 1: the last two
    elif case == "denormal":
        keys = (rng.standard_normal(n) * 1e-41).astype(F)      # subnormal magnitudes
        keys[::5] = 0.0
        k = 20_000
    else:
        numel = [8190, 3, 20_001, 1, 21_805]
        keys = rng.integers(1, 3, n).astype(F); k = 26_000
    _split_from_keys(keys, k, numel)


def test_split_element_guess_of_the_first_digit():
    """The first radix pass also refines the bucket the previous split's threshold fell into.
    Splits in a row on one context: budgets that keep the threshold in its bucket (the guess
    is right and the second pass is skipped), budgets and keys that move it (the guess is
    wrong and the second pass is made), budget 0 in between; every GIB against the oracle."""
    say("element split: guessed first digit")
    rng = np.random.default_rng(11)
    n = 300_000                                  # several histogram workgroups, ragged tail
    wl = W.custom([n - 7, 3, 4], 1, align=4, config_id=33)
    arena, off = wl.arena_elems(), wl.offsets()
    real = brute.real_mask(wl.numel, off, arena)
    P = np.zeros(arena, F); P[real] = 1.0
    o = OracleOSP(wl.numel, off, arena, 1, 0.0, 0.0); o.load_params(P)     # lr 0: P stays 1
    job = device_job(wl, element_keys=True, lr=0.0, mu=0.0, params=P)
    narrow = (1.0 + rng.random(n)).astype(F)                    # one binade: 4 first digits
    wide = (10.0 ** rng.uniform(-6, 2, n)).astype(F)            # many binades
    rounds = [(narrow, n // 2), (narrow, n // 2 + 11), (narrow, n // 2 - 5000), (narrow, 17),
              (narrow, n // 2), (wide, n // 2), (wide, n // 2 + 1), (wide, 0), (wide, n // 2),
              (narrow, n - 3), (narrow, n), (narrow, n // 2)]
    for r, (vals, k) in enumerate(rounds):
        g = np.zeros((1, arena), F); g[0, real] = vals
        gd = job.upload_grads(g)
        o.ps_aggregate_update(0, g); job.ctx.osp_ps_aggregate_update(0, gd, arena)
        o.split(GRAN_ELEMENT, k); job.ctx.osp_split(GRAN_ELEMENT, k)
        compare_gib(job, o, f"round {r}, budget {k}")
        assert np.array_equal(job.ctx.osp_get_keys()[real], o.keys()[real])


@pytest.mark.parametrize("ties,take", [(3000, 1234), (5, 2), (70_000, 69_999)])
def test_split_element_ties_cut_at_large_indices(ties, take):
    """Ties at the threshold spread over 8.4 M keys: the cut by arena index works through its
    11-bit digits up to bit 23 (few ties: the candidate list; 70 000: the per-tile counts).
    Keys go straight into the context-free entry point; expected bitmap: the oracle's sort."""
    import torch
    from paper_2306_16926_amd.binding import osp_split_element_static
    say("ties at large indices", ties, take)
    rng = np.random.default_rng(ties)
    n = (1 << 23) + 4096
    bits = (np.uint32(0x3F800000) + rng.permutation(n).astype(np.uint32))   # distinct, positive, finite
    T = np.uint32(0x3FC00000)
    bits[bits == T] = np.uint32(0x3F800000) + np.uint32(n)                   # (still distinct)
    where = rng.choice(n, ties, replace=False)
    where[:3] = [n - 1, (1 << 22) + 1, 5]                                    # both ends and a middle digit
    bits[where] = T
    k = int((bits < T).sum()) + take
    o = OracleOSP([n], [0], n, 1, 0.1, 0.0)
    o.q[:] = bits.view(F)
    assert np.array_equal(o.keys(), bits)
    o.split(GRAN_ELEMENT, k)
    keys = torch.from_numpy(bits.view(np.int32)).cuda()
    out = torch.zeros((n + 31) // 32, dtype=torch.int32, device="cuda")
    osp_split_element_static(keys, n, k, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, o.gib_bits), int((got != o.gib_bits).sum())
    s2 = np.unpackbits(got.view(np.uint8), bitorder="little")[:n] == 0
    assert int(s2.sum()) == k and int(s2[np.sort(where)][:take].sum()) == take


def test_split_layer_ties_nan_and_zero_layers():
    say("layer ties")
    wl = W.custom([8, 8, 8, 8, 8, 5000], 1, align=4, config_id=32)
    arena = wl.arena_elems(); off = wl.offsets()
    real = brute.real_mask(wl.numel, off, arena)
    P = np.zeros(arena, F); P[real] = 1.0
    g = np.zeros((1, arena), F)
    g[0, 0:8] = 1.0
    g[0, 24:32] = np.nan
    g[0, 32:40] = 0.5
    g[0, 40:5040] = 1e-3
    o = OracleOSP(wl.numel, off, arena, 1, 0.1, 0.0); o.load_params(P)
    job = device_job(wl, mu=0.0, params=P)
    gd = job.upload_grads(g)
    for budget in (8, 24, 5032, 5040):
        say("  budget", budget)
        oo = OracleOSP(wl.numel, off, arena, 1, 0.1, 0.0); oo.load_params(P)
        jj = device_job(wl, mu=0.0, params=P)
        with np.errstate(all="ignore"):
            oo.ps_aggregate_update(0, g)
        jj.ctx.osp_ps_aggregate_update(0, gd, arena)
        oo.split(GRAN_LAYER, budget); jj.ctx.osp_split(GRAN_LAYER, budget)
        compare_gib(jj, oo, f"budget {budget}")
        compare_state(jj, oo, f"budget {budget}")
        imp = jj.ctx.osp_get_importance()
        assert np.isnan(imp[3]) and imp[1] == 0.0 and imp[2] == 0.0
    del o, job


@pytest.mark.parametrize("n_layers", [1025, 2500, 4200])
def test_split_layer_many_layers(n_layers):
    """More layers than the ranking workgroup has threads (1024) and than one of its
    LDS tiles holds (2048); sizes repeat, so importances tie and the index decides."""
    say("many layers", n_layers)
    rng = np.random.default_rng(n_layers)
    numel = rng.integers(1, 40, n_layers).tolist()
    numel[7] = 3000
    wl = W.custom(numel, 2, 0.45, align=4, config_id=34)
    run_steps(wl, GRAN_LAYER, 3)
    run_steps(wl, GRAN_LAYER, 2, windows=True)
    # identical layers: every importance ties within its group
    wl = W.custom([16] * n_layers, 1, 0.5, align=4, config_id=35)
    arena = wl.arena_elems()
    P = np.ones(arena, F)
    g = np.zeros((1, arena), F)
    g[0, :] = 1e-3
    g[0, ::3 * 16] = 2e-3
    o = OracleOSP(wl.numel, wl.offsets(), arena, 1, 0.1, 0.0); o.load_params(P)
    job = device_job(wl, mu=0.0, params=P)
    gd = job.upload_grads(g)
    o.ps_aggregate_update(0, g); job.ctx.osp_ps_aggregate_update(0, gd, arena)
    for budget in (16 * 7, 16 * 1024, 16 * 1024 + 15, wl.budget):
        o.split(GRAN_LAYER, budget); job.ctx.osp_split(GRAN_LAYER, budget)
        compare_gib(job, o, f"ties, budget {budget}")
        o.ps_aggregate_update(0, g); job.ctx.osp_ps_aggregate_update(0, gd, arena)


def test_nonfinite_gradients_flow_through_every_call():
    say("nonfinite")
    wl = W.custom([3000, 7, 2049], 3, 0.5, align=4, config_id=33)
    o = make_oracle(wl); job = device_job(wl, element_keys=True)
    rng = np.random.default_rng(3)
    gib = random_bits(rng, wl.arena_elems(),
                      brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems()))
    o.set_gib(GRAN_ELEMENT, gib); job.ctx.osp_set_gib(GRAN_ELEMENT, gib)
    g = wl.make_grads(0, 0)
    g[0, 5] = np.inf; g[1, 5] = -np.inf; g[2, 9] = np.nan; g[1, 3001] = np.inf
    g[0, 100:110] = 1e38; g[1, 100:110] = 3e38        # overflow in the sum
    g[:, 200:260] = 1e-44                              # subnormal sums
    gd = job.upload_grads(g)
    with np.errstate(all="ignore"):
        o.sync_step(g, GRAN_ELEMENT, wl.budget)
    job.sync_step(gd, GRAN_ELEMENT, wl.budget)
    compare_state(job, o, "nonfinite")
    compare_gib(job, o, "nonfinite")


# --------------------------------------------------------------------------
# order-of-calls errors (need real launches to advance the state)
# --------------------------------------------------------------------------

def test_state_machine():
    say("state machine")
    from paper_2306_16926_amd import binding as B
    wl = W.get("tiny")
    job = device_job(wl)
    c = job.ctx
    g = wl.make_grads(0, 0); gd = job.upload_grads(g); s = g.shape[1]

    def bad(fn, *a):
        with pytest.raises(B.OspError) as e:
            fn(*a)
        assert e.value.status == B.OSP_ERR_BAD_STATE, e.value
    before = job.download()
    bad(c.osp_ps_aggregate_update, 1, gd, s)            # no GIB yet
    bad(c.osp_get_gib)
    c.osp_ps_aggregate_update(0, gd, s)                 # stage 0 needs none
    bad(c.osp_lgp_correct, gd, s)                       # LGP has no place in a BSP step
    c.osp_apply_stage(0); c.osp_split(B.OSP_GRAN_LAYER, wl.budget)
    bad(c.osp_split, B.OSP_GRAN_LAYER, wl.budget)       # nothing aggregated since
    bad(c.osp_ps_aggregate_update, 2, gd, s)            # stage 2 before stage 1
    bad(c.osp_apply_stage, 1)
    bad(c.osp_lgp_correct, gd, s)
    c.osp_ps_aggregate_update(1, gd, s)
    bad(c.osp_ps_aggregate_update, 1, gd, s)            # stage 2 pending
    bad(c.osp_ps_aggregate_update, 0, gd, s)
    bad(c.osp_set_gib, B.OSP_GRAN_LAYER, np.ones(wl.n_tensors, np.uint8))
    bad(c.osp_apply_stage, 2)
    bad(c.osp_split, B.OSP_GRAN_LAYER, wl.budget)
    with pytest.raises(B.OspError) as e:
        c.osp_split(B.OSP_GRAN_ELEMENT, wl.budget)       # element_keys off
    assert e.value.status == B.OSP_ERR_UNSUPPORTED
    c.osp_lgp_correct(gd, s)
    bad(c.osp_lgp_correct, gd, s)                       # twice
    c.osp_apply_stage(1)
    snap = job.download()
    bad(c.osp_ps_aggregate_update, 1, gd, s)
    after = job.download()
    for a, b in zip(snap, after):                       # a rejected call touches nothing
        assert np.array_equal(a, b)
    c.osp_ps_aggregate_update(2, gd, s)
    c.osp_apply_stage(2)
    bad(c.osp_lgp_correct, gd, s)                       # would undo the correction
    c.osp_ps_aggregate_update(1, gd, s)                 # split is optional: next iteration
    c.osp_ps_aggregate_update(2, gd, s)
    c.osp_split(B.OSP_GRAN_LAYER, 0)
    layer, _, n2 = c.osp_get_gib()
    assert n2 == 0 and layer.all()
    assert not np.array_equal(before[0], after[0])


def test_reference_traffic_kernels_move_what_they_say():
    """osp_stream_copy and osp_stream_pattern are bandwidth reference lines, not part of the
    step; they still have to do exactly the stated data movement."""
    import torch
    from paper_2306_16926_amd.binding import OspError, osp_stream_copy, osp_stream_pattern
    say("reference kernels")
    n, stride = 100_000, 100_064
    for n_read in (1, 3, 8, 16, 19):
        for n_rw in (1, 2):
            reads = torch.randint(-8, 9, (n_read, stride), device="cuda").float()
            rw = torch.randint(-8, 9, (n_rw, stride), device="cuda").float()
            want = rw.clone()
            want[:, :n] += reads[:, :n].sum(0)              # small integers: exact in any order
            osp_stream_pattern(reads, n_read, stride, rw, n_rw, stride, n)
            assert torch.equal(rw, want), (n_read, n_rw)
    src = torch.arange(1 << 16, device="cuda", dtype=torch.float32)
    dst = torch.zeros_like(src)
    osp_stream_copy(dst, src, src.numel() * 4)
    assert torch.equal(dst, src)
    with pytest.raises(OspError):
        osp_stream_pattern(reads, 3, n - 4, rw, 1, stride, n)   # stride below the stream length


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_learning_rate_schedule(gran):
    """osp_set_hyper between iterations (the learning rate is halved every 10 epochs, Sec. 5.1.3);
    refused between the two stages of one iteration."""
    from paper_2306_16926_amd.binding import OspError
    say("lr schedule", gran)
    wl = W.custom([5000, 3, 1029, 64, 2048, 30000], 4, 0.5, align=4, config_id=400)
    o = make_oracle(wl)
    job = device_job(wl, element_keys=True)
    c = job.ctx
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
    lr = wl.lr
    for step in range(6):
        if step in (2, 4):
            lr *= 0.5
            mu = wl.momentum if step == 2 else 0.5
            o.set_hyper(lr, mu); c.osp_set_hyper(lr, mu)
        g = wl.make_grads(0, step); gd = job.upload_grads(g); s_ = g.shape[1]
        if step % 2:
            o.sync_step(g, gran, wl.budget); job.sync_step_windows(gd, gran, wl.budget)
        else:
            o.ps_aggregate_update(1, g); c.osp_ps_aggregate_update(1, gd, s_)
            with pytest.raises(OspError):
                c.osp_set_hyper(0.01, 0.0)              # between the stages
            o.apply_stage(1); c.osp_apply_stage(1)
            o.lgp_correct(g); c.osp_lgp_correct(gd, s_)
            o.ps_aggregate_update(2, g); c.osp_ps_aggregate_update(2, gd, s_)
            o.apply_stage(2); c.osp_apply_stage(2)
            o.split(gran, wl.budget); c.osp_split(gran, wl.budget)
        compare_state(job, o, f"lr schedule step {step}")
        compare_gib(job, o, f"lr schedule step {step}")


def test_arena_beyond_2_to_31_elements():
    """A tensor of more than 2^31 elements: every index computation has to be 64-bit.  Too large
    for the oracle to hold, so the check is the closed form of a BSP step with mu = 0 (P - lr *
    mean gradient, V = mean gradient), evaluated by separately rounded torch operations on
    the GPU and compared bit for bit over the whole arena; then the two-stage calls with the small
    tensor in stage 2."""
    import torch
    from paper_2306_16926_amd.binding import Context
    say("2^31+ elements")
    big = (1 << 31) + 4096 + 36
    numel = [big, 1000]
    off = [0, -(-big // 1024) * 1024]
    arena = off[1] + 1024
    N, lr = 2, 0.25
    stride = arena + 1024
    dev = torch.device("cuda")
    ctx = Context(numel, off, arena, N, lr, 0.0)
    P = torch.empty(arena, dtype=torch.float32, device=dev)
    step = 1 << 26
    for a in range(0, arena, step):                       # a ramp that differs across 2^31
        n = min(step, arena - a)
        P[a:a + n] = torch.arange(a, a + n, device=dev, dtype=torch.float64).mul_(1e-9).float()
    P0 = P.clone()
    V = torch.zeros(arena, dtype=torch.float32, device=dev)
    Pw = torch.zeros((N, stride), dtype=torch.float32, device=dev)
    Pw[:, :arena] = P
    ws = torch.empty(ctx.osp_workspace_bytes(), dtype=torch.uint8, device=dev)
    ctx.osp_bind(P, V, Pw, stride, ws, replicas_in_sync=True)
    g = torch.empty((N, stride), dtype=torch.float32, device=dev)
    g[0].fill_(0.5); g[1].fill_(-0.25)
    g[0, big - 7:big] = 3.0                                # the tail of the big tensor, beyond 2^31
    g[1, 5] = 8.0
    ctx.osp_set_gib(0, np.array([1, 0], np.uint8))         # small tensor in stage 2
    gbar = (g[0, :arena] + g[1, :arena]) * 0.5             # sum, then times fl(1/2): exact here
    want_P = P0 - gbar * lr                                # two separately rounded operations
    want_P[big:off[1]] = P0[big:off[1]]; want_P[off[1] + 1000:] = P0[off[1] + 1000:]   # padding untouched
    ctx.osp_ps_aggregate_update(1, g, stride)
    ctx.osp_apply_stage(1)
    ctx.osp_lgp_correct(g, stride)
    torch.cuda.synchronize()
    assert torch.equal(P[:big], want_P[:big])
    assert torch.equal(P[big:], P0[big:])                  # stage 2 and padding not yet touched
    assert torch.equal(Pw[0, :big], want_P[:big]) and torch.equal(Pw[1, :big], want_P[:big])
    lgp1 = P0[off[1]:off[1] + 1000] - g[1, off[1]:off[1] + 1000] * lr
    assert torch.equal(Pw[1, off[1]:off[1] + 1000], lgp1)
    ctx.osp_ps_aggregate_update(2, g, stride)
    ctx.osp_apply_stage(2)
    torch.cuda.synchronize()
    assert torch.equal(P, want_P)
    assert torch.equal(V[:big], gbar[:big]) and torch.equal(V[off[1]:off[1] + 1000], gbar[off[1]:off[1] + 1000])
    assert torch.equal(Pw[0, :arena], want_P) and torch.equal(Pw[1, :arena], want_P)
    assert bool((Pw[:, arena:] == 0).all())
    # the split sees the big tensor's importance as the larger one: budget of 1000 picks the small tensor
    ctx.osp_split(0, 1000)
    layer, _, n2 = ctx.osp_get_gib()
    assert layer.tolist() == [1, 0] and n2 == 1000
    imp = ctx.osp_get_importance()
    want_imp = 0.0
    for a in range(0, big, step):                          # |fl(gbar * P)| summed in fp64, in pieces
        b = min(big, a + step)
        want_imp += (gbar[a:b] * P0[a:b]).abs().double().sum().item()
    assert abs(imp[0] - want_imp) <= 1e-9 * want_imp
