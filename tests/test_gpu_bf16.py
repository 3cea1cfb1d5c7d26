"""bfloat16 gradient arenas: the oracle is fed the widened values, the bar stays bit equality."""
import numpy as np
import pytest

from oracle.osp_oracle import GRAN_ELEMENT, GRAN_LAYER
from paper_2306_16926_amd import workloads as W
from tests.gpu_common import F, compare_gib, compare_state, device_job, say
from tests.helpers import make_oracle

pytestmark = pytest.mark.gpu

# --------------------------------------------------------------------------
# bfloat16 gradient arenas: the oracle is fed the widened values (exact), so
# the bar stays bit equality
# --------------------------------------------------------------------------

def run_steps_bf16(wl, gran, steps, weights=None, chunk_elems=0, align=None, seed=0, threads=4,
                   windows=False):
    o = make_oracle(wl, seed, align, weights)
    job = device_job(wl, seed, align, weights, element_keys=(gran == GRAN_ELEMENT),
                     chunk_elems=chunk_elems)
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); job.ctx.osp_set_gib(GRAN_LAYER, all1)
    sizes = []
    for step in range(steps):
        h = W.to_bf16(wl.make_grads(seed, step, align, threads=threads))
        g = W.from_bf16(h)
        gd = job.upload_grads_bf16(h)
        o.sync_step(g, gran, wl.budget)
        if windows:
            job.sync_step_windows_bf16(gd, gran, wl.budget)
        else:
            job.sync_step_bf16(gd, gran, wl.budget)
        compare_state(job, o, f"bf16 {wl.name} step {step}")
        compare_gib(job, o, f"bf16 {wl.name} step {step}")
        sizes.append(o.n_stage2)
    return sizes


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("weighted", [False, True])
def test_bf16_gradients_tiny(gran, weighted):
    say("bf16 tiny", gran, weighted)
    wl = W.get("tiny")
    wts = np.array([0.4, 0.1, 0.3, 0.2], F) if weighted else None
    sizes = run_steps_bf16(wl, gran, 3, weights=wts)
    assert sizes[0] > 0
    run_steps_bf16(wl, gran, 2, align=64, chunk_elems=1024)
    run_steps_bf16(wl, gran, 3, weights=wts, windows=True)


@pytest.mark.parametrize("n_workers", [1, 3, 8, 9, 16, 17])
def test_bf16_gradients_worker_counts(n_workers):
    say("bf16 workers", n_workers)
    wl = W.custom([5000, 3, 1029, 64, 2048, 1], n_workers, 0.4, align=4, config_id=240 + n_workers)
    run_steps_bf16(wl, GRAN_LAYER, 2)
    run_steps_bf16(wl, GRAN_ELEMENT, 2)
    run_steps_bf16(wl, GRAN_LAYER, 3, windows=True)
    run_steps_bf16(wl, GRAN_ELEMENT, 3, windows=True)


def test_bf16_gradients_lgp_paths_nonfinite_and_errors():
    """LGP per replica (replicas not declared in sync) and from the PS values; non-finite
    gradients; misaligned arenas are refused."""
    say("bf16 lgp paths")
    from paper_2306_16926_amd.binding import OspError
    wl = W.custom([5000, 3, 1029, 64, 70000], 5, 0.5, align=4, config_id=250)
    for in_sync in (True, False):
        o = make_oracle(wl)
        job = device_job(wl, element_keys=True, declare_in_sync=in_sync)
        c = job.ctx
        all1 = np.ones(wl.n_tensors, np.uint8)
        o.set_gib(GRAN_LAYER, all1); c.osp_set_gib(GRAN_LAYER, all1)
        for step in range(3):
            gf = wl.make_grads(0, step)
            if step == 2:
                gf[1, 7] = np.inf; gf[2, 5001] = np.nan; gf[0, 5010] = -np.inf
            h = W.to_bf16(gf); g = W.from_bf16(h); gd = job.upload_grads_bf16(h); s_ = g.shape[1]
            gran = GRAN_ELEMENT if step else GRAN_LAYER
            with np.errstate(all="ignore"):
                o.ps_aggregate_update(1, g); c.osp_ps_aggregate_update_bf16(1, gd, s_)
                o.lgp_correct(g); c.osp_lgp_correct_bf16(gd, s_)       # before the install
                compare_state(job, o, f"lgp in_sync={in_sync} step {step}")
                o.apply_stage(1); c.osp_apply_stage(1)
                o.ps_aggregate_update(2, g); c.osp_ps_aggregate_update_bf16(2, gd, s_)
                o.apply_stage(2); c.osp_apply_stage(2)
                compare_state(job, o, f"in_sync={in_sync} step {step}")
                o.split(gran, wl.budget); c.osp_split(gran, wl.budget)
            compare_gib(job, o, f"in_sync={in_sync} step {step}")
        with pytest.raises(OspError):
            c.osp_ps_aggregate_update_bf16(1, gd.data_ptr() + 2, s_)   # not 8-byte aligned


def test_bf16_gradients_cnn_shaped():
    say("bf16 resnet18")
    run_steps_bf16(W.get("resnet18"), GRAN_LAYER, 2, threads=8)
    run_steps_bf16(W.get("resnet18"), GRAN_ELEMENT, 2, threads=8)
    run_steps_bf16(W.get("resnet18"), GRAN_LAYER, 2, threads=8, windows=True)
    run_steps_bf16(W.get("resnet18"), GRAN_ELEMENT, 3, threads=8, windows=True)
