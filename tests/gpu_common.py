"""Plumbing shared by the GPU parity tests (no method arithmetic): building a device job,
comparing its state and GIB with the oracle's, and running chained steps on both sides.

Bar: the stage-1/stage-2 partition bit-exact; fp32 parameters within a relative
error of 1e-5 (they are in fact bit-identical, which is asserted too, because
both sides evaluate the same sequence of separately rounded fp32 operations);
fp64 layer importances within 1e-12 relative (different summation order)."""
import sys

import numpy as np

from oracle.osp_oracle import GRAN_ELEMENT, GRAN_LAYER
from tests import brute
from tests.helpers import make_oracle

F = np.float32
REL_TOL = 1e-5           # tolerance of record for fp32 parameters


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def device_job(wl, seed=0, align=None, weights=None, element_keys=False, chunk_elems=0,
               lr=None, mu=None, param_stride=None, pad_fill=None, params=None,
               declare_in_sync=True):
    from paper_2306_16926_amd.device import DeviceJob
    p = wl.make_params(seed, align) if params is None else params
    return DeviceJob(wl.numel, wl.offsets(align), wl.arena_elems(align), wl.n_workers,
                     wl.lr if lr is None else lr, wl.momentum if mu is None else mu, p,
                     worker_weight=weights, element_keys=element_keys, chunk_elems=chunk_elems,
                     param_stride=param_stride, pad_fill=pad_fill,
                     declare_in_sync=declare_in_sync)


def close_enough(got, want, what):
    """rel 1e-5 (the stated bar), then bit equality (what the design promises)."""
    got = np.asarray(got); want = np.asarray(want)
    assert got.shape == want.shape, what
    both_nan = np.isnan(got) & np.isnan(want)
    fin = ~both_nan
    err = np.abs(got[fin].astype(np.float64) - want[fin].astype(np.float64))
    bound = REL_TOL * np.abs(want[fin].astype(np.float64))
    with np.errstate(invalid="ignore"):
        bad = ~((err <= bound) | (got[fin] == want[fin]))
    assert not bad.any(), f"{what}: {int(bad.sum())} elements outside rel {REL_TOL}"
    assert np.array_equal(got, want, equal_nan=True), f"{what}: not bit-identical"


def compare_state(job, o, what):
    P, V, Pw = job.download()
    close_enough(P, o.P, what + " P")
    close_enough(V, o.V, what + " V")
    close_enough(Pw[:, :o.arena], o.Pw[:, :o.arena], what + " Pw")


def compare_gib(job, o, what):
    layer, bits, n2 = job.ctx.osp_get_gib()
    if o.granularity == GRAN_LAYER:
        assert np.array_equal(layer, o.gib_layer), what + " layer GIB"
    else:
        assert np.array_equal(bits, o.gib_bits), what + " element bitmap"
    assert n2 == o.n_stage2, what + " n_stage2"


def run_steps(wl, gran, steps, seed=0, align=None, weights=None, chunk_elems=0, budget=None,
              threads=4, windows=False):
    budget = wl.budget if budget is None else budget
    o = make_oracle(wl, seed, align, weights)
    job = device_job(wl, seed, align, weights, element_keys=(gran == GRAN_ELEMENT),
                     chunk_elems=chunk_elems)
    all1 = np.ones(wl.n_tensors, np.uint8)
    o.set_gib(GRAN_LAYER, all1); job.ctx.osp_set_gib(GRAN_LAYER, all1)
    sizes = []
    for step in range(steps):
        g = wl.make_grads(seed, step, align, threads=threads)
        gd = job.upload_grads(g)
        o.sync_step(g, gran, budget)
        if windows:
            job.sync_step_windows(gd, gran, budget)
        else:
            job.sync_step(gd, gran, budget)
        compare_state(job, o, f"{wl.name} step {step}")
        compare_gib(job, o, f"{wl.name} step {step}")
        if gran == GRAN_LAYER:
            imp = job.ctx.osp_get_importance()
            rel = np.abs(imp - o.importance) / np.maximum(np.abs(o.importance), 1e-300)
            assert rel.max() <= 1e-12, f"layer importance rel err {rel.max()}"
        else:
            real = brute.real_mask(wl.numel, wl.offsets(align), wl.arena_elems(align))
            keys = job.ctx.osp_get_keys()
            assert np.array_equal(keys[real], o.keys()[real]), "element keys"
            assert (keys[~real] == 0xFFFFFFFF).all()
        sizes.append(o.n_stage2)
        del gd
    return sizes


