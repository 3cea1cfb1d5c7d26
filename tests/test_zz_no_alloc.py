"""The allocation-free element split (osp_split_element_static: scratch in an array that is
part of the library's image) against osp_split(OSP_GRAN_ELEMENT) on a bound context, through
the C ABI: same keys, same budget, bitmaps bit for bit.  Two calls in a row share the one
scratch array, the second on a smaller input and with ties at the threshold."""
import numpy as np
import pytest

from paper_2306_16926_amd import workloads as W
from tests.gpu_common import device_job, say

pytestmark = pytest.mark.gpu

GRAN_ELEMENT = 1


def split_both_ways(wl, budget, grads_seed, quantise=False):
    import torch
    from paper_2306_16926_amd.binding import osp_split_element_static
    job = device_job(wl, element_keys=True)
    g = wl.make_grads(grads_seed, 0)
    if quantise:                                   # few distinct values: long runs of equal keys
        g = (np.round(g * np.float32(500.0)) / np.float32(500.0)).astype(np.float32)
        job.P.copy_(torch.sign(job.P) * 0.25)
    gd = job.upload_grads(g)
    job.ctx.osp_ps_aggregate_update(0, gd, gd.shape[1])
    job.ctx.osp_split(GRAN_ELEMENT, budget)
    _, want, n2 = job.ctx.osp_get_gib()
    assert n2 == budget
    keys = torch.from_numpy(job.ctx.osp_get_keys().view(np.int32)).cuda()
    arena = wl.arena_elems()
    words = (arena + 31) // 32
    out = torch.zeros(words, dtype=torch.int32, device="cuda")
    before = torch.cuda.memory_allocated()
    osp_split_element_static(keys, arena, budget, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got = out.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, want), f"{wl.name}: bitmaps differ in {int((got != want).sum())} words"
    if quantise:
        k = keys.cpu().numpy().view(np.uint32)
        s2 = np.unpackbits(got.view(np.uint8), bitorder="little")[:arena] == 0
        T = k[s2].max()
        assert ((k == T) & ~s2).any(), "the case is meant to cut a run of ties"


def test_static_scratch_split_matches_osp_split_twice_in_a_row():
    say("static split: resnet18-shaped, then tiny with ties")
    big = W.get("resnet18")
    split_both_ways(big, big.budget, 0)
    small = W.get("tiny")
    split_both_ways(small, small.budget, 3, quantise=True)
    say("static split: degenerate budgets on the same scratch")
    split_both_ways(small, 0, 4)
    split_both_ways(small, small.n_params, 5)
