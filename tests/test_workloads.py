"""The synthetic workloads reproduce the stated tensor and parameter counts."""
import numpy as np
import pytest

from paper_2306_16926_amd import workloads as W


@pytest.mark.parametrize("name", list(W.EXPECTED_COUNTS))
def test_counts(name):
    wl = W.get(name)
    assert (wl.n_tensors, wl.n_params) == W.EXPECTED_COUNTS[name]
    off = wl.offsets()
    assert (off % wl.align == 0).all() and (off % 4 == 0).all()
    ends = off + np.asarray(wl.numel)
    assert (off[1:] >= ends[:-1]).all() and ends[-1] <= wl.arena_elems()
    assert wl.worker_stride() >= wl.arena_elems() and wl.worker_stride() % 4 == 0


def test_seeded_and_distinct():
    wl = W.get("tiny")
    a = wl.make_grads(0, 0); b = wl.make_grads(0, 0); c = wl.make_grads(0, 1); d = wl.make_grads(1, 0)
    assert np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)
    assert not np.array_equal(a[0], a[1])
    t = wl.make_grads(0, 0, threads=4)
    assert np.array_equal(a, t)
    assert abs(float(a.std()) - 1e-3) < 1e-4
    assert abs(float(wl.make_params(0).std()) - 0.05) < 5e-3
