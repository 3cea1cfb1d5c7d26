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
    assert wl.replica_stride() >= wl.arena_elems() and wl.replica_stride() % 4 == 0
    # the measured layout: rows a multiple of 1 KiB apart, gradient rows 8 KiB past a round
    # number, replica rows 1 KiB past it and never a multiple of 8 MiB
    assert wl.replica_stride() % 256 == 0 and wl.worker_stride() % 256 == 0
    assert wl.worker_stride() % 1024 == 0 and wl.replica_stride() % 1024 == 256
    assert (wl.replica_stride() * 4) % (8 << 20) != 0


def test_seeded_and_distinct():
    wl = W.get("tiny")
    a = wl.make_grads(0, 0); b = wl.make_grads(0, 0); c = wl.make_grads(0, 1); d = wl.make_grads(1, 0)
    assert np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)
    assert not np.array_equal(a[0], a[1])
    t = wl.make_grads(0, 0, threads=4)
    assert np.array_equal(a, t)
    assert abs(float(a.std()) - 1e-3) < 1e-4
    assert abs(float(wl.make_params(0).std()) - 0.05) < 5e-3


def test_bf16_storage_rounds_like_torch_and_widens_exactly():
    import torch
    from paper_2306_16926_amd.workloads import from_bf16, to_bf16
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(200_000) * 10.0 ** rng.uniform(-8, 3, 200_000)).astype(np.float32)
    a[:6] = [np.inf, -np.inf, 0.0, -0.0, 3.3895314e38, 1e-40]      # overflow to inf, subnormal
    h = to_bf16(a)
    t = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(h, t.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(from_bf16(h), t.float().numpy())
    assert np.array_equal(to_bf16(from_bf16(h)), h)               # representable values are fixed points
    assert np.isnan(from_bf16(to_bf16(np.array([np.nan], np.float32))))[0]
