"""S(G^u) tuning (Sec. 4.1.2, Eq. 5, Algorithm 1): pins of the oracle against
the closed forms the paper states, then the library against the oracle.
Host-only functions: no GPU involved."""
import math

import numpy as np
import pytest

from oracle import osp_oracle as O
from paper_2306_16926_amd import binding as B


# ---- oracle pins ----------------------------------------------------------

def test_first_epoch_is_bsp():
    assert O.tune_budget(1, 2.3, 2.3, 1e6, 10_000_000) == 0
    assert O.tune_budget(1, 0.0, 2.3, 1e6, 10_000_000) == 0


def test_loss_equal_to_first_gives_zero_and_vanishing_loss_gives_umax():
    assert O.tune_budget(2, 2.0, 2.0, 600.0, 1000) == 0
    assert O.tune_budget(9, 0.0, 2.0, 600.0, 1000) == 600
    assert O.tune_budget(9, 1e-3, 2.0, 600.0, 1000) == 599        # (1 - 0.0005) * 600 = 599.7


def test_hand_values():
    # (1 - 0.5/2.0) * 600 = 450 ; U_max = 900 is capped at 0.8 * 1000 = 800 -> 600
    assert O.tune_budget(3, 0.5, 2.0, 600.0, 1000) == 450
    assert O.tune_budget(3, 0.5, 2.0, 900.0, 1000) == 600
    assert O.tune_budget(3, 1.0, 2.0, 900.0, 1000) == 400


def test_cap_at_80_percent_of_the_model():
    assert O.tune_budget(5, 0.0, 1.0, 1e12, 1000) == 800
    assert O.tune_budget(5, 0.0, 1.0, 799.0, 1000) == 799


def test_loss_above_first_never_goes_negative():
    assert O.tune_budget(4, 3.0, 2.0, 600.0, 1000) == 0


def test_grows_as_the_loss_falls():
    losses = np.linspace(2.0, 0.0, 41)
    s = [O.tune_budget(2 + i, float(l), 2.0, 5000.0, 100_000) for i, l in enumerate(losses)]
    assert s == sorted(s) and s[0] == 0 and s[-1] == 5000
    # linear in the loss
    assert s[20] == 2500


def test_upper_bound_closed_form():
    # 10 Gbit/s of fp32 elements, no loss, 0.1 s of compute, 8 workers
    b = 10e9 / 32
    assert O.ics_upper_bound(b, 0.0, 0.1, 8) == b * 0.1 / 8
    assert O.ics_upper_bound(b, 0.25, 0.1, 8) == b * 1.25 * 0.1 / 8
    # doubling the workers halves the bound; doubling compute time doubles it
    assert O.ics_upper_bound(b, 0.0, 0.1, 16) == O.ics_upper_bound(b, 0.0, 0.1, 8) / 2
    assert O.ics_upper_bound(b, 0.0, 0.2, 8) == O.ics_upper_bound(b, 0.0, 0.1, 8) * 2


# ---- library against the oracle -------------------------------------------

def test_library_matches_oracle_on_a_grid():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        epoch = int(rng.integers(1, 50))
        L = float(rng.uniform(0.1, 10.0))
        loss = float(rng.uniform(0.0, 1.3) * L)
        model = int(rng.integers(1, 200_000_000))
        u = float(rng.uniform(0.0, 1.5) * model)
        assert B.osp_tune_budget(epoch, loss, L, u, model) == O.tune_budget(epoch, loss, L, u, model)
    for _ in range(500):
        b, lr, tc = (float(x) for x in rng.uniform(0, 1, 3) * (1e9, 0.2, 2.0))
        n = int(rng.integers(1, 64))
        assert B.osp_ics_upper_bound(b, lr, tc, n) == O.ics_upper_bound(b, lr, tc, n)


def test_library_rejects_bad_arguments():
    assert B.osp_tune_budget(0, 1.0, 2.0, 10.0, 100) == -1
    assert B.osp_tune_budget(2, float("nan"), 2.0, 10.0, 100) == -1
    assert B.osp_tune_budget(2, 1.0, 0.0, 10.0, 100) == -1
    assert B.osp_tune_budget(2, 1.0, 2.0, -1.0, 100) == -1
    assert B.osp_tune_budget(2, 1.0, 2.0, 10.0, -5) == -1
    assert B.osp_ics_upper_bound(1e9, 0.0, 0.1, 0) == 0.0
    assert B.osp_ics_upper_bound(float("inf"), 0.0, 0.1, 4) == 0.0


def test_budget_feeds_split_range():
    # what the tuner returns is always a legal budget for osp_split: 0 <= S <= M
    for loss in (0.0, 0.3, 1.0, 5.0):
        s = B.osp_tune_budget(7, loss, 1.0, 1e18, 12345)
        assert 0 <= s <= 12345
