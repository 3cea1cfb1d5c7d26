"""Pins for the CPU oracle: each test checks the C oracle against something
that is not the oracle (a closed form, a library routine, a NumPy brute force
written separately, an invariant the paper states), so that a dropped term, a
wrong sign or index, or a transposed operand fails at least one of them."""
import math

import numpy as np
import pytest
import torch

from oracle.osp_oracle import GRAN_ELEMENT, GRAN_LAYER, OracleOSP
from paper_2306_16926_amd import workloads as W
from tests import brute
from tests.helpers import (bits_to_bool, make_oracle, random_bits, random_layer_gib,
                           read_fixture)

F = np.float32


def small_wl(n_workers=3, seed_id=7):
    # ragged sizes, a 1-element tensor, offsets only 4-aligned
    return W.custom([37, 1, 128, 5, 1000, 64, 3], n_workers, align=4, config_id=seed_id)


def same(a, b):
    return np.array_equal(a, b, equal_nan=True)


# --------------------------------------------------------------------------
# hand-worked example (tests/golden/hand_example.txt)
# --------------------------------------------------------------------------

def hand_oracle(fx):
    numel = fx["numel"].astype(np.int64)
    off = np.array([0, 4], np.int64)
    o = OracleOSP(numel, off, 8, 2, 0.5, 0.5)
    P = np.zeros(8, F); V = np.zeros(8, F)
    P[[0, 1, 4]] = fx["P"]; V[[0, 1, 4]] = fx["V"]
    o.load_params(P, V)
    g = np.zeros((2, 8), F)
    g[0, [0, 1, 4]] = fx["g0"]; g[1, [0, 1, 4]] = fx["g1"]
    return o, g


def test_hand_example_update_and_importance():
    fx = read_fixture("hand_example.txt")
    o, g = hand_oracle(fx)
    o.ps_aggregate_update(0, g)
    idx = [0, 1, 4]
    assert same(o.V[idx], fx["V_new"].astype(F))
    assert same(o.P[idx], fx["P_new"].astype(F))
    assert same(o.q[idx], fx["I_elem"].astype(F))
    assert same(o.layer_importance(), fx["I_layer"])
    # padding never written
    assert not o.P[[2, 3, 5, 6, 7]].any() and not o.V[[2, 3, 5, 6, 7]].any()


@pytest.mark.parametrize("budget", [1, 2, 3])
def test_hand_example_layer_split(budget):
    fx = read_fixture("hand_example.txt")
    o, g = hand_oracle(fx)
    o.ps_aggregate_update(0, g)
    n2 = o.split(GRAN_LAYER, budget)
    want = fx[f"gib_budget{budget}"].astype(np.uint8)
    assert same(o.gib_layer, want)
    assert n2 == int(np.array([2, 1])[want == 0].sum())


@pytest.mark.parametrize("budget", [1, 2])
def test_hand_example_element_split(budget):
    fx = read_fixture("hand_example.txt")
    o, g = hand_oracle(fx)
    o.ps_aggregate_update(0, g)
    o.split(GRAN_ELEMENT, budget)
    arena_idx = {0: 0, 1: 1, 2: 4}
    want = np.ones(32, bool)
    for e in fx[f"s2_elems_budget{budget}"].astype(int):
        want[arena_idx[e]] = False
    assert same(bits_to_bool(o.gib_bits, 32), want)


def test_hand_example_lgp():
    fx = read_fixture("hand_example.txt")
    o, g = hand_oracle(fx)
    o.set_gib(GRAN_LAYER, fx["gib_budget2"].astype(np.uint8))
    o.lgp_correct(g)
    assert same(o.Pw[0, [0, 1, 4]], fx["lgp_w0"].astype(F))
    assert same(o.Pw[1, [0, 1, 4]], fx["lgp_w1"].astype(F))


# --------------------------------------------------------------------------
# PS update: library special case, closed form, partition independence
# --------------------------------------------------------------------------

def test_bsp_step_matches_torch_sgd():
    """Empty stage 2 (Sec. 4.3: everything in RS is BSP) must be a plain
    SGD-with-momentum step on the mean gradient; checked against
    torch.optim.SGD over three chained steps."""
    wl = W.get("tiny")
    o = make_oracle(wl)
    p = torch.tensor(o.P.copy(), requires_grad=True)
    opt = torch.optim.SGD([p], lr=wl.lr, momentum=wl.momentum, dampening=0)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    for step in range(3):
        g = wl.make_grads(0, step)
        o.ps_aggregate_update(1, g)          # GIB all-important: stage 1 is everything
        o.ps_aggregate_update(2, g)          # empty
        p.grad = torch.tensor(g.astype(np.float64).mean(0).astype(F))
        opt.step()
        ref = p.detach().numpy()
        # rtol of a few fp32 ulps; atol covers parameters that land next to zero
        assert np.allclose(o.P[real], ref[real], rtol=2e-6, atol=1e-9)


def test_closed_form_single_worker_no_momentum():
    wl = small_wl(n_workers=1)
    o = make_oracle(wl, mu=0.0, lr=0.25)
    P0 = o.P.copy()
    g = wl.make_grads(0, 0)
    o.ps_aggregate_update(0, g)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    want = P0 - F(0.25) * g[0]
    assert same(o.P[real], want[real])
    assert same(o.V[real], g[0][real])       # V = 0*V + g
    assert same(o.P[~real], P0[~real])


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_partition_independence(gran):
    """No gradient is dropped (Sec. 2.2.2, 3.2): for any GIB, stage 1 followed
    by stage 2 leaves the PS exactly where one BSP step would."""
    wl = small_wl()
    rng = np.random.default_rng(5)
    g = wl.make_grads(0, 0)
    a = make_oracle(wl); b = make_oracle(wl)
    gib = random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER else random_bits(rng, wl.arena_elems())
    a.set_gib(gran, gib)
    a.ps_aggregate_update(1, g)
    mid = a.P.copy()
    a.ps_aggregate_update(2, g)
    b.ps_aggregate_update(0, g)
    assert same(a.P, b.P) and same(a.V, b.V) and same(a.q, b.q)
    assert not same(mid, a.P)                # stage 2 did do something
    # each element updated exactly once: a third call on stage 1 changes state again
    c = make_oracle(wl); c.set_gib(gran, gib); c.ps_aggregate_update(1, g)
    assert same(c.P, mid)


@pytest.mark.parametrize("weighted", [False, True])
def test_aggregate_matches_bruteforce(weighted):
    wl = small_wl(n_workers=5)
    wts = None
    if weighted:
        wts = np.array([0.1, 0.3, 0.05, 0.35, 0.2], F)
    o = make_oracle(wl, weights=wts)
    b = brute.Brute(wl.numel, wl.offsets(), wl.arena_elems(), 5, wl.lr, wl.momentum, wts)
    b.load(o.P.copy())
    for step in range(2):
        g = wl.make_grads(0, step)
        o.ps_aggregate_update(0, g); b.agg(0, g)
        assert same(o.P, b.P) and same(o.V, b.V) and same(o.q, b.q)


@pytest.mark.parametrize("weighted", [False, True])
def test_worker_and_replica_strides_are_honoured(weighted):
    """Gradient arenas and replicas that are further apart than one arena: a full
    step must match the brute force (which slices the arena out of every row),
    and the gap between arenas must stay untouched."""
    wl = small_wl(n_workers=3)
    arena = wl.arena_elems()
    gs, ps = arena + 12, arena + 8
    wts = np.array([0.5, 0.125, 0.375], F) if weighted else None
    o = make_oracle(wl, weights=wts, param_stride=ps)
    o.Pw[:, arena:] = 77.0
    b = brute.Brute(wl.numel, wl.offsets(), arena, 3, wl.lr, wl.momentum, wts)
    b.load(o.P.copy())
    rng = np.random.default_rng(1)
    gib = random_layer_gib(rng, wl.n_tensors)
    o.set_gib(GRAN_LAYER, gib)
    b.s2 = brute.stage2_mask_from_layer_gib(gib, wl.numel, wl.offsets(), arena)
    g = np.full((3, gs), 5.0, F)                 # garbage in the gap
    g[:, :arena] = wl.make_grads(0, 0)
    for call in ("agg1", "apply1", "lgp", "agg2", "apply2"):
        if call.startswith("agg"):
            o.ps_aggregate_update(int(call[-1]), g); b.agg(int(call[-1]), g)
        elif call.startswith("apply"):
            o.apply_stage(int(call[-1])); b.apply(int(call[-1]))
        else:
            o.lgp_correct(g); b.lgp(g)
        assert same(o.P, b.P) and same(o.V, b.V) and same(o.Pw[:, :arena], b.Pw), call
    assert (o.Pw[:, arena:] == 77.0).all()


def test_power_of_two_weights_equal_plain_mean():
    """alpha_w = 1/4 for four workers: scaling by a power of two commutes with
    rounding, so the weighted form must reproduce the unweighted one bit for bit
    (catches a weight applied to the wrong worker or a missing 1/N)."""
    wl = small_wl(n_workers=4)
    g = wl.make_grads(0, 0)
    a = make_oracle(wl); b = make_oracle(wl, weights=np.full(4, 0.25, F))
    a.ps_aggregate_update(0, g); b.ps_aggregate_update(0, g)
    assert same(a.P, b.P) and same(a.V, b.V)


def test_weights_attach_to_the_right_worker():
    wl = small_wl(n_workers=3)
    g = wl.make_grads(0, 0)
    wts = np.array([0.0, 1.0, 0.0], F)
    o = make_oracle(wl, weights=wts, mu=0.0, lr=1.0)
    P0 = o.P.copy()
    o.ps_aggregate_update(0, g)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    assert same(o.P[real], (P0 - g[1])[real])


def test_momentum_carries_over_steps():
    """Constant gradient c, P0 = 0: V_t = c (1 + mu + ... + mu^(t-1)) and
    P_t = -lr sum V_i; with c = 1, mu = 0.5, lr = 0.5 all values are dyadic."""
    wl = W.custom([8], 2, align=4)
    o = OracleOSP(wl.numel, wl.offsets(), wl.arena_elems(), 2, 0.5, 0.5)
    o.load_params(np.zeros(wl.arena_elems(), F))
    g = np.ones((2, wl.arena_elems()), F)
    vs, ps = [], []
    for _ in range(3):
        o.ps_aggregate_update(0, g)
        vs.append(float(o.V[0])); ps.append(float(o.P[0]))
    assert vs == [1.0, 1.5, 1.75]
    assert ps == [-0.5, -1.25, -2.125]


# --------------------------------------------------------------------------
# LGP, apply, Eq. 7
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_lgp_is_stale_minus_lr_local_gradient(gran):
    wl = small_wl(n_workers=4)
    rng = np.random.default_rng(11)
    o = make_oracle(wl)
    arena = wl.arena_elems()
    gib = random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER else random_bits(rng, arena)
    o.set_gib(gran, gib)
    stale = o.Pw.copy()
    g = wl.make_grads(0, 0)
    o.lgp_correct(g)
    if gran == GRAN_LAYER:
        s2 = brute.stage2_mask_from_layer_gib(gib, wl.numel, wl.offsets(), arena)
    else:
        s2 = brute.stage2_mask_from_bits(gib, wl.numel, wl.offsets(), arena)
    assert s2.any() and (~s2).any()
    want = stale - F(wl.lr) * g
    for w in range(4):
        assert same(o.Pw[w][s2], want[w][s2])            # every stage-2 element, exactly
        assert same(o.Pw[w][~s2], stale[w][~s2])         # stage 1 and padding untouched
    assert o.n_stage2 == int(s2.sum())


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_full_step_restores_consistency_and_eq7(gran):
    """After the stage-2 correction every replica equals the PS on every
    element, and Eq. 7 evaluated literally lands on the same values."""
    wl = small_wl(n_workers=4)
    rng = np.random.default_rng(3)
    o = make_oracle(wl)
    arena = wl.arena_elems()
    gib = random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER else random_bits(rng, arena)
    o.set_gib(gran, gib)
    g = wl.make_grads(0, 0)
    o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
    # after the RS window: stage-1 elements already global, stage-2 carry the estimate
    assert not same(o.Pw[0], o.Pw[1])
    P_old = o.P.copy()
    o.ps_aggregate_update(2, g)
    lit = o.eq7_literal(g, P_old, o.P)
    o.apply_stage(2)
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    for w in range(4):
        assert same(o.Pw[w][real], o.P[real])
        rel = np.abs(lit[w][real] - o.P[real]) / np.maximum(np.abs(o.P[real]), 1e-3)
        assert rel.max() < 1e-6


def test_single_worker_no_momentum_estimate_is_already_global():
    wl = small_wl(n_workers=1)
    o = make_oracle(wl, mu=0.0)
    o.set_gib(GRAN_LAYER, np.zeros(wl.n_tensors, np.uint8))   # everything in stage 2
    g = wl.make_grads(0, 0)
    o.ps_aggregate_update(1, g); o.apply_stage(1); o.lgp_correct(g)
    est = o.Pw.copy()
    o.ps_aggregate_update(2, g); o.apply_stage(2)
    assert same(est, o.Pw)


def test_degrades_to_bsp_and_asp():
    """Sec. 4.3: budget 0 is BSP; budget M leaves the PS untouched during the RS
    window while every worker takes its own local step (ASP-like)."""
    wl = W.get("tiny")
    g = wl.make_grads(0, 0)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    # BSP
    a = make_oracle(wl); b = make_oracle(wl)
    a.ps_aggregate_update(0, g); a.split(GRAN_LAYER, 0)
    assert a.n_stage2 == 0 and a.gib_layer.all()
    b.set_gib(GRAN_LAYER, a.gib_layer)
    b.sync_step(g, GRAN_LAYER, 0)
    assert same(a.P, b.P)
    for w in range(wl.n_workers):
        assert same(b.Pw[w][real], b.P[real])
    # ASP
    c = make_oracle(wl)
    c.ps_aggregate_update(0, g); c.split(GRAN_LAYER, wl.n_params)
    assert c.n_stage2 == wl.n_params and not c.gib_layer.any()
    c2 = make_oracle(wl); c2.set_gib(GRAN_LAYER, c.gib_layer)
    P0 = c2.P.copy()
    c2.ps_aggregate_update(1, g); c2.apply_stage(1); c2.lgp_correct(g)
    assert same(c2.P, P0)
    for w in range(wl.n_workers):
        assert same(c2.Pw[w][real], (P0 - F(wl.lr) * g[w][:wl.arena_elems()])[real])


# --------------------------------------------------------------------------
# importance (Eq. 3 / Eq. 4)
# --------------------------------------------------------------------------

def test_layer_importance_matches_fsum():
    wl = W.get("tiny")
    o = make_oracle(wl)
    g = wl.make_grads(0, 0)
    P0 = o.P.copy()
    o.ps_aggregate_update(0, g)
    gbar = brute.aggregate(g[:, :wl.arena_elems()])
    imp = o.layer_importance()
    for l, (a, n) in enumerate(zip(wl.offsets(), wl.numel)):
        vals = np.abs(gbar[a:a + n] * P0[a:a + n])           # fp32 product, pre-update P
        want = math.fsum(float(v) for v in vals)
        assert abs(imp[l] - want) <= 1e-12 * want
        assert same(o.q[a:a + n], vals)


def test_importance_uses_pre_update_parameters_and_aggregated_gradient():
    wl = W.custom([4], 2, align=4)
    o = OracleOSP(wl.numel, wl.offsets(), 4, 2, 0.5, 0.0)
    o.load_params(np.array([1, 2, -4, 8], F))
    g = np.array([[1, 1, 1, 1], [3, -1, 1, 0]], F)
    o.ps_aggregate_update(0, g)
    assert same(o.q, np.array([2, 0, 4, 4], F))              # |mean(g) * P_before|
    assert o.layer_importance()[0] == 10.0


def test_compensated_sum_keeps_small_terms():
    """2^30 followed by 2^20 copies of 2^-30: a naive fp32 or a sloppy fp64 loop
    would still pass, but a sum that drops or reorders layers would not; the
    value is exact in fp64."""
    n = 1 << 12
    wl = W.custom([n + 1], 1, align=4)
    o = OracleOSP(wl.numel, wl.offsets(), wl.arena_elems(), 1, 0.1, 0.0)
    o.load_params(np.ones(wl.arena_elems(), F))
    g = np.zeros((1, wl.arena_elems()), F)
    g[0, 0] = 2.0 ** 30
    g[0, 1:n + 1] = 2.0 ** -30
    o.ps_aggregate_update(0, g)
    assert o.layer_importance()[0] == 2.0 ** 30 + n * 2.0 ** -30


# --------------------------------------------------------------------------
# split
# --------------------------------------------------------------------------

@pytest.mark.parametrize("frac", [0.0, 0.1, 0.3, 0.5, 0.9, 1.0])
def test_split_layer_matches_bruteforce_and_invariants(frac):
    wl = W.get("tiny")
    o = make_oracle(wl)
    b = brute.Brute(wl.numel, wl.offsets(), wl.arena_elems(), wl.n_workers, wl.lr, wl.momentum)
    b.load(o.P.copy())
    g = wl.make_grads(0, 0)
    o.ps_aggregate_update(0, g); b.agg(0, g)
    budget = int(frac * wl.n_params)
    n2 = o.split(GRAN_LAYER, budget)
    gib, taken, rank = b.split_layer(budget)
    assert same(o.gib_layer, gib) and n2 == taken
    assert list(o.order) == rank
    # invariants: within budget; the next layer in rank would not fit
    assert n2 <= budget
    nxt = [l for l in rank if gib[l] == 1]
    if nxt:
        assert n2 + wl.numel[nxt[0]] > budget
    # stage 2 is a prefix of the ranking
    flags = [gib[l] for l in rank]
    assert flags == sorted(flags)


def test_split_layer_ties_and_nan():
    wl = W.custom([8, 8, 8, 8, 8], 1, align=4)
    o = OracleOSP(wl.numel, wl.offsets(), wl.arena_elems(), 1, 0.1, 0.0)
    o.load_params(np.ones(wl.arena_elems(), F))
    g = np.zeros((1, wl.arena_elems()), F)
    g[0, 0:8] = 1.0          # layer 0: importance 8
    # layers 1 and 2: all-zero gradients, importance exactly 0 -> tie, lower index first
    g[0, 24:32] = np.nan     # layer 3: NaN ranks last
    g[0, 32:40] = 0.5        # layer 4: importance 4
    o.ps_aggregate_update(0, g)
    o.split(GRAN_LAYER, 8)
    assert list(o.order) == [1, 2, 4, 0, 3]
    assert list(o.gib_layer) == [1, 0, 1, 1, 1]
    o.split(GRAN_LAYER, 40)
    assert not o.gib_layer.any()


def _element_case(keys_f32, budget):
    n = len(keys_f32)
    wl = W.custom([n], 1, align=4)
    arena = wl.arena_elems()
    o = OracleOSP(wl.numel, wl.offsets(), arena, 1, 0.1, 0.0)
    o.load_params(np.ones(arena, F))
    g = np.zeros((1, arena), F)
    g[0, :n] = keys_f32
    o.ps_aggregate_update(0, g)
    o.split(GRAN_ELEMENT, budget)
    return bits_to_bool(o.gib_bits, arena)[:n], o


@pytest.mark.parametrize("case", ["all_equal", "all_zero", "k0", "kM", "inside_ties",
                                  "ties_across_word", "nan_inf", "neg_zero", "nan_payloads"])
def test_split_element_adversarial(case):
    n = 200
    rng = np.random.default_rng(2)
    if case == "all_equal":
        keys, k = np.full(n, 3.0, F), 77
    elif case == "all_zero":
        keys, k = np.zeros(n, F), 33
    elif case == "k0":
        keys, k = rng.standard_normal(n).astype(F), 0
    elif case == "kM":
        keys, k = rng.standard_normal(n).astype(F), n
    elif case == "inside_ties":
        keys = rng.integers(0, 4, n).astype(F); k = 90
    elif case == "ties_across_word":
        keys = np.ones(n, F); keys[:20] = 0.5; k = 20 + 30      # ties run across bit 32|33
    elif case == "nan_inf":
        keys = rng.standard_normal(n).astype(F)
        keys[5] = np.nan; keys[100] = np.inf; keys[150] = -np.inf; keys[160] = np.nan
        k = n - 3
    elif case == "nan_payloads":
        # NaNs with different payloads are ONE value: among them the index decides.
        # The NaN at the lower index carries the larger payload, so an order on raw
        # bit patterns would put it last instead of first.
        keys = rng.standard_normal(n).astype(F)
        bits = keys.view(np.uint32)
        bits[10] = 0x7FFFFFFF; bits[60] = 0x7FC00001; bits[120] = 0xFFC12345
        k = n - 2                                # exactly one NaN goes to stage 2: the first
    else:
        keys = np.zeros(n, F); keys[::2] = -0.0; keys[7] = 1.0; k = 100
    imp, o = _element_case(keys, k)
    mag = np.abs(keys)
    kk = mag.view(np.uint32).copy()
    kk[np.isnan(mag)] = 0x7FC00000
    order = np.lexsort((np.arange(n), kk))
    want = np.ones(n, bool)
    want[order[:k]] = False
    assert same(imp, want)
    assert int((~imp).sum()) == k == o.n_stage2
    if 0 < k < n:
        assert kk[~imp].max() <= kk[imp].min()
    if case == "nan_inf":
        # NaN above Inf above finite: with k = n-3 the three left in stage 1 are
        # the two NaNs and ... one of the two infinities (the later index)
        assert imp[5] and imp[160] and imp[150] and not imp[100]
    if case == "all_equal":
        assert not imp[:k].any() and imp[k:].all()
    if case == "nan_payloads":
        assert not imp[10] and imp[60] and imp[120]


@pytest.mark.parametrize("frac", [0.0, 0.3, 0.5, 1.0])
def test_split_element_matches_bruteforce_tiny(frac):
    wl = W.get("tiny")
    o = make_oracle(wl)
    b = brute.Brute(wl.numel, wl.offsets(), wl.arena_elems(), wl.n_workers, wl.lr, wl.momentum)
    b.load(o.P.copy())
    g = wl.make_grads(0, 0)
    o.ps_aggregate_update(0, g); b.agg(0, g)
    budget = int(frac * wl.n_params)
    o.split(GRAN_ELEMENT, budget)
    bits = b.split_element(budget)
    assert same(o.gib_bits, bits)
    assert same(o.keys()[b.real], b.keys()[b.real])


@pytest.mark.parametrize("frac", [0.0, 0.3, 1.0])
@pytest.mark.parametrize("ties", [False, True])
def test_split_by_selection_equals_the_full_sort(frac, ties):
    """OracleOSP.split_element_by_selection (used where the full sort takes too long) against
    split(), the definition."""
    wl = W.get("tiny")
    o = make_oracle(wl)
    g = wl.make_grads(0, 0)
    if ties:                                      # few distinct magnitudes: long runs of equal keys
        g = (np.round(g * F(2000.0)) / F(2000.0)).astype(F)
        o.P[:] = np.sign(o.P) * F(0.25)
    o.ps_aggregate_update(0, g)
    budget = int(frac * wl.n_params)
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    if ties:
        assert np.unique(o.keys()[real]).size < 200
    assert o.split_element_by_selection(budget) == budget
    got = o.gib_bits.copy()
    o.split(GRAN_ELEMENT, budget)
    assert same(got, o.gib_bits)
    assert o.n_stage2 == budget


def test_split_by_selection_adversarial():
    """All keys equal, the cut inside a run of ties that crosses a bitmap word, NaN on top."""
    wl = small_wl(2)
    o = make_oracle(wl)
    n = wl.n_params
    for case in range(4):
        q = np.zeros(o.arena, F)
        real = brute.real_mask(o.numel, o.offset, o.arena)
        vals = {0: np.ones(n, F), 1: np.zeros(n, F),
                2: np.random.default_rng(1).integers(0, 3, n).astype(F),
                3: np.random.default_rng(2).standard_normal(n).astype(F)}[case]
        if case == 3:
            vals[3] = np.nan; vals[n // 2] = np.inf
        q[real] = np.abs(vals)
        o.q[:] = q
        for budget in (0, 1, n // 3, n - 1, n):
            o.split_element_by_selection(budget)
            got = o.gib_bits.copy()
            o.split(GRAN_ELEMENT, budget)
            assert same(got, o.gib_bits), (case, budget)


def test_split_element_rejects_bad_budget():
    wl = W.get("tiny")
    o = make_oracle(wl)
    with pytest.raises(ValueError):
        o.split(GRAN_ELEMENT, wl.n_params + 1)
    with pytest.raises(ValueError):
        o.split(GRAN_ELEMENT, -1)


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_partition_invariant_under_power_of_two_gradient_scaling(gran):
    wl = W.get("tiny")
    g = wl.make_grads(0, 0)
    a = make_oracle(wl); b = make_oracle(wl)
    a.ps_aggregate_update(0, g); b.ps_aggregate_update(0, g * F(64.0))
    a.split(gran, wl.budget); b.split(gran, wl.budget)
    assert same(a.gib_layer, b.gib_layer) and same(a.gib_bits, b.gib_bits)


def test_gib_is_under_1kb_below_1k_layers():
    # Sec. 4.1.2: below 1K layers the GIB is smaller than 1 KB
    wl = W.get("resnet152")
    assert wl.n_tensors < 1000
    assert np.ones(wl.n_tensors, np.uint8).nbytes < 1024


def test_learning_rate_schedule_matches_torch_sgd():
    """Halving the learning rate between iterations (Sec. 5.1.3): the momentum buffer carries
    over, as in torch.optim.SGD whose param_group lr is changed."""
    wl = small_wl(2)
    o = make_oracle(wl, lr=0.1, mu=0.9)
    o.set_gib(GRAN_LAYER, np.ones(wl.n_tensors, np.uint8))
    p = torch.tensor(o.P.copy(), dtype=torch.float32, requires_grad=True)
    opt = torch.optim.SGD([p], lr=0.1, momentum=0.9)
    lr = 0.1
    for step in range(4):
        if step == 2:
            lr = 0.05
            o.set_hyper(lr, 0.9)
            opt.param_groups[0]["lr"] = lr
        g = wl.make_grads(0, step)
        o.ps_aggregate_update(0, g)
        p.grad = torch.tensor((g[0, :wl.arena_elems()] + g[1, :wl.arena_elems()]) * F(0.5))
        opt.step()
    real = brute.real_mask(wl.numel, wl.offsets(), wl.arena_elems())
    assert np.allclose(o.P[real], p.detach().numpy()[real], rtol=2e-6, atol=1e-9)


# --------------------------------------------------------------------------
# gradient splitter (Sec. 4.5): dense G^i / G^u, and the PS update fed by them
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
def test_split_gradients_is_boolean_indexing(gran):
    """NumPy's boolean indexing is the definition: the stage's elements, in arena order."""
    wl = small_wl(4)
    rng = np.random.default_rng(3)
    arena = wl.arena_elems(); off = wl.offsets()
    real = brute.real_mask(wl.numel, off, arena)
    o = make_oracle(wl)
    if gran == GRAN_LAYER:
        gib = random_layer_gib(rng, wl.n_tensors)
        s2 = brute.stage2_mask_from_layer_gib(gib, wl.numel, off, arena)
    else:
        gib = random_bits(rng, arena, real)
        s2 = brute.stage2_mask_from_bits(gib, wl.numel, off, arena)
    o.set_gib(gran, gib)
    g = wl.make_grads(0, 0)
    g[:, ~real] = 9.0                        # padding must not reach either part
    g_i, g_u = o.split_gradients(g)
    assert g_i.shape[1] + g_u.shape[1] == wl.n_params and g_u.shape[1] == int(s2.sum())
    for w in range(wl.n_workers):
        assert same(g_i[w], g[w, :arena][real & ~s2])
        assert same(g_u[w], g[w, :arena][s2])
    # nothing dropped, nothing duplicated (Sec. 3.2): scattering both parts back gives g
    back = np.zeros(arena, F)
    back[real & ~s2] = g_i[1]; back[s2] = g_u[1]
    assert same(back[real], g[1, :arena][real])


def test_split_gradients_hand_example():
    # arena [a b . . c . . .], layers {a b} and {c}; element bitmap: a, c important, b not
    numel = np.array([2, 1], np.int64); off = np.array([0, 4], np.int64)
    o = OracleOSP(numel, off, 8, 2, 0.5, 0.5)
    o.load_params(np.zeros(8, F))
    g = np.zeros((2, 8), F)
    g[0, [0, 1, 4]] = [1.0, 2.0, 3.0]; g[1, [0, 1, 4]] = [-1.0, -2.0, -3.0]
    o.set_gib(GRAN_ELEMENT, np.array([0b11111101], np.uint32))
    g_i, g_u = o.split_gradients(g)
    assert g_i.tolist() == [[1.0, 3.0], [-1.0, -3.0]] and g_u.tolist() == [[2.0], [-2.0]]
    o.set_gib(GRAN_LAYER, np.array([0, 1], np.uint8))
    g_i, g_u = o.split_gradients(g)
    assert g_i.tolist() == [[3.0], [-3.0]] and g_u.tolist() == [[1.0, 2.0], [-1.0, -2.0]]
    # degenerate GIBs: one part is empty
    o.set_gib(GRAN_LAYER, np.array([1, 1], np.uint8))
    g_i, g_u = o.split_gradients(g)
    assert g_i.shape == (2, 3) and g_u.shape == (2, 0)


@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("weighted", [False, True])
def test_update_from_packed_gradients_equals_update_in_place(gran, weighted):
    """Feeding the PS the dense parts gives, bit for bit, what the gradients give in place,
    which in turn is pinned against torch.optim.SGD and the brute force above."""
    wl = small_wl(3)
    rng = np.random.default_rng(5)
    arena = wl.arena_elems()
    real = brute.real_mask(wl.numel, wl.offsets(), arena)
    wts = np.array([0.5, 0.2, 0.3], F) if weighted else None
    a = make_oracle(wl, weights=wts); b = make_oracle(wl, weights=wts)
    for step in range(2):
        gib = (random_layer_gib(rng, wl.n_tensors) if gran == GRAN_LAYER
               else random_bits(rng, arena, real))
        a.set_gib(gran, gib); b.set_gib(gran, gib)
        g = wl.make_grads(0, step)
        g_i, g_u = b.split_gradients(g)
        # strides larger than the part, garbage behind it
        pad_i = np.full((wl.n_workers, g_i.shape[1] + 5), 7.0, F); pad_i[:, :g_i.shape[1]] = g_i
        pad_u = np.full((wl.n_workers, g_u.shape[1] + 3), 7.0, F); pad_u[:, :g_u.shape[1]] = g_u
        a.ps_aggregate_update(1, g); b.ps_aggregate_update_packed(1, pad_i)
        assert same(a.P, b.P) and same(a.V, b.V) and same(a.q, b.q)
        a.ps_aggregate_update(2, g); b.ps_aggregate_update_packed(2, pad_u)
        assert same(a.P, b.P) and same(a.V, b.V) and same(a.q, b.q)


# --------------------------------------------------------------------------
# chained sync steps against the independent brute force
# --------------------------------------------------------------------------

@pytest.mark.parametrize("gran", [GRAN_LAYER, GRAN_ELEMENT])
@pytest.mark.parametrize("weighted", [False, True])
def test_three_chained_steps_match_bruteforce(gran, weighted):
    wl = W.get("tiny")
    wts = np.array([0.4, 0.1, 0.3, 0.2], F) if weighted else None
    o = make_oracle(wl, weights=wts)
    b = brute.Brute(wl.numel, wl.offsets(), wl.arena_elems(), wl.n_workers, wl.lr, wl.momentum, wts)
    b.load(o.P.copy())
    sizes = []
    for step in range(3):
        g = wl.make_grads(0, step)
        n2 = o.sync_step(g, gran, wl.budget)
        b.step(g, gran, wl.budget)
        assert same(o.P, b.P) and same(o.V, b.V) and same(o.Pw[:, :wl.arena_elems()], b.Pw)
        s2_o = (brute.stage2_mask_from_layer_gib(o.gib_layer, wl.numel, wl.offsets(), wl.arena_elems())
                if gran == GRAN_LAYER else
                brute.stage2_mask_from_bits(o.gib_bits, wl.numel, wl.offsets(), wl.arena_elems()))
        assert same(s2_o, b.s2)
        assert n2 == int(b.s2.sum())
        sizes.append(n2)
    assert sizes[0] > 0                      # the second and third step really ran two-stage
    if gran == GRAN_ELEMENT:
        assert sizes == [wl.budget] * 3


def test_openmp_build_is_bit_identical():
    wl = W.get("tiny")
    a = make_oracle(wl); b = make_oracle(wl, omp=True)
    for step in range(2):
        g = wl.make_grads(0, step)
        a.sync_step(g, GRAN_LAYER, wl.budget); b.sync_step(g, GRAN_LAYER, wl.budget)
    assert same(a.P, b.P) and same(a.V, b.V) and same(a.Pw, b.Pw) and same(a.gib_layer, b.gib_layer)
