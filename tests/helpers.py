"""Shared test plumbing (no method arithmetic)."""
import os

import numpy as np

from oracle.osp_oracle import OracleOSP
from paper_2306_16926_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_fixture(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = np.array([float(x) for x in v.split()])
    return out


def make_oracle(wl, seed=0, align=None, weights=None, lr=None, mu=None, omp=False,
                param_stride=None):
    off = wl.offsets(align)
    o = OracleOSP(wl.numel, off, wl.arena_elems(align), wl.n_workers,
                  wl.lr if lr is None else lr, wl.momentum if mu is None else mu,
                  worker_weight=weights, omp=omp, param_stride=param_stride)
    o.load_params(wl.make_params(seed, align))
    return o


def random_layer_gib(rng, L):
    g = (rng.random(L) < 0.5).astype(np.uint8)
    return g


def random_bits(rng, arena, real=None):
    """Random element bitmap; with `real` (bool per arena element) the padding
    bits are set to 1, the normal form both sides report."""
    words = (arena + 31) // 32
    bits = rng.integers(0, 2**32, words, dtype=np.uint64).astype(np.uint32)
    if real is not None:
        pad = np.ones(words * 32, np.uint8)
        pad[:arena] = ~real
        bits |= np.packbits(pad, bitorder="little").view(np.uint32)
    return bits


def bits_to_bool(bits, arena):
    return np.unpackbits(np.asarray(bits, np.uint32).view(np.uint8), bitorder="little")[:arena] == 1
