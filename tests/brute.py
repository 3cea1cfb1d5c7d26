"""NumPy brute force of one OSP iteration, used only to pin the C oracle.

Written independently of oracle/osp_oracle.c: whole-array NumPy operations on
boolean stage masks instead of per-element loops, fp32 arrays so that every
NumPy ufunc call is one IEEE binary32 rounding per element.
"""
import math

import numpy as np

F = np.float32


def real_mask(numel, offset, arena):
    m = np.zeros(arena, bool)
    for a, n in zip(offset, numel):
        m[int(a):int(a) + int(n)] = True
    return m


def layer_of(numel, offset, arena):
    lay = np.full(arena, -1, np.int64)
    for l, (a, n) in enumerate(zip(offset, numel)):
        lay[int(a):int(a) + int(n)] = l
    return lay


def stage2_mask_from_layer_gib(gib, numel, offset, arena):
    lay = layer_of(numel, offset, arena)
    m = np.zeros(arena, bool)
    ok = lay >= 0
    m[ok] = np.asarray(gib)[lay[ok]] == 0
    return m


def stage2_mask_from_bits(bits, numel, offset, arena):
    b = np.unpackbits(np.asarray(bits, np.uint32).view(np.uint8), bitorder="little")[:arena]
    return (b == 0) & real_mask(numel, offset, arena)


def aggregate(grads, weights=None):
    """Sequential fp32 sum over workers in ascending index (Sec. 2.1.1)."""
    n = grads.shape[0]
    if weights is None:
        acc = grads[0].copy()
        for w in range(1, n):
            acc = acc + grads[w]
        return acc * (F(1.0) / F(n))
    acc = F(weights[0]) * grads[0]
    for w in range(1, n):
        acc = acc + F(weights[w]) * grads[w]
    return acc


class Brute:
    def __init__(self, numel, offset, arena, n_workers, lr, mu, weights=None):
        self.numel, self.offset, self.arena = list(map(int, numel)), list(map(int, offset)), arena
        self.N, self.lr, self.mu, self.weights = n_workers, F(lr), F(mu), weights
        self.real = real_mask(numel, offset, arena)
        self.s2 = np.zeros(arena, bool)           # iteration 1: everything important
        self.P = np.zeros(arena, F)
        self.V = np.zeros(arena, F)
        self.Pw = np.zeros((n_workers, arena), F)
        self.q = np.zeros(arena, F)

    def load(self, P):
        self.P[:] = P
        self.V[:] = 0
        self.Pw[:] = P[None, :]

    def _sel(self, stage):
        if stage == 0:
            return self.real
        return self.real & (self.s2 if stage == 2 else ~self.s2)

    def agg(self, stage, grads):
        sel = self._sel(stage)
        g = aggregate(grads[:, :self.arena], self.weights)
        with np.errstate(all="ignore"):
            self.q[sel] = np.abs(g[sel] * self.P[sel])
            v = self.mu * self.V + g
            p = self.P - self.lr * v
        self.V[sel] = v[sel]
        self.P[sel] = p[sel]

    def apply(self, stage):
        sel = self._sel(stage)
        self.Pw[:, sel] = self.P[sel][None, :]

    def lgp(self, grads):
        sel = self._sel(2)
        with np.errstate(all="ignore"):
            new = self.Pw - self.lr * grads[:, :self.arena]
        self.Pw[:, sel] = new[:, sel]

    # ---- importance and split --------------------------------------------
    def keys(self):
        k = np.abs(self.q).view(np.uint32).copy()
        k[np.isnan(self.q)] = 0x7FC00000
        return k

    def layer_importance(self):
        out = []
        for a, n in zip(self.offset, self.numel):
            vals = [float(x) for x in self.q[a:a + n]]
            out.append(math.fsum(vals) if all(math.isfinite(v) for v in vals)
                       else float(np.sum(np.asarray(vals, np.float64))))
        return np.asarray(out)

    def split_layer(self, budget):
        imp = self.layer_importance()
        rank = sorted(range(len(imp)),
                      key=lambda l: (1 if math.isnan(imp[l]) else 0,
                                     0.0 if math.isnan(imp[l]) else imp[l], l))
        gib = np.ones(len(imp), np.uint8)
        taken = 0
        for l in rank:
            if taken + self.numel[l] > budget:
                break
            taken += self.numel[l]
            gib[l] = 0
        self.s2 = stage2_mask_from_layer_gib(gib, self.numel, self.offset, self.arena)
        return gib, taken, rank

    def split_element(self, budget):
        idx = np.nonzero(self.real)[0]
        k = self.keys()[idx]
        order = np.lexsort((idx, k))              # primary key, then index
        chosen = idx[order[:budget]]
        self.s2 = np.zeros(self.arena, bool)
        self.s2[chosen] = True
        words = (self.arena + 31) // 32
        bit = np.ones(words * 32, np.uint8)
        bit[chosen] = 0
        return np.packbits(bit, bitorder="little").view(np.uint32).copy()

    def step(self, grads, gran, budget):
        self.agg(1, grads); self.apply(1); self.lgp(grads)
        self.agg(2, grads); self.apply(2)
        return self.split_layer(budget)[0] if gran == 0 else self.split_element(budget)
