"""ctypes wrapper around the plain-C OSP oracle.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It shares nothing with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "osp_oracle.c")
_LIB = os.path.join(_HERE, "libosp_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libosp_oracle_omp.so")

# -ffp-contract=off: one rounding per operator (no fused multiply-add)
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra"]

GRAN_LAYER = 0
GRAN_ELEMENT = 1


def build(force: bool = False) -> None:
    """Compile the oracle (serial build, and the same loops under OpenMP)."""
    for lib, extra in ((_LIB, []), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
            subprocess.check_call(["gcc", *_CFLAGS, *extra, _SRC, "-o", lib, "-lm"])


class _Model(C.Structure):
    _fields_ = [("n_workers", C.c_int32), ("n_tensors", C.c_int32),
                ("numel", C.POINTER(C.c_int64)), ("offset", C.POINTER(C.c_int64)),
                ("arena_elems", C.c_int64), ("lr", C.c_float), ("momentum", C.c_float),
                ("worker_weight", C.POINTER(C.c_float))]


class _Gib(C.Structure):
    _fields_ = [("granularity", C.c_int32), ("layer", C.POINTER(C.c_uint8)),
                ("bits", C.POINTER(C.c_uint32))]


def _fp(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


_libs = {}


def _load(omp: bool):
    if omp not in _libs:
        # OSP_ORACLE_LIB: load this library instead (the test that plants mistakes into
        # copies of the oracle source uses it to show that the pins notice them)
        override = os.environ.get("OSP_ORACLE_LIB")
        if override:
            lib = C.CDLL(override)
        else:
            build()
            lib = C.CDLL(_LIB_OMP if omp else _LIB)
        mp, gp, fp = C.POINTER(_Model), C.POINTER(_Gib), C.POINTER(C.c_float)
        lib.osp_oracle_aggregate_update.argtypes = [mp, gp, C.c_int, fp, fp, fp, C.c_int64, fp]
        lib.osp_oracle_aggregate_update.restype = None
        lib.osp_oracle_apply_stage.argtypes = [mp, gp, C.c_int, fp, fp, C.c_int64]
        lib.osp_oracle_apply_stage.restype = None
        lib.osp_oracle_lgp_correct.argtypes = [mp, gp, fp, C.c_int64, fp, C.c_int64]
        lib.osp_oracle_lgp_correct.restype = None
        lib.osp_oracle_split_gradients.argtypes = [mp, gp, fp, fp, fp]
        lib.osp_oracle_split_gradients.restype = C.c_int64
        lib.osp_oracle_aggregate_update_packed.argtypes = [mp, gp, C.c_int, fp, fp, fp, C.c_int64, fp]
        lib.osp_oracle_aggregate_update_packed.restype = None
        lib.osp_oracle_eq7_literal.argtypes = [mp, gp, fp, C.c_int64, fp, C.c_int64, fp, fp,
                                               C.POINTER(C.c_double)]
        lib.osp_oracle_eq7_literal.restype = None
        lib.osp_oracle_layer_importance.argtypes = [mp, fp, C.POINTER(C.c_double)]
        lib.osp_oracle_layer_importance.restype = None
        lib.osp_oracle_split_layer.argtypes = [mp, C.POINTER(C.c_double), C.c_int64,
                                               C.POINTER(C.c_uint8), C.POINTER(C.c_int32)]
        lib.osp_oracle_split_layer.restype = C.c_int64
        lib.osp_oracle_keys.argtypes = [mp, fp, C.POINTER(C.c_uint32)]
        lib.osp_oracle_keys.restype = None
        lib.osp_oracle_split_element.argtypes = [mp, fp, C.c_int64, C.POINTER(C.c_uint32)]
        lib.osp_oracle_split_element.restype = C.c_int64
        lib.osp_oracle_ics_upper_bound.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int]
        lib.osp_oracle_ics_upper_bound.restype = C.c_double
        lib.osp_oracle_tune_budget.argtypes = [C.c_int, C.c_double, C.c_double, C.c_double, C.c_int64]
        lib.osp_oracle_tune_budget.restype = C.c_int64
        _libs[omp] = lib
    return _libs[omp]


def ics_upper_bound(b: float, loss_rate: float, t_c: float, n_workers: int) -> float:
    """Eq. 5."""
    return float(_load(False).osp_oracle_ics_upper_bound(b, loss_rate, t_c, n_workers))


def tune_budget(epoch: int, loss_i: float, L: float, u_max: float, model_elems: int) -> int:
    """Algorithm 1, one epoch."""
    return int(_load(False).osp_oracle_tune_budget(epoch, loss_i, L, u_max, model_elems))


class OracleOSP:
    """Host-memory state of one OSP job (PS + N workers) driven by the C oracle.

    Arrays (all owned here, fp32 unless noted):
      P, V            [arena]            PS parameters and momentum
      Pw              [N, param_stride]  worker replicas
      q               [arena]            |gbar * P| of the current iteration
      gib_layer       [L] uint8          1 = important (stage 1)
      gib_bits        [ceil(arena/32)] uint32, bit per element, 1 = important
    """

    def __init__(self, numel, offset, arena_elems: int, n_workers: int, lr: float,
                 momentum: float, worker_weight: Optional[np.ndarray] = None,
                 param_stride: Optional[int] = None, omp: bool = False):
        self.lib = _load(omp)
        self.omp = omp
        self.numel = np.ascontiguousarray(numel, dtype=np.int64)
        self.offset = np.ascontiguousarray(offset, dtype=np.int64)
        self.L = int(self.numel.shape[0])
        self.N = int(n_workers)
        self.arena = int(arena_elems)
        self.param_stride = int(param_stride) if param_stride else self.arena
        self.ww = None if worker_weight is None else np.ascontiguousarray(worker_weight, np.float32)
        self.model = _Model(self.N, self.L,
                            self.numel.ctypes.data_as(C.POINTER(C.c_int64)),
                            self.offset.ctypes.data_as(C.POINTER(C.c_int64)),
                            self.arena, lr, momentum,
                            None if self.ww is None else _fp(self.ww))
        self.P = np.zeros(self.arena, np.float32)
        self.V = np.zeros(self.arena, np.float32)
        self.Pw = np.zeros((self.N, self.param_stride), np.float32)
        self.q = np.zeros(self.arena, np.float32)
        self.words = (self.arena + 31) // 32
        self.granularity = GRAN_LAYER
        self.gib_layer = np.ones(self.L, np.uint8)          # iteration 1: all important
        self.gib_bits = np.full(self.words, 0xFFFFFFFF, np.uint32)
        self.n_stage2 = 0

    # -- state -----------------------------------------------------------
    def set_hyper(self, lr: float, momentum: float) -> None:
        """New learning rate / momentum from the next call on (the schedule of Sec. 5.1.3
        halves the learning rate every 10 epochs)."""
        self.model.lr = lr
        self.model.momentum = momentum

    def load_params(self, P: np.ndarray, V: Optional[np.ndarray] = None) -> None:
        self.P[:] = P
        self.V[:] = 0.0 if V is None else V
        self.Pw[:, :self.arena] = self.P[None, :]

    def set_gib(self, granularity: int, gib: np.ndarray) -> None:
        self.granularity = granularity
        if granularity == GRAN_LAYER:
            self.gib_layer[:] = np.asarray(gib, np.uint8)
            self.n_stage2 = int(self.numel[self.gib_layer == 0].sum())
        else:
            self.gib_bits[:] = np.asarray(gib, np.uint32)
            bits = np.unpackbits(self.gib_bits.view(np.uint8), bitorder="little")
            self.n_stage2 = int(sum(int(n) - int(bits[int(a):int(a) + int(n)].sum())
                                    for a, n in zip(self.offset, self.numel)))

    def _gib(self) -> _Gib:
        return _Gib(self.granularity,
                    self.gib_layer.ctypes.data_as(C.POINTER(C.c_uint8)),
                    self.gib_bits.ctypes.data_as(C.POINTER(C.c_uint32)))

    # -- the calls of one synchronization step ------------------------------
    def ps_aggregate_update(self, stage: int, grads: np.ndarray) -> None:
        assert grads.dtype == np.float32 and grads.ndim == 2 and grads.shape[0] == self.N
        assert grads.flags.c_contiguous and grads.shape[1] >= self.arena
        g = self._gib()
        self.lib.osp_oracle_aggregate_update(C.byref(self.model), C.byref(g), stage,
                                             _fp(self.P), _fp(self.V), _fp(grads),
                                             grads.shape[1], _fp(self.q))

    def split_gradients(self, grads: np.ndarray):
        """Gradient splitter (Sec. 4.5): per worker the dense arrays G^i and G^u.
        Returns (g_i [N, E1], g_u [N, E2])."""
        assert grads.dtype == np.float32 and grads.ndim == 2 and grads.shape[0] == self.N
        n_real = int(np.sum(self.numel))
        e2 = self.n_stage2
        g_i = np.zeros((self.N, n_real - e2), np.float32)
        g_u = np.zeros((self.N, e2), np.float32)
        g = self._gib()
        for w in range(self.N):
            row = np.ascontiguousarray(grads[w])
            got = self.lib.osp_oracle_split_gradients(C.byref(self.model), C.byref(g), _fp(row),
                                                      _fp(g_i[w]) if g_i.shape[1] else None,
                                                      _fp(g_u[w]) if g_u.shape[1] else None)
            assert got == e2
        return g_i, g_u

    def ps_aggregate_update_packed(self, stage: int, packed: np.ndarray) -> None:
        """Stage 1 or 2 fed by the dense arrays of split_gradients."""
        assert stage in (1, 2) and packed.dtype == np.float32 and packed.ndim == 2
        assert packed.flags.c_contiguous and packed.shape[0] == self.N
        g = self._gib()
        self.lib.osp_oracle_aggregate_update_packed(C.byref(self.model), C.byref(g), stage,
                                                    _fp(self.P), _fp(self.V), _fp(packed),
                                                    packed.shape[1], _fp(self.q))

    def apply_stage(self, stage: int) -> None:
        g = self._gib()
        self.lib.osp_oracle_apply_stage(C.byref(self.model), C.byref(g), stage,
                                        _fp(self.P), _fp(self.Pw), self.param_stride)

    def lgp_correct(self, grads: np.ndarray) -> None:
        assert grads.dtype == np.float32 and grads.flags.c_contiguous
        g = self._gib()
        self.lib.osp_oracle_lgp_correct(C.byref(self.model), C.byref(g), _fp(self.Pw),
                                        self.param_stride, _fp(grads), grads.shape[1])

    def eq7_literal(self, grads: np.ndarray, P_old: np.ndarray, P_new: np.ndarray) -> np.ndarray:
        out = np.zeros((self.N, self.param_stride), np.float64)
        g = self._gib()
        self.lib.osp_oracle_eq7_literal(C.byref(self.model), C.byref(g), _fp(self.Pw),
                                        self.param_stride, _fp(grads), grads.shape[1],
                                        _fp(np.ascontiguousarray(P_old, np.float32)),
                                        _fp(np.ascontiguousarray(P_new, np.float32)),
                                        out.ctypes.data_as(C.POINTER(C.c_double)))
        return out

    def layer_importance(self) -> np.ndarray:
        imp = np.zeros(self.L, np.float64)
        self.lib.osp_oracle_layer_importance(C.byref(self.model), _fp(self.q),
                                             imp.ctypes.data_as(C.POINTER(C.c_double)))
        return imp

    def keys(self) -> np.ndarray:
        key = np.full(self.arena, 0xFFFFFFFF, np.uint32)
        self.lib.osp_oracle_keys(C.byref(self.model), _fp(self.q),
                                 key.ctypes.data_as(C.POINTER(C.c_uint32)))
        return key

    def split(self, granularity: int, budget_elems: int) -> int:
        """Compute the next GIB from this iteration's importances and install it."""
        if granularity == GRAN_LAYER:
            imp = self.layer_importance()
            gib = np.ones(self.L, np.uint8)
            self.order = np.zeros(self.L, np.int32)
            n2 = self.lib.osp_oracle_split_layer(
                C.byref(self.model), imp.ctypes.data_as(C.POINTER(C.c_double)), budget_elems,
                gib.ctypes.data_as(C.POINTER(C.c_uint8)),
                self.order.ctypes.data_as(C.POINTER(C.c_int32)))
            self.importance = imp
            self.granularity = GRAN_LAYER
            self.gib_layer[:] = gib
        else:
            bits = np.zeros(self.words, np.uint32)
            n2 = self.lib.osp_oracle_split_element(
                C.byref(self.model), _fp(self.q), budget_elems,
                bits.ctypes.data_as(C.POINTER(C.c_uint32)))
            if n2 < 0:
                raise ValueError("budget outside [0, number of parameters]")
            self.granularity = GRAN_ELEMENT
            self.gib_bits[:] = bits
        self.n_stage2 = int(n2)
        return self.n_stage2

    def split_element_by_selection(self, budget_elems: int) -> int:
        """The partition split(GRAN_ELEMENT, budget) defines (the first `budget` parameters in
        the order: key ascending, arena index ascending), found by selection on this oracle's
        keys instead of the full sort, for the sizes where the sort takes minutes: T = the
        budget-th smallest key; every key below T is in stage 2; of the keys equal to T the
        first budget - (number below) in index order are.  Pinned to split() by
        tests/test_oracle_pins.py; split() stays the definition."""
        n_real = int(np.sum(self.numel))
        if budget_elems < 0 or budget_elems > n_real:
            raise ValueError("budget outside [0, number of parameters]")
        keys = self.keys()
        real = np.zeros(self.arena, bool)
        for a, n in zip(self.offset, self.numel):
            real[int(a):int(a) + int(n)] = True
        s2 = np.zeros(self.words * 32, bool)
        if budget_elems > 0:
            T = np.partition(keys[real], budget_elems - 1)[budget_elems - 1]
            below = real & (keys < T)
            r = budget_elems - int(below.sum())
            ties = np.nonzero(real & (keys == T))[0]
            assert 1 <= r <= ties.size
            s2[:self.arena] = below
            s2[ties[:r]] = True
        self.granularity = GRAN_ELEMENT
        self.gib_bits[:] = np.packbits(~s2, bitorder="little").view(np.uint32)
        self.n_stage2 = int(budget_elems)
        return self.n_stage2

    def sync_step(self, grads: np.ndarray, granularity: int, budget_elems: int,
                  element_by_selection: bool = False) -> int:
        """One full step in the paper's order (Sec. 3.1, Eq. 5 ordering):
        RS window = aggregate stage 1, hand back, LGP; ICS window = aggregate
        stage 2, correct the local estimate, compute the next GIB."""
        self.ps_aggregate_update(1, grads)
        self.apply_stage(1)
        self.lgp_correct(grads)
        self.ps_aggregate_update(2, grads)
        self.apply_stage(2)
        if granularity == GRAN_ELEMENT and element_by_selection:
            return self.split_element_by_selection(budget_elems)
        return self.split(granularity, budget_elems)
