"""Thin ctypes binding of libosp.so: argument marshalling only.

Function names and argument order follow include/osp.h.  Every step of the
synchronization path runs in the library's HIP kernels; this module only turns
torch tensors into device pointers and statuses into exceptions.  There is no
fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# OSP_LIB: load this build of the library instead of the in-tree one
LIB_PATH = os.environ.get("OSP_LIB") or os.path.join(_HERE, "libosp.so")

OSP_OK, OSP_ERR_INVALID_ARG, OSP_ERR_BAD_STATE, OSP_ERR_NOMEM, OSP_ERR_HIP, OSP_ERR_UNSUPPORTED = range(6)
OSP_GRAN_LAYER, OSP_GRAN_ELEMENT = 0, 1

STATUS_NAMES = {0: "OSP_OK", 1: "OSP_ERR_INVALID_ARG", 2: "OSP_ERR_BAD_STATE",
                3: "OSP_ERR_NOMEM", 4: "OSP_ERR_HIP", 5: "OSP_ERR_UNSUPPORTED"}


class OspError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class osp_config(C.Structure):
    _fields_ = [("n_workers", C.c_int32), ("n_tensors", C.c_int32),
                ("numel", C.POINTER(C.c_int64)), ("offset", C.POINTER(C.c_int64)),
                ("arena_elems", C.c_int64), ("lr", C.c_float), ("momentum", C.c_float),
                ("worker_weight", C.POINTER(C.c_float)),
                ("element_keys", C.c_int32), ("chunk_elems", C.c_int32)]


class osp_buffers(C.Structure):
    _fields_ = [("ps_param", C.c_void_p), ("ps_momentum", C.c_void_p),
                ("worker_param", C.c_void_p), ("worker_param_stride", C.c_int64),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("replicas_in_sync", C.c_int32)]


def _load() -> C.CDLL:
    # PyTorch ships its own copy of the HIP runtime (same soname as the system one).  Two
    # copies in one process do not share a device context: memory allocated by torch would be
    # foreign to this library, and the second copy reports that it finds no device.  Importing
    # torch first makes libosp.so bind to the runtime torch has already loaded.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        # nothing built yet: build once (hipcc cross-compiles without a GPU); no CPU fallback
        try:
            from . import build as _build
            _build.build(force=True)
        except Exception as e:
            raise ImportError(
                f"{LIB_PATH} is not built and building it failed ({e}); run "
                "`python -c 'import __graft_entry__ as g; g.build()'` (there is no CPU fallback)") from e
    lib = C.CDLL(LIB_PATH)
    vp, i64 = C.c_void_p, C.c_int64
    lib.osp_create.argtypes = [C.POINTER(osp_config), C.POINTER(vp)]
    lib.osp_create.restype = C.c_int
    lib.osp_destroy.argtypes = [vp]
    lib.osp_destroy.restype = None
    lib.osp_workspace_bytes.argtypes = [vp]
    lib.osp_workspace_bytes.restype = C.c_size_t
    lib.osp_bind.argtypes = [vp, C.POINTER(osp_buffers), vp]
    lib.osp_bind.restype = C.c_int
    lib.osp_set_hyper.argtypes = [vp, C.c_float, C.c_float]
    lib.osp_set_hyper.restype = C.c_int
    lib.osp_split.argtypes = [vp, C.c_int, i64, vp]
    lib.osp_split.restype = C.c_int
    lib.osp_split_element_static.argtypes = [vp, i64, i64, vp, vp]
    lib.osp_split_element_static.restype = C.c_int
    lib.osp_get_gib.argtypes = [vp, vp, vp, C.POINTER(i64), vp]
    lib.osp_get_gib.restype = C.c_int
    lib.osp_read_n_stage2_async.argtypes = [vp, vp, vp]
    lib.osp_read_n_stage2_async.restype = C.c_int
    lib.osp_set_stage2_log.argtypes = [vp, vp, i64, vp]
    lib.osp_set_stage2_log.restype = C.c_int
    lib.osp_n_stage2.argtypes = [vp, C.POINTER(i64)]
    lib.osp_n_stage2.restype = C.c_int
    lib.osp_set_gib.argtypes = [vp, C.c_int, vp, vp]
    lib.osp_set_gib.restype = C.c_int
    lib.osp_ps_aggregate_update.argtypes = [vp, C.c_int, vp, i64, vp]
    lib.osp_ps_aggregate_update.restype = C.c_int
    lib.osp_lgp_correct.argtypes = [vp, vp, i64, vp]
    lib.osp_lgp_correct.restype = C.c_int
    lib.osp_ps_aggregate_update_bf16.argtypes = [vp, C.c_int, vp, i64, vp]
    lib.osp_ps_aggregate_update_bf16.restype = C.c_int
    lib.osp_lgp_correct_bf16.argtypes = [vp, vp, i64, vp]
    lib.osp_lgp_correct_bf16.restype = C.c_int
    lib.osp_apply_stage.argtypes = [vp, C.c_int, vp]
    lib.osp_apply_stage.restype = C.c_int
    lib.osp_split_gradients.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp]
    lib.osp_split_gradients.restype = C.c_int
    lib.osp_ps_aggregate_update_packed.argtypes = [vp, C.c_int, vp, i64, vp]
    lib.osp_ps_aggregate_update_packed.restype = C.c_int
    lib.osp_split_gradients_bf16.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp]
    lib.osp_split_gradients_bf16.restype = C.c_int
    lib.osp_ps_aggregate_update_packed_bf16.argtypes = [vp, C.c_int, vp, i64, vp]
    lib.osp_ps_aggregate_update_packed_bf16.restype = C.c_int
    lib.osp_set_keep_stage2_aggregate.argtypes = [vp, C.c_int32]
    lib.osp_set_keep_stage2_aggregate.restype = C.c_int
    lib.osp_drop_kept_aggregate.argtypes = [vp]
    lib.osp_drop_kept_aggregate.restype = C.c_int
    lib.osp_lgp_kept_aggregate.argtypes = [vp]
    lib.osp_lgp_kept_aggregate.restype = C.c_int32
    lib.osp_rs_window.argtypes = [vp, vp, i64, vp]
    lib.osp_rs_window.restype = C.c_int
    lib.osp_ics_window.argtypes = [vp, vp, i64, C.c_int, i64, vp]
    lib.osp_ics_window.restype = C.c_int
    lib.osp_rs_window_bf16.argtypes = [vp, vp, i64, vp]
    lib.osp_rs_window_bf16.restype = C.c_int
    lib.osp_ics_window_bf16.argtypes = [vp, vp, i64, C.c_int, i64, vp]
    lib.osp_ics_window_bf16.restype = C.c_int
    lib.osp_sync_step.argtypes = [vp, vp, i64, C.c_int, i64, vp]
    lib.osp_sync_step.restype = C.c_int
    lib.osp_get_importance.argtypes = [vp, vp, vp]
    lib.osp_get_importance.restype = C.c_int
    lib.osp_get_keys.argtypes = [vp, vp, vp]
    lib.osp_get_keys.restype = C.c_int
    lib.osp_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.osp_stream_copy.restype = C.c_int
    lib.osp_stream_pattern.argtypes = [vp, C.c_int32, i64, vp, C.c_int32, i64, i64, vp]
    lib.osp_stream_pattern.restype = C.c_int
    lib.osp_ics_upper_bound.argtypes = [C.c_double, C.c_double, C.c_double, C.c_int32]
    lib.osp_ics_upper_bound.restype = C.c_double
    lib.osp_tune_budget.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double, i64]
    lib.osp_tune_budget.restype = i64
    lib.osp_last_error.argtypes = [vp]
    lib.osp_last_error.restype = C.c_char_p
    lib.osp_lgp_read_shared.argtypes = [vp]
    lib.osp_lgp_read_shared.restype = C.c_int32
    lib.osp_windows_fused.argtypes = [vp]
    lib.osp_windows_fused.restype = C.c_int32
    lib.osp_chunk_elems.argtypes = [vp]
    lib.osp_chunk_elems.restype = C.c_int32
    lib.osp_n_chunks.argtypes = [vp]
    lib.osp_n_chunks.restype = C.c_int64
    return lib


lib = _load()

EXPORTS = ["osp_create", "osp_destroy", "osp_workspace_bytes", "osp_bind", "osp_set_hyper",
           "osp_split", "osp_split_element_static", "osp_get_gib", "osp_read_n_stage2_async", "osp_set_stage2_log", "osp_n_stage2", "osp_set_gib", "osp_ps_aggregate_update",
           "osp_lgp_correct", "osp_apply_stage", "osp_rs_window", "osp_ics_window", "osp_sync_step",
           "osp_split_gradients", "osp_ps_aggregate_update_packed",
           "osp_split_gradients_bf16", "osp_ps_aggregate_update_packed_bf16",
           "osp_ps_aggregate_update_bf16", "osp_lgp_correct_bf16",
           "osp_rs_window_bf16", "osp_ics_window_bf16",
           "osp_get_importance", "osp_get_keys",
           "osp_stream_copy", "osp_stream_pattern", "osp_ics_upper_bound", "osp_tune_budget",
           "osp_last_error", "osp_chunk_elems", "osp_n_chunks", "osp_lgp_read_shared", "osp_windows_fused",
           "osp_set_keep_stage2_aggregate", "osp_lgp_kept_aggregate", "osp_drop_kept_aggregate"]


def _ptr(t) -> int:
    """Device (or host) address of a torch tensor / numpy array, or a raw int."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Context:
    """Owns one osp_ctx.  Methods carry the C entry points' names."""

    def __init__(self, numel: Sequence[int], offset: Sequence[int], arena_elems: int,
                 n_workers: int, lr: float, momentum: float,
                 worker_weight: Optional[Sequence[float]] = None,
                 element_keys: bool = False, chunk_elems: int = 0):
        self._numel = np.ascontiguousarray(numel, dtype=np.int64)
        self._offset = np.ascontiguousarray(offset, dtype=np.int64)
        self._ww = None if worker_weight is None else np.ascontiguousarray(worker_weight, np.float32)
        self.n_tensors = int(self._numel.shape[0])
        self.n_workers = int(n_workers)
        self.arena_elems = int(arena_elems)
        self.n_words = (self.arena_elems + 31) // 32
        cfg = osp_config(
            self.n_workers, self.n_tensors,
            self._numel.ctypes.data_as(C.POINTER(C.c_int64)),
            self._offset.ctypes.data_as(C.POINTER(C.c_int64)),
            self.arena_elems, lr, momentum,
            None if self._ww is None else self._ww.ctypes.data_as(C.POINTER(C.c_float)),
            1 if element_keys else 0, int(chunk_elems))
        h = C.c_void_p()
        st = lib.osp_create(C.byref(cfg), C.byref(h))
        if st != OSP_OK:
            raise OspError(st, lib.osp_last_error(None).decode())
        self._h = h
        self._keep = None

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib.osp_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, st: int) -> None:
        if st != OSP_OK:
            raise OspError(st, lib.osp_last_error(self._h).decode())

    # ---- C entry points --------------------------------------------------
    def osp_workspace_bytes(self) -> int:
        return int(lib.osp_workspace_bytes(self._h))

    def osp_chunk_elems(self) -> int:
        return int(lib.osp_chunk_elems(self._h))

    def osp_n_stage2(self) -> int:
        out = C.c_int64(0)
        self._check(lib.osp_n_stage2(self._h, C.byref(out)))
        return int(out.value)

    def osp_lgp_read_shared(self) -> bool:
        return bool(lib.osp_lgp_read_shared(self._h))

    def osp_windows_fused(self) -> int:
        return int(lib.osp_windows_fused(self._h))

    def osp_set_keep_stage2_aggregate(self, on: bool) -> None:
        self._check(lib.osp_set_keep_stage2_aggregate(self._h, 1 if on else 0))

    def osp_drop_kept_aggregate(self) -> None:
        self._check(lib.osp_drop_kept_aggregate(self._h))

    def osp_lgp_kept_aggregate(self) -> bool:
        return bool(lib.osp_lgp_kept_aggregate(self._h))

    def osp_n_chunks(self) -> int:
        return int(lib.osp_n_chunks(self._h))

    def osp_bind(self, ps_param, ps_momentum, worker_param, worker_param_stride: int,
                 workspace, workspace_bytes: Optional[int] = None, stream=None,
                 replicas_in_sync: bool = False) -> None:
        if workspace_bytes is None:
            workspace_bytes = workspace.numel() * workspace.element_size()
        buf = osp_buffers(_ptr(ps_param), _ptr(ps_momentum), _ptr(worker_param),
                          int(worker_param_stride), _ptr(workspace), int(workspace_bytes),
                          1 if replicas_in_sync else 0)
        self._check(lib.osp_bind(self._h, C.byref(buf), _stream(stream)))
        self._keep = (ps_param, ps_momentum, worker_param, workspace)   # borrowed buffers stay alive

    def osp_set_hyper(self, lr: float, momentum: float) -> None:
        self._check(lib.osp_set_hyper(self._h, lr, momentum))

    def osp_split(self, granularity: int, budget_elems: int, stream=None) -> None:
        self._check(lib.osp_split(self._h, granularity, int(budget_elems), _stream(stream)))

    def osp_set_gib(self, granularity: int, gib_host: np.ndarray, stream=None) -> None:
        dt = np.uint8 if granularity == OSP_GRAN_LAYER else np.uint32
        want = self.n_tensors if granularity == OSP_GRAN_LAYER else self.n_words
        g = np.ascontiguousarray(gib_host, dtype=dt)
        if g.shape != (want,):
            raise ValueError(f"gib must have {want} entries")
        self._check(lib.osp_set_gib(self._h, granularity, g.ctypes.data, _stream(stream)))

    def osp_get_gib(self, stream=None):
        """Returns (layer_gib uint8[L], elem_bitmap uint32[words], n_stage2); the array
        that does not match the current granularity is left all-ones."""
        layer = np.ones(self.n_tensors, np.uint8)
        bits = np.full(self.n_words, 0xFFFFFFFF, np.uint32)
        n2 = C.c_int64(0)
        self._check(lib.osp_get_gib(self._h, layer.ctypes.data, bits.ctypes.data, C.byref(n2),
                                    _stream(stream)))
        return layer, bits, int(n2.value)

    def osp_read_n_stage2_async(self, out_host, stream=None) -> None:
        """out_host: address (or pinned int64 tensor / array element) the count is copied to."""
        self._check(lib.osp_read_n_stage2_async(self._h, _ptr(out_host), _stream(stream)))

    def osp_set_stage2_log(self, log, capacity: Optional[int] = None, stream=None) -> None:
        """log: int64 device tensor (or device address) every later split appends its stage-2
        size to, round robin; None takes the log away."""
        if capacity is None:
            capacity = 0 if log is None else log.numel()
        self._check(lib.osp_set_stage2_log(self._h, _ptr(log), int(capacity), _stream(stream)))
        self._log = log                         # borrowed buffer stays alive

    def osp_ps_aggregate_update(self, stage: int, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_ps_aggregate_update(self._h, stage, _ptr(grads), int(worker_stride),
                                                _stream(stream)))

    def osp_lgp_correct(self, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_lgp_correct(self._h, _ptr(grads), int(worker_stride), _stream(stream)))

    def osp_ps_aggregate_update_bf16(self, stage: int, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_ps_aggregate_update_bf16(self._h, stage, _ptr(grads), int(worker_stride),
                                                     _stream(stream)))

    def osp_lgp_correct_bf16(self, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_lgp_correct_bf16(self._h, _ptr(grads), int(worker_stride),
                                             _stream(stream)))

    def osp_apply_stage(self, stage: int, stream=None) -> None:
        self._check(lib.osp_apply_stage(self._h, stage, _stream(stream)))

    def osp_split_gradients(self, grads, worker_stride: int, g_important, important_stride: int,
                            g_unimportant, unimportant_stride: int, stream=None) -> None:
        self._check(lib.osp_split_gradients(self._h, _ptr(grads), int(worker_stride),
                                            _ptr(g_important), int(important_stride),
                                            _ptr(g_unimportant), int(unimportant_stride),
                                            _stream(stream)))

    def osp_ps_aggregate_update_packed(self, stage: int, packed, packed_stride: int,
                                       stream=None) -> None:
        self._check(lib.osp_ps_aggregate_update_packed(self._h, stage, _ptr(packed),
                                                       int(packed_stride), _stream(stream)))

    def osp_split_gradients_bf16(self, grads, worker_stride: int, g_important, important_stride: int,
                                 g_unimportant, unimportant_stride: int, stream=None) -> None:
        self._check(lib.osp_split_gradients_bf16(self._h, _ptr(grads), int(worker_stride),
                                                 _ptr(g_important), int(important_stride),
                                                 _ptr(g_unimportant), int(unimportant_stride),
                                                 _stream(stream)))

    def osp_ps_aggregate_update_packed_bf16(self, stage: int, packed, packed_stride: int,
                                            stream=None) -> None:
        self._check(lib.osp_ps_aggregate_update_packed_bf16(self._h, stage, _ptr(packed),
                                                            int(packed_stride), _stream(stream)))

    def osp_rs_window(self, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_rs_window(self._h, _ptr(grads), int(worker_stride), _stream(stream)))

    def osp_ics_window(self, grads, worker_stride: int, granularity: int, budget_elems: int,
                       stream=None) -> None:
        self._check(lib.osp_ics_window(self._h, _ptr(grads), int(worker_stride), int(granularity),
                                       int(budget_elems), _stream(stream)))

    def osp_rs_window_bf16(self, grads, worker_stride: int, stream=None) -> None:
        self._check(lib.osp_rs_window_bf16(self._h, _ptr(grads), int(worker_stride), _stream(stream)))

    def osp_ics_window_bf16(self, grads, worker_stride: int, granularity: int, budget_elems: int,
                            stream=None) -> None:
        self._check(lib.osp_ics_window_bf16(self._h, _ptr(grads), int(worker_stride),
                                            int(granularity), int(budget_elems), _stream(stream)))

    def osp_sync_step(self, grads, worker_stride: int, granularity: int, budget_elems: int,
                      stream=None) -> None:
        self._check(lib.osp_sync_step(self._h, _ptr(grads), int(worker_stride), int(granularity),
                                      int(budget_elems), _stream(stream)))

    def osp_get_importance(self, stream=None) -> np.ndarray:
        imp = np.zeros(self.n_tensors, np.float64)
        self._check(lib.osp_get_importance(self._h, imp.ctypes.data, _stream(stream)))
        return imp

    def osp_get_keys(self, stream=None) -> np.ndarray:
        key = np.zeros(self.arena_elems, np.uint32)
        self._check(lib.osp_get_keys(self._h, key.ctypes.data, _stream(stream)))
        return key


def osp_split_element_static(keys, n_elems: int, budget_elems: int, elem_bitmap, stream=None) -> None:
    st = lib.osp_split_element_static(_ptr(keys), int(n_elems), int(budget_elems),
                                      _ptr(elem_bitmap), _stream(stream))
    if st != OSP_OK:
        raise OspError(st, lib.osp_last_error(None).decode())


def osp_stream_copy(dst, src, nbytes: int, stream=None) -> None:
    st = lib.osp_stream_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream))
    if st != OSP_OK:
        raise OspError(st, "osp_stream_copy")


def osp_stream_pattern(reads, n_read: int, read_stride: int, rw, n_rw: int, rw_stride: int,
                       n_elems: int, stream=None) -> None:
    st = lib.osp_stream_pattern(_ptr(reads), int(n_read), int(read_stride), _ptr(rw), int(n_rw),
                                int(rw_stride), int(n_elems), _stream(stream))
    if st != OSP_OK:
        raise OspError(st, "osp_stream_pattern")


def osp_ics_upper_bound(bandwidth_elems_per_s, loss_rate, t_compute_s, n_workers) -> float:
    return float(lib.osp_ics_upper_bound(bandwidth_elems_per_s, loss_rate, t_compute_s, n_workers))


def osp_tune_budget(epoch, loss_i, loss_1, u_max, model_elems) -> int:
    return int(lib.osp_tune_budget(epoch, loss_i, loss_1, u_max, model_elems))
