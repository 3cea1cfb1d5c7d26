"""The C-ABI library loads, exports every symbol the header declares, and its
host-side validation works with no GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2306_16926_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "osp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(osp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert {"osp_split", "osp_ps_aggregate_update", "osp_lgp_correct", "osp_apply_stage"} <= set(names)
    raw = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(B.EXPORTS) == names


def mk(**kw):
    args = dict(numel=[10, 7], offset=[0, 12], arena_elems=20, n_workers=2, lr=0.1, momentum=0.9)
    args.update(kw)
    return B.Context(**args)


def test_create_and_geometry():
    c = mk(numel=[5000, 7], offset=[0, 5000], arena_elems=5008, chunk_elems=1024)
    assert c.osp_chunk_elems() == 1024
    assert c.osp_n_chunks() == 5 + 1
    assert c.osp_workspace_bytes() > 0 and c.osp_workspace_bytes() % 256 == 0
    small = c.osp_workspace_bytes()
    c2 = mk(numel=[5000, 7], offset=[0, 5000], arena_elems=5008, chunk_elems=1024, element_keys=True)
    assert c2.osp_workspace_bytes() >= small + 4 * 5008 + 5008 // 8
    c.close(); c.close()


@pytest.mark.parametrize("bad", [
    dict(n_workers=0), dict(numel=[0, 7]), dict(offset=[0, 9]), dict(offset=[0, 8]),
    dict(arena_elems=18), dict(arena_elems=16), dict(momentum=1.0), dict(momentum=-0.1),
    dict(lr=float("nan")), dict(chunk_elems=1000), dict(chunk_elems=128),
    dict(numel=[], offset=[]),
])
def test_create_rejects(bad):
    with pytest.raises(B.OspError) as e:
        mk(**bad)
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    assert len(str(e.value)) > len("OSP_ERR_INVALID_ARG: ")


def test_calls_before_bind_fail_cleanly():
    c = mk()
    g = np.zeros(64, np.float32)            # host memory: must never be dereferenced
    addr = g.ctypes.data - (g.ctypes.data % 16) + 16
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(1, addr, 20, stream=0)
    assert e.value.status == B.OSP_ERR_BAD_STATE
    with pytest.raises(B.OspError) as e:
        c.osp_apply_stage(1, stream=0)
    assert e.value.status == B.OSP_ERR_BAD_STATE
    with pytest.raises(B.OspError) as e:
        c.osp_lgp_correct(addr, 20, stream=0)
    assert e.value.status == B.OSP_ERR_BAD_STATE
    with pytest.raises(B.OspError) as e:
        c.osp_split(B.OSP_GRAN_LAYER, 5, stream=0)
    assert e.value.status == B.OSP_ERR_BAD_STATE
    with pytest.raises(B.OspError) as e:
        c.osp_get_gib(stream=0)
    assert e.value.status == B.OSP_ERR_BAD_STATE


def test_argument_errors_come_before_state_errors():
    c = mk()
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(3, 16, 20, stream=0)
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(1, 0, 20, stream=0)          # NULL grads
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(1, 24, 20, stream=0)         # misaligned
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(1, 16, 16, stream=0)         # stride < arena
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_ps_aggregate_update(1, 16, 22, stream=0)         # stride not multiple of 4
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_split(B.OSP_GRAN_LAYER, 18, stream=0)            # budget > 17 parameters
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_split(B.OSP_GRAN_LAYER, -1, stream=0)
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_split(B.OSP_GRAN_ELEMENT, 5, stream=0)           # element_keys off
    assert e.value.status == B.OSP_ERR_UNSUPPORTED
    with pytest.raises(B.OspError) as e:
        c.osp_split(7, 5, stream=0)
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    with pytest.raises(B.OspError) as e:
        c.osp_set_hyper(0.1, 1.5)
    assert e.value.status == B.OSP_ERR_INVALID_ARG
    c.osp_set_hyper(0.05, 0.5)


def test_bind_validation_without_gpu():
    c = mk()
    ok = dict(ps_param=256, ps_momentum=512, worker_param=1024, worker_param_stride=20,
              workspace=4096, workspace_bytes=1 << 20, stream=0)
    for bad in (dict(ps_param=0), dict(ps_param=260), dict(worker_param_stride=16),
                dict(worker_param_stride=21), dict(workspace=4100), dict(workspace_bytes=8),
                dict(workspace=0)):
        with pytest.raises(B.OspError) as e:
            c.osp_bind(**{**ok, **bad})
        assert e.value.status == B.OSP_ERR_INVALID_ARG, bad


def test_null_context_is_harmless():
    assert B.lib.osp_workspace_bytes(None) == 0
    B.lib.osp_destroy(None)
    assert B.lib.osp_apply_stage(None, 1, None) == B.OSP_ERR_INVALID_ARG


def test_newer_entry_points_validate_before_touching_anything():
    """Windows, gradient splitter, packed and bfloat16 inputs, reference traffic kernels:
    NULL context, bad arguments and an unbound context are answered on the host."""
    L = B.lib
    assert L.osp_rs_window(None, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_ics_window(None, 16, 20, 0, 1, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_split_gradients(None, 16, 20, 16, 20, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_ps_aggregate_update_packed(None, 1, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_split_gradients_bf16(None, 16, 20, 16, 20, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_ps_aggregate_update_packed_bf16(None, 1, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_ps_aggregate_update_bf16(None, 1, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_lgp_correct_bf16(None, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_rs_window_bf16(None, 16, 20, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_ics_window_bf16(None, 16, 20, 0, 1, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_sync_step(None, 16, 20, 0, 1, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_n_stage2(None, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_windows_fused(None) == 0
    c = mk()
    cases = [
        (lambda: c.osp_rs_window(0, 20, stream=0), B.OSP_ERR_INVALID_ARG),            # NULL grads
        (lambda: c.osp_rs_window(16, 20, stream=0), B.OSP_ERR_BAD_STATE),             # not bound
        (lambda: c.osp_ics_window(16, 20, 9, 5, stream=0), B.OSP_ERR_INVALID_ARG),    # granularity
        (lambda: c.osp_ics_window(16, 20, 0, 18, stream=0), B.OSP_ERR_INVALID_ARG),   # budget > 17
        (lambda: c.osp_ics_window(16, 20, 1, 5, stream=0), B.OSP_ERR_UNSUPPORTED),    # element keys off
        (lambda: c.osp_ics_window(16, 20, 0, 5, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_split_gradients(16, 20, 0, 0, 0, 0, stream=0), B.OSP_ERR_INVALID_ARG),
        (lambda: c.osp_split_gradients(16, 20, 16, 20, 16, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_ps_aggregate_update_packed(0, 16, 20, stream=0), B.OSP_ERR_INVALID_ARG),
        (lambda: c.osp_ps_aggregate_update_packed(1, 18, 20, stream=0), B.OSP_ERR_INVALID_ARG),
        (lambda: c.osp_ps_aggregate_update_packed(1, 16, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_split_gradients_bf16(12, 20, 16, 20, 16, 20, stream=0), B.OSP_ERR_INVALID_ARG),  # arena alignment
        (lambda: c.osp_split_gradients_bf16(8, 20, 17, 20, 16, 20, stream=0), B.OSP_ERR_INVALID_ARG),   # odd output
        (lambda: c.osp_split_gradients_bf16(8, 20, 18, 20, 16, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_ps_aggregate_update_packed_bf16(1, 17, 20, stream=0), B.OSP_ERR_INVALID_ARG),
        (lambda: c.osp_ps_aggregate_update_packed_bf16(1, 18, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_ps_aggregate_update_bf16(1, 12, 20, stream=0), B.OSP_ERR_INVALID_ARG),  # 8-byte alignment
        (lambda: c.osp_ps_aggregate_update_bf16(1, 8, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_lgp_correct_bf16(8, 16, stream=0), B.OSP_ERR_INVALID_ARG),      # stride < arena
        (lambda: c.osp_lgp_correct_bf16(8, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_n_stage2(), B.OSP_ERR_BAD_STATE),                               # no GIB
        (lambda: c.osp_set_stage2_log(16, 0, stream=0), B.OSP_ERR_INVALID_ARG),        # no room
        (lambda: c.osp_set_stage2_log(20, 4, stream=0), B.OSP_ERR_INVALID_ARG),        # alignment
        (lambda: c.osp_set_stage2_log(16, 4, stream=0), B.OSP_ERR_BAD_STATE),          # not bound
        (lambda: c.osp_rs_window_bf16(12, 20, stream=0), B.OSP_ERR_INVALID_ARG),       # 8-byte alignment
        (lambda: c.osp_rs_window_bf16(8, 20, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_ics_window_bf16(8, 20, 0, 5, stream=0), B.OSP_ERR_BAD_STATE),
        (lambda: c.osp_sync_step(16, 20, 0, 18, stream=0), B.OSP_ERR_INVALID_ARG),
        (lambda: c.osp_sync_step(16, 20, 0, 5, stream=0), B.OSP_ERR_BAD_STATE),
    ]
    for i, (call, want) in enumerate(cases):
        with pytest.raises(B.OspError) as e:
            call()
        assert e.value.status == want, i
    # the allocation-free element split: every argument error is answered before any GPU call
    for a, want in (((0, 64, 8, 16), B.OSP_ERR_INVALID_ARG), ((16, 64, 8, 0), B.OSP_ERR_INVALID_ARG),
                    ((24, 64, 8, 16), B.OSP_ERR_INVALID_ARG), ((16, 64, 8, 18), B.OSP_ERR_INVALID_ARG),
                    ((16, 0, 0, 16), B.OSP_ERR_INVALID_ARG), ((16, 62, 8, 16), B.OSP_ERR_INVALID_ARG),
                    ((16, 64, 65, 16), B.OSP_ERR_INVALID_ARG), ((16, 64, -1, 16), B.OSP_ERR_INVALID_ARG),
                    ((16, (1 << 28) + 4, 8, 16), B.OSP_ERR_UNSUPPORTED)):
        assert L.osp_split_element_static(a[0], a[1], a[2], a[3], None) == want, a
        assert len(L.osp_last_error(None)) > 0
    # reference kernels: argument checks only (no launch for bad shapes)
    assert L.osp_stream_pattern(0, 1, 16, 16, 1, 16, 16, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_stream_pattern(16, 0, 16, 16, 1, 16, 16, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_stream_pattern(16, 1, 16, 16, 3, 16, 16, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_stream_pattern(16, 1, 12, 16, 1, 16, 16, None) == B.OSP_ERR_INVALID_ARG
    assert L.osp_stream_pattern(16, 1, 16, 16, 1, 16, 18, None) == B.OSP_ERR_INVALID_ARG
