"""Host-side checks of bench.py: the byte counts it credits and its refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

SIX = ("agg1", "apply1", "lgp", "agg2", "apply2", "split")


@pytest.mark.parametrize("N,M,E2", [(16, 138_357_544, 35_597_096), (8, 60_192_808, 41_957_416), (4, 100_000, 0)])
def test_layer_step_bytes_are_the_stated_formula(N, M, E2):
    b = bench.step_bytes(N, M, E2, element=False)
    assert sum(b[n] for n in SIX) == 4 * M * (2 * N + 5) + 12 * N * E2
    assert b["rs_window"] + b["ics_window"] == sum(b[n] for n in SIX)
    assert b["split_gradients"] == 8 * N * M


def test_element_step_bytes_add_keys_and_selection_floor():
    N, M, E2 = 16, 138_357_544, 69_178_772
    layer = bench.step_bytes(N, M, E2, element=False)
    elem = bench.step_bytes(N, M, E2, element=True)
    extra = sum(elem[n] - layer[n] for n in SIX)
    assert extra == 4 * M + (4 * M + M // 8)            # key write per element, then one key read + bitmap


def test_bf16_gradients_halve_only_the_gradient_reads():
    N, M, E2 = 8, 1000, 400
    f32 = bench.step_bytes(N, M, E2, element=False, gb=4)
    b16 = bench.step_bytes(N, M, E2, element=False, gb=2)
    assert sum(f32[n] - b16[n] for n in SIX) == 2 * N * M + 2 * N * E2


def test_bytes_moved_are_itemised():
    """LGP that keeps the stage-2 aggregate: N grads + P read, N replicas + aggregate written;
    stage 2 then reads P, V, aggregate and writes P, V.  Never more than the metric credits."""
    N, M, E2 = 16, 4000, 1000
    b = bench.step_bytes(N, M, E2, element=False)
    kept = bench.moved_bytes(N, M, E2, False, 4, True, True, False, False)
    assert kept["lgp"] + kept["agg2"] == 4 * (N + 1) * E2 + 4 * (N + 1) * E2 + 12 * E2 + 8 * E2
    shared = bench.moved_bytes(N, M, E2, False, 4, True, False, False, False)
    assert b["lgp"] - shared["lgp"] == 4 * (N - 1) * E2 and shared["agg2"] == b["agg2"]
    plain = bench.moved_bytes(N, M, E2, False, 4, False, False, False, False)
    for n in SIX:
        assert plain[n] == b[n]
        assert kept[n] <= b[n] and shared[n] <= b[n]
    assert plain["rs_window"] == b["rs_window"] and plain["ics_window"] == b["ics_window"]
    # bfloat16 arenas: gradients are 2 bytes
    kept2 = bench.moved_bytes(N, M, E2, False, 2, True, True, False, False)
    assert kept2["lgp"] + kept2["agg2"] == (2 * N + 4) * E2 + 4 * (N + 1) * E2 + 12 * E2 + 8 * E2


def test_element_windows_move_one_pass_each():
    """Fused element-granular RS window: N gradients, P, V and the bitmap read; P, V, keys, the
    kept aggregate and N replicas written; all over whole arenas."""
    N, M, E2 = 16, 3200, 1600
    mv = bench.moved_bytes(N, M, E2, True, 4, True, False, True, False)
    assert mv["rs_window"] == (4 * N + 8) * M + M // 8 + (16 + 4 * N) * M
    assert mv["ics_window"] == (20 * M + M // 8) + 4 * (N + 1) * M + (8 * M + M // 8)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
