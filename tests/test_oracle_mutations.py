"""The pins have teeth: plausible mistakes planted into COPIES of the oracle
source (on the CPU, never in the product or on the GPU) must each make the pin
suite fail.  The oracle file itself is not touched."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "osp_oracle.c")
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math"]

# (name, text in the oracle, replacement): each is one plausible slip
MUTATIONS = [
    ("pgp_uses_updated_parameter",
     "    float prod = gbar * P[k];\n    q[k] = fabsf(prod);\n    float mv = m->momentum * V[k];\n    float v = mv + gbar;\n    float step = m->lr * v;\n    V[k] = v;\n    P[k] = P[k] - step;",
     "    float mv = m->momentum * V[k];\n    float v = mv + gbar;\n    float step = m->lr * v;\n    V[k] = v;\n    P[k] = P[k] - step;\n    float prod = gbar * P[k];\n    q[k] = fabsf(prod);"),
    ("momentum_dropped", "float mv = m->momentum * V[k];", "float mv = 0.0f * V[k];"),
    ("update_sign", "P[k] = P[k] - step;", "P[k] = P[k] + step;"),
    ("mean_missing", "gbar = acc * inv_n;", "gbar = acc;"),
    ("weight_of_wrong_worker",
     "float term = m->worker_weight[w] * g[(int64_t)w * stride];",
     "float term = m->worker_weight[w - 1] * g[(int64_t)w * stride];"),
    ("worker_stride_ignored", "acc = acc + g[(int64_t)w * stride];",
     "acc = acc + g[(int64_t)w * m->arena_elems];"),
    ("lgp_sign", "*p = *p - step;", "*p = *p + step;"),
    ("lgp_on_wrong_stage", "if (stage_of(gib, l, k) != 2)\n                    continue;\n                float step",
     "if (stage_of(gib, l, k) != 1)\n                    continue;\n                float step"),
    ("lgp_uses_momentum_free_global", "float step = m->lr * grads[(int64_t)w * worker_stride + k];",
     "float step = m->lr * grads[k];"),
    ("gib_polarity", "return important ? 1 : 2;", "return important ? 2 : 1;"),
    ("importance_without_abs", "q[k] = fabsf(prod);", "q[k] = prod;"),
    ("layer_rank_descending", "if (a != b)\n        return a < b;", "if (a != b)\n        return a > b;"),
    ("layer_tie_break", "        return a < b;\n    return ia < ib;", "        return a < b;\n    return ia > ib;"),
    ("prefix_rule_skips", "            break;                           /* prefix rule: stop at the first misfit */",
     "            continue;"),
    ("budget_off_by_one", "if (taken + m->numel[l] > budget_elems)", "if (taken + m->numel[l] >= budget_elems)"),
    ("element_tie_break", "return x->index < y->index ? -1 : 1;", "return x->index < y->index ? 1 : -1;"),
    ("element_takes_largest", "return x->key < y->key ? -1 : 1;", "return x->key < y->key ? 1 : -1;"),
    ("nan_not_canonical", "if (isnan(q))\n        return 0x7FC00000u;", "if (0)\n        return 0x7FC00000u;"),
    ("apply_wrong_source", "Pw[(int64_t)w * param_stride + k] = P[k];", "Pw[(int64_t)w * param_stride + k] = P[k + 1 < m->arena_elems ? k + 1 : k];"),
    ("tuner_cap", "double limit = 0.8 * (double)model_elems;", "double limit = 0.9 * (double)model_elems;"),
    ("tuner_first_epoch", "    if (epoch == 1)\n        return 0;\n    double share", "    if (epoch == 0)\n        return 0;\n    double share"),
    ("tuner_share_inverted", "double share = 1.0 - loss_i / L;", "double share = loss_i / L;"),
    ("tuner_bound_divides_by_workers", "return b * (1.0 + loss_rate) * t_c / (double)n_workers;", "return b * (1.0 + loss_rate) * t_c;"),
    ("splitter_parts_swapped", "if (stage_of(gib, l, k) == 1) {\n                if (g_i)", "if (stage_of(gib, l, k) == 2) {\n                if (g_i)"),
    ("splitter_reads_tensor_local_index", "                    g_u[n_u] = g[k];", "                    g_u[n_u] = g[j];"),
    ("packed_update_wrong_stage", "            if (stage_of(gib, l, k) != stage)\n                continue;", "            if (stage_of(gib, l, k) == stage)\n                continue;"),
    ("packed_update_position_not_advanced", "            ++i;\n        }\n}", "        }\n}"),
    ("packed_update_uses_arena_index", "aggregate_element(m, packed + i, packed_stride)", "aggregate_element(m, packed + k, packed_stride)"),
    ("layer_sum_drops_last", "for (int64_t j = 0; j < m->numel[l]; ++j) {\n            double x", "for (int64_t j = 0; j + 1 < m->numel[l]; ++j) {\n            double x"),
]


def test_every_mutation_target_exists():
    text = open(SRC).read()
    for name, old, _ in MUTATIONS:
        assert text.count(old) == 1, f"{name}: target text must occur exactly once in the oracle"


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    text = open(SRC).read()
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", *CFLAGS, str(src), "-o", str(lib), "-lm"])
    env = dict(os.environ, OSP_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_tuner.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert b"failed" in r.stdout or b"error" in r.stdout.lower()
