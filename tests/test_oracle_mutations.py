"""The pins must be able to fail: plant one plausible mistake at a time in a copy of the
oracle's source (on the CPU, in a temporary build) and require that some pin rejects it."""
import ctypes
import importlib.util
import os
import subprocess

import pytest

import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")

MUTATIONS = [
    ("cost sign flipped", "s += X[(size_t)i * d + c] * Z[(size_t)t * d + c]",
     "s -= X[(size_t)i * d + c] * Z[(size_t)t * d + c]"),
    ("token mass dropped from the f-update", "f[i] = eps * (log(a[i]) - logsumexp(col, r, 1))",
     "f[i] = eps * (0.0 - logsumexp(col, r, 1))"),
    ("pivot mass dropped from the g-update", "g[t] = eps * (log(b[t]) - logsumexp(col, n, 1))",
     "g[t] = eps * (0.0 - logsumexp(col, n, 1))"),
    ("wrong start", "for (int t = 0; t < r; ++t) g[t] = 0.0;", "for (int t = 0; t < r; ++t) g[t] = 0.3 * t;"),
    ("maximum not added back", "return m + log(s);", "return log(s);"),
    ("eps multiplies instead of divides", "exp((C[(size_t)i * r + t] + f[i] + g[t]) / eps)",
     "exp((C[(size_t)i * r + t] + f[i] + g[t]) * eps)"),
    ("factor n missing", "O[(size_t)i * d_v + c] = (double)n * s;\n        }\n    free(Y);",
     "O[(size_t)i * d_v + c] = s;\n        }\n    free(Y);"),
    ("1/beta missing in the factored apply", "Y[(size_t)t * d_v + c] /= beta[t];", "Y[(size_t)t * d_v + c] /= 1.0;"),
    ("1/beta missing in the dense plan", "s += gamma1[(size_t)i * r + t] / beta[t] * gamma2[(size_t)t * n + j];",
     "s += gamma1[(size_t)i * r + t] * gamma2[(size_t)t * n + j];"),
    ("key side solved with the queries", "lot_oracle_cost(K, Z, n, r, d_k, C);", "lot_oracle_cost(Q, Z, n, r, d_k, C);"),
    ("pivot measure indexed by batch", "int h = p % H;", "int h = p / H;"),
    ("key coupling applied to the wrong token", "gamma2[(size_t)t * n + j] * V[(size_t)j * d_v + c]",
     "gamma2[(size_t)t * n + (n - 1 - j)] * V[(size_t)j * d_v + c]"),
]


def _mutated_oracle(tmp_path, old, new):
    src = open(os.path.join(ORACLE_DIR, "lot_oracle.c")).read()
    assert src.count(old) == 1, "mutation target not found exactly once: %r" % old
    c_file = tmp_path / "mut.c"
    c_file.write_text(src.replace(old, new))
    so = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so),
                           str(c_file), "-lm"])
    spec = importlib.util.spec_from_file_location("lot_oracle_mut", os.path.join(ORACLE_DIR, "lot_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._lib = ctypes.CDLL(str(so))
    mod._lib.lot_oracle_attention.restype = ctypes.c_int
    return mod


def _run_all_pins(oracle):
    """Run every pin (with a reduced parameter set); return the names of those that fail."""
    cases = [
        (pins.test_cost_is_x_zt, ()),
        (pins.test_iterates_equal_scaling_form, (3,)),
        (pins.test_converged_coupling_maximises_entropic_objective, ()),
        (pins.test_two_by_two_closed_form, ()),
        (pins.test_scaling_form_cross_ratios, (3,)),
        (pins.test_gluing_identities_hold_at_every_T, (2,)),
        (pins.test_doubly_stochastic_at_convergence, ()),
        (pins.test_rank_at_most_r_and_generically_r, (1,)),
        (pins.test_factored_dense_and_outer_product_forms_agree, (1, 16, 8)),
        (pins.test_single_pivot_gives_mean_of_v, (1, 1.0)),
        (pins.test_degenerate_costs_give_product_coupling, ()),
        (pins.test_symmetries, ()),
        (pins.test_batch_layout_and_per_head_pivots, ()),
    ]
    failed = []
    for fn, args in cases:
        try:
            fn(oracle, *args)
        except Exception:                                   # noqa: BLE001 - any failure counts
            failed.append(fn.__name__)
    return failed


def test_unmutated_source_passes(oracle):
    assert _run_all_pins(oracle) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    failed = _run_all_pins(_mutated_oracle(tmp_path, old, new))
    assert failed, "no pin noticed: " + name
