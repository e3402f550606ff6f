"""Mutation check of the oracle (CPU only): plant one plausible mistake at a time in a COPY of the
oracle -- a text substitution in oracle/bcq_ref.c compiled to a temporary library, or in
oracle/quantizer.py executed as a temporary module -- run the pins against the copy, and require that
the pins named for that mistake fail.  Shows that the pins of tests/test_oracle_pins.py and
tests/test_oracle_quantizer.py can tell the oracle from its near misses (a dropped term, a wrong sign
or index, a transposed operand).  Nothing here touches the GPU path or the real oracle files."""
import os
import subprocess
import types

import pytest

from oracle import build as oracle_build, quantizer, ref
from tests import test_oracle_pins as P
from tests import test_oracle_quantizer as PQ

# name -> callable; the parametrised pins are called on one representative case
C_PINS = {
    "half_to_double_all_patterns": P.test_half_to_double_all_patterns,
    "round_trip_fused_form": lambda: P.test_round_trip_fused_form_is_exact(3, 2),
    "round_trip_general_scale": P.test_round_trip_general_scale_within_half_ulp_of_offset,
    "q1_sign_matrix": P.test_q1_sign_matrix_against_int64_matvec,
    "popcount_closed_form": P.test_popcount_closed_form_with_all_ones_input,
    "column_probe": P.test_column_probe_fixes_bit_order_and_group_index,
    "transposition": P.test_transposition_would_be_caught,
    "gemm_against_brute": lambda: P.test_gemm_against_brute_force(33, 96, 3),
    "linearity": P.test_linearity_in_x,
    "plane_flip": P.test_flipping_a_plane_negates_its_alpha,
    "plane_permutation": P.test_plane_permutation_and_zero_alpha_plane,
    "no_offset_equals_zero_offset": P.test_no_offset_equals_zero_offset,
    "subnormal_alpha": P.test_subnormal_alpha_is_kept,
    "exact_layer": P.test_exact_layer_is_integer_valued_and_matches_brute,
}

# (name, text in bcq_ref.c, replacement, pins that must fail)
C_MUTATIONS = [
    ("bit order inside a word reversed",
     "return ((word >> (k & 31)) & 1u) ? 1.0 : -1.0;", "return ((word >> (31 - (k & 31))) & 1u) ? 1.0 : -1.0;",
     ["column_probe", "gemm_against_brute"]),
    ("sign encoding swapped (bit 1 -> -1)",
     "return ((word >> (k & 31)) & 1u) ? 1.0 : -1.0;", "return ((word >> (k & 31)) & 1u) ? -1.0 : 1.0;",
     ["q1_sign_matrix", "popcount_closed_form", "round_trip_fused_form"]),
    ("alpha indexed [m][plane][group] instead of [m][group][plane]",
     "double a = bcq_ref_half_to_double(alpha[(m * G + grp) * q + i]);",
     "double a = bcq_ref_half_to_double(alpha[(m * q + i) * G + grp]);",
     ["column_probe", "round_trip_fused_form"]),
    ("group index off by one",
     "int64_t grp = k / g;", "int64_t grp = (k / g + 1) % G;",
     ["column_probe", "popcount_closed_form"]),
    ("offset subtracted",
     "w += bcq_ref_half_to_double(z[m * G + grp]);", "w -= bcq_ref_half_to_double(z[m * G + grp]);",
     ["round_trip_fused_form", "popcount_closed_form"]),
    ("offset dropped",
     "w += bcq_ref_half_to_double(z[m * G + grp]);", "(void)z;",
     ["round_trip_fused_form", "popcount_closed_form"]),
    ("subnormal binary16 values flushed to zero",
     "v = ldexp((double)frac, -24);            /* subnormal or zero */", "v = 0.0;",
     ["half_to_double_all_patterns", "subnormal_alpha"]),
    ("binary16 exponent bias off by one",
     "v = ldexp((double)(1024 + frac), expo - 25);", "v = ldexp((double)(1024 + frac), expo - 24);",
     ["half_to_double_all_patterns"]),
    ("last plane dropped",
     "        for (int i = 0; i < q; ++i) {\n            double a = bcq_ref_half_to_double(alpha[(m * G + grp) * q + i]);",
     "        for (int i = 0; i < q - 1; ++i) {\n            double a = bcq_ref_half_to_double(alpha[(m * G + grp) * q + i]);",
     ["round_trip_fused_form", "q1_sign_matrix", "gemm_against_brute"]),
    ("output written transposed",
     "Y[j * M + m] = acc;", "Y[m * b + j] = acc;",
     ["transposition", "linearity"]),
    ("activation row ignored (always row 0)",
     "acc += wrow[k] * xd[j * N + k];", "acc += wrow[k] * xd[k];",
     ["linearity", "gemm_against_brute"]),
]


def _run(pins):
    failed = []
    for name, fn in pins.items():
        try:
            fn()
        except AssertionError:
            failed.append(name)
        except Exception:  # a mutation may also break a shape or produce NaN handling errors
            failed.append(name)
    return failed


@pytest.fixture
def mutated_c_oracle(tmp_path, monkeypatch):
    """Returns load(old, new): compiles the mutated source and points oracle.ref at it."""
    src = open(oracle_build.SRC).read()

    def load(old, new):
        assert src.count(old) >= 1, f"mutation target not found in bcq_ref.c: {old!r}"
        c_path = tmp_path / "bcq_ref_mutant.c"
        so_path = tmp_path / "libbcq_ref_mutant.so"
        c_path.write_text(src.replace(old, new))
        subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", str(c_path), "-o", str(so_path), "-lm"], check=True)
        monkeypatch.setattr(oracle_build, "LIB", str(so_path))
        monkeypatch.setattr(ref, "_lib", None)
        ref.lib()

    yield load
    monkeypatch.undo()
    ref._lib = None  # the next user reloads the real library


def test_the_unmutated_oracle_passes_every_pin_used_here():
    assert _run(C_PINS) == []
    assert _run(Q_PINS) == []


@pytest.mark.parametrize("name,old,new,expected", C_MUTATIONS, ids=[m[0] for m in C_MUTATIONS])
def test_c_oracle_mutation_is_caught(mutated_c_oracle, name, old, new, expected):
    mutated_c_oracle(old, new)
    failed = _run(C_PINS)
    assert failed, f"no pin notices: {name}"
    missing = [p for p in expected if p not in failed]
    assert not missing, f"{name}: expected {expected} to fail, but {missing} passed (failed: {failed})"


# ---- oracle/quantizer.py ----------------------------------------------------------------------------
Q_PINS = {
    "eq7_interval": PQ.test_scale_grid_stays_inside_the_interval_of_eq7,
    "eq6_example": PQ.test_quant_row_reproduces_the_papers_example,
    "search_brute_force": PQ.test_search_is_the_brute_force_argmin,
    "diagonal_h_round_to_nearest": PQ.test_gptq_with_uncorrelated_inputs_is_round_to_nearest,
    "eq2_least_squares": PQ.test_eq2_is_the_least_squares_compensation,
    "cholesky_equals_definition": PQ.test_cholesky_form_equals_the_definition,
    "compensation_lowers_error": PQ.test_compensation_lowers_the_output_error,
    "search_then_fuse": PQ.test_search_then_fuse_round_trip,
    "constant_row": PQ.test_constant_row_is_reproduced,
    "follow_replays": PQ.test_gptq_follow_replays_gptq_and_reports_forced_columns,
}

Q_MUTATIONS = [
    ("sign of the Cholesky-form update",
     "            err = (W[m, j] - (S[m] * wq + qbias[m])) / U[j, j]\n            W[m, j:] -= err * U[j, j:]\n    return Wq",
     "            err = (W[m, j] - (S[m] * wq + qbias[m])) / U[j, j]\n            W[m, j:] += err * U[j, j:]\n    return Wq",
     ["cholesky_equals_definition"]),
    ("1/U[j][j] missing in the Cholesky-form update",
     "            err = (W[m, j] - (S[m] * wq + qbias[m])) / U[j, j]\n            W[m, j:] -= err * U[j, j:]\n    return Wq",
     "            err = (W[m, j] - (S[m] * wq + qbias[m]))\n            W[m, j:] -= err * U[j, j:]\n    return Wq",
     ["cholesky_equals_definition"]),
    ("sign of Eq. 2 in the literal form",
     "return -err / Hinv[0, 0] * Hinv[:, 0]", "return err / Hinv[0, 0] * Hinv[:, 0]",
     ["eq2_least_squares", "cholesky_equals_definition"]),
    ("Eq. 2 without the division by the diagonal of the inverse Hessian",
     "return -err / Hinv[0, 0] * Hinv[:, 0]", "return -err * Hinv[:, 0]",
     ["eq2_least_squares", "cholesky_equals_definition"]),
    ("Eq. 2 takes a row of the wrong matrix (the Hessian itself, not its inverse)",
     "Hinv = np.linalg.inv(H[j:, j:])                # H_F^-1, F = columns j .. N-1", "Hinv = H[j:, j:]",
     ["cholesky_equals_definition"]),
    ("both forms of the update with the wrong sign",
     None, None, ["compensation_lowers_error"]),
    ("lower bound of Eq. 7 uses 2^n - 1",
     "lo = (w_max - w_min) / (2 ** (n + 1) - 1)", "lo = (w_max - w_min) / (2 ** n - 1)",
     ["eq7_interval"]),
    ("upper bound of Eq. 7 uses 2^n - 1",
     "hi = (w_max - w_min) / (2 ** (n - 1) - 1)", "hi = (w_max - w_min) / (2 ** n - 1)",
     ["eq7_interval"]),
    ("Hessian dropped from the search criterion",
     "err = float(d @ G @ d)", "err = float(d @ d)",
     ["search_brute_force"]),
    ("search keeps the last instead of the first smallest... of a worse candidate (>)",
     "if err < best[0]:", "if err > best[0] or best[1] is None:",
     ["search_brute_force"]),
    ("dampening left out",
     "    H = H + damp * np.mean(np.diag(H)) * np.eye(N)\n    U = np.linalg.cholesky", "    U = np.linalg.cholesky",
     ["cholesky_equals_definition"]),
    ("H = X X^T without the factor 2",
     "return 2.0 * X @ X.T", "return X @ X.T",
     ["search_brute_force"]),
]


BOTH_SIGNS = [("return -err / Hinv[0, 0] * Hinv[:, 0]", "return err / Hinv[0, 0] * Hinv[:, 0]"),
              ("            W[m, j:] -= err * U[j, j:]\n    return Wq", "            W[m, j:] += err * U[j, j:]\n    return Wq")]


def _mutant_quantizer(old, new):
    src = open(quantizer.__file__).read()
    pairs = BOTH_SIGNS if old is None else [(old, new)]
    for o, n_ in pairs:
        assert src.count(o) == 1, f"mutation target not found exactly once in quantizer.py: {o!r}"
        src = src.replace(o, n_)
    mod = types.ModuleType("oracle.quantizer_mutant")
    mod.__file__ = quantizer.__file__
    mod.__package__ = "oracle"
    exec(compile(src, quantizer.__file__, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name,old,new,expected", Q_MUTATIONS, ids=[m[0] for m in Q_MUTATIONS])
def test_quantizer_oracle_mutation_is_caught(monkeypatch, name, old, new, expected):
    monkeypatch.setattr(PQ, "Q", _mutant_quantizer(old, new))
    failed = _run(Q_PINS)
    assert failed, f"no pin notices: {name}"
    missing = [p for p in expected if p not in failed]
    assert not missing, f"{name}: expected {expected} to fail, but {missing} passed (failed: {failed})"
