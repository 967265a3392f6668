"""Checks that the oracle's pins have teeth: plant one plausible mistake at a time
in a copy of the C oracle (on the CPU), and require that at least one pin test of
tests/test_oracle_instances.py / test_oracle_scan.py / test_oracle_capsule.py fails for every planted mistake.  CPU only."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_instances as pins
import test_oracle_capsule as capsule_pins
import test_oracle_scan as scan_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "mdh_oracle.c")

# (name, text in the source, replacement)
MUTANTS = [
    ("dot_drops_last", "for (int64_t k = 0; k < K; ++k) {\n    double t = (double)x[k] * (double)y[k];", "for (int64_t k = 0; k < K - 1; ++k) {\n    double t = (double)x[k] * (double)y[k];"),
    ("matvec_x_indexed_by_row", "(double)A[i * K + k] * (double)x[k]", "(double)A[i * K + k] * (double)x[(k + i) % K]"),
    ("matvec_abs_forgotten", "aabs += fabs(t);\n    }\n    y[i] = acc;", "aabs += t;\n    }\n    y[i] = acc;"),
    ("matmul_B_column_mirrored", "(double)B[k * N + j];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C[i * N + j]",
     "(double)B[k * N + (N - 1 - j)];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C[i * N + j]"),
    ("matmul_k_mismatched", "double t = (double)A[i * K + k] * (double)B[k * N + j];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C[i * N + j]",
     "double t = (double)A[i * K + (K - 1 - k)] * (double)B[k * N + j];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C[i * N + j]"),
    ("matmul_drops_last_k", "for (int64_t k = 0; k < K; ++k) {\n        double t = (double)A[i * K + k] * (double)B[k * N + j];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C[",
     "for (int64_t k = 0; k < K - 1; ++k) {\n        double t = (double)A[i * K + k] * (double)B[k * N + j];\n        acc += t;\n        aabs += fabs(t);\n      }\n      C["),
    ("matmul_abs_forgotten", "aabs += fabs(t);\n      }\n      C[i * N + j] = acc;", "aabs += t;\n      }\n      C[i * N + j] = acc;"),
    ("jacobi_wrong_neighbour", "(double)c[-sx] + (double)c[sx]", "(double)c[-sx] + (double)c[sy]"),
    ("jacobi_sign", "d0 * (double)c[0] + d1 * nb", "d0 * (double)c[0] - d1 * nb"),
    ("jacobi_centre_shift", "in + (i + 1) * sx + (j + 1) * sy + (k + 1)", "in + (i + 1) * sx + (j + 1) * sy + k"),
    ("jacobi_coeffs_swapped", "d0 * (double)c[0] + d1 * nb", "d1 * (double)c[0] + d0 * nb"),
    ("mcc_filter_flipped", "filt[((k * R + r) * S + s) * C + c]", "filt[((k * R + (R - 1 - r)) * S + s) * C + c]"),
    ("mcc_stride_on_filter_index", "(p * sh + r)) * W + (q * sw + s)", "(p + r * sh)) * W + (q * sw + s)"),
    ("mcc_r_s_swapped_in_input", "(p * sh + r)) * W + (q * sw + s)", "(p * sh + s % R)) * W + (q * sw + r % S)"),
    ("mcc_drops_channel", "for (int64_t c = 0; c < C; ++c)\n    for (int64_t r", "for (int64_t c = 1; c < C; ++c)\n    for (int64_t r"),
    ("prl_tie_break_largest", "s2 == *s1 && b2 < *b1", "s2 == *s1 && b2 > *b1"),
    ("prl_weights_swapped", "(ra[f] == rb[f]) ? wp[f] : wm[f]", "(ra[f] == rb[f]) ? wm[f] : wp[f]"),
    ("prl_skips_last_b", "for (int64_t b = 1; b < nB; ++b)\n      maxidx(&bs, &bi, wght(nF, A + a * nF, B + b * nF", "for (int64_t b = 1; b < nB - 1; ++b)\n      maxidx(&bs, &bi, wght(nF, A + a * nF, B + b * nF"),
    ("prl_min_instead_of_max", "if (s2 > *s1) {", "if (s2 < *s1) {"),
    ("scan_exclusive", "out[i * n + j] = acc;", "out[i * n + j] = acc - (double)x[i * n + j];"),
    ("scan_abs_forgotten", "aabs += fabs((double)x[i * n + j]);", "aabs += (double)x[i * n + j];"),
    ("scan_row_stride", "acc += (double)x[i * n + j];", "acc += (double)x[i * (n - 1) + j];"),
    ("capsule_filter_matrix_transposed", "* MK + mk) * MJ + mj];", "* MK + mj % MK) * MJ + mk % MJ];"),
    ("capsule_drops_first_mk", "for (int64_t mk = 0; mk < MK; ++mk) {", "for (int64_t mk = 1; mk < MK; ++mk) {"),
    ("capsule_input_matrix_transposed", "* MI + mi) * MK + mk];", "* MI + mk % MI) * MK + mi % MK];"),
    ("capsule_stride_on_tap", "(n * H + (p * sh + r)) * W + (q * sw + s)) * C + c) * MI", "(n * H + (p + r * sh)) * W + (q * sw + s)) * C + c) * MI"),
    ("prl_field_dropped", "for (int32_t f = 0; f < nF; ++f) s +=", "for (int32_t f = 0; f < nF - 1; ++f) s +="),
]

PIN_TESTS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]
PIN_TESTS += [getattr(scan_pins, n) for n in dir(scan_pins) if n.startswith("test_")]
PIN_TESTS += [getattr(capsule_pins, n) for n in dir(capsule_pins) if n.startswith("test_")]


def _any_pin_fails():
    for t in PIN_TESTS:
        try:
            t()
        except Exception:  # assertion or anything else a broken oracle provokes
            return t.__name__
    return None


def test_pins_pass_on_the_real_oracle():
    assert _any_pin_fails() is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found: " + name
    mutated = text.replace(old, new, 1)
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    real = oracle._load()
    oracle._lib = ctypes.CDLL(str(so))
    try:
        caught_by = _any_pin_fails()
    finally:
        oracle._lib = real
    assert caught_by is not None, "no pin notices the planted mistake " + name
