"""The pins must bite: each plausible mistake planted in a copy of the oracle's source (a dropped
term, a wrong sign or index, an unstable order, a wrong tie rule) has to make at least one pin
fail.  The broken copies are compiled on the CPU into a temporary directory; nothing here touches
the GPU or the real oracle."""
import os

import pytest

import oracle
import test_oracle_pins as pins
import test_oracle_reduce_pins as rpins
import test_oracle_scale_pins as spins

SRC = os.path.join(os.path.dirname(oracle.__file__), "isp_oracle.c")

# (name, text in isp_oracle.c, replacement, pins of which at least one must fail)
MUTANTS = [
    ("spmm: sign of the accumulated product",
     "        y[k] += t;\n        if (m) m[k] += fabs(t);", "        y[k] -= t;\n        if (m) m[k] += fabs(t);",
     [pins.test_hand_worked_example]),
    ("spmm: gathers the row's own X row instead of the column's",
     "      const float* x = X + (int64_t)indices[p] * ldx;", "      const float* x = X + (i % 2 ? (int64_t)indices[p] : 0) * ldx;",
     [pins.test_spmm_matches_dense_bruteforce]),
    ("spmm: magnitude without the absolute value",
     "        if (m) m[k] += fabs(t);\n      }\n    }\n  }\n}\n\n/* Backward of SpMM in scatter form", "        if (m) m[k] += t;\n      }\n    }\n  }\n}\n\n/* Backward of SpMM in scatter form",
     [pins.test_spmm_matches_dense_bruteforce]),
    ("transpose: entries of a column in reverse source order (not stable)",
     "  for (int64_t i = 0; i < n_rows; ++i) {\n    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {\n      const int64_t q = cursor[indices[p]]++;",
     "  for (int64_t i = n_rows - 1; i >= 0; --i) {\n    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {\n      const int64_t q = cursor[indices[p]]++;",
     [pins.test_transpose_properties, pins.test_hand_worked_example]),
    ("transpose: t_values not permuted",
     "      if (t_values) t_values[q] = values ? values[p] : 1.0f;", "      if (t_values) t_values[q] = values ? values[q] : 1.0f;",
     [pins.test_transpose_properties]),
    ("scatter backward: adds into the row instead of the column",
     "      double* o = dX + (int64_t)indices[p] * d;\n      for (int32_t k = 0; k < d; ++k) o[k] += a * (double)g[k];",
     "      double* o = dX + (int64_t)(indices[p] / 2) * d;\n      for (int32_t k = 0; k < d; ++k) o[k] += a * (double)g[k];",
     [pins.test_backward_adjoint_and_scatter]),
    ("sddmm: last feature dropped from the dot product",
     "      double acc = 0.0, am = 0.0;\n      for (int32_t k = 0; k < d; ++k) {", "      double acc = 0.0, am = 0.0;\n      for (int32_t k = 0; k + 1 < d || (d == 1 && k < 1); ++k) {",
     [pins.test_sddmm_bruteforce_and_identity]),
    ("sddmm: scale flag ignored",
     "      const double a = (scale_by_a && values) ? (double)values[p] : 1.0;\n      out[p] = a * acc;", "      const double a = 1.0;\n      out[p] = a * acc;",
     [pins.test_hand_worked_example]),
    ("fusedmm: sigmoid of +z replaced by sigmoid of -z",
     "return op == 0 ? 1.0 / (1.0 + exp(-z)) :", "return op == 0 ? 1.0 / (1.0 + exp(z)) :",
     [pins.test_fusedmm_forward_is_unfused_composition]),
    ("fusedmm backward: the path through z into x_j dropped",
     "        oj[k] += a * s * (double)gi[k] + dz * (double)xi[k];", "        oj[k] += a * s * (double)gi[k];",
     [lambda: pins.test_fusedmm_backward_finite_differences(0, "sigmoid")]),
    ("fusedmm backward: derivative of the sigmoid with the wrong sign inside",
     "return s * (1.0 - s); }", "return s * (1.0 + s); }",
     [lambda: pins.test_fusedmm_backward_finite_differences(1, "sigmoid")]),
    ("fusedmm backward: direct term uses the gradient of the wrong row",
     "    const float* gi = dY + i * ldg;\n    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {\n      const int64_t j = indices[p];",
     "    const float* gi = dY + i * ldg;\n    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {\n      const int64_t j = indices[p];\n      gi = dY + j * ldg;",
     [lambda: pins.test_fusedmm_backward_finite_differences(2, "dot")]),
    ("mean: divides by the row length plus one",
     "        y[k] = e > s ? acc / (double)(e - s) : 0.0;", "        y[k] = e > s ? acc / (double)(e - s + 1) : 0.0;",
     [rpins.test_mean_closed_forms]),
    ("min / max: the last of equal entries wins instead of the first",
     "(reduce == 2 ? tv < best : tv > best)", "(reduce == 2 ? tv <= best : tv >= best)",
     [rpins.test_mean_closed_forms, rpins.test_reduce_matches_bruteforce]),
    ("min / max backward: the entry's value is not applied",
     "        const double t = (values ? (double)values[p] : 1.0) * (double)g[k];\n        dX[(int64_t)indices[p] * d + k] += t;",
     "        const double t = (double)g[k];\n        dX[(int64_t)indices[p] * d + k] += t;",
     [rpins.test_reduce_backward_is_the_adjoint_of_the_selected_linear_map]),
    ("mean backward: weight without the division by the row length",
     "        const double w = (values ? (double)values[p] : 1.0) / (double)(e - s);", "        const double w = (values ? (double)values[p] : 1.0);",
     [rpins.test_reduce_backward_is_the_adjoint_of_the_selected_linear_map]),
    # ---- the error scales (mag) the FusedMM / reduction parity tests divide by
    ("fusedmm scale: doubled",
     "        if (m) m[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);",
     "        if (m) m[k] += 2.0 * fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);",
     [spins.test_fusedmm_forward_scale]),
    ("fusedmm scale: edge value without the absolute value",
     "        if (m) m[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);",
     "        if (m) m[k] += a * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);",
     [spins.test_fusedmm_forward_scale]),
    ("fusedmm scale: the dot product's share (L1 term) dropped",
     "        if (m) m[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)xj[k]);",
     "        if (m) m[k] += fabs(a) * fabs(s) * fabs((double)xj[k]);",
     [spins.test_fusedmm_forward_scale]),
    ("fusedmm scale: derivative bound of the sigmoid inflated",
     "static double edge_l1(int op) { return op == 0 ? 0.25 :", "static double edge_l1(int op) { return op == 0 ? 250.0 :",
     [spins.test_fusedmm_forward_scale]),
    ("fusedmm scale: za accumulated without the absolute value",
     "        z += t;\n        za += fabs(t);", "        z += t;\n        za += t;",
     [spins.test_fusedmm_forward_scale]),
    ("fusedmm backward scale: dz bound doubled",
     "      const double dzm = fabs(a) * gda * (fabs(edge_df(op, z)) + edge_l2(op) * za);",
     "      const double dzm = 2.0 * fabs(a) * gda * (fabs(edge_df(op, z)) + edge_l2(op) * za);",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: second-derivative (L2) term dropped",
     "      const double dzm = fabs(a) * gda * (fabs(edge_df(op, z)) + edge_l2(op) * za);",
     "      const double dzm = fabs(a) * gda * fabs(edge_df(op, z));",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: second-derivative bound inflated",
     "static double edge_l2(int op) { return op == 0 ? 0.1 : 0.0; }", "static double edge_l2(int op) { return op == 0 ? 100.0 : 0.0; }",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: row term multiplied by 1000",
     "          mi[k] += dzm * fabs((double)xj[k]);", "          mi[k] += 1000.0 * dzm * fabs((double)xj[k]);",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: direct term of the column part doubled",
     "          mj[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);",
     "          mj[k] += 2.0 * fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: L1 term of the column part dropped",
     "          mj[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);",
     "          mj[k] += fabs(a) * fabs(s) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: the z path of the column part dropped",
     "          mj[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]) + dzm * fabs((double)xi[k]);",
     "          mj[k] += fabs(a) * (fabs(s) + edge_l1(op) * za) * fabs((double)gi[k]);",
     [spins.test_fusedmm_backward_scale]),
    ("fusedmm backward scale: |g x| accumulated without the absolute value",
     "        gda += fabs(t);", "        gda += t;",
     [spins.test_fusedmm_backward_scale]),
    ("mean scale: not divided by the row length",
     "        if (m) m[k] = e > s ? am / (double)(e - s) : 0.0;", "        if (m) m[k] = e > s ? am : 0.0;",
     [spins.test_mean_scale]),
    ("mean scale: doubled",
     "          am += fabs(t);", "          am += 2.0 * fabs(t);",
     [spins.test_mean_scale]),
    ("mean backward scale: doubled",
     "          if (m) m[k] += fabs(w * (double)g[k]);", "          if (m) m[k] += 2.0 * fabs(w * (double)g[k]);",
     [spins.test_reduce_backward_scale]),
    ("min / max backward scale: doubled",
     "        if (mag) mag[(int64_t)indices[p] * d + k] += fabs(t);", "        if (mag) mag[(int64_t)indices[p] * d + k] += 2.0 * fabs(t);",
     [spins.test_reduce_backward_scale]),
    ("min / max backward scale: without the absolute value",
     "        if (mag) mag[(int64_t)indices[p] * d + k] += fabs(t);", "        if (mag) mag[(int64_t)indices[p] * d + k] += t;",
     [spins.test_reduce_backward_scale]),
    ("min / max: products compared in fp64 but reported position of the last near-tie",
     "(reduce == 2 ? tv < best : tv > best)", "(reduce == 2 ? tv <= best : tv >= best)",
     [spins.test_minmax_against_the_fp64_definition]),
]


@pytest.fixture
def restore_oracle():
    yield
    oracle.use_library(None)


@pytest.mark.parametrize("name,old,new,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pin_catches_planted_mistake(name, old, new, checks, tmp_path, restore_oracle):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found exactly once: " + name
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = oracle.compile_source(str(src), str(tmp_path / "libmutant.so"))
    oracle.use_library(lib)
    caught = False
    for check in checks:
        try:
            check()
        except Exception:  # an AssertionError, or hypothesis' group of several distinct failures
            caught = True
            break
    oracle.use_library(None)
    assert caught, "no pin noticed the planted mistake: " + name


def test_the_unmodified_oracle_passes_the_same_pins(restore_oracle):
    oracle.use_library(None)
    for _, _, _, checks in MUTANTS:
        for check in checks:
            check()
