"""The pins must notice a broken oracle: plant one plausible mistake at a time in a COPY of the
oracle's source (a dropped term, a wrong index, a wrong triangle, a forgotten scalar), build it,
and require that tests/test_oracle_pins.py fails against it.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "blas3_ref.c")

MUTANTS = {
    "gemm_drops_beta_term": ("            if (beta != 0.0) v += beta * (double)C[p];                              \\\n            C[p] = (T)v;                                                            \\\n        }                                                                           \\\n        free(acc);",
                             "            C[p] = (T)v;                                                            \\\n        }                                                                           \\\n        free(acc);"),
    "gemm_transposed_b_index": ("double b = is_tr(tb) ? (double)B[at(order, j, l, ldb)]", "double b = is_tr(tb) ? (double)B[at(order, l, j, ldb)]"),
    "gemm_transposed_a_index": ("double a = is_tr(ta) ? (double)A[at(order, l, i, lda)]", "double a = is_tr(ta) ? (double)A[at(order, i, l, lda)]"),
    "gemm_alpha_applied_to_c": ("double v = (alpha != 0.0) ? alpha * acc[i] : 0.0;                       \\\n            if (beta != 0.0) v += beta * (double)C[p];",
                                "double v = (alpha != 0.0) ? alpha * acc[i] : 0.0;                       \\\n            if (beta != 0.0) v += alpha * beta * (double)C[p];"),
    "gemm_float_accumulation": ("acc[i] += a * b;", "acc[i] = (float)(acc[i] + a * b);"),
    "row_major_index_swapped": ("                        : (size_t)r * (size_t)ld + (size_t)c;", "                        : (size_t)c * (size_t)ld + (size_t)r;"),
    "syrk_writes_whole_matrix": ("long i0 = (uplo == LO) ? j : 0;", "long i0 = 0;"),
    "syrk_wrong_triangle": ("long i1 = (uplo == LO) ? N : j + 1;", "long i1 = (uplo == LO) ? N : j;"),
    "syr2k_drops_second_product": ("s += ai * bj + bi * aj;", "s += ai * bj;"),
    "syr2k_same_product_twice": ("s += ai * bj + bi * aj;", "s += ai * bj + ai * bj;"),
    "symm_reads_other_triangle": ("int stored = (uplo == LO) ? (r >= c) : (r <= c);", "int stored = 1;"),
    "symm_right_uses_left_indices": ("long r = (side == LEFT) ? i : l, c = (side == LEFT) ? l : j;", "long r = i, c = l;"),
    "tri_reads_unit_diagonal": ("if (r == c) return diag == UNIT ? 1.0 : (double)A[at(order, r, r, lda)];", "if (r == c) return (double)A[at(order, r, r, lda)];"),
    "tri_wrong_triangle": ("int inside = (uplo == LO) ? (r > c) : (r < c);", "int inside = (uplo == LO) ? (r < c) : (r > c);"),
    "tri_ignores_transpose": ("return is_tr(trans) ? tri_##SFX(order, uplo, diag, A, lda, c, r)", "return is_tr(trans) ? tri_##SFX(order, uplo, diag, A, lda, r, c)"),
    "trmm_forgets_alpha": ("B[at(order, i, j, ldb)] = (T)((alpha != 0.0) ? alpha * s : 0.0);", "B[at(order, i, j, ldb)] = (T)s;"),
    "trsm_forgets_alpha": ("double s = (alpha != 0.0) ? alpha * (double)B[at(order, i, j, ldb)] : 0.0;", "double s = (double)B[at(order, i, j, ldb)];"),
    "trsm_right_wrong_direction": ("long c = eff_lower ? N - 1 - t : t;", "long c = eff_lower ? t : N - 1 - t;"),
    # mistakes in the single-precision instantiations only (the double-precision pins cannot see them)
    "ssyrk_instantiated_for_double": ("DEFINE_SYRK(ref_ssyrk, float)", "DEFINE_SYRK(ref_ssyrk, double)"),
    "ssyr2k_instantiated_for_double": ("DEFINE_SYR2K(ref_ssyr2k, float)", "DEFINE_SYR2K(ref_ssyr2k, double)"),
    "ssymm_instantiated_for_double": ("DEFINE_SYMM(ref_ssymm, float)", "DEFINE_SYMM(ref_ssymm, double)"),
    "strmm_reads_the_triangle_as_double": ("DEFINE_TRMM(ref_strmm, float, s)", "DEFINE_TRMM(ref_strmm, float, d)"),
    "strsm_reads_the_triangle_as_double": ("DEFINE_TRSM(ref_strsm, float, s)", "DEFINE_TRSM(ref_strsm, float, d)"),
    "single_precision_triangle_ignores_unit_diagonal": (
        "DEFINE_TRI(float, s)",
        "static inline double tri_s(int order, int uplo, int diag, const float *A, long lda, long r, long c)\n"
        "{ (void)diag; if (r == c) return (double)A[at(order, r, r, lda)];\n"
        "  int inside = (uplo == LO) ? (r > c) : (r < c); return inside ? (double)A[at(order, r, c, lda)] : 0.0; }\n"
        "static inline double top_s(int order, int uplo, int trans, int diag, const float *A, long lda, long r, long c)\n"
        "{ return is_tr(trans) ? tri_s(order, uplo, diag, A, lda, c, r) : tri_s(order, uplo, diag, A, lda, r, c); }"),
    "syrk_accumulates_in_float": ("            double s = 0.0;                                                         \\\n            if (alpha != 0.0)                                                       \\\n                for (long l = 0; l < K; ++l) {                                      \\\n                    double x = is_tr(trans)",
                                  "            float s = 0.0f;                                                         \\\n            if (alpha != 0.0)                                                       \\\n                for (long l = 0; l < K; ++l) {                                      \\\n                    double x = is_tr(trans)"),
    "trsm_skips_division": ("x[i] = s / top_##SFX(order, uplo, trans, diag, A, lda, i, i);", "x[i] = s;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_fail_on_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found: the oracle changed, update this test"
    mutated = text.replace(old, new, 1)
    src = tmp_path / "blas3_ref_mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(mutated)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(src)])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(lib), OMP_NUM_THREADS="2")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # a failed assertion or a crash (an out-of-bounds index) both count as noticed
    assert run.returncode != 0, "the pins did not notice mutant %r\n%s" % (name, run.stdout[-2000:])
