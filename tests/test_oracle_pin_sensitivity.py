"""Do the pins of the oracle bite?  Each case plants one plausible mistake in a
copy of ``oracle/mhcl_oracle.c`` (a dropped term, a missing factor, a
transposed index, a swapped order), builds it on the side and runs the pin
suites against that library in a child process: at least one pin must fail.
Everything here runs on the CPU; the oracle in the tree is never touched.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mhcl_oracle.c")
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_subset_pins.py", "tests/test_oracle_diag_pins.py"]

# (name, text in the source, replacement, which occurrence)
MUTANTS = [
    ("eps_outside_the_root", "1.0 / sqrt(ss / (double)nC + eps)", "1.0 / (sqrt(ss / (double)nC) + eps)", 0),
    ("sum_instead_of_mean_square", "1.0 / sqrt(ss / (double)nC + eps)", "1.0 / sqrt(ss + eps)", 0),
    ("h_post_without_factor_two", "H_post[(size_t)t * n + j] = 2.0 * sigmoid(z[R + n + j]);",
     "H_post[(size_t)t * n + j] = sigmoid(z[R + n + j]);", 0),
    ("permutation_matrices_transposed", "acc += a[k] * P[((size_t)k * n + i) * n + j];",
     "acc += a[k] * P[((size_t)k * n + j) * n + i];", 0),
    ("post_update_uses_h_res_transposed",
     "acc += H_res[((size_t)t * n + i) * n + j] * x[((size_t)t * n + j) * C + c];",
     "acc += H_res[((size_t)t * n + j) * n + i] * x[((size_t)t * n + j) * C + c];", 0),
    ("sk_rows_before_columns",
     "for (int i = 0; i < n; ++i) s += X[i * n + j];\n            for (int i = 0; i < n; ++i) X[i * n + j] /= s;",
     "for (int i = 0; i < n; ++i) s += X[j * n + i];\n            for (int i = 0; i < n; ++i) X[j * n + i] /= s;", 0),
    ("softmax_backward_without_the_mean", "a[k] * (g_a[k] - mean);", "a[k] * g_a[k];", 0),
    ("post_gate_backward_without_factor_two",
     "g_H_post[(size_t)t * n + j] * 2.0 * sq * (1.0 - sq);", "g_H_post[(size_t)t * n + j] * sq * (1.0 - sq);", 0),
    ("norm_backward_without_projection_term", "+= r * gxn[k] - coef * xh[k];", "+= r * gxn[k];", 0),
    ("g_W_from_unnormalised_input", "acc += rr[t] * x[(size_t)t * nC + k] * v[(size_t)t * M + m];",
     "acc += x[(size_t)t * nC + k] * v[(size_t)t * M + m];", 0),
    ("g_alpha_without_the_logit", "g_alpha[g] += g_z[(size_t)t * M + m] * uu[(size_t)t * M + m];",
     "g_alpha[g] += g_z[(size_t)t * M + m];", 0),
    ("sk_backward_row_step_without_its_sum",
     "for (int j = 0; j < n; ++j) g[i * n + j] = (g[i * n + j] - d) / s[i];",
     "for (int j = 0; j < n; ++j) g[i * n + j] = g[i * n + j] / s[i];", 0),
    ("sk_backward_column_step_divides_by_row_sums",
     "for (int i = 0; i < n; ++i) g[i * n + j] = (g[i * n + j] - d) / s[j];",
     "for (int i = 0; i < n; ++i) g[i * n + j] = (g[i * n + j] - d) / s[i];", 0),
    ("sk_backward_forgets_the_exponential", "g_z[(size_t)t * M + e] = g[e] * E[e];",
     "g_z[(size_t)t * M + e] = g[e];", 0),
    ("relative_range_upside_down", "nu[t] = mn / mx;", "nu[t] = mx / mn;", 0),
    ("layer_product_on_the_other_side", "s += Hl[i * n + k] * Q[k * n + j];", "s += Q[i * n + k] * Hl[k * n + j];", 0),
    ("g_y_with_unit_gates", "acc += H_post[(size_t)t * n + i] * gt[(size_t)i * C + c];",
     "acc += gt[(size_t)i * C + c];", 0),
    ("subset_table_read_as_inverse",
     "for (int i = 0; i < n; ++i) P[((size_t)k * n + i) * n + sigma[k * n + i]] = 1.0;",
     "for (int i = 0; i < n; ++i) P[((size_t)k * n + sigma[k * n + i]) * n + i] = 1.0;", 0),
]


def _nth(text, old, which):
    pos = -1
    for _ in range(which + 1):
        pos = text.index(old, pos + 1)
    return pos


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new, which):
    text = open(SRC).read()
    pos = _nth(text, old, which)
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(text[:pos] + new + text[pos + len(old):])
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    "-o", str(lib), str(mutant_c), "-lm"], check=True)
    env = dict(os.environ, MHCLO_LIB=str(lib), OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider",
                        "-m", "not gpu"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1 and " failed" in r.stdout, \
        f"{name}: the pins did not notice (exit {r.returncode})\n{r.stdout[-800:]}"


def test_the_unchanged_source_passes_the_same_way(tmp_path):
    """The side build itself is sound: the untouched source, built the same way, passes."""
    lib = tmp_path / "libsame.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    "-o", str(lib), SRC, "-lm"], check=True)
    env = dict(os.environ, MHCLO_LIB=str(lib), OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider",
                        "-m", "not gpu"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-800:]
