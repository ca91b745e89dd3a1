"""Do the pins have teeth?  Each case plants ONE plausible mistake in a copy of
the oracle's C source (never in the oracle itself, never on a GPU), compiles
the copy and requires that at least one pin fails on it.  CPU only."""
import os
import subprocess

import pytest

from oracle import came_oracle as O
from oracle_pins import ALL_PINS

SRC = os.path.join(os.path.dirname(O.__file__), "came_oracle.c")

# (name, exact text in came_oracle.c, replacement, how many occurrences to replace [0 = all])
MUTATIONS = [
    ("row_mean_instead_of_sum",
     "r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * rowsum;",
     "r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * rowsum / (double)m;", 1),
    ("v_without_normaliser",
     "v[i * m + j] = r[i] * c[j] / sum_r;", "v[i * m + j] = r[i] * c[j];", 1),
    ("eps1_dropped",
     "G[i * m + j] = g[i * m + j] * g[i * m + j] + h->eps1;",
     "G[i * m + j] = g[i * m + j] * g[i * m + j];", 1),
    ("eps1_outside_the_sum",
     "r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * rowsum;",
     "r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * (rowsum - (m - 1) * h->eps1);", 1),
    ("clip_min_instead_of_max",
     "const double denom = fmax(1.0, rms_u / h->clip_d);\n    for (int64_t k = 0; k < nm; ++k) uh[k] = u[k] / denom;",
     "const double denom = fmin(1.0, rms_u / h->clip_d);\n    for (int64_t k = 0; k < nm; ++k) uh[k] = u[k] / denom;", 1),
    ("clip_inverted_ratio",
     "const double denom = fmax(1.0, rms_u / h->clip_d);\n    for (int64_t k = 0; k < nm; ++k) uh[k] = u[k] / denom;",
     "const double denom = fmax(1.0, h->clip_d / rms_u);\n    for (int64_t k = 0; k < nm; ++k) uh[k] = u[k] / denom;", 1),
    ("rms_not_a_mean",
     "return sqrt(ss / (double)count);", "return sqrt(ss);", 1),
    ("momentum_coefficients_swapped",
     "M[k] = h->beta1 * M[k] + (1.0 - h->beta1) * uh[k];\n\n    /* instability",
     "M[k] = (1.0 - h->beta1) * M[k] + h->beta1 * uh[k];\n\n    /* instability", 1),
    ("instability_from_unclipped_u",
     "U[k] = (uh[k] - M[k]) * (uh[k] - M[k]);", "U[k] = (u[k] - M[k]) * (u[k] - M[k]);", 1),
    ("instability_not_squared",
     "U[k] = (uh[k] - M[k]) * (uh[k] - M[k]);", "U[k] = fabs(uh[k] - M[k]);", 1),
    ("eps2_dropped_rows",
     "rowsum += U[i * m + j] + h->eps2;", "rowsum += U[i * m + j];", 1),
    ("eps2_dropped_cols",
     "colsum += U[i * m + j] + h->eps2;", "colsum += U[i * m + j];", 1),
    ("confidence_uses_beta2",
     "R[i] = h->beta3 * R[i] + (1.0 - h->beta3) * rowsum;",
     "R[i] = h->beta2 * R[i] + (1.0 - h->beta2) * rowsum;", 1),
    ("second_moment_forgets_history",
     "c[j] = h->beta2 * c[j] + (1.0 - h->beta2) * colsum;\n    }\n\n    /* rank-one second moment",
     "c[j] = (1.0 - h->beta2) * colsum;\n    }\n\n    /* rank-one second moment", 1),
    ("S_without_normaliser",
     "S[i * m + j] = R[i] * C[j] / sum_R;", "S[i * m + j] = R[i] * C[j];", 1),
    ("S_not_under_sqrt",
     "theta[k] = theta[k] - h->lr / sqrt(S[k]) * M[k];", "theta[k] = theta[k] - h->lr / S[k] * M[k];", 1),
    ("update_sign",
     "theta[k] = theta[k] - h->lr / sqrt(S[k]) * M[k];", "theta[k] = theta[k] + h->lr / sqrt(S[k]) * M[k];", 1),
    ("update_uses_u_hat_not_momentum",
     "theta[k] = theta[k] - h->lr / sqrt(S[k]) * M[k];", "theta[k] = theta[k] - h->lr / sqrt(S[k]) * uh[k];", 1),
    ("column_sum_over_wrong_axis",
     "for (int64_t i = 0; i < n; ++i) colsum += G[i * m + j];",
     "for (int64_t i = 0; i < n; ++i) colsum += G[i * m + (j + 1) % m];", 1),
    ("vector_confidence_dropped",
     "theta[i] = theta[i] - h->lr / sqrt(s[i]) * M[i];", "theta[i] = theta[i] - h->lr * M[i];", 1),
    ("vector_second_moment_is_a_sum",
     "v[i] = h->beta2 * v[i] + (1.0 - h->beta2) * (g[i] * g[i] + h->eps1);",
     "v[i] = v[i] + (g[i] * g[i] + h->eps1);", 1),
    ("adafactor_applies_confidence",
     "theta[k] = theta[k] - h->lr * M[k];", "theta[k] = theta[k] - h->lr * M[k] / sqrt(fabs(M[k]) + 1.0);", 1),
    ("bf16_truncates",
     "nearbyint(ldexp(f, -q))", "trunc(ldexp(f, -q))", 1),
    ("bf16_rounds_half_away",
     "nearbyint(ldexp(f, -q))", "round(ldexp(f, -q))", 1),
    ("bf16_keeps_nine_bits",
     "int q = e - 8; ", "int q = e - 9; ", 1),
    ("bf16_subnormals_too_fine",
     "if (q < -133) q = -133;", "", 1),
    ("bf16_never_overflows",
     "if (fabs(y) >= ldexp(1.0, 128)) return copysign(INFINITY, y);", "", 1),
    ("bf16_rounds_the_double_not_the_binary32",
     "const double f = (double)(float)x; ", "const double f = x; ", 1),
    ("decay_grows_the_parameter",
     "theta[k] = theta[k] - lr * weight_decay * theta[k];", "theta[k] = theta[k] + lr * weight_decay * theta[k];", 1),
    ("decay_ignores_the_learning_rate",
     "theta[k] = theta[k] - lr * weight_decay * theta[k];", "theta[k] = theta[k] - weight_decay * theta[k];", 1),
    ("list_driver_skips_vectors",
     "e = came_oracle_vector_step(rows[t], theta[t], g[t], M[t], r[t], R[t], h, NULL);",
     "e = 0;", 1),
]


@pytest.mark.parametrize("name,old,new,count", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, count, tmp_path):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target not found in oracle source: {old!r}"
    mutated = text.replace(old, new, count) if count else text.replace(old, new)
    assert mutated != text
    src = tmp_path / f"mut_{name}.c"
    src.write_text(mutated)
    lib_path = str(tmp_path / f"libmut_{name}.so")
    subprocess.run(["gcc", "-std=c99", "-O1", "-fPIC", "-shared", "-fopenmp", str(src), "-o", lib_path,
                    "-lm"], check=True)
    lib = O.load(lib_path)
    caught = []
    for pin in ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"
