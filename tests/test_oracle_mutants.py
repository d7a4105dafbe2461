"""Shows that the pins in test_oracle_pins.py have teeth: each plausible mistake
below is planted in a copy of the oracle's source (on the CPU, in a temporary
directory), the copy is compiled, and the pin suite is run against it in a child
process.  Every mutant must make at least one pin fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "hcsa_oracle.c")

MUTANTS = {
    "unfused_multiply_add": ("acc = fmaf(qsum[d], widen(k, dtype, krow + d), acc);",
                             "acc = acc + qsum[d] * widen(k, dtype, krow + d);"),
    "descending_d": ("for (int d = 0; d < D; ++d)\n                acc = fmaf(",
                     "for (int d = D - 1; d >= 0; --d)\n                acc = fmaf("),
    "block_rows_descending": ("for (int64_t i = 0; i < nq; ++i)\n                a = a + widen(q, dtype, ((q0 + i) * Hq + h) * D + d);",
                              "for (int64_t i = nq - 1; i >= 0; --i)\n                a = a + widen(q, dtype, ((q0 + i) * Hq + h) * D + d);"),
    "ties_to_higher_position": ("if (x->s < y->s) return 1;\n    return (x->j > y->j) - (x->j < y->j);",
                                "if (x->s < y->s) return 1;\n    return (x->j < y->j) - (x->j > y->j);"),
    "smallest_scores_kept": ("if (x->s > y->s) return -1;\n    if (x->s < y->s) return 1;",
                             "if (x->s > y->s) return 1;\n    if (x->s < y->s) return -1;"),
    "scale_dropped": ("z[t] = softmax_scale * dot;", "z[t] = dot;"),
    "logit_sign": ("const double p = exp(z[t] - zmax);", "const double p = exp(zmax - z[t]);"),
    "values_from_keys": ("out[d] += p * (double)widen(v, dtype, vrow + d);",
                         "out[d] += p * (double)widen(k, dtype, vrow + d);"),
    "not_normalised": ("for (int d = 0; d < D; ++d) out[d] /= denom;", ""),
    "gqa_head_map_in_attend": ("const int h = (int)(rh % Hq), g = h / G;", "const int h = (int)(rh % Hq), g = h % Hkv;"),
    "gqa_head_map_in_score": ("const int b = bh / Hq, h = bh % Hq, g = h / G;", "const int b = bh / Hq, h = bh % Hq, g = h % Hkv;"),
    "sequence_offset_dropped": ("const int64_t vrow = ((k0 + j) * Hkv + g) * D;", "const int64_t vrow = (j * Hkv + g) * D;"),
    "pool_window_lopsided": ("int64_t hi = j + half > L - 1 ? L - 1 : j + half;",
                             "int64_t hi = j + half - 1 > L - 1 ? L - 1 : (j + half - 1 < lo ? lo : j + half - 1);"),
    "query_dims_transposed": ("const int64_t qrow = (row * Hq + h) * D;\n        double zmax",
                              "const int64_t qrow = (row * Hq + (Hq - 1 - h)) * D;\n        double zmax"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    "-o", str(lib), str(mutated), "-lm"], check=True)
    env = dict(os.environ, HCSA_ORACLE_LIB_OVERRIDE=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, f"mutant '{name}' passed every pin:\n{r.stdout[-2000:]}"
    assert "failed" in r.stdout, r.stdout[-2000:]
