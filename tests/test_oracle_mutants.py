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
    "forced_tail_positions_shifted": ("idx_out[(int64_t)h * total_k + o0 + kc + t] = (int32_t)(Lc + t);",
                                      "idx_out[(int64_t)h * total_k + o0 + kc + t] = (int32_t)(Lc + t - 1);"),
    "pool_window_reaches_into_the_forced_block": ("int64_t hi = j + half > Lc - 1 ? Lc - 1 : j + half;",
                                                  "int64_t hi = j + half > L - 1 ? L - 1 : j + half;"),
    "head_sum_descending_heads": ("for (int h = 0; h < Hq; ++h) sc = sc + pooled[(int64_t)h * Lc + j];",
                                  "for (int h = Hq - 1; h >= 0; --h) sc = sc + pooled[(int64_t)h * Lc + j];"),
    "head_sum_list_only_to_head_0": ("for (int h = head_sum ? 0 : li; h < (head_sum ? Hq : li + 1); ++h) {",
                                     "for (int h = li; h < li + 1; ++h) {"),
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


# ---- the packing oracle is plain Python: its mutants are functions put in its place

def _pack_with(rows_of, head_of):
    import numpy as np

    def pack(k, v, cu_kv, idx, cu_k):
        Hq, Hkv, D = idx.shape[0], k.shape[1], k.shape[2]
        kp = np.zeros((Hq, int(cu_k[-1]), D), dtype=k.dtype)
        vp = np.zeros((Hq, int(cu_k[-1]), D), dtype=v.dtype)
        for h in range(Hq):
            for b in range(len(cu_k) - 1):
                lst = rows_of(idx[h, int(cu_k[b]):int(cu_k[b + 1])], int(cu_kv[b]))
                for t, row in enumerate(lst):
                    kp[h, int(cu_k[b]) + t] = k[row, head_of(h, Hq, Hkv)]
                    vp[h, int(cu_k[b]) + t] = v[row, head_of(h, Hq, Hkv)]
        return kp, vp
    return pack


PACK_MUTANTS = {
    "rows_in_position_order_not_list_order": _pack_with(lambda l, k0: sorted(k0 + int(j) for j in l), lambda h, Hq, Hkv: h // (Hq // Hkv)),
    "sequence_offset_dropped": _pack_with(lambda l, k0: [int(j) for j in l], lambda h, Hq, Hkv: h // (Hq // Hkv)),
    "kv_head_by_modulo": _pack_with(lambda l, k0: [k0 + int(j) for j in l], lambda h, Hq, Hkv: h % Hkv),
}


def test_pack_mutant_harness_accepts_the_real_thing(monkeypatch):
    import oracle
    from tests import test_oracle_pins as pins
    faithful = _pack_with(lambda l, k0: [k0 + int(j) for j in l], lambda h, Hq, Hkv: h // (Hq // Hkv))
    monkeypatch.setattr(oracle, "pack", faithful)
    pins.test_pack_then_dense_attention_equals_attention_over_kept_rows()


@pytest.mark.parametrize("name", sorted(PACK_MUTANTS))
def test_pins_catch_pack_mutant(name, monkeypatch):
    import oracle
    from tests import test_oracle_pins as pins
    monkeypatch.setattr(oracle, "pack", PACK_MUTANTS[name])
    with pytest.raises(AssertionError):
        pins.test_pack_then_dense_attention_equals_attention_over_kept_rows()


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle built with -fsanitize=address,undefined runs the whole pin suite without a report
    (out-of-bounds reads, signed overflow, misaligned access ... in the checker would end the child)."""
    import oracle
    lib = oracle.build(sanitize=True, out=str(tmp_path / "libhcsa_oracle_san.so"))
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       env=oracle.sanitizer_env(lib), cwd=ROOT, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
