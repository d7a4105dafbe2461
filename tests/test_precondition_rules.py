"""The rules of the optional device-side precondition checks (csrc/precondition_rules.h), compiled for the
host with gcc and driven through ctypes: the same text the checked library's validators run on the GPU."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_17077_amd", "csrc")
CU_Q, CU_KV, CU_K, K_OVER_L, FORCED, IDX = 1, 2, 4, 8, 16, 32

HARNESS = r'''
#include "precondition_rules.h"
unsigned all_sequences(const int32_t* cu_q, const int32_t* cu_kv, const int32_t* cu_k, const uint8_t* mode, int batch,
                       int total_q, int total_kv, int total_k, int max_q, int max_kv, int max_k, int forced_tail) {
  unsigned e = 0;
  for (int b = 0; b < batch; ++b)
    e |= dllm_rule_sequence(cu_q, cu_kv, cu_k, mode, b, batch, total_q, total_kv, total_k, max_q, max_kv, max_k, forced_tail);
  return e;
}
int owner(const int32_t* cu_k, int batch, int t) { return dllm_rule_owner(cu_k, batch, t); }
unsigned all_indices(const int32_t* idx, int heads, const int32_t* cu_kv, const int32_t* cu_k, const uint8_t* mode,
                     int batch, int total_k) {
  unsigned e = 0;
  for (int h = 0; h < heads; ++h)
    for (int t = 0; t < total_k; ++t)
      e |= dllm_rule_index(idx[(long)h * total_k + t], cu_kv, mode, dllm_rule_owner(cu_k, batch, t));
  return e;
}
'''


@pytest.fixture(scope="module")
def rules(tmp_path_factory):
    d = tmp_path_factory.mktemp("rules")
    src = d / "harness.c"
    src.write_text(HARNESS)
    lib = d / "librules.so"
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Werror", "-shared", "-fPIC", "-I", CSRC, str(src), "-o", str(lib)],
                   check=True)
    return ctypes.CDLL(str(lib))


def i32(x):
    return np.ascontiguousarray(x, dtype=np.int32)


def p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def seq_errors(L, cu_q, cu_kv, cu_k, mode=None, forced_tail=0, max_q=None, max_kv=None, max_k=None, totals=None):
    cu_q, cu_kv = i32(cu_q), i32(cu_kv)
    cu_k = None if cu_k is None else i32(cu_k)
    mode = None if mode is None else np.ascontiguousarray(mode, dtype=np.uint8)
    batch = len(cu_q) - 1
    tq, tkv, tk = totals or (int(cu_q[-1]), int(cu_kv[-1]), 0 if cu_k is None else int(cu_k[-1]))
    return L.all_sequences(p(cu_q), p(cu_kv), p(cu_k), p(mode), batch, tq, tkv, tk,
                           max_q if max_q is not None else int(np.diff(cu_q).max()),
                           max_kv if max_kv is not None else int(np.diff(cu_kv).max()),
                           max_k if max_k is not None else (0 if cu_k is None else max(0, int(np.diff(cu_k).max()))),
                           forced_tail)


def test_valid_batches_pass(rules):
    assert seq_errors(rules, [0, 32, 64, 64], [0, 100, 400, 400], [0, 100, 150, 150]) == 0
    assert seq_errors(rules, [0, 32], [0, 100], None) == 0
    assert seq_errors(rules, [0, 5, 37], [0, 10, 500], [0, 10, 60], forced_tail=10) == 0
    # a dense sequence may carry any count in cu_k: its list is never read
    assert seq_errors(rules, [0, 32, 64], [0, 100, 200], [0, 50, 250], mode=[0, 1], max_k=200) == 0


@pytest.mark.parametrize("kw,bit", [
    (dict(cu_q=[1, 32, 64]), CU_Q), (dict(cu_q=[0, 40, 30], totals=(30, 300, 60)), CU_Q), (dict(max_q=31), CU_Q),
    (dict(totals=(65, 300, 60)), CU_Q),
    (dict(cu_kv=[0, 200, 100], totals=(64, 300, 60)), CU_KV), (dict(max_kv=199), CU_KV), (dict(totals=(64, 301, 60)), CU_KV),
    (dict(cu_k=[0, 50, 40], totals=(64, 300, 40)), CU_K), (dict(max_k=29), CU_K), (dict(totals=(64, 300, 61)), CU_K),
    (dict(cu_k=[2, 30, 60]), CU_K),
    (dict(cu_k=[0, 101, 131], max_k=200), K_OVER_L),
    (dict(forced_tail=31), FORCED),
])
def test_each_violation_sets_its_bit(rules, kw, bit):
    args = dict(cu_q=[0, 32, 64], cu_kv=[0, 100, 300], cu_k=[0, 30, 60])
    args.update(kw)
    e = seq_errors(rules, **args)
    assert e & bit, (kw, e)


def test_forced_tail_applies_only_where_rows_are_kept_and_lists_are_read(rules):
    assert seq_errors(rules, [0, 32, 64], [0, 100, 300], [0, 0, 40], forced_tail=8) == 0          # k_b == 0: skipped
    assert seq_errors(rules, [0, 32, 64], [0, 100, 300], [0, 4, 44], forced_tail=8) & FORCED        # k_b < tail
    assert seq_errors(rules, [0, 32, 64], [0, 5, 305], [0, 5, 45], forced_tail=8) & FORCED          # L_b < tail
    assert seq_errors(rules, [0, 32, 64], [0, 5, 305], [0, 5, 45], mode=[1, 0], forced_tail=8) == 0  # dense: not read


def test_owner_is_the_sequence_holding_the_list_position(rules):
    rng = np.random.default_rng(3)
    for _ in range(20):
        keep = rng.integers(0, 9, size=rng.integers(1, 40))
        cu_k = i32(np.concatenate([[0], np.cumsum(keep)]))
        for t in range(int(cu_k[-1])):
            b = rules.owner(p(cu_k), len(keep), t)
            assert cu_k[b] <= t < cu_k[b + 1]
            assert b == np.searchsorted(cu_k, t, side="right") - 1


def test_index_rule(rules):
    cu_kv, cu_k = i32([0, 10, 30]), i32([0, 3, 7])
    good = i32([[0, 9, 5, 19, 0, 1, 2], [1, 2, 3, 4, 5, 6, 7]])
    assert rules.all_indices(p(good), 2, p(cu_kv), p(cu_k), None, 2, 7) == 0
    for h, t, bad in ((0, 1, 10), (1, 0, -1), (0, 6, 20), (1, 3, 1 << 30)):
        idx = good.copy()
        idx[h, t] = bad
        assert rules.all_indices(p(idx), 2, p(cu_kv), p(cu_k), None, 2, 7) == IDX
        mode = np.array([t < 3, t >= 3], np.uint8)      # the owning sequence flagged dense: its list is not read
        assert rules.all_indices(p(idx), 2, p(cu_kv), p(cu_k), p(mode), 2, 7) == 0
