/* The rules the optional precondition checks apply, as plain functions with no GPU construct in them, so
 * that the validators of the checked build and a CPU test share one text.  Offsets are int32 prefix sums
 * of [batch+1] entries; an error is a set of DLLM_CHECK_* bits (dllm_hcsa.h). */
#ifndef DLLM_PRECONDITION_RULES_H
#define DLLM_PRECONDITION_RULES_H
#include <stdint.h>

#ifdef __HIPCC__
#define DLLM_RULE __host__ __device__ static inline
#else
#define DLLM_RULE static inline
#endif

#define DLLM_RULE_CU_Q 1u        /* cu_q does not start at 0, decreases, exceeds max_q per sequence, or does not end at total_q */
#define DLLM_RULE_CU_KV 2u       /* the same for cu_kv, max_kv, total_kv */
#define DLLM_RULE_CU_K 4u        /* the same for cu_k, max_k, total_k */
#define DLLM_RULE_K_OVER_L 8u    /* a sparse sequence keeps more rows than it has */
#define DLLM_RULE_FORCED 16u     /* a sequence with kept rows keeps, or has, fewer than forced_tail */
#define DLLM_RULE_IDX 32u        /* an index outside [0, L_b) */

/* one prefix-sum array at position b (0 <= b < batch): the step b -> b+1, plus the two ends */
DLLM_RULE uint32_t dllm_rule_prefix(const int32_t* cu, int32_t b, int32_t batch, int32_t total, int32_t max_len,
                                    uint32_t bit) {
  uint32_t e = 0;
  if (b == 0 && cu[0] != 0) e |= bit;
  const int32_t lo = cu[b], hi = cu[b + 1];
  if (hi < lo || hi - lo > max_len) e |= bit;
  if (b == batch - 1 && hi != total) e |= bit;
  return e;
}

/* everything about sequence b that needs no index list; cu_k may be NULL (then nothing is kept anywhere) */
DLLM_RULE uint32_t dllm_rule_sequence(const int32_t* cu_q, const int32_t* cu_kv, const int32_t* cu_k,
                                      const uint8_t* seq_mode, int32_t b, int32_t batch, int32_t total_q,
                                      int32_t total_kv, int32_t total_k, int32_t max_q, int32_t max_kv, int32_t max_k,
                                      int32_t forced_tail) {
  uint32_t e = dllm_rule_prefix(cu_q, b, batch, total_q, max_q, DLLM_RULE_CU_Q) |
               dllm_rule_prefix(cu_kv, b, batch, total_kv, max_kv, DLLM_RULE_CU_KV);
  if (cu_k != 0) {
    e |= dllm_rule_prefix(cu_k, b, batch, total_k, max_k, DLLM_RULE_CU_K);
    const int sparse = seq_mode == 0 || seq_mode[b] == 0;
    const int64_t kb = (int64_t)cu_k[b + 1] - cu_k[b], L = (int64_t)cu_kv[b + 1] - cu_kv[b];
    if (sparse && kb > L) e |= DLLM_RULE_K_OVER_L;
    if (sparse && kb > 0 && (kb < forced_tail || L < forced_tail)) e |= DLLM_RULE_FORCED;
  }
  return e;
}

/* the sequence that owns list position t (0 <= t < total_k): largest b with cu_k[b] <= t.  Only called once
 * cu_k has passed dllm_rule_prefix everywhere (0 at the start, non-decreasing, total_k at the end). */
DLLM_RULE int32_t dllm_rule_owner(const int32_t* cu_k, int32_t batch, int32_t t) {
  int32_t lo = 0, hi = batch;   /* invariant: cu_k[lo] <= t < cu_k[hi] */
  while (hi - lo > 1) {
    const int32_t mid = lo + (hi - lo) / 2;
    if (cu_k[mid] <= t) lo = mid;
    else hi = mid;
  }
  return lo;
}

/* one entry of one head's index list */
DLLM_RULE uint32_t dllm_rule_index(int32_t row, const int32_t* cu_kv, const uint8_t* seq_mode, int32_t b) {
  if (seq_mode != 0 && seq_mode[b] != 0) return 0;   /* dense sequences do not read their lists */
  const int32_t L = cu_kv[b + 1] - cu_kv[b];
  return (row < 0 || row >= L) ? DLLM_RULE_IDX : 0u;
}

#endif
