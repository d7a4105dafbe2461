// Internal declarations shared by the HIP translation units of libdllm_hcsa (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dllm_hcsa.h"

namespace dllm {

constexpr int kWave = 64;

// 16 bytes as a native vector: loads and stores of it stay plain vector moves in every address
// space, so register tiles built from it are always promoted out of private memory
typedef __attribute__((ext_vector_type(4))) unsigned int v4u;
typedef __attribute__((ext_vector_type(2))) unsigned int v2u;

// Element strides and sizes every kernel needs; built once per call on the host.
struct Shape {
  int32_t batch, hq, hkv, group, d;
  int64_t q_tok, q_head, kv_tok, kv_head;  // element strides
  int32_t total_q, total_kv, max_q, max_kv;
  float scale;
};

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// ---- selection (select_kernels.hip)
struct SelectPlan {
  size_t off_scores, off_summed, bytes;
};
SelectPlan plan_select(const Shape& s);
hipError_t launch_select(const Shape& s, dllm_dtype dt, const void* q, const void* k, const int32_t* cu_q,
                         const int32_t* cu_kv, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                         int32_t pool_w, int32_t forced_tail, int32_t head_sum, int32_t* idx_out, void* ws,
                         hipStream_t st);

// the form a selection call of this shape takes under the current setting (ONE_LAUNCH or TWO_LAUNCHES)
int32_t select_form_of(const Shape& s, dllm_dtype dt, int32_t pool_w, int32_t head_sum);
int32_t set_select_form(int32_t form);   // DLLM_SELECT_FORM_*; returns the previous one, -1 if form is not one of them

// ---- packing of the kept rows (pack_kernels.hip)
hipError_t launch_pack(const Shape& s, dllm_dtype dt, const void* k, const void* v, const int32_t* cu_kv,
                       const int32_t* idx, const int32_t* cu_k, int32_t total_k, int32_t max_k, void* kp, void* vp,
                       hipStream_t st);

// ---- attention over kept rows / all rows (attend_*.hip)
struct AttendPlan {
  int32_t chunk_rows;  // kept rows one workgroup walks
  int32_t n_chunks;    // upper bound on chunks per (sequence, head)
  int32_t max_k;       // the caller's bound on kept rows per (sequence, head)
  size_t off_po, off_pm, off_pl, bytes;
};
AttendPlan plan_attend(const Shape& s, dllm_dtype dt, int32_t max_k);

// `which` selects the sequences a launch works on: 0 = those not flagged dense (all, if seq_mode
// is NULL), attended over their kept rows; 1 = those flagged dense; 2 = every sequence, as dense.
hipError_t launch_attend_f32(const Shape& s, const void* q, const void* k, const void* v, const int32_t* cu_q,
                             const int32_t* cu_kv, const int32_t* idx, const int32_t* cu_k, int32_t total_k,
                             const uint8_t* seq_mode, int which, void* o, hipStream_t st);
hipError_t launch_zero_sparse_outputs(const Shape& s, dllm_dtype dt, const int32_t* cu_q, const uint8_t* seq_mode,
                                      void* o, hipStream_t st);
hipError_t launch_attend_sparse_bf16(const Shape& s, const AttendPlan& p, const void* q, const void* k,
                                     const void* v, const int32_t* cu_q, const int32_t* cu_kv, const int32_t* idx,
                                     const int32_t* cu_k, int32_t total_k, const uint8_t* seq_mode, void* o,
                                     void* ws, hipStream_t st);
hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st);

// ---- optional device-side precondition checks (checks.hip; built with -DDLLM_CHECK_PRECONDITIONS)
// In that build every entry point first runs validators over the offset arrays and the index lists, which
// set bits in an error word, and every kernel takes that word's address as its last argument and returns
// at once if it is not zero: a violating input is reported and nothing is read or written through it.
#ifdef DLLM_CHECK_PRECONDITIONS
#define DLLM_CHECK_PARAM , const uint32_t* __restrict__ check_word
#define DLLM_CHECK_PASS , dllm::check_word()
#define DLLM_CHECK_EXIT() \
  if (*check_word != 0) return
uint32_t* check_word();   // device address of the current GPU's error word; NULL if it cannot be had
#else
#define DLLM_CHECK_PARAM
#define DLLM_CHECK_PASS
#define DLLM_CHECK_EXIT()
#endif
// Runs the validators (a no-op in the release build).  cu_k, idx and seq_mode may be NULL.
hipError_t validate_inputs(const Shape& s, const int32_t* cu_q, const int32_t* cu_kv, const int32_t* cu_k,
                           const int32_t* idx, const uint8_t* seq_mode, int32_t total_k, int32_t max_k,
                           int32_t forced_tail, hipStream_t st);

// ---- device helpers
// 16-byte load of data that is read once per launch (K/V rows streamed or gathered from HBM): the
// non-temporal hint keeps such lines from displacing reusable data in the caches, which measurably
// raises the HBM read rate on MI355X.
#ifndef DLLM_STREAM_NT
#define DLLM_STREAM_NT 1
#endif
__device__ __forceinline__ v4u load_once(const void* p) {
#if DLLM_STREAM_NT
  return __builtin_nontemporal_load(static_cast<const v4u*>(p));
#else
  return *static_cast<const v4u*>(p);
#endif
}
// Inclusive prefix sum over the 64 lanes of a wave (all lanes active) through the data-parallel
// primitives: shifts by 1, 2, 4, 8 within each row of 16 lanes, then the last lane of row 0 (2) is
// added to row 1 (3), then lane 31 to rows 2 and 3.  A lane without a source adds zero.
template <int Ctrl, int RowMask>
__device__ __forceinline__ uint32_t dpp_add(uint32_t x) {
  return x + uint32_t(__builtin_amdgcn_update_dpp(0, int(x), Ctrl, RowMask, 0xf, false));
}
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x) {
  x = dpp_add<0x111, 0xf>(x);   // row_shr:1
  x = dpp_add<0x112, 0xf>(x);   // row_shr:2
  x = dpp_add<0x114, 0xf>(x);   // row_shr:4
  x = dpp_add<0x118, 0xf>(x);   // row_shr:8
  x = dpp_add<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (inputs are finite here)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

}  // namespace dllm
