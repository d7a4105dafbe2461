// Packing of the kept rows (Section 4.5, "Decoupling Logical Sparsity from Physical Layout"): at
// Refresh time every head's kept K and V rows are copied, in list order, into dense buffers of shape
// [n_q_heads, total_k, head_dim], so that the Reuse steps that follow read them sequentially.
//
// Pure data movement, bound by HBM: per kept (head, row) pair one K row and one V row are gathered
// (16-byte non-temporal loads, a row's chunks in neighbouring lanes) and written out contiguously.
// A workgroup takes a run of consecutive list positions of one (sequence, head), so its stores cover
// one contiguous span (written with non-temporal stores: the packed rows are not read again soon);
// several rows per lane group are in flight before the first store.
#include "common.h"

namespace dllm {

constexpr int kPackThreads = 256;
#ifndef DLLM_PACK_INFLIGHT
#define DLLM_PACK_INFLIGHT 4
#endif
constexpr int kPackInFlight = DLLM_PACK_INFLIGHT;   // rows per lane group gathered before any is stored

// CH: 16-byte chunks per row (head_dim * element size / 16)
template <int CH>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(
    const char* __restrict__ k, const char* __restrict__ v, const int32_t* __restrict__ cu_kv,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cu_k, int32_t total_k, char* __restrict__ kp,
    char* __restrict__ vp, int es, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int ROWS = kPackThreads / CH;                 // rows per pass of the workgroup
  constexpr int ROWS_PER_WG = ROWS * kPackInFlight;
  const int h = blockIdx.y, b = blockIdx.z;
  const int ko0 = cu_k[b], kb = cu_k[b + 1] - ko0;
  const int t0 = blockIdx.x * ROWS_PER_WG;
  if (t0 >= kb) return;
  const int kv0 = cu_kv[b];
  const int g = h / s.group;
  const int sub = threadIdx.x / CH, c = threadIdx.x % CH;
  const int32_t* __restrict__ rows = idx + int64_t(h) * total_k + ko0;
  const int64_t pitch = s.kv_tok * es;
  const char* kbase = k + (int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head) * es + c * 16;
  const char* vbase = v + (int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head) * es + c * 16;
  const int64_t out_row = int64_t(CH) * 16;
  char* kout = kp + (int64_t(h) * total_k + ko0) * out_row + c * 16;
  char* vout = vp + (int64_t(h) * total_k + ko0) * out_row + c * 16;

  v4u kr[kPackInFlight], vr[kPackInFlight];
#pragma unroll
  for (int p = 0; p < kPackInFlight; ++p) {
    const int t = min(t0 + p * ROWS + sub, kb - 1);   // past the end: the last row again, never stored
    const int64_t r = rows[t];
    kr[p] = load_once(kbase + r * pitch);
    vr[p] = load_once(vbase + r * pitch);
  }
#pragma unroll
  for (int p = 0; p < kPackInFlight; ++p) {
    const int t = t0 + p * ROWS + sub;
    if (t < kb) {
      __builtin_nontemporal_store(kr[p], reinterpret_cast<v4u*>(kout + t * out_row));
      __builtin_nontemporal_store(vr[p], reinterpret_cast<v4u*>(vout + t * out_row));
    }
  }
}

hipError_t launch_pack(const Shape& s, dllm_dtype dt, const void* k, const void* v, const int32_t* cu_kv,
                       const int32_t* idx, const int32_t* cu_k, int32_t total_k, int32_t max_k, void* kp, void* vp,
                       hipStream_t st) {
  const int es = dt == DLLM_F32 ? 4 : 2;
  const int ch = s.d * es / 16;   // 8, 16 or 32
  const int rows_per_wg = kPackThreads / ch * kPackInFlight;
  dim3 grid((max_k + rows_per_wg - 1) / rows_per_wg, s.hq, s.batch);
  const char *kc = static_cast<const char*>(k), *vc = static_cast<const char*>(v);
  char *kpc = static_cast<char*>(kp), *vpc = static_cast<char*>(vp);
  if (ch == 8)
    pack_kernel<8><<<grid, kPackThreads, 0, st>>>(kc, vc, cu_kv, idx, cu_k, total_k, kpc, vpc, es, s DLLM_CHECK_PASS);
  else if (ch == 16)
    pack_kernel<16><<<grid, kPackThreads, 0, st>>>(kc, vc, cu_kv, idx, cu_k, total_k, kpc, vpc, es, s DLLM_CHECK_PASS);
  else
    pack_kernel<32><<<grid, kPackThreads, 0, st>>>(kc, vc, cu_kv, idx, cu_k, total_k, kpc, vpc, es, s DLLM_CHECK_PASS);
  return hipGetLastError();
}

}  // namespace dllm
