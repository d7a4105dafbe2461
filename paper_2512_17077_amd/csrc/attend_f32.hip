// fp32 attention (Section 2.3, Eq. 3 and Eq. 4) with plain fp32 vector arithmetic.
//
// fp32 inputs are held to 1e-5 absolute, which rules out the reduced-precision matrix paths, and
// the fp32 workload is a few hundred kilobytes, so this kernel aims at correctness and full
// coalescing of the V reads, not at a roofline: one wave per query row, lanes over keys for the
// logits, lanes over head_dim for the weighted sum, online softmax in between.
#include "common.h"

namespace dllm {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// which: 0 = sequences flagged sparse (or all, if seq_mode is NULL); 1 = sequences flagged dense;
//        2 = every sequence, treated as dense
template <int D>
__global__ __launch_bounds__(256) void attend_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cu_k, int32_t total_k, const uint8_t* __restrict__ seq_mode, int which,
    float* __restrict__ o, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  const int b = blockIdx.z, h = blockIdx.y;
  const bool flagged_dense = seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE;
  if (which == 0 && flagged_dense) return;
  if (which == 1 && !flagged_dense) return;
  const bool dense = which != 0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  const int i = blockIdx.x * 4 + wave;
  if (i >= nq) return;
  const int kv0 = cu_kv[b], L = cu_kv[b + 1] - kv0;
  const int o0 = dense ? 0 : cu_k[b];
  const int n = dense ? L : cu_k[b + 1] - o0;
  const int g = h / s.group;
  // a NULL idx stands for the identity lists (kept rows 0 .. k_b-1): then a row is its own list position
  const bool direct = dense || idx == nullptr;
  const int32_t* __restrict__ rows = direct ? nullptr : idx + int64_t(h) * total_k + o0;

  float qr[D];
  const float* qp = q + int64_t(q0 + i) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
  for (int d = 0; d < D; d += 4) {
    const float4 x = *reinterpret_cast<const float4*>(qp + d);
    qr[d] = x.x; qr[d + 1] = x.y; qr[d + 2] = x.z; qr[d + 3] = x.w;
  }
  const float* kb = k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head;
  const float* vb = v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head;

  constexpr int NO = D / 64;
  float m = -INFINITY, l = 0.0f, acc[NO];
#pragma unroll
  for (int t = 0; t < NO; ++t) acc[t] = 0.0f;

  for (int t0 = 0; t0 < n; t0 += 64) {
    const int t = t0 + lane;
    const bool ok = t < n;
    const int r = ok ? (direct ? t : rows[t]) : 0;
    float z = -INFINITY;
    if (ok) {
      const float* kr = kb + int64_t(r) * s.kv_tok;
      float dot = 0.0f;
#pragma unroll
      for (int d = 0; d < D; d += 4) {
        const float4 x = *reinterpret_cast<const float4*>(kr + d);
        dot = fmaf(qr[d], x.x, dot);
        dot = fmaf(qr[d + 1], x.y, dot);
        dot = fmaf(qr[d + 2], x.z, dot);
        dot = fmaf(qr[d + 3], x.w, dot);
      }
      z = dot * s.scale;
    }
    const float m_new = fmaxf(m, wave_max(z));
    const float alpha = expf(m - m_new);       // first tile: exp(-inf) = 0
    const float p = ok ? expf(z - m_new) : 0.0f;
    l = l * alpha + wave_sum(p);
#pragma unroll
    for (int u = 0; u < NO; ++u) acc[u] *= alpha;
    const int cnt = min(64, n - t0);
    for (int tt = 0; tt < cnt; ++tt) {
      const float pt = __shfl(p, tt);
      const int rt = __shfl(r, tt);
      const float* vr = vb + int64_t(rt) * s.kv_tok;
#pragma unroll
      for (int u = 0; u < NO; ++u) acc[u] = fmaf(pt, vr[lane + 64 * u], acc[u]);
    }
    m = m_new;
  }
  float* op = o + (int64_t(q0 + i) * s.hq + h) * D;
  const float inv = n > 0 ? 1.0f / l : 0.0f;
#pragma unroll
  for (int u = 0; u < NO; ++u) op[lane + 64 * u] = acc[u] * inv;
}

// o rows of the sequences not flagged dense := 0 (what attention over an empty kept list is defined as);
// used when a call passes no cu_k at all.  es: element bytes.
__global__ __launch_bounds__(256) void zero_sparse_outputs_kernel(const int32_t* __restrict__ cu_q,
                                                                  const uint8_t* __restrict__ seq_mode,
                                                                  char* __restrict__ o, int row_bytes DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  const int b = blockIdx.y;
  if (seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE) return;
  const int64_t lo = int64_t(cu_q[b]) * row_bytes, hi = int64_t(cu_q[b + 1]) * row_bytes;   // multiples of 16
  for (int64_t e = lo + (int64_t(blockIdx.x) * 256 + threadIdx.x) * 16; e < hi; e += int64_t(gridDim.x) * 256 * 16)
    *reinterpret_cast<v4u*>(o + e) = v4u{0u, 0u, 0u, 0u};
}

hipError_t launch_zero_sparse_outputs(const Shape& s, dllm_dtype dt, const int32_t* cu_q, const uint8_t* seq_mode,
                                      void* o, hipStream_t st) {
  if (s.max_q == 0) return hipSuccess;
  const int row_bytes = s.hq * s.d * (dt == DLLM_F32 ? 4 : 2);
  const int64_t per_seq = int64_t(s.max_q) * row_bytes / (256 * 16) + 1;
  zero_sparse_outputs_kernel<<<dim3(unsigned(per_seq < 64 ? per_seq : 64), s.batch), 256, 0, st>>>(
      cu_q, seq_mode, static_cast<char*>(o), row_bytes DLLM_CHECK_PASS);
  return hipGetLastError();
}

hipError_t launch_attend_f32(const Shape& s, const void* q, const void* k, const void* v, const int32_t* cu_q,
                             const int32_t* cu_kv, const int32_t* idx, const int32_t* cu_k, int32_t total_k,
                             const uint8_t* seq_mode, int which, void* o, hipStream_t st) {
  if (s.max_q == 0) return hipSuccess;   // no sequence has a query: nothing to write
  dim3 grid((s.max_q + 3) / 4, s.hq, s.batch);
  const float *qf = static_cast<const float*>(q), *kf = static_cast<const float*>(k),
              *vf = static_cast<const float*>(v);
  if (s.d == 128)
    attend_f32_kernel<128><<<grid, 256, 0, st>>>(qf, kf, vf, cu_q, cu_kv, idx, cu_k, total_k, seq_mode, which,
                                                static_cast<float*>(o), s DLLM_CHECK_PASS);
  else
    attend_f32_kernel<64><<<grid, 256, 0, st>>>(qf, kf, vf, cu_q, cu_kv, idx, cu_k, total_k, seq_mode, which,
                                               static_cast<float*>(o), s DLLM_CHECK_PASS);
  return hipGetLastError();
}

}  // namespace dllm
