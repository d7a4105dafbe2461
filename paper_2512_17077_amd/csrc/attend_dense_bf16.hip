// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput.
//
// A workgroup of four waves owns 128 query rows of one (sequence, head); each wave keeps its 32
// queries as the B operand in registers for the whole pass.  K/V tiles of 64 keys are loaded by all
// 256 threads (16-byte loads, whole rows per 16 lanes), prefetched one tile ahead into registers,
// and staged in LDS with an XOR swizzle.  Per tile and wave:
//   S^T (64 keys x 32 queries) = K_tile * Q^T          v_mfma_f32_32x32x16_bf16, A from LDS
//   online softmax per query column, base 2
//   O^T (D x 32 queries)      += V_tile^T * P^T         P^T = S^T accumulators re-used in place
#include "common.h"

namespace dllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kDenseWaves = 4;
constexpr int kDenseQ = kDenseWaves * 32;   // query rows per workgroup
constexpr int kDenseK = 64;                 // keys per tile
constexpr float kLog2eD = 1.4426950408889634f;

template <int CH>
__device__ __forceinline__ int swz_d(int row) {
  constexpr int rows_per_line = CH >= 16 ? 1 : 16 / CH;
  return (row / rows_per_line) & (CH - 1);
}

// which: 1 = only sequences flagged dense in seq_mode; 2 = every sequence
template <int D>
__global__ __launch_bounds__(kDenseWaves * 64) void attend_dense_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const uint8_t* __restrict__ seq_mode,
    int which, uint16_t* __restrict__ o, Shape s) {
  constexpr int CH = D / 8;
  constexpr int NLD = kDenseK * CH / (kDenseWaves * 64);   // 16-byte loads per thread, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  constexpr int NKB = kDenseK / 32;

  __shared__ uint4 ktile[kDenseK * CH];
  __shared__ uint4 vtile[kDenseK * CH];

  const int b = blockIdx.z, h = blockIdx.y;
  if (which == 1 && !(seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE)) return;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  const int qbase = blockIdx.x * kDenseQ;
  if (qbase >= nq) return;
  const int kv0 = cu_kv[b], L = cu_kv[b + 1] - kv0;
  const int g = h / s.group;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int qi = qbase + wave * 32 + col;

  if (L == 0) {   // nothing to attend to: zeros
    for (int e = tid; e < kDenseQ * D; e += kDenseWaves * 64) {
      const int r = qbase + e / D;
      if (r < nq) o[(int64_t(q0 + r) * s.hq + h) * D + e % D] = 0;
    }
    return;
  }

  uint4 qreg[NT];
  {
    const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      qreg[t] = make_uint4(0, 0, 0, 0);
      if (qi < nq) qreg[t] = *reinterpret_cast<const uint4*>(qp + 16 * t + 8 * hf);
    }
  }
  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const int64_t pitch = s.kv_tok * 2;
  const float zscale = s.scale * kLog2eD;
  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(vtile);

  float m = -INFINITY, l = 0.0f;
  f32x16 acc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[db][i] = 0.0f;

  uint4 kr[NLD], vr[NLD];
  auto fetch = [&](int t0) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int f = i * (kDenseWaves * 64) + tid, row = f / CH, c = f % CH;
      kr[i] = make_uint4(0, 0, 0, 0);
      vr[i] = make_uint4(0, 0, 0, 0);
      if (t0 + row < L) {
        kr[i] = *reinterpret_cast<const uint4*>(kbase + (t0 + row) * pitch + c * 16);
        vr[i] = *reinterpret_cast<const uint4*>(vbase + (t0 + row) * pitch + c * 16);
      }
    }
  };

  fetch(0);
  for (int t0 = 0; t0 < L; t0 += kDenseK) {
    __syncthreads();   // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int f = i * (kDenseWaves * 64) + tid, row = f / CH, c = f % CH;
      ktile[row * CH + (c ^ swz_d<CH>(row))] = kr[i];
      vtile[row * CH + (c ^ swz_d<CH>(row))] = vr[i];
    }
    if (t0 + kDenseK < L) fetch(t0 + kDenseK);
    __syncthreads();

    f32x16 st[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) st[kb][i] = 0.0f;
      const int key = kb * 32 + col;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const uint4 a = ktile[key * CH + ((2 * t + hf) ^ swz_d<CH>(key))];
        st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                         __builtin_bit_cast(bf16x8, qreg[t]), st[kb], 0, 0, 0);
      }
    }
    const int nvalid = L - t0;
    float mloc = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kb * 32 + 8 * (i / 4) + 4 * hf + (i % 4);
        st[kb][i] = key < nvalid ? st[kb][i] * zscale : -INFINITY;
        mloc = fmaxf(mloc, st[kb][i]);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m, mloc);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    float psum = 0.0f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        st[kb][i] = __builtin_amdgcn_exp2f(st[kb][i] - m_new);
        psum += st[kb][i];
      }
    l = l * alpha + psum;
    m = m_new;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][i] *= alpha;

#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        uint4 pb;
        pb.x = pack_bf16x2(st[kb][8 * u + 0], st[kb][8 * u + 1]);
        pb.y = pack_bf16x2(st[kb][8 * u + 2], st[kb][8 * u + 3]);
        pb.z = pack_bf16x2(st[kb][8 * u + 4], st[kb][8 * u + 5]);
        pb.w = pack_bf16x2(st[kb][8 * u + 6], st[kb][8 * u + 7]);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int d = db * 32 + col;
          uint32_t w[4];
#pragma unroll
          for (int sp = 0; sp < 4; ++sp) {
            const int s0 = 2 * sp, s1 = 2 * sp + 1;
            const int key0 = kb * 32 + 16 * u + 8 * (s0 / 4) + 4 * hf + (s0 % 4);
            const int key1 = kb * 32 + 16 * u + 8 * (s1 / 4) + 4 * hf + (s1 % 4);
            const uint32_t lo = vt16[(key0 * CH + ((d >> 3) ^ swz_d<CH>(key0))) * 8 + (d & 7)];
            const uint32_t hi = vt16[(key1 * CH + ((d >> 3) ^ swz_d<CH>(key1))) * 8 + (d & 7)];
            w[sp] = lo | (hi << 16);
          }
          const uint4 a = make_uint4(w[0], w[1], w[2], w[3]);
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                          __builtin_bit_cast(bf16x8, pb), acc[db], 0, 0, 0);
        }
      }
  }

  l += __shfl_xor(l, 32);
  if (qi < nq) {
    const float inv = 1.0f / l;
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      uint16_t* op = o + (int64_t(q0 + qi) * s.hq + h) * D + db * 32 + 4 * hf;
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        uint2 w2;
        w2.x = pack_bf16x2(acc[db][4 * i4 + 0] * inv, acc[db][4 * i4 + 1] * inv);
        w2.y = pack_bf16x2(acc[db][4 * i4 + 2] * inv, acc[db][4 * i4 + 3] * inv);
        *reinterpret_cast<uint2*>(op + 8 * i4) = w2;
      }
    }
  }
}

hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st) {
  dim3 grid((s.max_q + kDenseQ - 1) / kDenseQ, s.hq, s.batch);
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  if (s.d == 128)
    attend_dense_bf16_kernel<128><<<grid, kDenseWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, seq_mode, which,
                                                                    static_cast<uint16_t*>(o), s);
  else
    attend_dense_bf16_kernel<64><<<grid, kDenseWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, seq_mode, which,
                                                                   static_cast<uint16_t*>(o), s);
  return hipGetLastError();
}

}  // namespace dllm
