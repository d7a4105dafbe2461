// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput,
// with the softmax's exponentials on the vector ALUs as the co-bottleneck.
//
// A workgroup of four waves owns 256 query rows of one (sequence, head); each wave keeps its 64
// queries (two 32-column blocks) as B operands in registers for the whole pass, so every K / V^T
// operand fetched from LDS feeds two MFMAs.  K/V tiles of 64 keys are loaded by all 256 threads
// (16-byte loads, whole rows per 16 lanes), prefetched one tile ahead into registers and staged in
// a double-buffered, XOR-swizzled LDS tile: one barrier per tile.  Per tile and wave:
//   S^T (64 keys x 64 queries) = K_tile * Q^T     32 MFMAs, A by ds_read_b128
//   softmax, base 2, with a lazily updated running maximum (rescale O only when the maximum of some
//            query of the wave grew by more than 2^8; until then probabilities may exceed 1)
//   O^T (D x 64 queries)     += V_tile^T * P^T    32 MFMAs, A by ds_read_b64_tr_b16, B = S^T in place
#include "attn_tile.h"

namespace dllm {

constexpr int kDenseK = 64;                         // keys per tile
constexpr float kLazyStep = 8.0f;                   // log2 of the growth that forces a rescale

// which: 1 = only sequences flagged dense in seq_mode; 2 = every sequence
// NQB: 32-query blocks per wave; WAVES: waves per workgroup (WAVES * NQB * 32 query rows)
template <int D, int NQB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void attend_dense_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const uint8_t* __restrict__ seq_mode,
    int which, uint16_t* __restrict__ o, Shape s) {
  constexpr int CH = D / 8;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kDenseK * ROWB;
  constexpr int kDenseWaves = WAVES;
  constexpr int kDenseQ = WAVES * 32 * NQB;
  constexpr int NLD = kDenseK * CH / (kDenseWaves * 64);   // 16-byte loads per thread, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  constexpr int NKB = kDenseK / 32;

  __shared__ __attribute__((aligned(16))) char smem[2][2][TILEB];   // [buffer][K, V]

  const int b = blockIdx.z, h = blockIdx.y;
  if (which == 1 && !(seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE)) return;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  const int qbase = blockIdx.x * kDenseQ;
  if (qbase >= nq) return;
  const int kv0 = cu_kv[b], L = cu_kv[b + 1] - kv0;
  const int g = h / s.group;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 31, hf = lane >> 5;

  if (L == 0) {   // nothing to attend to: zeros
    for (int e = tid; e < kDenseQ * D; e += kDenseWaves * 64) {
      const int r = qbase + e / D;
      if (r < nq) o[(int64_t(q0 + r) * s.hq + h) * D + e % D] = 0;
    }
    return;
  }

  // Q^T operands: lane (col = query, hf) holds Q[query][16t + 8hf .. +8) for every step t
  v4u qreg[NQB][NT];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      qreg[qb][t] = v4u{0u, 0u, 0u, 0u};
      if (qi < nq) qreg[qb][t] = *reinterpret_cast<const v4u*>(qp + 16 * t + 8 * hf);
    }
  }
  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const int64_t pitch = s.kv_tok * 2;
  const float zscale = s.scale * kLog2e;

  // per-lane LDS offsets (tile-relative)
  KAddr<D> ka;
  ka.init(lane);
  VtAddr<D> vt;
  vt.init(lane);
  int woff[NLD];   // where this thread's loaded chunks go
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * (kDenseWaves * 64) + tid;
    woff[i] = tile_off<D>(f / CH, f % CH);
  }

  float m_used[NQB], lsum[NQB];
  f32x16 acc[NQB][NDB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_used[qb] = -INFINITY;
    lsum[qb] = 0.0f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[qb][db][i] = 0.0f;
  }

  v4u kr[NLD], vr[NLD];
  auto fetch = [&](int t0) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int f = i * (kDenseWaves * 64) + tid, row = f / CH, c = f % CH;
      kr[i] = v4u{0u, 0u, 0u, 0u};
      vr[i] = v4u{0u, 0u, 0u, 0u};
      if (t0 + row < L) {
        kr[i] = *reinterpret_cast<const v4u*>(kbase + (t0 + row) * pitch + c * 16);
        vr[i] = *reinterpret_cast<const v4u*>(vbase + (t0 + row) * pitch + c * 16);
      }
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      *reinterpret_cast<v4u*>(&smem[buf][0][woff[i]]) = kr[i];
      *reinterpret_cast<v4u*>(&smem[buf][1][woff[i]]) = vr[i];
    }
  };

  auto tile = [&](const int buf, const int t0) {
    const char* kt = smem[buf][0];
    const char* vtile = smem[buf][1];
    const int nvalid = L - t0;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {   // 32 keys at a time keeps S^T at 16 registers per query block
      f32x16 st[NQB];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) st[qb][i] = 0.0f;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const v4u a = *reinterpret_cast<const v4u*>(kt + ka.off(t) + kb * 32 * ROWB);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) st[qb] = mfma_bf16(a, qreg[qb][t], st[qb]);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (nvalid < kb * 32 + 32) {   // ragged last tile: keys past the end get no weight
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = kb * 32 + 8 * (i / 4) + 4 * hf + (i % 4);
            if (key >= nvalid) st[qb][i] = -INFINITY;
          }
      }
      v4u pb[NQB][2];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float tmax = fmaxf(st[qb][0], st[qb][1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, st[qb][i]), st[qb][i + 1]);
        tmax = max_across_halves(tmax) * zscale;   // zscale >= 0
        if (__builtin_amdgcn_ballot_w64(tmax > m_used[qb] + kLazyStep) != 0) {
          // -inf only if every key so far was masked, which a tile with a valid key rules out later
          const float m_new = fmaxf(m_used[qb], tmax);
          const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_used[qb] - m_new);
          m_used[qb] = m_new;
          lsum[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[qb][db][i] *= alpha;
        }
        const float neg_m = m_used[qb] == -INFINITY ? 0.0f : -m_used[qb];
        float ls = lsum[qb];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint32_t w[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[qb][8 * u + 2 * j], zscale, neg_m));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[qb][8 * u + 2 * j + 1], zscale, neg_m));
            w[j] = cvt_pk_bf16(p0, p1);
            ls = add_pair_bf16(w[j], ls);
          }
          pb[qb][u] = v4u{w[0], w[1], w[2], w[3]};
        }
        lsum[qb] = ls;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int step = (kb * 32 + 16 * u) * ROWB;
          const v2u lo = lds_read_tr16(vtile + vt.off(0, db) + step);
          const v2u hi = lds_read_tr16(vtile + vt.off(1, db) + step);
          const v4u a = v4u{lo.x, lo.y, hi.x, hi.y};
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) acc[qb][db] = mfma_bf16(a, pb[qb][u], acc[qb][db]);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  fetch(0);
  stage(0);
  __syncthreads();
  int buf = 0;
  for (int t0 = 0; t0 < L; t0 += kDenseK) {
    const bool more = t0 + kDenseK < L;
    if (more) fetch(t0 + kDenseK);
    if (buf == 0) tile(0, t0); else tile(1, t0);
    if (more) stage(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const float l = sum_across_halves(lsum[qb]);
    if (qi < nq) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        uint16_t* op = o + (int64_t(q0 + qi) * s.hq + h) * D + db * 32 + 4 * hf;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          v2u w2;
          w2.x = cvt_pk_bf16(acc[qb][db][4 * i4 + 0] * inv, acc[qb][db][4 * i4 + 1] * inv);
          w2.y = cvt_pk_bf16(acc[qb][db][4 * i4 + 2] * inv, acc[qb][db][4 * i4 + 3] * inv);
          *reinterpret_cast<v2u*>(op + 8 * i4) = w2;
        }
      }
    }
  }
}

constexpr int kQB = 1, kWavesPerGroup = 8;

hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st) {
  constexpr int rows = kWavesPerGroup * 32 * kQB;
  dim3 grid((s.max_q + rows - 1) / rows, s.hq, s.batch);
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  if (s.d == 128)
    attend_dense_bf16_kernel<128, kQB, kWavesPerGroup><<<grid, kWavesPerGroup * 64, 0, st>>>(
        qh, kh, vh, cu_q, cu_kv, seq_mode, which, static_cast<uint16_t*>(o), s);
  else
    attend_dense_bf16_kernel<64, kQB, kWavesPerGroup><<<grid, kWavesPerGroup * 64, 0, st>>>(
        qh, kh, vh, cu_q, cu_kv, seq_mode, which, static_cast<uint16_t*>(o), s);
  return hipGetLastError();
}

}  // namespace dllm
