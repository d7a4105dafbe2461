// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput,
// with the softmax's exponentials on the vector ALUs as the co-bottleneck (about as many VALU
// cycles as MFMA cycles per step), so the two have to overlap.
//
// A workgroup owns WAVES * NQB * 32 query rows of one (sequence, head); each wave keeps its queries
// as B operands in registers for the whole pass.  K/V tiles of 64 keys are loaded by all threads
// (16-byte loads, whole rows per 16 lanes), prefetched into registers three tiles ahead of their use
// and staged in a three-deep ring of XOR-swizzled LDS tiles: one barrier per tile.
//
// Each wave walks the keys in steps of 32 with a software pipeline, so that every stretch of MFMAs
// has independent vector work issued between them:
//   stage 1   S^T(i+1) = K * Q^T          (MFMA, A by ds_read_b128)  ||  exp2 of step i, keys 0..15
//   stage 2   O^T += V^T P^T, keys 0..15  (MFMA, A by ds_read_b64_tr) ||  exp2 of step i, keys 16..31
//   stage 3   O^T += V^T P^T, keys 16..31 (MFMA)                      ||  row maxima of step i+1
// The running maximum is updated lazily: the accumulators are rescaled only when some query's
// maximum grew by more than 2^8 (probabilities may exceed 1 until then), and that rare rescale runs
// outside the hot loop, which then resumes at the next step.
#include "attn_tile.h"

namespace dllm {

constexpr int kDenseK = 64;          // keys per LDS tile
constexpr int kDenseRing = 3;        // LDS tiles in flight
constexpr float kLazyStep = 8.0f;    // log2 of the growth that forces a rescale

// NQB: 32-query blocks per wave; WAVES: waves per workgroup
// which: 1 = only sequences flagged dense in seq_mode; 2 = every sequence
template <int D, int NQB, int WAVES>
__global__ __launch_bounds__(WAVES * 64, (NQB == 1 ? 2 : 1)) void attend_dense_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const uint8_t* __restrict__ seq_mode,
    int which, uint16_t* __restrict__ o, Shape s) {
  constexpr int CH = D / 8;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kDenseK * ROWB;
  constexpr int NTHREADS = WAVES * 64;
  constexpr int QROWS = WAVES * 32 * NQB;
  constexpr int NLD = kDenseK * CH / NTHREADS;   // 16-byte loads per thread, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  static_assert(NLD >= 1, "too many threads for one tile");

  __shared__ __attribute__((aligned(16))) char smem[kDenseRing][2][TILEB];   // [ring slot][K, V]

  // Workgroups are handed to the eight XCDs round-robin by launch order, and each XCD has its own
  // L2.  Renumber so that the query tiles of one (sequence, head), which all stream the same K/V,
  // land on one XCD (launch ids equal modulo 8) and share its L2 instead of fetching K/V eight
  // times, while consecutive (sequence, head) pairs still go to different XCDs.
  const int nx = gridDim.x, groups = gridDim.y * gridDim.z;
  const int n = blockIdx.x + nx * (blockIdx.y + gridDim.y * blockIdx.z);
  int qtile = blockIdx.x, gi = blockIdx.y + gridDim.y * blockIdx.z;
  if ((groups & 7) == 0) {
    const int j = n >> 3;   // position in this XCD's own launch sequence
    qtile = j % nx;
    gi = (j / nx) * 8 + (n & 7);
  }
  const int h = gi % gridDim.y, b = gi / gridDim.y;
  if (which == 1 && !(seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE)) return;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  const int qbase = qtile * QROWS;
  if (qbase >= nq) return;
  const int kv0 = cu_kv[b], L = cu_kv[b + 1] - kv0;
  const int g = h / s.group;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 31, hf = lane >> 5;

  if (L == 0) {   // nothing to attend to: zeros
    for (int e = tid; e < QROWS * D; e += NTHREADS) {
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
  const float zscale = s.scale * kLog2e;   // > 0

  KAddr<D> ka;
  ka.init(lane);
  VtAddr<D> vt;
  vt.init(lane);
  int woff[NLD];   // where this thread's loaded chunks go inside a tile
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * NTHREADS + tid;
    woff[i] = tile_off<D>(f / CH, f % CH);
  }

  float m_used[NQB], lsum[NQB], tmax[NQB];
  f32x16 acc[NQB][NDB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_used[qb] = -INFINITY;
    lsum[qb] = 0.0f;
    tmax[qb] = -INFINITY;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[qb][db][i] = 0.0f;
  }

  v4u kr[NLD], vr[NLD];
  auto fetch = [&](int tile) {   // rows past the end of the sequence are zero-filled
    const int t0 = tile * kDenseK;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int f = i * NTHREADS + tid, row = f / CH, c = f % CH;
      kr[i] = v4u{0u, 0u, 0u, 0u};
      vr[i] = v4u{0u, 0u, 0u, 0u};
      if (t0 + row < L) {
        kr[i] = *reinterpret_cast<const v4u*>(kbase + (t0 + row) * pitch + c * 16);
        vr[i] = *reinterpret_cast<const v4u*>(vbase + (t0 + row) * pitch + c * 16);
      }
    }
  };
  auto stage = [&](int slot) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      *reinterpret_cast<v4u*>(&smem[slot][0][woff[i]]) = kr[i];
      *reinterpret_cast<v4u*>(&smem[slot][1][woff[i]]) = vr[i];
    }
  };
  // scores of one 32-key step for this wave's queries: rows = keys, columns = queries
  auto scores = [&](f32x16 (&st)[NQB], int step) {
    const char* kt = smem[(step >> 1) % kDenseRing][0] + (step & 1) * 32 * ROWB;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[qb][i] = 0.0f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const v4u a = *reinterpret_cast<const v4u*>(kt + ka.off(t));
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) st[qb] = mfma_bf16(a, qreg[qb][t], st[qb]);
    }
  };
  auto mask_tail = [&](f32x16 (&st)[NQB], int nvalid) {   // keys past the end get no weight
    asm volatile("" ::: "memory");   // keep the caller's test a real (uniform) branch
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = 8 * (i / 4) + 4 * hf + (i % 4);
        if (key >= nvalid) st[qb][i] = -INFINITY;
      }
  };
  // row maxima of a step; true if some query of this wave needs its running maximum raised
  auto maxima = [&](const f32x16 (&st)[NQB]) -> bool {
    bool gr = false;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float mx = fmaxf(st[qb][0], st[qb][1]);
#pragma unroll
      for (int i = 2; i < 16; i += 2) mx = fmaxf(fmaxf(mx, st[qb][i]), st[qb][i + 1]);
      tmax[qb] = max_across_halves(mx) * zscale;
      gr = gr || (tmax[qb] > m_used[qb] + kLazyStep);
    }
    return __builtin_amdgcn_ballot_w64(gr) != 0;
  };
  // probabilities of keys 16u .. 16u+15 of a step, packed as the B operand of the P*V MFMAs
  auto probs = [&](const f32x16 (&st)[NQB], int u, v4u (&pb)[NQB]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float neg_m = -m_used[qb];
      uint32_t w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[qb][8 * u + 2 * j], zscale, neg_m));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[qb][8 * u + 2 * j + 1], zscale, neg_m));
        w[j] = cvt_pk_bf16(p0, p1);
        lsum[qb] = add_pair_bf16(w[j], lsum[qb]);
      }
      pb[qb] = v4u{w[0], w[1], w[2], w[3]};
    }
  };
  auto accumulate = [&](const char* vtile, int u, const v4u (&pb)[NQB]) {
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const v2u lo = lds_read_tr16(vtile + vt.off(0, db) + 16 * u * ROWB);
      const v2u hi = lds_read_tr16(vtile + vt.off(1, db) + 16 * u * ROWB);
      const v4u a = v4u{lo.x, lo.y, hi.x, hi.y};
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) acc[qb][db] = mfma_bf16(a, pb[qb], acc[qb][db]);
    }
  };

  const int rem = L % 32;
  const int nsteps = L / 32 + (rem ? 1 : 0);
  const int ntiles = (L + kDenseK - 1) / kDenseK;

  fetch(0);
  stage(0);
  if (ntiles > 1) { fetch(1); stage(1); }
  if (ntiles > 2) fetch(2);
  __syncthreads();

  f32x16 st_cur[NQB];
  scores(st_cur, 0);
  if (nsteps == 1 && rem) mask_tail(st_cur, rem);
  bool grow = maxima(st_cur);   // always true here: the running maxima start at -inf
  int i = 0;
  for (;;) {
    if (grow) {   // rare after the first step: raise the running maxima, rescale what was accumulated
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float m_new = fmaxf(m_used[qb], tmax[qb]);
        const float alpha = __builtin_amdgcn_exp2f(m_used[qb] - m_new);   // exp2(-inf) = 0 the first time
        m_used[qb] = m_new;
        lsum[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[qb][db][e] *= alpha;
      }
      grow = false;
    }
    while (i < nsteps) {
      const int tile = i >> 1, kb = i & 1;
      if (kb == 0) {   // tile boundary: everyone is done with tile-1; tile+1 (staged a tile ago) becomes visible
        __syncthreads();
        if (tile + 2 < ntiles) stage((tile + 2) % kDenseRing);
        if (tile + 3 < ntiles) fetch(tile + 3);
      }
      const int inext = min(i + 1, nsteps - 1);   // past the end: a valid step again, result unused
      const char* vtile = smem[tile % kDenseRing][1] + kb * 32 * ROWB;
      f32x16 st_next[NQB];
      v4u pb0[NQB], pb1[NQB];
      // stage 1
      scores(st_next, inext);
      probs(st_cur, 0, pb0);
      // stage 2
      accumulate(vtile, 0, pb0);
      probs(st_cur, 1, pb1);
      // stage 3
      if (rem && i + 2 == nsteps) mask_tail(st_next, rem);
      accumulate(vtile, 1, pb1);
      const bool gr = maxima(st_next);
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) st_cur[qb] = st_next[qb];
      ++i;
      if (__builtin_expect(gr && i < nsteps, 0)) {
        grow = true;
        break;
      }
    }
    if (!grow) break;
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

// Two waves per SIMD (eight per workgroup, one 32-query block each) measured fastest on MI355X: the
// second wave fills the issue slots the first leaves while it waits on LDS or on a dependent MFMA.
constexpr int kDenseQB = 1, kDenseWaves = 8;

hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st) {
  constexpr int rows = kDenseWaves * 32 * kDenseQB;
  dim3 grid((s.max_q + rows - 1) / rows, s.hq, s.batch);
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  if (s.d == 128)
    attend_dense_bf16_kernel<128, kDenseQB, kDenseWaves><<<grid, kDenseWaves * 64, 0, st>>>(
        qh, kh, vh, cu_q, cu_kv, seq_mode, which, static_cast<uint16_t*>(o), s);
  else
    attend_dense_bf16_kernel<64, kDenseQB, kDenseWaves><<<grid, kDenseWaves * 64, 0, st>>>(
        qh, kh, vh, cu_q, cu_kv, seq_mode, which, static_cast<uint16_t*>(o), s);
  return hipGetLastError();
}

}  // namespace dllm
