// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput,
// with the softmax's exponentials on the vector ALUs as the co-bottleneck: one v_exp_f32 per score
// costs a quarter-rate issue slot, which alone is half of the MFMA time of a step.  Everything else
// on the vector ALUs is therefore kept to a minimum:
//   - Q is scaled by softmax_scale * log2(e) once, when it is loaded (rounded to bf16 again), and the
//     score MFMA chain starts from the accumulator value -m (the running maximum) instead of 0, so
//     the scores leave the matrix core ready for exp2: no multiply-add per score;
//   - the running maximum is raised lazily (only when a score exceeds it by more than 2^8, so
//     probabilities may exceed 1 until then) and that rare rescale sits behind a uniform branch;
//   - the key loop is unrolled over one turn of the LDS ring (six 32-key steps), so every LDS
//     address is a register fixed before the loop plus an immediate offset;
//   - the row sums come from the packed bf16 probabilities (two per v_dot2c), the same values the
//     P*V product uses.
//
// A workgroup owns WAVES * NQB * 32 query rows of one (sequence, head); each wave keeps its queries
// as B operands in registers for the whole pass.  K/V tiles of 64 keys are loaded by all threads
// (16-byte loads, whole rows per 16 lanes), prefetched into registers three tiles ahead of their use
// and staged in a three-deep ring of XOR-swizzled LDS tiles: one barrier per tile.
//
// Each wave walks the keys in steps of 32 with a software pipeline, so that every stretch of MFMAs
// has independent vector work issued between them:
//   stage 1   S^T(i+1) = K * Q^T - m      (MFMA, A by ds_read_b128)  ||  exp2 of step i, keys 0..15
//   stage 2   O^T += V^T P^T, keys 0..15  (MFMA, A by ds_read_b64_tr) ||  exp2 of step i, keys 16..31
//   stage 3   O^T += V^T P^T, keys 16..31 (MFMA)                      ||  row maxima of step i+1
#include <type_traits>

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
  constexpr int VBASE = kDenseRing * TILEB;      // V tiles follow the K tiles
  constexpr int NTHREADS = WAVES * 64;
  constexpr int QROWS = WAVES * 32 * NQB;
  constexpr int NLD = kDenseK * CH / NTHREADS;   // 16-byte loads per thread, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  constexpr int ROUND = 2 * kDenseRing;          // steps in one turn of the ring
  static_assert(NLD >= 1, "too many threads for one tile");

  __shared__ __attribute__((aligned(16))) char smem[2 * kDenseRing * TILEB];   // K ring, then V ring

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

  // Q^T operands: lane (col = query, hf) holds zscale * Q[query][16t + 8hf .. +8) for every step t
  const float zscale = s.scale * kLog2e;   // > 0
  v4u qreg[NQB][NT];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      v4u x = v4u{0u, 0u, 0u, 0u};
      if (qi < nq) x = *reinterpret_cast<const v4u*>(qp + 16 * t + 8 * hf);
      qreg[qb][t] = v4u{cvt_pk_bf16(bf16_lo(x.x) * zscale, bf16_hi(x.x) * zscale),
                        cvt_pk_bf16(bf16_lo(x.y) * zscale, bf16_hi(x.y) * zscale),
                        cvt_pk_bf16(bf16_lo(x.z) * zscale, bf16_hi(x.z) * zscale),
                        cvt_pk_bf16(bf16_lo(x.w) * zscale, bf16_hi(x.w) * zscale)};
    }
  }
  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const int64_t pitch = s.kv_tok * 2;

  // LDS addresses, fixed for the whole pass; ring slot, 32-key half and 16-key quarter are immediates
  int ka[NT], va[2][NDB];
  {
    KAddr<D> kaddr;
    kaddr.init(lane);
    VtAddr<D> vaddr;
    vaddr.init(lane);
#pragma unroll
    for (int t = 0; t < NT; ++t) ka[t] = kaddr.off(t);
#pragma unroll
    for (int rd = 0; rd < 2; ++rd)
#pragma unroll
      for (int db = 0; db < NDB; ++db) va[rd][db] = VBASE + vaddr.off(rd, db);
  }
  int woff[NLD];   // where this thread's loaded chunks go inside a tile
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * NTHREADS + tid;
    woff[i] = tile_off<D>(f / CH, f % CH);
  }

  // running maximum m (base-2 logits), kept negated in all 16 registers of an accumulator so that
  // it can seed the score MFMA chain; row sum; output accumulators
  f32x16 negm[NQB];
  float lsum[NQB];
  f32x16 acc[NQB][NDB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    lsum[qb] = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) negm[qb][i] = 0.0f;
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
      *reinterpret_cast<v4u*>(smem + slot * TILEB + woff[i]) = kr[i];
      *reinterpret_cast<v4u*>(smem + VBASE + slot * TILEB + woff[i]) = vr[i];
    }
  };
  // scores of the 32-key step at byte offset `koff` of the K ring, relative to the running maxima:
  // rows = keys, columns = this wave's queries
  auto scores = [&](f32x16 (&st)[NQB], int koff) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) st[qb] = negm[qb];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#ifdef DLLM_ABL_NOLDSREAD
      const v4u a = qreg[0][(t + 1) % NT];
#else
      const v4u a = *reinterpret_cast<const v4u*>(smem + ka[t] + koff);
#endif
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
  // largest score of a step per lane (a query's scores sit in the lane pair l, l ^ 32)
  auto lane_max = [&](const f32x16& st) -> float {
    float mx = fmaxf(st[0], st[1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) mx = fmaxf(fmaxf(mx, st[i]), st[i + 1]);
    return mx;
  };
  // Raise the running maxima by delta >= 0 per query and rescale what was accumulated under the old
  // ones, including the scores `st` already computed relative to them.
  auto raise = [&](f32x16 (&st)[NQB], const float (&delta)[NQB]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float alpha = __builtin_amdgcn_exp2f(-delta[qb]);
      lsum[qb] *= alpha;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        negm[qb][i] -= delta[qb];
        st[qb][i] -= delta[qb];
      }
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[qb][db][e] *= alpha;
    }
  };
  // probabilities of keys 16u .. 16u+15 of a step, packed as the B operand of the P*V MFMAs
  auto probs = [&](const f32x16 (&st)[NQB], int u, v4u (&pb)[NQB]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      uint32_t w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#ifdef DLLM_ABL_NOEXP
        const float p0 = st[qb][8 * u + 2 * j], p1 = st[qb][8 * u + 2 * j + 1];
#else
        const float p0 = __builtin_amdgcn_exp2f(st[qb][8 * u + 2 * j]);
        const float p1 = __builtin_amdgcn_exp2f(st[qb][8 * u + 2 * j + 1]);
#endif
        w[j] = cvt_pk_bf16(p0, p1);
        lsum[qb] = add_pair_bf16(w[j], lsum[qb]);
      }
      pb[qb] = v4u{w[0], w[1], w[2], w[3]};
    }
  };
  auto accumulate = [&](int voff, const v4u (&pb)[NQB]) {
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
#ifdef DLLM_ABL_NOLDSREAD
      const v4u a = qreg[0][db];
#else
      const v2u lo = lds_read_tr16(smem + va[0][db] + voff);
      const v2u hi = lds_read_tr16(smem + va[1][db] + voff);
      const v4u a = v4u{lo.x, lo.y, hi.x, hi.y};
#endif
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

  f32x16 st_a[NQB], st_b[NQB];
  scores(st_a, 0);
  if (nsteps == 1 && rem) mask_tail(st_a, rem);
  {   // the first step sets the maxima outright (they may be negative)
    float delta[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) delta[qb] = max_across_halves(lane_max(st_a[qb]));
    raise(st_a, delta);
  }

  // One 32-key step.  R (0..5) is its position in the turn of the ring, which fixes every LDS offset:
  // the step reads V of ring slot R/2, half R%2, and computes the scores of the step after it.
  int i = 0;
  auto step = [&](auto rc, f32x16 (&cur)[NQB], f32x16 (&nxt)[NQB]) {
    constexpr int R = decltype(rc)::value;
    constexpr int slot = R / 2, kb = R % 2;
    constexpr int RN = (R + 1) % ROUND;
    const int tile = i >> 1;
    if (kb == 0) {   // tile boundary: everyone is done with tile-1; tile+1 (staged a tile ago) becomes visible
      __syncthreads();
#ifndef DLLM_ABL_NOSTAGE
      if (tile + 2 < ntiles) stage((slot + 2) % kDenseRing);
      if (tile + 3 < ntiles) fetch(tile + 3);
#endif
    }
    constexpr int voff = slot * TILEB + kb * 32 * ROWB;
    v4u pb0[NQB], pb1[NQB];
    // stage 1 (past the last step the scores are computed from stale LDS and never used)
    scores(nxt, (RN / 2) * TILEB + (RN % 2) * 32 * ROWB);
    probs(cur, 0, pb0);
    // stage 2
    accumulate(voff, pb0);
    probs(cur, 1, pb1);
    // stage 3
    if (rem && i + 2 == nsteps) mask_tail(nxt, rem);
    accumulate(voff + 16 * ROWB, pb1);
    bool grow = false;
    float mx[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      mx[qb] = lane_max(nxt[qb]);
      grow = grow || (mx[qb] > kLazyStep);
    }
    ++i;
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0 && i < nsteps, 0)) {
      float delta[NQB];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) delta[qb] = fmaxf(max_across_halves(mx[qb]), 0.0f);
      raise(nxt, delta);
    }
  };
  for (;;) {
    if (i >= nsteps) break;
    step(std::integral_constant<int, 0>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 1>{}, st_b, st_a);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 2>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 3>{}, st_b, st_a);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 4>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 5>{}, st_b, st_a);
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

// Two waves per SIMD (eight per workgroup, one 32-query block each): the second wave fills the
// issue slots the first leaves while it waits on LDS or on a dependent MFMA.
#ifndef DLLM_DENSE_QB
#define DLLM_DENSE_QB 1
#endif
#ifndef DLLM_DENSE_WAVES
#define DLLM_DENSE_WAVES 8
#endif
constexpr int kDenseQB = DLLM_DENSE_QB, kDenseWaves = DLLM_DENSE_WAVES;

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
