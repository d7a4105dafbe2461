// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput.
// Measured on MI355X, MFMA co-issues with v_exp_f32 and plain vector work almost for free; what costs
// time is everything that makes waves wait: the start and end of a workgroup, workgroup barriers,
// staging K/V through registers, and LDS read latency.  Hence:
//   - a workgroup is four waves (128 query rows of one (sequence, head)) and uses 80 KB of LDS, so two
//     workgroups share a compute unit and run out of phase: one's prologue, epilogue and barrier waits
//     are covered by the other's matrix work;
//   - K/V tiles of 64 keys go from global memory straight into LDS (global_load_lds, 16 bytes per
//     lane), issued right after the tile barrier and due one tile later: no staging registers, no LDS
//     writes, and the prologue's loads (Q, two K tiles, one V tile) are all in flight at once.  LDS
//     tiles are XOR-swizzled by row; since the LDS side of such a load is lane-contiguous, the swizzle
//     is applied to the global chunk each lane fetches (a permutation inside one 2*D-byte row);
//   - K lives in a ring of three tiles (its scores are computed one step ahead), V in a ring of two;
//   - the score MFMA chain starts from the accumulator value -m (the running maximum of the raw
//     scores) instead of 0, so the scores leave the matrix core with the maximum subtracted; one
//     multiply by softmax_scale * log2(e) per score, done in the stage that has vector slots to
//     spare, makes them base-2 logits (Q is NOT pre-scaled: rounding the scaled queries to bf16
//     again costs 2e-2 of output accuracy at logits around 20);
//   - the running maximum is raised lazily (only when a score exceeds it by more than 2^8, so
//     probabilities may exceed 1 until then) behind a uniform branch;
//   - the key loop is unrolled over one common turn of both rings (twelve 32-key steps), so every LDS
//     address is a register fixed before the loop plus an immediate offset.
//
// Each wave keeps its 32 queries as MFMA B operands in registers for the whole pass and walks the keys
// in steps of 32 with a software pipeline:
//   stage 1   S^T(i+1) = K * Q^T - m      (MFMA, A by ds_read_b128)  ||  exp2 of step i, keys 0..15
//   stage 2   O^T += V^T P^T, keys 0..15  (MFMA, A by ds_read_b64_tr) ||  exp2 of step i, keys 16..31
//   stage 3   O^T += V^T P^T, keys 16..31 (MFMA)                      ||  scale, row maxima of step i+1
#include <type_traits>

#include "attn_tile.h"


namespace dllm {

#ifndef DLLM_S3V
#define DLLM_S3V 7
#endif
constexpr int kDenseK = 64;          // keys per LDS tile
constexpr int kDenseRingK = 3;       // K tiles resident in LDS
constexpr int kDenseRingV = 2;       // V tiles resident in LDS
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
  constexpr int VBASE = kDenseRingK * TILEB;     // V tiles follow the K tiles
  constexpr int NTHREADS = WAVES * 64;
  constexpr int QROWS = WAVES * 32 * NQB;
  constexpr int NLD = kDenseK * CH / NTHREADS;   // 16-byte loads per lane, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  constexpr int ROUND = 2 * kDenseRingK * kDenseRingV;   // steps in one common turn of both rings
  static_assert(NLD >= 1 && kDenseK * CH % NTHREADS == 0, "tile does not split evenly over the threads");

  __shared__ __attribute__((aligned(16))) char smem[(kDenseRingK + kDenseRingV) * TILEB];   // K ring, V ring

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
  // Global side of the tile loads: this lane's chunk f = i * NTHREADS + tid of a tile lands at LDS
  // byte 16 * f, i.e. row f / CH, chunk slot f % CH, and must hold chunk (slot ^ swizzle(row)) of
  // that row.  Rows past the end of the sequence re-read its last row (their keys are masked).
  int ld_row[NLD], ld_col[NLD];
  uint32_t ld_off[NLD];   // byte offset of the chunk from the tile's first row (fits: checked on the host)
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * NTHREADS + tid, row = f / CH;
    ld_row[i] = row;
    ld_col[i] = ((f % CH) ^ tile_swz<D>(row)) << 4;
    ld_off[i] = uint32_t(row) * uint32_t(pitch) + uint32_t(ld_col[i]);
  }
  // this wave's slice of each load round, as an LDS byte address
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_addr(smem) + wave * 64 * 16);
  auto load_tile = [&](const char* base, int tile, int lds_off) {
    const int t0 = tile * kDenseK;
    if (t0 + kDenseK <= L) {   // whole tile inside the sequence: uniform tile address + fixed lane offsets
      const char* tbase = base + int64_t(t0) * pitch;
#pragma unroll
      for (int i = 0; i < NLD; ++i) load16_to_lds(tbase, ld_off[i], wave_lds + lds_off + i * NTHREADS * 16);
    } else {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int row = min(t0 + ld_row[i], L - 1);
        load16_to_lds(base + row * pitch + ld_col[i], wave_lds + lds_off + i * NTHREADS * 16);
      }
    }
  };

  // the first tiles are requested before anything else, so their latency overlaps the Q loads
  const int rem = L % 32;
  const int nsteps = L / 32 + (rem ? 1 : 0);
  const int ntiles = (L + kDenseK - 1) / kDenseK;
  load_tile(kbase, 0, 0);
  load_tile(vbase, 0, VBASE);
  if (ntiles > 1) load_tile(kbase, 1, TILEB);

  // Q^T operands: lane (col = query, hf) holds Q[query][16t + 8hf .. +8) for every step t, as given:
  // scaling them here would round them to bf16 a second time, an error in the logit that grows with
  // the logit (2e-2 in the output at logits around 20); the scale is applied to the fp32 scores
  const float zscale = s.scale * kLog2e;   // > 0; scores * zscale are base-2 logits
  const float inv_zscale = 1.0f / zscale;
  v4u qreg[NQB][NT];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      v4u x = v4u{0u, 0u, 0u, 0u};
      if (qi < nq) x = *reinterpret_cast<const v4u*>(qp + 16 * t + 8 * hf);
      qreg[qb][t] = x;
    }
  }

  // running maximum m (of the raw scores q.k), kept negated in all 16 registers of an accumulator so
  // that it can seed the score MFMA chain; row sum; output accumulators
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

  // A operands of one step's score chain: rows = 32 keys at byte offset `koff` of the K ring
  auto k_operands = [&](v4u (&kop)[NT], int koff) {
#pragma unroll
    for (int t = 0; t < NT; ++t) kop[t] = *reinterpret_cast<const v4u*>(smem + ka[t] + koff);
  };
  // scores of a 32-key step relative to the running maxima: rows = keys, columns = this wave's queries
  auto score_chain = [&](f32x16 (&st)[NQB], const v4u (&kop)[NT]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) st[qb] = negm[qb];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) st[qb] = mfma_bf16(kop[t], qreg[qb][t], st[qb]);
  };
  // raw scores minus the running maximum -> base-2 logits
  auto to_logits = [&](f32x16 (&st)[NQB]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[qb][i] *= zscale;
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
  // Raise the running maxima by delta >= 0 (in base-2 logits) per query and rescale what was
  // accumulated under the old ones, including the logits `st` already computed relative to them.
  auto raise = [&](f32x16 (&st)[NQB], const float (&delta)[NQB]) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float alpha = __builtin_amdgcn_exp2f(-delta[qb]);
      const float delta_raw = delta[qb] * inv_zscale;
      lsum[qb] *= alpha;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        negm[qb][i] -= delta_raw;
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
        const float p0 = __builtin_amdgcn_exp2f(st[qb][8 * u + 2 * j]);
        const float p1 = __builtin_amdgcn_exp2f(st[qb][8 * u + 2 * j + 1]);
        w[j] = cvt_pk_bf16(p0, p1);
        lsum[qb] = add_pair_bf16(w[j], lsum[qb]);
      }
      pb[qb] = v4u{w[0], w[1], w[2], w[3]};
    }
  };
  // A operands of one 16-key slice of O^T += V^T P^T: V^T blocks of 32 head_dim rows x 16 keys
  auto v_operands = [&](v4u (&vop)[NDB], int voff) {
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const v2u lo = lds_read_tr16(smem + va[0][db] + voff);
      const v2u hi = lds_read_tr16(smem + va[1][db] + voff);
      vop[db] = v4u{lo.x, lo.y, hi.x, hi.y};
    }
  };
  auto accumulate = [&](const v4u (&vop)[NDB], const v4u (&pb)[NQB]) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) acc[qb][db] = mfma_bf16(vop[db], pb[qb], acc[qb][db]);
  };

  wait_tile_loads();
  __syncthreads();

  // Issue-order hints: inside a stage, spread the vector and LDS work between the MFMAs so that the
  // matrix pipe always has the next MFMA waiting behind work that does not depend on it.
#define DLLM_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
  constexpr int kMfma = 0x008, kValu = 0x002, kTrans = 0x400, kDsRead = 0x100;

  f32x16 st_a[NQB], st_b[NQB];
  v4u kop[NT];   // K operands of the next score chain, fetched a stage ahead of their use
  k_operands(kop, 0);
  score_chain(st_a, kop);
  to_logits(st_a);
  if (nsteps == 1 && rem) mask_tail(st_a, rem);
  // the first step sets the maxima outright (they may be negative); nothing is accumulated yet
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const float first = max_across_halves(lane_max(st_a[qb]));
    const float first_raw = first * inv_zscale;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      negm[qb][i] = -first_raw;
      st_a[qb][i] -= first;
    }
  }
  k_operands(kop, 32 * ROWB);   // step 1 (stale LDS if there is none; then unused)

  // One 32-key step.  R is its position in the common turn of the rings, which fixes every LDS
  // offset.  The step multiplies P of step i with V tile (R/2) % 2, half R%2, computes the scores of
  // step i+1 from K operands fetched during step i-1, and fetches those of step i+2.
  int i = 0;
  auto step = [&](auto rc, f32x16 (&cur)[NQB], f32x16 (&nxt)[NQB]) {
    constexpr int R = decltype(rc)::value;
    constexpr int T = R / 2, kb = R % 2;   // tile index modulo the turn
    constexpr int RN2 = (R + 2) % ROUND;
    const int tile = i >> 1;
    if (kb == 0) {
      // Tile boundary: everyone is done with tile-1, and the loads issued a tile ago (K of tile+1,
      // V of this tile) have landed.  The slots of tile-1 take K of tile+2 and V of tile+1.
      wait_tile_loads();
      __syncthreads();
      if (tile + 2 < ntiles) load_tile(kbase, tile + 2, ((T + 2) % kDenseRingK) * TILEB);
      if (tile + 1 < ntiles) load_tile(vbase, tile + 1, VBASE + ((T + 1) % kDenseRingV) * TILEB);
    }
    constexpr int voff = (T % kDenseRingV) * TILEB + kb * 32 * ROWB;
    v4u pb0[NQB], pb1[NQB], vop0[NDB], vop1[NDB];
    __builtin_amdgcn_sched_barrier(0);
    // stage 1: S^T(i+1) chain || exp2 of keys 0..15 of step i || fetch V^T operands of keys 0..15
    v_operands(vop0, voff);
    score_chain(nxt, kop);
    probs(cur, 0, pb0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {   // one group per pair of probabilities packed together
      DLLM_SGB(kMfma, NT * NQB / 4);
      DLLM_SGB(kDsRead, 2 * NDB / 4);
      DLLM_SGB(kTrans, 2 * NQB);
      DLLM_SGB(kValu, 2 * NQB);
    }
    __builtin_amdgcn_sched_barrier(0);
    // stage 2: O^T += V^T P^T, keys 0..15 || exp2 of keys 16..31 || fetch V^T operands of keys 16..31
    // the two stages that feed the output accumulators run at raised wave priority: of the two waves
    // of a SIMD the one in its P*V half gets the issue slots (measured: 1 % on the Refresh workload)
    __builtin_amdgcn_s_setprio(3);
    v_operands(vop1, voff + 16 * ROWB);
    accumulate(vop0, pb0);
    probs(cur, 1, pb1);
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      DLLM_SGB(kMfma, NQB);
      DLLM_SGB(kDsRead, 2);
      DLLM_SGB(kTrans, 8 * NQB / NDB);
      DLLM_SGB(kValu, 8 * NQB / NDB);
    }
    __builtin_amdgcn_sched_barrier(0);
    // stage 3: O^T += V^T P^T, keys 16..31 || row maxima of step i+1 || fetch K operands of step i+2
    k_operands(kop, ((RN2 / 2) % kDenseRingK) * TILEB + (RN2 % 2) * 32 * ROWB);
    accumulate(vop1, pb1);
    to_logits(nxt);
    bool grow = false;
    float mx[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      mx[qb] = lane_max(nxt[qb]);
      grow = grow || (mx[qb] > kLazyStep);
    }
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      DLLM_SGB(kMfma, NQB);
      DLLM_SGB(kDsRead, NT / NDB);
      DLLM_SGB(kValu, DLLM_S3V * NQB);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
    ++i;
    // Rare path, one uniform branch: the next step is the ragged last one (mask the keys past the end,
    // which were scored from a repeated row), or some score outgrew its running maximum.
    const bool ragged = rem != 0 && i + 1 == nsteps;
    if (__builtin_expect((__builtin_amdgcn_ballot_w64(grow) != 0 || ragged) && i < nsteps, 0)) {
      if (ragged) {
        mask_tail(nxt, rem);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) mx[qb] = lane_max(nxt[qb]);
      }
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
    if (i >= nsteps) break;
    step(std::integral_constant<int, 6>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 7>{}, st_b, st_a);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 8>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 9>{}, st_b, st_a);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 10>{}, st_a, st_b);
    if (i >= nsteps) break;
    step(std::integral_constant<int, 11>{}, st_b, st_a);
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

// Four waves per workgroup, one 32-query block each; two workgroups per compute unit (two waves per SIMD).
#ifndef DLLM_DENSE_QB
#define DLLM_DENSE_QB 1
#endif
#ifndef DLLM_DENSE_WAVES
#define DLLM_DENSE_WAVES 4
#endif
constexpr int kDenseQB = DLLM_DENSE_QB, kDenseWaves = DLLM_DENSE_WAVES;

hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st) {
  constexpr int rows = kDenseWaves * 32 * kDenseQB;
  if (s.max_q == 0) return hipSuccess;   // no sequence has a query: nothing to write
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
