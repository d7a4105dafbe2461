// Reuse-phase attention over each head's kept rows (Section 2.3 Eq. 4 restricted to the kept set of
// Section 4.5), bf16 inputs, fp32 softmax state and accumulators, on the gfx950 matrix cores.
//
// The step is bound by HBM: every kept (head, row) pair costs one 2*D-byte K row and one V row and
// only 4*Bq*D flop.  What decides its speed is how many gathered rows are in flight, so the registers
// go to the gathers: a workgroup of four waves walks one chunk of one (sequence, head)'s kept rows,
// each wave owns its own 32-row tiles (no workgroup barrier in the loop) and keeps its next tile of K
// and V rows in flight in registers; the queries, which every step needs again, live in LDS instead.
//   gather   idx -> row offsets (32-bit, from a uniform base); 16-byte non-temporal loads with a row's
//            chunks in neighbouring lanes (whole 256-byte rows per 16 lanes)
//   stage    registers -> the wave's private LDS tile, XOR-swizzled by row; the freed registers are
//            refilled with the next tile at once
//   S^T      = K_tile (32 keys x D) * Q^T (D x 32 queries): A and B by ds_read_b128
//   softmax  online, base 2, lazily rescaled, per query column
//   O^T     += V_tile^T * P^T: A by ds_read_b64_tr_b16, B = the S^T accumulators in place
// After the loop the four waves merge (m, l, O) through LDS (one barrier).  A (sequence, head) whose kept rows fit
// one chunk writes O directly; otherwise chunks write fp32 partials and a small kernel merges them.
//
// Two kernels share that tile arithmetic: attend_sparse_bf16_kernel gives every (sequence, head, chunk)
// a workgroup of its own; attend_sparse_multi_bf16_kernel, for batches with more lists than compute
// units and lists of unequal length, runs one eight-wave workgroup per compute unit that walks a
// length-balanced share of the lists back to back.
#include "attn_tile.h"

namespace dllm {

constexpr int kTile = 32;        // kept rows per wave tile
constexpr int kWaves = 4;
constexpr int kWavesMulti = 8;        // waves of a workgroup that walks several lists, one after the other
constexpr int kMultiTilesPerWave = 8; // chunk_rows <= kMultiTilesPerWave * kWavesMulti * kTile there
constexpr float kLazyStepS = 8.0f;
constexpr int kMaxTilesPerWave = 16;  // chunk_rows <= kMaxTilesPerWave * kWaves * kTile
#ifndef DLLM_SPARSE_DEPTH
#define DLLM_SPARSE_DEPTH 1
#endif
constexpr int kDepth = DLLM_SPARSE_DEPTH;   // tiles of gathered rows a wave keeps in flight in registers
// The k-th tile wave `wave` takes of a pass after its first (tile w is wave w's first).  Two waves share
// a SIMD and the older one (waves 0-3) wins the arbitration for memory instructions, so with equal
// shares four waves finish early and wait at the merge.  The later tiles are therefore dealt in periods
// of 20 of which each of waves 0-3 takes three and each of waves 4-7 two, always the same ones, so the
// result does not depend on timing (measured on the batched Reuse workload: 40.9 -> 39.9 us; 4 : 3 and a
// shared counter that deals tiles as waves come free measure the same, 5 : 4 and 2 : 1 less).
__device__ __forceinline__ int later_tile(int wave, int k) {
  constexpr int F = 3, S = 2, P = 4 * (F + S);
  // rounds of a period: the first S rounds go to all eight waves, the other F - S to waves 0-3 only
  if (wave < 4) {
    const int p = k / F, r = k % F;
    return kWavesMulti + P * p + (r < S ? 8 * r + wave : 8 * S + 4 * (r - S) + wave);
  }
  const int p = k / S, r = k % S;
  return kWavesMulti + P * p + 8 * r + wave;
}
constexpr int kRankBatch = 64;        // batches up to this size are walked longest kept list first

// A (sequence, head) with kb kept rows is cut into n = ceil(kb / chunk_rows) chunks of equal size
// (rounded up to the 128 rows four waves take per step), so no chunk is a short leftover.
struct ChunkGeom {
  int n, rows;
};
__device__ __forceinline__ ChunkGeom chunk_geom(int kb, int chunk_rows) {
  ChunkGeom g;
  g.n = 1;
  g.rows = chunk_rows;
  if (kb > chunk_rows) {
    g.n = int(uint32_t(kb + chunk_rows - 1) / uint32_t(chunk_rows));
    g.rows = int((uint32_t(kb + g.n - 1) / uint32_t(g.n) + 127u) / 128u * 128u);
  }
  return g;
}

// Per-sequence offsets a workgroup needs, fetched for the whole (small) batch in one round of
// loads: lane i holds sequence i's entries, and the chosen sequence's are read back by lane index.
struct SeqInfo {
  int b, ko0, kb, q0, nq, kv0;
};

// The batch's offsets as one workgroup holds them: lane i holds sequence i's entries and its rank in
// descending order of kept rows (ties: lower sequence first); every workgroup derives the same order
// from cu_k.  Batches of more than kRankBatch sequences are not ranked and read their entries per use.
struct BatchInfo {
  int ko0, kb, q0, nq, kv0, rank;
};
__device__ __forceinline__ BatchInfo load_batch(const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv,
                                                const int32_t* __restrict__ cu_k, int batch, int lane, bool ranked) {
  BatchInfo bi = {0, 0, 0, 0, 0, 0};
  if (batch > kRankBatch) return bi;
  const int i = lane < batch ? lane : batch - 1;
  bi.ko0 = cu_k[i]; bi.kb = cu_k[i + 1] - bi.ko0;
  bi.q0 = cu_q[i]; bi.nq = cu_q[i + 1] - bi.q0;
  bi.kv0 = cu_kv[i];
  if (ranked) {
    const int mine = lane < batch ? bi.kb : -1;
    int rank = 0;
    for (int j = 0; j < batch; ++j) {
      const int other = __builtin_amdgcn_readlane(mine, j);
      rank += (other > mine) || (other == mine && j < lane);
    }
    bi.rank = rank;
  }
  return bi;
}

// Sequence handled by slot z.  With `ranked` set (small batches whose workgroups do not all fit on the
// chip at once, or that are shared out by length) it is the z-th in descending order of kept rows, so
// the longest lists start first and the short ones fill the compute units that free up.
__device__ __forceinline__ SeqInfo sequence_of_slot(const BatchInfo& bi, const int32_t* __restrict__ cu_q,
                                                    const int32_t* __restrict__ cu_kv,
                                                    const int32_t* __restrict__ cu_k, int batch, int z, int lane,
                                                    bool ranked) {
  SeqInfo si;
  if (batch > kRankBatch) {
    si.b = z;
    si.ko0 = cu_k[z]; si.kb = cu_k[z + 1] - si.ko0;
    si.q0 = cu_q[z]; si.nq = cu_q[z + 1] - si.q0;
    si.kv0 = cu_kv[z];
    return si;
  }
  int b = z;
  if (ranked) b = __builtin_ctzll(__builtin_amdgcn_ballot_w64(lane < batch && bi.rank == z));
  si.b = b;
  si.ko0 = __builtin_amdgcn_readlane(bi.ko0, b);
  si.kb = __builtin_amdgcn_readlane(bi.kb, b);
  si.q0 = __builtin_amdgcn_readlane(bi.q0, b);
  si.nq = __builtin_amdgcn_readlane(bi.nq, b);
  si.kv0 = __builtin_amdgcn_readlane(bi.kv0, b);
  return si;
}
__device__ __forceinline__ SeqInfo sequence_of_slot(const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv,
                                                    const int32_t* __restrict__ cu_k, int batch, int z, int lane,
                                                    bool ranked) {
  return sequence_of_slot(load_batch(cu_q, cu_kv, cu_k, batch, lane, ranked), cu_q, cu_kv, cu_k, batch, z, lane,
                          ranked);
}

// One 32-key tile that lies in LDS (K rows in ktile, V rows in vtile, the 32 queries in qtile, all in the
// swizzled tile layout): S^T = K Q^T, online softmax over the first nvalid keys, O^T += V^T P^T.
template <int D>
__device__ __forceinline__ void sparse_tile_math(const char* ktile, const char* vtile, const char* qtile,
                                                 const KAddr<D>& ka, const VtAddr<D>& vt, int hf, int nvalid,
                                                 float zscale, float& m_used, float& lsum, f32x16 (&acc)[D / 32]) {
  constexpr int ROWB = 2 * D;
  constexpr int NT = D / 16;    // MFMA steps along head_dim
  constexpr int NDB = D / 32;   // 32-wide blocks of head_dim in the output
  // S^T tile: rows = keys, columns = queries
  f32x16 st;
#pragma unroll
  for (int i = 0; i < 16; ++i) st[i] = 0.0f;
#pragma unroll
  for (int t = 0; t < NT; ++t)
    st = mfma_bf16(*reinterpret_cast<const v4u*>(ktile + ka.off(t)),
                   *reinterpret_cast<const v4u*>(qtile + ka.off(t)), st);
  // issue order: operand fetches just ahead of their MFMA, so few operand registers are live
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
  }
  __builtin_amdgcn_sched_barrier(0);

  if (nvalid < kTile) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = 8 * (i / 4) + 4 * hf + (i % 4);
      if (key >= nvalid) st[i] = -INFINITY;
    }
  }
  float tmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, st[i]), st[i + 1]);
  tmax = max_across_halves(tmax) * zscale;   // zscale >= 0
  if (__builtin_amdgcn_ballot_w64(tmax > m_used + kLazyStepS) != 0) {
    const float m_new = fmaxf(m_used, tmax);
    const float alpha = __builtin_amdgcn_exp2f(m_used - m_new);   // first tile: exp2(-inf) = 0
    m_used = m_new;
    lsum *= alpha;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][i] *= alpha;
  }
  const float neg_m = -m_used;
  v4u pb[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    uint32_t w[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[8 * u + 2 * jj], zscale, neg_m));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[8 * u + 2 * jj + 1], zscale, neg_m));
      w[jj] = cvt_pk_bf16(p0, p1);
      lsum = add_pair_bf16(w[jj], lsum);
    }
    pb[u] = v4u{w[0], w[1], w[2], w[3]};
  }
  // O^T += V^T P^T, 16 keys per step
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const v2u lo = lds_read_tr16(vtile + vt.off(0, db) + 16 * u * ROWB);
      const v2u hi = lds_read_tr16(vtile + vt.off(1, db) + 16 * u * ROWB);
      acc[db] = mfma_bf16(v4u{lo.x, lo.y, hi.x, hi.y}, pb[u], acc[db]);
    }
#pragma unroll
  for (int i = 0; i < 2 * NDB; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
  }
}

template <int D>
__global__ __launch_bounds__(kWaves * 64, 2) void attend_sparse_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cu_k, int32_t total_k, const uint8_t* __restrict__ seq_mode,
    uint16_t* __restrict__ o, float* __restrict__ po, float* __restrict__ pm, float* __restrict__ pl,
    int32_t chunk_rows, int ranked, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int CH = D / 8;             // 16-byte chunks per row
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kTile * ROWB;
  constexpr int NLD = kTile * CH / 64;  // 16-byte loads per lane per tile and tensor
  constexpr int NDB = D / 32;           // 32-wide blocks of head_dim in the output

  // per wave: K tile then V tile; reused as fp32 merge space afterwards
  __shared__ __attribute__((aligned(16))) char lds[kWaves][2 * TILEB];
  // the 32 queries of the current query tile (same swizzled layout as a K tile)
  __shared__ __attribute__((aligned(16))) char qtile[TILEB];
  // kept-row ids of each wave's tiles; after the loop each wave leaves its (m, l) pairs in its own part
  __shared__ int sm_rows[kWaves][kMaxTilesPerWave * kTile];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  // Every kernel argument is fetched now, next to the loads of the batch's offsets, and not where it
  // is first used: the gathers cannot start before the last of them has arrived.
  {
    auto fetch_now = [](auto x) { asm volatile("" ::"s"(x)); };
    fetch_now(q); fetch_now(k); fetch_now(v); fetch_now(idx); fetch_now(seq_mode); fetch_now(o);
    fetch_now(total_k); fetch_now(chunk_rows); fetch_now(ranked);
    fetch_now(s.batch); fetch_now(s.hq); fetch_now(s.group); fetch_now(s.q_tok); fetch_now(s.q_head);
    fetch_now(s.kv_tok); fetch_now(s.kv_head); fetch_now(s.total_q); fetch_now(s.scale);
  }
  const int chunk = blockIdx.x, h = blockIdx.y;
  const SeqInfo si = sequence_of_slot(cu_q, cu_kv, cu_k, s.batch, blockIdx.z, lane, ranked != 0);
  const int b = si.b;
  if (seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE) return;
  const int ko0 = si.ko0, kb = si.kb;
  const ChunkGeom cg = chunk_geom(kb, chunk_rows);
  const int c0 = chunk * cg.rows;
  if (c0 >= kb && !(chunk == 0 && kb == 0)) return;
  const int c1 = min(kb, c0 + cg.rows);
  const int nch_b = cg.n;
  const int q0 = si.q0, nq = si.nq;
  const int kv0 = si.kv0;
  const int g = h / s.group;

  if (kb == 0) {  // nothing kept: defined as zeros
    for (int e = threadIdx.x; e < nq * D; e += kWaves * 64)
      o[(int64_t(q0 + e / D) * s.hq + h) * D + e % D] = 0;
    return;
  }

  const int32_t* __restrict__ rows = idx + int64_t(h) * total_k + ko0;
  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const uint32_t pitch = uint32_t(s.kv_tok) * 2u;   // a sequence's K spans < 4 GiB (checked on the host)
  const float zscale = s.scale * kLog2e;
  const int ntiles = (c1 - c0 + kTile - 1) / kTile;
  char* ktile = lds[wave];
  char* vtile = lds[wave] + TILEB;

  KAddr<D> ka;
  ka.init(lane);
  VtAddr<D> vt;
  vt.init(lane);
  const uint32_t coff = (lane % CH) * 16;   // this lane's byte offset inside a gathered row
  // Registers are what bounds the number of gathered rows in flight, so per-lane LDS offsets are not
  // kept in registers across the loop: each round derives them again (one XOR each) from three values
  // it first passes through opaque(), which keeps the compiler from hoisting the derived ones.
  auto opaque = [](int x) {
    asm volatile("" : "+v"(x));
    return x;
  };

  for (int qt = 0; qt * 32 < nq; ++qt) {
    // Q tile -> LDS: thread f takes chunk f % CH of query row f / CH (zeros past the last query)
    {
      constexpr int NQL = kTile * CH / (kWaves * 64);
#pragma unroll
      for (int i = 0; i < NQL; ++i) {
        const int f = i * kWaves * 64 + threadIdx.x, r = f / CH, c = f % CH;
        const int qi = qt * 32 + r;
        v4u x = v4u{0u, 0u, 0u, 0u};
        if (qi < nq)
          x = *reinterpret_cast<const v4u*>(q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head + c * 8);
        *reinterpret_cast<v4u*>(qtile + tile_off<D>(r, c)) = x;
      }
    }
    float m_used = -INFINITY, lsum = 0.0f;
    f32x16 acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][i] = 0.0f;

    // Kept-row ids of every tile this wave will walk go to LDS once (positions past the end repeat
    // the last kept row; such rows are masked out of the softmax below).
    int* my_rows = sm_rows[wave];
#pragma unroll
    for (int j = 0; j < kMaxTilesPerWave / 2; ++j) {
      const int slot = j * 64 + lane;   // tile slot / 32, row slot % 32 of this wave
      const int t = min(c0 + (wave + (slot >> 5) * kWaves) * kTile + (slot & 31), c1 - 1);
      my_rows[slot] = idx != nullptr ? rows[t] : t;   // NULL idx: identity lists (a packed cache)
    }
    __syncthreads();   // Q tile and row ids are in place
    // gather the wave's j-th tile into a register buffer
    auto fetch = [&](v4u (&kr)[NLD], v4u (&vr)[NLD], int j) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const uint32_t off = __umul24(uint32_t(my_rows[j * kTile + (i * 64 + lane) / CH]), pitch) + coff;
        kr[i] = load_once(kbase + off);
        vr[i] = load_once(vbase + off);
      }
    };
    // one tile: registers -> LDS, refill the registers with the tile after next, then the math
    auto round = [&](v4u (&kr)[NLD], v4u (&vr)[NLD], int j, int tile) {
      KAddr<D> kar;
      kar.base = opaque(ka.base);
      VtAddr<D> vtr;
      vtr.base[0] = opaque(vt.base[0]);
      vtr.base[1] = opaque(vt.base[1]);
      const int lane_o = opaque(lane);
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int f = i * 64 + lane_o, woff = tile_off<D>(f / CH, f % CH);
        *reinterpret_cast<v4u*>(ktile + woff) = kr[i];
        *reinterpret_cast<v4u*>(vtile + woff) = vr[i];
      }
      if (tile + kDepth * kWaves < ntiles) fetch(kr, vr, j + kDepth);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      sparse_tile_math<D>(ktile, vtile, qtile, kar, vtr, hf, c1 - (c0 + tile * kTile), zscale, m_used, lsum, acc);
      __builtin_amdgcn_wave_barrier();
    };

    if constexpr (kDepth == 2) {
      v4u kra[NLD], vra[NLD], krb[NLD], vrb[NLD];
      int tile = wave, j = 0;
      if (tile < ntiles) fetch(kra, vra, 0);
      if (tile + kWaves < ntiles) fetch(krb, vrb, 1);
      while (tile < ntiles) {
        round(kra, vra, j, tile);
        tile += kWaves;
        ++j;
        if (tile >= ntiles) break;
        round(krb, vrb, j, tile);
        tile += kWaves;
        ++j;
      }
    } else {
      v4u kra[NLD], vra[NLD];
      int tile = wave;
      if (tile < ntiles) fetch(kra, vra, 0);
      for (int j = 0; tile < ntiles; ++j, tile += kWaves) round(kra, vra, j, tile);
    }

    // ---- merge the four waves' (m, l, O^T) through LDS.  Every wave leaves its own running maximum,
    // row sum and unscaled accumulators in LDS that only it has used (its kept-row ids and its tile
    // buffers), so one barrier is enough; the wave that reduces a head_dim block applies the factors
    // exp2(m_w - m) while it adds.
    const float l = sum_across_halves(lsum);
    float* sm_ml = reinterpret_cast<float*>(&sm_rows[0][0]);   // [wave][m: 32 | l: 32], row stride = a wave's id area
    constexpr int kMlStride = kMaxTilesPerWave * kTile;
    if (hf == 0) {
      sm_ml[wave * kMlStride + col] = m_used;
      sm_ml[wave * kMlStride + 32 + col] = l;
    }
    float4* mrg = reinterpret_cast<float4*>(&lds[0][0]);         // [wave][db][quad][lane], 16 bytes per lane
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        mrg[((wave * NDB + db) * 4 + i4) * 64 + lane] =
            make_float4(acc[db][4 * i4 + 0], acc[db][4 * i4 + 1], acc[db][4 * i4 + 2], acc[db][4 * i4 + 3]);
    __syncthreads();
    if (wave < NDB) {
      const int db = wave;
      float m_all = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, sm_ml[w * kMlStride + col]);
      float f[kWaves];
      float l_all = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        f[w] = __builtin_amdgcn_exp2f(sm_ml[w * kMlStride + col] - m_all);   // 0 for a wave that saw no tile
        l_all += sm_ml[w * kMlStride + 32 + col] * f[w];
      }
      float outv[16];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float4 x = mrg[((w * NDB + db) * 4 + i4) * 64 + lane];
          a.x += x.x * f[w]; a.y += x.y * f[w]; a.z += x.z * f[w]; a.w += x.w * f[w];
        }
        outv[4 * i4 + 0] = a.x; outv[4 * i4 + 1] = a.y; outv[4 * i4 + 2] = a.z; outv[4 * i4 + 3] = a.w;
      }
      const int qi = qt * 32 + col;
      if (qi < nq) {
        if (nch_b == 1) {
          const float inv = 1.0f / l_all;
          uint16_t* op = o + (int64_t(q0 + qi) * s.hq + h) * D + db * 32 + 4 * hf;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            v2u w2;
            w2.x = cvt_pk_bf16(outv[4 * i4 + 0] * inv, outv[4 * i4 + 1] * inv);
            w2.y = cvt_pk_bf16(outv[4 * i4 + 2] * inv, outv[4 * i4 + 3] * inv);
            *reinterpret_cast<v2u*>(op + 8 * i4) = w2;
          }
        } else {
          const int64_t slot = (int64_t(chunk) * s.total_q + (q0 + qi)) * s.hq + h;
          float* pp = po + slot * D + db * 32 + 4 * hf;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4)
            *reinterpret_cast<float4*>(pp + 8 * i4) =
                make_float4(outv[4 * i4 + 0], outv[4 * i4 + 1], outv[4 * i4 + 2], outv[4 * i4 + 3]);
          if (db == 0 && hf == 0) { pm[slot] = m_all; pl[slot] = l_all; }
        }
      }
    }
    if ((qt + 1) * 32 < nq) __syncthreads();   // merge space becomes tile space again
  }
}

// The same computation for batches with more lists than compute units and lists of unequal length.
// A one-dimensional grid of one eight-wave workgroup per compute unit shares out all (sequence, head,
// chunk) items, sequences sorted by descending number of kept rows, in serpentine order (item i of turn
// r goes to workgroup i or gridDim.x - 1 - i), so that every workgroup walks about the same number of kept
// rows; a workgroup walks its items shortest first, each with all its waves (a "pass" is one query
// tile of one item).  Passes are pipelined: while one is walked, the queries and the kept-row ids of
// the next go from global memory straight into a second pair of LDS buffers, and a wave's last round
// already gathers its first tile of the next pass, so that those rows are in flight while the waves
// merge.  LDS holds the eight waves' tiles, two query tiles and two sets of ids: 160 KB at D = 128.
// STREAM: the lists are the identity (idx = NULL: a packed cache, rows cu_k[b] .. cu_k[b+1]-1 of every head in
// place).  No ids are fetched, staged or read back: a wave's tile is 32 consecutive rows from one base.
template <int D, bool STREAM>
__global__ __launch_bounds__(kWavesMulti * 64, 1) void attend_sparse_multi_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cu_k, int32_t total_k, const uint8_t* __restrict__ seq_mode,
    uint16_t* __restrict__ o, float* __restrict__ po, float* __restrict__ pm, float* __restrict__ pl,
    int32_t chunk_rows, int32_t n_chunks, int32_t n_wg, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int WAVES = kWavesMulti;   // n_wg: the size of the grid, as an argument like the others
  constexpr int CH = D / 8;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kTile * ROWB;
  constexpr int NLD = kTile * CH / 64;
  constexpr int NDB = D / 32;
  constexpr int kIds = kMultiTilesPerWave * kTile;   // ids per wave and pass

  __shared__ __attribute__((aligned(16))) char lds[WAVES][2 * TILEB];   // per wave: K tile, V tile; merge space
  __shared__ __attribute__((aligned(16))) char qtile[2][TILEB];          // queries of the current and the next pass
  __shared__ __attribute__((aligned(16))) int sm_rows[2][WAVES][kIds];   // kept-row ids of both; (m, l) at the merge

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  // Every kernel argument is fetched now, next to the loads of the batch's offsets, and not where it
  // is first used: the first pass cannot start before the last of them has arrived.
  {
    auto fetch_now = [](auto x) { asm volatile("" ::"s"(x)); };
    fetch_now(q); fetch_now(k); fetch_now(v); fetch_now(idx); fetch_now(seq_mode); fetch_now(o);
    fetch_now(total_k); fetch_now(chunk_rows); fetch_now(n_chunks); fetch_now(n_wg);
    fetch_now(s.batch); fetch_now(s.hq); fetch_now(s.group); fetch_now(s.q_tok); fetch_now(s.q_head);
    fetch_now(s.kv_tok); fetch_now(s.kv_head); fetch_now(s.total_q); fetch_now(s.scale);
  }
  const BatchInfo bi = load_batch(cu_q, cu_kv, cu_k, s.batch, lane, true);
  const int n_items = n_chunks * s.hq * s.batch;
  const uint32_t pitch = uint32_t(s.kv_tok) * 2u;
  const float zscale = s.scale * kLog2e;

  struct Pass {
    int h, chunk, qt, q0, nq, c0, c1, nch, ntiles;
    const int32_t* rows;
    const char *kbase, *vbase;
  };
  // the next pass of this workgroup: the next query tile of the item, else the next item that has work
  int turn = (n_items + n_wg - 1) / n_wg;
  auto next_pass = [&](Pass& p, bool have) -> bool {
    if (have && (p.qt + 1) * 32 < p.nq) {
      ++p.qt;
      return true;
    }
    while (--turn >= 0) {
      const int item = turn * n_wg + ((turn & 1) ? n_wg - 1 - int(blockIdx.x) : int(blockIdx.x));
      if (item >= n_items) continue;
      // (unsigned divisions, and none by n_chunks when every list is one chunk: this runs before the
      // first load of a pass can be issued)
      const uint32_t pair = n_chunks == 1 ? uint32_t(item) : uint32_t(item) / uint32_t(n_chunks);
      const int chunk = n_chunks == 1 ? 0 : int(uint32_t(item) - pair * uint32_t(n_chunks));
      const int z = int(pair / uint32_t(s.hq)), h = int(pair - uint32_t(z) * uint32_t(s.hq));
      const SeqInfo si = sequence_of_slot(bi, cu_q, cu_kv, cu_k, s.batch, z, lane, true);
      if (seq_mode != nullptr && seq_mode[si.b] == DLLM_SEQ_DENSE) continue;
      const ChunkGeom cg = chunk_geom(si.kb, chunk_rows);
      const int c0 = chunk * cg.rows;
      if (c0 >= si.kb && !(chunk == 0 && si.kb == 0)) continue;
      if (si.kb == 0) {   // nothing kept: defined as zeros
        for (int e = threadIdx.x; e < si.nq * D; e += WAVES * 64)
          o[(int64_t(si.q0 + e / D) * s.hq + h) * D + e % D] = 0;
        continue;
      }
      if (si.nq == 0) continue;
      const int g = h / s.group;
      p.h = h; p.chunk = chunk; p.qt = 0; p.q0 = si.q0; p.nq = si.nq;
      p.c0 = c0; p.c1 = min(si.kb, c0 + cg.rows); p.nch = cg.n;
      p.ntiles = (p.c1 - p.c0 + kTile - 1) / kTile;
      p.rows = idx + int64_t(h) * total_k + si.ko0;
      p.kbase = reinterpret_cast<const char*>(k + int64_t(si.kv0) * s.kv_tok + int64_t(g) * s.kv_head);
      p.vbase = reinterpret_cast<const char*>(v + int64_t(si.kv0) * s.kv_tok + int64_t(g) * s.kv_head);
      return true;
    }
    return false;
  };
  // queries and this wave's kept-row ids of pass p -> LDS buffers bf, without passing through registers
  // (positions past the end repeat the last kept row, rows past the last query repeat the last query:
  // such rows are masked out of the softmax, such columns are never stored)
  auto prefetch = [&](const Pass& p, int bf) {
    if constexpr (!STREAM) {
#pragma unroll
      for (int j = 0; j < kIds / 64; ++j) {
        const int slot = j * 64 + lane;
        const int t = min(p.c0 + (wave + (slot >> 5) * WAVES) * kTile + (slot & 31), p.c1 - 1);
        load4_to_lds(p.rows + t, __builtin_amdgcn_readfirstlane(lds_addr(&sm_rows[bf][wave][j * 64])));
      }
    }
    if (kTile * CH >= WAVES * 64 || threadIdx.x < kTile * CH) {
      const int r = threadIdx.x / CH, c = (threadIdx.x % CH) ^ tile_swz<D>(r);
      const int qi = min(p.qt * 32 + r, p.nq - 1);
      load16_to_lds(q + int64_t(p.q0 + qi) * s.q_tok + int64_t(p.h) * s.q_head + c * 8,
                    __builtin_amdgcn_readfirstlane(lds_addr(qtile[bf]) + wave * 1024));
    }
  };
  static_assert(kTile * CH <= WAVES * 64, "one 16-byte query chunk per thread");

  char* ktile = lds[wave];
  char* vtile = lds[wave] + TILEB;
  KAddr<D> ka;
  ka.init(lane);
  VtAddr<D> vt;
  vt.init(lane);
  const uint32_t coff = (lane % CH) * 16;
  auto opaque = [](int x) {
    asm volatile("" : "+v"(x));
    return x;
  };
  // gather tile `tile` of pass p (its ids lie where the wave tile % WAVES put them)
  auto fetch = [&](v4u (&kr)[NLD], v4u (&vr)[NLD], const Pass& p, int bf, int tile) {
    if constexpr (STREAM) {
      // rows c0 + tile * 32 ..: positions past the end repeat the last row (masked in the softmax)
      const int first = p.c0 + tile * kTile;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const uint32_t off = __umul24(uint32_t(min(first + (i * 64 + lane) / CH, p.c1 - 1)), pitch) + coff;
        kr[i] = load_once(p.kbase + off);
        vr[i] = load_once(p.vbase + off);
      }
    } else {
      const int* my_rows = sm_rows[bf][tile % WAVES] + (tile / WAVES) * kTile;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const uint32_t off = __umul24(uint32_t(my_rows[(i * 64 + lane) / CH]), pitch) + coff;
        kr[i] = load_once(p.kbase + off);
        vr[i] = load_once(p.vbase + off);
      }
    }
  };

  Pass cur, nxt;
  if (!next_pass(cur, false)) return;
  int bf = 0;
  v4u kra[NLD], vra[NLD];
  if constexpr (STREAM) {   // nothing to wait for before the first rows are asked for
    if (wave < cur.ntiles) fetch(kra, vra, cur, 0, wave);
    prefetch(cur, 0);
    wait_tile_loads();
  } else {
    prefetch(cur, 0);
    wait_tile_loads();
    if (wave < cur.ntiles) fetch(kra, vra, cur, 0, wave);
  }
  __syncthreads();   // the queries are in place
  for (;;) {
    nxt = cur;
    const bool more = next_pass(nxt, true);
    if (more) prefetch(nxt, bf ^ 1);
    // what a wave does once its own tiles of this pass are on their way: its first tile of the next
    auto start_next = [&]() {
      if (more) {
        wait_tile_loads();   // the next pass's ids (nothing else is outstanding here)
        if (wave < nxt.ntiles) fetch(kra, vra, nxt, bf ^ 1, wave);
      }
    };
    float m_used = -INFINITY, lsum = 0.0f;
    f32x16 acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][i] = 0.0f;
    if (wave >= cur.ntiles) start_next();
    // A wave's first tile of a pass is tile `wave` (gathered before the pass starts, from ids the wave
    // loaded itself); the later ones (later_tile) may have ids another wave loaded, which are in place:
    // every wave waited for its id loads before the barrier that opened this pass.
    int taken = 0;   // tiles of this pass this wave has taken after its first
    for (int tile = wave; tile < cur.ntiles;) {
      KAddr<D> kar;
      kar.base = opaque(ka.base);
      VtAddr<D> vtr;
      vtr.base[0] = opaque(vt.base[0]);
      vtr.base[1] = opaque(vt.base[1]);
      const int lane_o = opaque(lane);
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int f = i * 64 + lane_o, woff = tile_off<D>(f / CH, f % CH);
        *reinterpret_cast<v4u*>(ktile + woff) = kra[i];
        *reinterpret_cast<v4u*>(vtile + woff) = vra[i];
      }
      const int next = later_tile(wave, taken++);
      if (next < cur.ntiles) fetch(kra, vra, cur, bf, next);
      else start_next();
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      sparse_tile_math<D>(ktile, vtile, qtile[bf], kar, vtr, hf, cur.c1 - (cur.c0 + tile * kTile), zscale, m_used,
                          lsum, acc);
      __builtin_amdgcn_wave_barrier();
      tile = next;
    }

    // ---- merge the eight waves' (m, l, O^T) through LDS (see attend_sparse_bf16_kernel)
    const float l = sum_across_halves(lsum);
    float* sm_ml = reinterpret_cast<float*>(&sm_rows[bf][0][0]);   // [wave][m: 32 | l: 32]
    if (hf == 0) {
      sm_ml[wave * kIds + col] = m_used;
      sm_ml[wave * kIds + 32 + col] = l;
    }
    float4* mrg = reinterpret_cast<float4*>(&lds[0][0]);
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        mrg[((wave * NDB + db) * 4 + i4) * 64 + lane] =
            make_float4(acc[db][4 * i4 + 0], acc[db][4 * i4 + 1], acc[db][4 * i4 + 2], acc[db][4 * i4 + 3]);
    __syncthreads();
    {
      // every wave reduces a quarter or an eighth of the tile: head_dim block db, register quads i4_0 ...
      constexpr int PARTS = WAVES / NDB, NQ4 = 4 / PARTS;
      static_assert(WAVES % NDB == 0 && 4 % PARTS == 0, "the waves split the output evenly");
      const int db = wave % NDB, i4_0 = (wave / NDB) * NQ4;
      float m_all = -INFINITY;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) m_all = fmaxf(m_all, sm_ml[w * kIds + col]);
      float f[WAVES];
      float l_all = 0.0f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        f[w] = __builtin_amdgcn_exp2f(sm_ml[w * kIds + col] - m_all);   // 0 for a wave that saw no tile
        l_all += sm_ml[w * kIds + 32 + col] * f[w];
      }
      float outv[4 * NQ4];
#pragma unroll
      for (int n = 0; n < NQ4; ++n) {
        float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
          const float4 x = mrg[((w * NDB + db) * 4 + i4_0 + n) * 64 + lane];
          a.x += x.x * f[w]; a.y += x.y * f[w]; a.z += x.z * f[w]; a.w += x.w * f[w];
        }
        outv[4 * n + 0] = a.x; outv[4 * n + 1] = a.y; outv[4 * n + 2] = a.z; outv[4 * n + 3] = a.w;
      }
      const int qi = cur.qt * 32 + col;
      if (qi < cur.nq) {
        if (cur.nch == 1) {
          const float inv = 1.0f / l_all;
          uint16_t* op = o + (int64_t(cur.q0 + qi) * s.hq + cur.h) * D + db * 32 + 4 * hf;
#pragma unroll
          for (int n = 0; n < NQ4; ++n) {
            v2u w2;
            w2.x = cvt_pk_bf16(outv[4 * n + 0] * inv, outv[4 * n + 1] * inv);
            w2.y = cvt_pk_bf16(outv[4 * n + 2] * inv, outv[4 * n + 3] * inv);
            *reinterpret_cast<v2u*>(op + 8 * (i4_0 + n)) = w2;
          }
        } else {
          const int64_t slot = (int64_t(cur.chunk) * s.total_q + (cur.q0 + qi)) * s.hq + cur.h;
          float* pp = po + slot * D + db * 32 + 4 * hf;
#pragma unroll
          for (int n = 0; n < NQ4; ++n)
            *reinterpret_cast<float4*>(pp + 8 * (i4_0 + n)) =
                make_float4(outv[4 * n + 0], outv[4 * n + 1], outv[4 * n + 2], outv[4 * n + 3]);
          if (wave == 0 && hf == 0) { pm[slot] = m_all; pl[slot] = l_all; }
        }
      }
    }
    if (!more) break;
    __syncthreads();   // merge space becomes tile space again; the next pass's queries are in place
    cur = nxt;
    bf ^= 1;
  }
}

// Merge the chunk partials of every (sequence, head) that needed more than one chunk.
// One workgroup per (head, sequence): 8 threads per query row, each owning D/8 output elements,
// so all loads of a row are independent and issued together.
template <int D>
__global__ __launch_bounds__(256) void attend_sparse_combine_kernel(
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k, const uint8_t* __restrict__ seq_mode,
    const float* __restrict__ po, const float* __restrict__ pm, const float* __restrict__ pl,
    uint16_t* __restrict__ o, int32_t chunk_rows, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  const int h = blockIdx.x, b = blockIdx.y;
  if (seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE) return;
  const int kb = cu_k[b + 1] - cu_k[b];
  const int nch = chunk_geom(kb, chunk_rows).n;
  if (nch <= 1) return;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  constexpr int EPT = D / 8;   // elements per thread
  const int sub = threadIdx.x & 7;
  for (int i = threadIdx.x >> 3; i < nq; i += 32) {
    float m_all = -INFINITY;
    for (int c = 0; c < nch; ++c) m_all = fmaxf(m_all, pm[(int64_t(c) * s.total_q + (q0 + i)) * s.hq + h]);
    float l_all = 0.0f, a[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) a[e] = 0.0f;
    for (int c = 0; c < nch; ++c) {
      const int64_t slot = (int64_t(c) * s.total_q + (q0 + i)) * s.hq + h;
      const float w = __builtin_amdgcn_exp2f(pm[slot] - m_all);
      l_all += pl[slot] * w;
      const float4* src = reinterpret_cast<const float4*>(po + slot * D + sub * EPT);
#pragma unroll
      for (int e = 0; e < EPT / 4; ++e) {
        const float4 x = src[e];
        a[4 * e + 0] += x.x * w; a[4 * e + 1] += x.y * w; a[4 * e + 2] += x.z * w; a[4 * e + 3] += x.w * w;
      }
    }
    const float inv = 1.0f / l_all;
    uint16_t* op = o + (int64_t(q0 + i) * s.hq + h) * D + sub * EPT;
#pragma unroll
    for (int e = 0; e < EPT; e += 2)
      *reinterpret_cast<uint32_t*>(op + e) = cvt_pk_bf16(a[e] * inv, a[e + 1] * inv);
  }
}

hipError_t launch_attend_sparse_bf16(const Shape& s, const AttendPlan& p, const void* q, const void* k,
                                     const void* v, const int32_t* cu_q, const int32_t* cu_kv, const int32_t* idx,
                                     const int32_t* cu_k, int32_t total_k, const uint8_t* seq_mode, void* o,
                                     void* ws, hipStream_t st) {
  if (s.max_q == 0) return hipSuccess;   // no sequence has a query: nothing to write
  char* w = static_cast<char*>(ws);
  float* po = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_po) : nullptr;
  float* pm = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_pm) : nullptr;
  float* pl = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_pl) : nullptr;
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  uint16_t* oh = static_cast<uint16_t*>(o);
  // More lists than compute units, and lists of unequal length (the longest at least 1.5 times the mean
  // over the batch): one eight-wave workgroup per compute unit walks its share of them.  With lists of
  // equal length one list per workgroup is faster (40 against 44 us on the mixed workload's Reuse part).
  int dev = 0, n_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  const int64_t n_items = int64_t(p.n_chunks) * s.hq * s.batch;
  const bool multi = n_items > n_cu && n_items < (int64_t(1) << 30) &&
                     p.chunk_rows <= kMultiTilesPerWave * kWavesMulti * kTile &&
                     2 * int64_t(p.max_k) * s.batch >= 3 * int64_t(total_k);
  if (multi) {
    auto launch = [&](auto kernel) {
      kernel<<<n_cu, kWavesMulti * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k, seq_mode, oh, po, pm, pl,
                                                 p.chunk_rows, p.n_chunks, n_cu, s DLLM_CHECK_PASS);
    };
    if (idx == nullptr) {
      if (s.d == 128) launch(attend_sparse_multi_bf16_kernel<128, true>);
      else launch(attend_sparse_multi_bf16_kernel<64, true>);
    } else {
      if (s.d == 128) launch(attend_sparse_multi_bf16_kernel<128, false>);
      else launch(attend_sparse_multi_bf16_kernel<64, false>);
    }
  } else {
    dim3 grid(p.n_chunks, s.hq, s.batch);
    // the start order only matters when the workgroups cannot all be resident at once (two per compute unit)
    const int ranked = n_items > 512 ? 1 : 0;
    if (s.d == 128)
      attend_sparse_bf16_kernel<128><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                                  seq_mode, oh, po, pm, pl, p.chunk_rows, ranked, s DLLM_CHECK_PASS);
    else
      attend_sparse_bf16_kernel<64><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                                 seq_mode, oh, po, pm, pl, p.chunk_rows, ranked, s DLLM_CHECK_PASS);
  }
  e = hipGetLastError();
  if (e != hipSuccess || p.n_chunks <= 1) return e;
  dim3 cgrid(s.hq, s.batch);
  if (s.d == 128)
    attend_sparse_combine_kernel<128><<<cgrid, 256, 0, st>>>(cu_q, cu_k, seq_mode, po, pm, pl, oh, p.chunk_rows, s DLLM_CHECK_PASS);
  else
    attend_sparse_combine_kernel<64><<<cgrid, 256, 0, st>>>(cu_q, cu_k, seq_mode, po, pm, pl, oh, p.chunk_rows, s DLLM_CHECK_PASS);
  return hipGetLastError();
}

}  // namespace dllm
