// Reuse-phase attention over each head's kept rows (Section 2.3 Eq. 4 restricted to the kept set of
// Section 4.5), bf16 inputs, fp32 softmax state and accumulators, on the gfx950 matrix cores.
//
// The step is bound by HBM: every kept (head, row) pair costs one 2*D-byte K row and one V row and
// only 4*Bq*D flop.  What decides its speed is how many gathered rows are in flight, so the registers
// go to the gathers: a workgroup of four waves walks one chunk of one (sequence, head)'s kept rows,
// each wave owns its own 32-row tiles (no workgroup barrier in the loop) and keeps TWO tiles of K and
// V rows in flight in registers; the queries, which every step needs again, live in LDS instead.
//   gather   idx -> row offsets (32-bit, from a uniform base); 16-byte non-temporal loads with a row's
//            chunks in neighbouring lanes (whole 256-byte rows per 16 lanes)
//   stage    registers -> the wave's private LDS tile, XOR-swizzled by row; the freed registers are
//            refilled with the tile after next at once
//   S^T      = K_tile (32 keys x D) * Q^T (D x 32 queries): A and B by ds_read_b128
//   softmax  online, base 2, lazily rescaled, per query column
//   O^T     += V_tile^T * P^T: A by ds_read_b64_tr_b16, B = the S^T accumulators in place
// After the loop the four waves merge (m, l, O) through LDS (one barrier).  A (sequence, head) whose kept rows fit
// one chunk writes O directly; otherwise chunks write fp32 partials and a small kernel merges them.
#include "attn_tile.h"

namespace dllm {

constexpr int kTile = 32;        // kept rows per wave tile
constexpr int kWaves = 4;
constexpr float kLazyStepS = 8.0f;
constexpr int kMaxTilesPerWave = 16;  // chunk_rows <= kMaxTilesPerWave * kWaves * kTile
#ifndef DLLM_SPARSE_DEPTH
#define DLLM_SPARSE_DEPTH 1
#endif
constexpr int kDepth = DLLM_SPARSE_DEPTH;   // tiles of gathered rows a wave keeps in flight in registers
constexpr int kRankBatch = 64;        // batches up to this size are walked longest kept list first

// A (sequence, head) with kb kept rows is cut into n = ceil(kb / chunk_rows) chunks of equal size
// (rounded up to the 128 rows four waves take per step), so no chunk is a short leftover.
struct ChunkGeom {
  int n, rows;
};
__device__ __forceinline__ ChunkGeom chunk_geom(int kb, int chunk_rows) {
  ChunkGeom g;
  g.n = (kb + chunk_rows - 1) / chunk_rows;
  g.rows = g.n <= 1 ? chunk_rows : ((kb + g.n - 1) / g.n + 127) / 128 * 128;
  return g;
}

// Per-sequence offsets a workgroup needs, fetched for the whole (small) batch in one round of
// loads: lane i holds sequence i's entries, and the chosen sequence's are read back by lane index.
struct SeqInfo {
  int b, ko0, kb, q0, nq, kv0;
};

// Sequence handled by grid slot z.  With `ranked` set (small batches whose workgroups do not all fit
// on the chip at once) sequences are taken in descending order of kept rows (ties: lower sequence
// first), so the longest lists start first and the short ones fill the compute units that free up;
// every workgroup derives the same order from cu_k.
__device__ __forceinline__ SeqInfo sequence_of_slot(const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv,
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
  const int i = lane < batch ? lane : batch - 1;
  const int ko0 = cu_k[i], kb = cu_k[i + 1] - ko0;
  const int q0 = cu_q[i], nq = cu_q[i + 1] - q0;
  const int kv0 = cu_kv[i];
  int b = z;
  if (ranked) {
    const int mine = lane < batch ? kb : -1;
    int rank = 0;
    for (int j = 0; j < batch; ++j) {
      const int other = __builtin_amdgcn_readlane(mine, j);
      rank += (other > mine) || (other == mine && j < lane);
    }
    b = __builtin_ctzll(__builtin_amdgcn_ballot_w64(lane < batch && rank == z));
  }
  si.b = b;
  si.ko0 = __builtin_amdgcn_readlane(ko0, b);
  si.kb = __builtin_amdgcn_readlane(kb, b);
  si.q0 = __builtin_amdgcn_readlane(q0, b);
  si.nq = __builtin_amdgcn_readlane(nq, b);
  si.kv0 = __builtin_amdgcn_readlane(kv0, b);
  return si;
}

template <int D>
__global__ __launch_bounds__(kWaves * 64, 2) void attend_sparse_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cu_k, int32_t total_k, const uint8_t* __restrict__ seq_mode,
    uint16_t* __restrict__ o, float* __restrict__ po, float* __restrict__ pm, float* __restrict__ pl,
    int32_t chunk_rows, int ranked, Shape s) {
  constexpr int CH = D / 8;             // 16-byte chunks per row
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kTile * ROWB;
  constexpr int NLD = kTile * CH / 64;  // 16-byte loads per lane per tile and tensor
  constexpr int NT = D / 16;            // MFMA steps along head_dim
  constexpr int NDB = D / 32;           // 32-wide blocks of head_dim in the output

  // per wave: K tile then V tile; reused as fp32 merge space afterwards
  __shared__ __attribute__((aligned(16))) char lds[kWaves][2 * TILEB];
  // the 32 queries of the current query tile (same swizzled layout as a K tile)
  __shared__ __attribute__((aligned(16))) char qtile[TILEB];
  // kept-row ids of each wave's tiles; after the loop each wave leaves its (m, l) pairs in its own part
  __shared__ int sm_rows[kWaves][kMaxTilesPerWave * kTile];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
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

      // S^T tile: rows = keys, columns = queries
      f32x16 st;
#pragma unroll
      for (int i = 0; i < 16; ++i) st[i] = 0.0f;
#pragma unroll
      for (int t = 0; t < NT; ++t)
        st = mfma_bf16(*reinterpret_cast<const v4u*>(ktile + kar.off(t)),
                       *reinterpret_cast<const v4u*>(qtile + kar.off(t)), st);
      // issue order: operand fetches just ahead of their MFMA, so few operand registers are live
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);

      const int nvalid = c1 - (c0 + tile * kTile);
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
          const v2u lo = lds_read_tr16(vtile + vtr.off(0, db) + 16 * u * ROWB);
          const v2u hi = lds_read_tr16(vtile + vtr.off(1, db) + 16 * u * ROWB);
          acc[db] = mfma_bf16(v4u{lo.x, lo.y, hi.x, hi.y}, pb[u], acc[db]);
        }
#pragma unroll
      for (int i = 0; i < 2 * NDB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
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

// Merge the chunk partials of every (sequence, head) that needed more than one chunk.
// One workgroup per (head, sequence): 8 threads per query row, each owning D/8 output elements,
// so all loads of a row are independent and issued together.
template <int D>
__global__ __launch_bounds__(256) void attend_sparse_combine_kernel(
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k, const uint8_t* __restrict__ seq_mode,
    const float* __restrict__ po, const float* __restrict__ pm, const float* __restrict__ pl,
    uint16_t* __restrict__ o, int32_t chunk_rows, Shape s) {
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
  dim3 grid(p.n_chunks, s.hq, s.batch);
  // the start order only matters when the workgroups cannot all be resident at once (two per compute unit)
  const int ranked = int64_t(p.n_chunks) * s.hq * s.batch > 512 ? 1 : 0;
  if (s.d == 128)
    attend_sparse_bf16_kernel<128><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                                seq_mode, oh, po, pm, pl, p.chunk_rows, ranked, s);
  else
    attend_sparse_bf16_kernel<64><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                               seq_mode, oh, po, pm, pl, p.chunk_rows, ranked, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.n_chunks <= 1) return e;
  dim3 cgrid(s.hq, s.batch);
  if (s.d == 128)
    attend_sparse_combine_kernel<128><<<cgrid, 256, 0, st>>>(cu_q, cu_k, seq_mode, po, pm, pl, oh, p.chunk_rows, s);
  else
    attend_sparse_combine_kernel<64><<<cgrid, 256, 0, st>>>(cu_q, cu_k, seq_mode, po, pm, pl, oh, p.chunk_rows, s);
  return hipGetLastError();
}

}  // namespace dllm
