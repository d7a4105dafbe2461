// Reuse-phase attention over each head's kept rows (Section 2.3 Eq. 4 restricted to the kept set of
// Section 4.5), bf16 inputs, fp32 softmax state and accumulators, on the gfx950 matrix cores.
//
// The step is bound by HBM: every kept (head, row) pair costs one 2*D-byte K row and one V row and
// only 4*Bq*D flop.  A workgroup of four waves walks one chunk of one (sequence, head)'s kept rows;
// each wave owns its own 32-row tiles, so no workgroup barrier sits in the loop:
//   gather   idx -> row addresses; 16-byte loads with a row's chunks in neighbouring lanes (whole
//            256-byte rows per 16 lanes), prefetched one tile ahead into registers
//   stage    registers -> the wave's private LDS tile, XOR-swizzled by row
//   S^T      = K_tile (32 keys x D) * Q^T (D x 32 queries): v_mfma_f32_32x32x16_bf16, A from LDS, B = Q in registers
//   softmax  online, base 2, per query column: 16 registers in-lane plus one cross-half exchange
//   O^T     += V_tile^T (D x 32 keys) * P^T: P^T is the S^T accumulator re-used in place as B operand,
//            V^T gathered from the LDS tile in the matching key order
// After the loop the four waves merge (m, l, O) through LDS.  A (sequence, head) whose kept rows fit
// one chunk writes O directly; otherwise chunks write fp32 partials and a small kernel merges them.
#include "common.h"

namespace dllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTile = 32;        // kept rows per wave tile
constexpr int kWaves = 4;
constexpr float kLog2e = 1.4426950408889634f;

template <int CH>
__device__ __forceinline__ int swz_rows(int row) {
  constexpr int rows_per_line = CH >= 16 ? 1 : 16 / CH;
  return (row / rows_per_line) & (CH - 1);
}

template <int D>
__global__ __launch_bounds__(kWaves * 64) void attend_sparse_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cu_k, int32_t total_k, const uint8_t* __restrict__ seq_mode,
    uint16_t* __restrict__ o, float* __restrict__ po, float* __restrict__ pm, float* __restrict__ pl,
    int32_t chunk_rows, Shape s) {
  constexpr int CH = D / 8;          // 16-byte chunks per row
  constexpr int NLD = kTile * CH / 64;  // 16-byte loads per lane per tile and tensor
  constexpr int NT = D / 16;         // MFMA steps along head_dim
  constexpr int NDB = D / 32;        // 32-wide blocks of head_dim in the output

  // per wave: K tile then V tile (kTile*CH uint4 each); reused as fp32 merge space afterwards
  __shared__ uint4 lds[kWaves][2 * kTile * CH];
  __shared__ float sm_m[kWaves][32], sm_l[kWaves][32];

  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE) return;
  const int ko0 = cu_k[b], kb = cu_k[b + 1] - ko0;
  const int c0 = chunk * chunk_rows;
  if (c0 >= kb && !(chunk == 0 && kb == 0)) return;
  const int c1 = min(kb, c0 + chunk_rows);
  const int nch_b = (kb + chunk_rows - 1) / chunk_rows;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  const int kv0 = cu_kv[b];
  const int g = h / s.group;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;

  if (kb == 0) {  // nothing kept: defined as zeros
    for (int e = threadIdx.x; e < nq * D; e += kWaves * 64)
      o[(int64_t(q0 + e / D) * s.hq + h) * D + e % D] = 0;
    return;
  }

  const int32_t* __restrict__ rows = idx + int64_t(h) * total_k + ko0;
  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const int64_t pitch = s.kv_tok * 2;
  const float zscale = s.scale * kLog2e;
  const int ntiles = (c1 - c0 + kTile - 1) / kTile;
  uint4* ktile = lds[wave];
  uint4* vtile = lds[wave] + kTile * CH;
  const uint16_t* vt16 = reinterpret_cast<const uint16_t*>(vtile);

  for (int qt = 0; qt * 32 < nq; ++qt) {
    // Q^T operand: lane (col = query, hf) holds Q[query][16t + 8hf .. +8) for every step t
    uint4 qreg[NT];
    {
      const int qi = qt * 32 + col;
      const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        qreg[t] = make_uint4(0, 0, 0, 0);
        if (qi < nq) qreg[t] = *reinterpret_cast<const uint4*>(qp + 16 * t + 8 * hf);
      }
    }
    float m = -INFINITY, l = 0.0f;
    f32x16 acc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][i] = 0.0f;

    uint4 kr[NLD], vr[NLD];
    auto fetch = [&](int tile, int my_row) {
      // my_row: this lane's kept-row id for tile row (lane & 31), or -1 past the end
      (void)tile;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int f = i * 64 + lane, row = f / CH, c = f % CH;
        const int r = __shfl(my_row, row);
        kr[i] = make_uint4(0, 0, 0, 0);
        vr[i] = make_uint4(0, 0, 0, 0);
        if (r >= 0) {
          kr[i] = *reinterpret_cast<const uint4*>(kbase + r * pitch + c * 16);
          vr[i] = *reinterpret_cast<const uint4*>(vbase + r * pitch + c * 16);
        }
      }
    };
    auto row_of = [&](int tile) -> int {
      const int t = c0 + tile * kTile + col;
      return (tile < ntiles && t < c1) ? rows[t] : -1;
    };

    int tile = wave;
    int row_next = row_of(tile);
    if (tile < ntiles) fetch(tile, row_next);
    row_next = row_of(tile + kWaves);

    for (; tile < ntiles; tile += kWaves) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int f = i * 64 + lane, row = f / CH, c = f % CH;
        ktile[row * CH + (c ^ swz_rows<CH>(row))] = kr[i];
        vtile[row * CH + (c ^ swz_rows<CH>(row))] = vr[i];
      }
      if (tile + kWaves < ntiles) fetch(tile + kWaves, row_next);
      row_next = row_of(tile + 2 * kWaves);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // S^T tile: rows = keys, columns = queries
      f32x16 st;
#pragma unroll
      for (int i = 0; i < 16; ++i) st[i] = 0.0f;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const uint4 a = ktile[col * CH + ((2 * t + hf) ^ swz_rows<CH>(col))];
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                     __builtin_bit_cast(bf16x8, qreg[t]), st, 0, 0, 0);
      }
      // accumulator register i of lane (col, hf) is key 8*(i/4) + 4*hf + i%4 of the tile
      const int nvalid = c1 - (c0 + tile * kTile);
      float mloc = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = 8 * (i / 4) + 4 * hf + (i % 4);
        st[i] = key < nvalid ? st[i] * zscale : -INFINITY;
        mloc = fmaxf(mloc, st[i]);
      }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
      const float m_new = fmaxf(m, mloc);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      float psum = 0.0f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        st[i] = __builtin_amdgcn_exp2f(st[i] - m_new);
        psum += st[i];
      }
      l = l * alpha + psum;
      m = m_new;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] *= alpha;

      // O^T += V^T P^T, 16 keys per step; slot sl of lane half hf is key 16u + 8*(sl/4) + 4*hf + sl%4
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        uint4 pb;
        pb.x = pack_bf16x2(st[8 * u + 0], st[8 * u + 1]);
        pb.y = pack_bf16x2(st[8 * u + 2], st[8 * u + 3]);
        pb.z = pack_bf16x2(st[8 * u + 4], st[8 * u + 5]);
        pb.w = pack_bf16x2(st[8 * u + 6], st[8 * u + 7]);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int d = db * 32 + col;
          uint32_t w[4];
#pragma unroll
          for (int sp = 0; sp < 4; ++sp) {
            const int s0 = 2 * sp, s1 = 2 * sp + 1;
            const int key0 = 16 * u + 8 * (s0 / 4) + 4 * hf + (s0 % 4);
            const int key1 = 16 * u + 8 * (s1 / 4) + 4 * hf + (s1 % 4);
            const uint32_t lo = vt16[(key0 * CH + ((d >> 3) ^ swz_rows<CH>(key0))) * 8 + (d & 7)];
            const uint32_t hi = vt16[(key1 * CH + ((d >> 3) ^ swz_rows<CH>(key1))) * 8 + (d & 7)];
            w[sp] = lo | (hi << 16);
          }
          const uint4 a = make_uint4(w[0], w[1], w[2], w[3]);
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                          __builtin_bit_cast(bf16x8, pb), acc[db], 0, 0, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();
    }

    // ---- merge the four waves' (m, l, O^T) through LDS
    l += __shfl_xor(l, 32);
    __syncthreads();                       // every wave is done with its tile buffers
    if (hf == 0) { sm_m[wave][col] = m; sm_l[wave][col] = l; }
    __syncthreads();
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, sm_m[w][col]);
    float l_all = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) l_all += sm_l[w][col] * __builtin_amdgcn_exp2f(sm_m[w][col] - m_all);
    const float mine = __builtin_amdgcn_exp2f(m - m_all);   // 0 for a wave that saw no tile
    float* mrg = reinterpret_cast<float*>(&lds[0][0]);      // [wave][db][reg][lane]
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) mrg[((wave * NDB + db) * 16 + i) * 64 + lane] = acc[db][i] * mine;
    __syncthreads();
    if (wave < NDB) {
      const int db = wave;
      float outv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float a = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) a += mrg[((w * NDB + db) * 16 + i) * 64 + lane];
        outv[i] = a;
      }
      const int qi = qt * 32 + col;
      if (qi < nq) {
        if (nch_b == 1) {
          const float inv = 1.0f / l_all;
          uint16_t* op = o + (int64_t(q0 + qi) * s.hq + h) * D + db * 32 + 4 * hf;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            uint2 w2;
            w2.x = pack_bf16x2(outv[4 * i4 + 0] * inv, outv[4 * i4 + 1] * inv);
            w2.y = pack_bf16x2(outv[4 * i4 + 2] * inv, outv[4 * i4 + 3] * inv);
            *reinterpret_cast<uint2*>(op + 8 * i4) = w2;
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
    __syncthreads();                       // merge space becomes tile space again
  }
}

// Merge the chunk partials of every (sequence, head) that needed more than one chunk.
template <int D>
__global__ __launch_bounds__(256) void attend_sparse_combine_kernel(
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k, const uint8_t* __restrict__ seq_mode,
    const float* __restrict__ po, const float* __restrict__ pm, const float* __restrict__ pl,
    uint16_t* __restrict__ o, int32_t chunk_rows, Shape s) {
  const int h = blockIdx.x, b = blockIdx.y;
  if (seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE) return;
  const int kb = cu_k[b + 1] - cu_k[b];
  const int nch = (kb + chunk_rows - 1) / chunk_rows;
  if (nch <= 1) return;
  const int q0 = cu_q[b], nq = cu_q[b + 1] - q0;
  constexpr int RPB = 256 / D;   // query rows per pass
  const int d = threadIdx.x % D;
  for (int i = threadIdx.x / D; i < nq; i += RPB) {
    float m_all = -INFINITY;
    for (int c = 0; c < nch; ++c) m_all = fmaxf(m_all, pm[(int64_t(c) * s.total_q + (q0 + i)) * s.hq + h]);
    float l_all = 0.0f, a = 0.0f;
    for (int c = 0; c < nch; ++c) {
      const int64_t slot = (int64_t(c) * s.total_q + (q0 + i)) * s.hq + h;
      const float w = __builtin_amdgcn_exp2f(pm[slot] - m_all);
      l_all += pl[slot] * w;
      a += po[slot * D + d] * w;
    }
    o[(int64_t(q0 + i) * s.hq + h) * D + d] = uint16_t(f32_to_bf16_bits(a / l_all));
  }
}

hipError_t launch_attend_sparse_bf16(const Shape& s, const AttendPlan& p, const void* q, const void* k,
                                     const void* v, const int32_t* cu_q, const int32_t* cu_kv, const int32_t* idx,
                                     const int32_t* cu_k, int32_t total_k, const uint8_t* seq_mode, void* o,
                                     void* ws, hipStream_t st) {
  char* w = static_cast<char*>(ws);
  float* po = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_po) : nullptr;
  float* pm = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_pm) : nullptr;
  float* pl = p.n_chunks > 1 ? reinterpret_cast<float*>(w + p.off_pl) : nullptr;
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  uint16_t* oh = static_cast<uint16_t*>(o);
  dim3 grid(p.n_chunks, s.hq, s.batch);
  if (s.d == 128)
    attend_sparse_bf16_kernel<128><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                                seq_mode, oh, po, pm, pl, p.chunk_rows, s);
  else
    attend_sparse_bf16_kernel<64><<<grid, kWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, idx, cu_k, total_k,
                                                               seq_mode, oh, po, pm, pl, p.chunk_rows, s);
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
