// Selection: per-head importance scores (Section 4.5, Eq. 6) and per-head top-k.
//
// Kernels on the caller's stream:
//   score_kernel        qsum[h,:] = sum of the sequence's block queries (fp32, ascending rows), then
//                       one pass over K: s[h,j] = fma chain over d of qsum[h,d] * K[j, h/G, d]
//   head_sum_kernel     (head-summed selection only, Section 2.4 Eq. 5) the pooled scores summed over heads
//   topk_reg_kernel     per (sequence, head), lists of up to 4096 candidates: pooled keys in registers,
//                       radix select of the k-th largest, ordered compaction (ties to the lower
//                       position, output ascending)
//   topk_kernel         the same for longer lists, with the keys in LDS
//
// The score arithmetic is fixed (one fused multiply-add per d, ascending d, one lane owns one key),
// because the kept set must be reproducible bit for bit.  To keep the HBM reads coalesced while one
// lane owns a whole row, each wave stages 64 rows through LDS: 16-byte chunks are loaded so that a
// row's chunks sit in neighbouring lanes, written to LDS with an XOR swizzle, and read back one row
// per lane without bank conflicts.
#include <atomic>
#include <type_traits>
#include <utility>

#include "common.h"

namespace dllm {

// ------------------------------------------------------------------ score
constexpr int kScoreWaves = 4;
constexpr int kScoreRowsPerBlock = kScoreWaves * 64;

template <int CH>
__device__ __forceinline__ int swz(int row) {
  // chunk permutation that spreads 16 consecutive rows over the 16 sixteen-byte bank groups
  constexpr int rows_per_line = CH >= 16 ? 1 : 16 / CH;
  return (row / rows_per_line) & (CH - 1);
}

// ES: element bytes (2 = bf16, 4 = fp32); D: head_dim; GT: query heads scored per pass over the tile.
// Each wave walks `tiles_per_wave` consecutive 64-row tiles; while it scores one tile out of LDS the
// next tile's rows are already in flight into registers.
// acc += q[J + e] * kv[e] for e = 0 .. N-1 in this order, one fused multiply-add each, where q[j] is
// what lane j of this lane's row of 16 lanes holds in `vq`: v_fmac_f32 with the DPP row broadcast
// applied to its first operand, so the block sums reach the multiplier without scalar loads (which
// return out of order: every wait for one is a wait for all) and without an instruction of their own.
// The leading s_nop covers the two wait states a DPP read needs after a vector write of its source,
// should the compiler have copied `vq` just before.
template <int J, int N>
__device__ __forceinline__ float fma_row_bcast(float acc, float vq, const float (&kv)[N]) {
  static_assert(N == 4 || N == 8, "one 16-byte chunk of fp32 or bf16");
  static_assert(J % N == 0 && J + N <= 16, "the chunk lies inside one row of 16 sums");
  if constexpr (N == 8) {
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %1, %2 row_newbcast:%10 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %3 row_newbcast:%11 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %4 row_newbcast:%12 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %5 row_newbcast:%13 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %6 row_newbcast:%14 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %7 row_newbcast:%15 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %8 row_newbcast:%16 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %9 row_newbcast:%17 row_mask:0xf bank_mask:0xf"
        : "+v"(acc)
        : "v"(vq), "v"(kv[0]), "v"(kv[1]), "v"(kv[2]), "v"(kv[3]), "v"(kv[4]), "v"(kv[5]), "v"(kv[6]), "v"(kv[7]),
          "n"(J), "n"(J + 1), "n"(J + 2), "n"(J + 3), "n"(J + 4), "n"(J + 5), "n"(J + 6), "n"(J + 7));
  } else {
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %1, %2 row_newbcast:%6 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %3 row_newbcast:%7 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %4 row_newbcast:%8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %1, %5 row_newbcast:%9 row_mask:0xf bank_mask:0xf"
        : "+v"(acc)
        : "v"(vq), "v"(kv[0]), "v"(kv[1]), "v"(kv[2]), "v"(kv[3]), "n"(J), "n"(J + 1), "n"(J + 2), "n"(J + 3));
  }
  return acc;
}

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ... in order
template <typename F, int... C>
__device__ __forceinline__ void for_each_index(F& f, std::integer_sequence<int, C...>) {
  (f(std::integral_constant<int, C>{}), ...);
}

template <int ES, int D, int GT>
__global__ __launch_bounds__(kScoreWaves * 64, (ES * D <= 256 ? 2 : 1)) void score_kernel(
    const char* __restrict__ k, const char* __restrict__ q, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k, float* __restrict__ scores,
    int tiles_per_wave, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int ROWB = D * ES;
  constexpr int CH = ROWB / 16;   // 16-byte chunks per row
  constexpr int EPC = 16 / ES;    // elements per chunk
  __shared__ v4u tile[kScoreWaves][64 * CH];
  extern __shared__ __attribute__((aligned(16))) float sums[];   // [group][D]: block sums of this KV head's query heads

  // KV head is the fastest grid index: workgroups launched together read neighbouring 2*D-byte
  // slices of the same token rows, which keeps the DRAM pages they open busy.  Consecutive workgroups
  // go to consecutive XCDs, so the head is rotated by the sequence: otherwise an XCD would only ever
  // fetch the same 1/8 of the 256-byte columns (measured: 4 % on the batched workload).  Within a
  // sequence an XCD keeps its heads, so their block queries are fetched into its L2 once (rotating by
  // the row block as well cost 12 % more bytes fetched on the grouped-query workload).
  const int b = blockIdx.z, g = (blockIdx.x + blockIdx.z) % s.hkv;
  // All offsets in one round trip: the memory system is busy with the K stream, and every dependent
  // scalar load before the first tile request costs this workgroup a microsecond or more.
  int ck0 = cu_k[b], ck1 = cu_k[b + 1], kv0 = cu_kv[b], kv1 = cu_kv[b + 1], q0 = cu_q[b], q1 = cu_q[b + 1];
  asm volatile("" : "+s"(ck0), "+s"(ck1), "+s"(kv0), "+s"(kv1), "+s"(q0), "+s"(q1));   // keeps the loads above the branches
  if (ck1 == ck0) return;
  const int L = kv1 - kv0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (blockIdx.y * kScoreWaves * tiles_per_wave * 64 >= L) return;   // the whole workgroup lies past the end
  const int first = (blockIdx.y * kScoreWaves + wave) * tiles_per_wave * 64;
  const int ntiles = first < L ? min(tiles_per_wave, (L - first + 63) / 64) : 0;   // 0: only helps with the sums
  const char* base = k + (int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head) * ES + (lane % CH) * 16;
  const int64_t row_pitch = s.kv_tok * ES;
  v4u* mine = tile[wave];
  const int sw = swz<CH>(lane);

  v4u regs[CH];
  // rows past the end of the sequence re-read its last row; their scores are never stored
  auto fetch = [&](int r0) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int row = min(r0 + (i * 64 + lane) / CH, L - 1);
      regs[i] = load_once(base + row * row_pitch);
    }
  };
  if (ntiles > 0) fetch(first);

  // While the first rows are on their way: the block sums of this KV head's query heads,
  // sum[hh][d] = sum over the block's query rows in ascending row order, fp32 (the canonical order).
  // Every workgroup computes the few hundred sums it needs itself (the block's queries are a few KB
  // and stay in L2), so selection needs no reduction launch of its own.
  {
    const int nq = q1 - q0;
    const int64_t qpitch = s.q_tok * ES;
    auto widen = [](const char* p) -> float {
      if constexpr (ES == 2)
        return __uint_as_float(uint32_t(*reinterpret_cast<const uint16_t*>(p)) << 16);
      else
        return *reinterpret_cast<const float*>(p);
    };
    for (int e = threadIdx.x; e < s.group * D; e += kScoreWaves * 64) {
      const char* p = q + (int64_t(q0) * s.q_tok + int64_t(g * s.group + e / D) * s.q_head + e % D) * ES;
      float a = 0.0f;
      int i = 0;
      for (; i + 32 <= nq; i += 32) {   // a whole block of 32 queries: all loads in flight, then the adds in row order
        float x[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) x[j] = widen(p + (i + j) * qpitch);
#pragma unroll
        for (int j = 0; j < 32; ++j) a = a + x[j];
      }
      for (; i + 16 <= nq; i += 16) {
        float x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) x[j] = widen(p + (i + j) * qpitch);
#pragma unroll
        for (int j = 0; j < 16; ++j) a = a + x[j];
      }
      for (; i < nq; ++i) a = a + widen(p + i * qpitch);
      sums[e] = a;
    }
    __syncthreads();
  }

  // Sums of the GT query heads scored per pass, 16 per register: lane l holds sum[16 i + l % 16] in
  // vq[t][i] (the same in all four rows of 16 lanes).  With one pass per tile (group == GT) they are
  // read once, here; with several, at the start of every pass.
  constexpr int NQ = D / 16;
  float vq[GT][NQ];
  auto load_sums = [&](int hh) {
    const float* qs = sums + hh * D + (lane & 15);
#pragma unroll
    for (int t = 0; t < GT; ++t)
#pragma unroll
      for (int i = 0; i < NQ; ++i) vq[t][i] = qs[t * D + 16 * i];
  };
  const bool one_pass = s.group == GT;
  if (one_pass) load_sums(0);

  for (int it = 0; it < ntiles; ++it) {
    const int r0 = first + it * 64;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int f = i * 64 + lane, row = f / CH, c = f % CH;
      mine[row * CH + (c ^ swz<CH>(row))] = regs[i];
    }
    if (it + 1 < ntiles) fetch(r0 + 64);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    for (int hh = 0; hh < s.group; hh += GT) {
      const int h0 = g * s.group + hh;
      if (!one_pass) load_sums(hh);
      float acc[GT];
#pragma unroll
      for (int t = 0; t < GT; ++t) acc[t] = 0.0f;
      // one key per lane: its row, 16 bytes at a time, against the sums in ascending d
      auto chunk = [&](auto cc) {
        constexpr int c = decltype(cc)::value;
        const v4u x = mine[lane * CH + (c ^ sw)];
        float kv[EPC];
        if constexpr (ES == 2) {
          kv[0] = bf16_lo(x.x); kv[1] = bf16_hi(x.x); kv[2] = bf16_lo(x.y); kv[3] = bf16_hi(x.y);
          kv[4] = bf16_lo(x.z); kv[5] = bf16_hi(x.z); kv[6] = bf16_lo(x.w); kv[7] = bf16_hi(x.w);
        } else {
          kv[0] = __uint_as_float(x.x); kv[1] = __uint_as_float(x.y);
          kv[2] = __uint_as_float(x.z); kv[3] = __uint_as_float(x.w);
        }
#pragma unroll
        for (int t = 0; t < GT; ++t) acc[t] = fma_row_bcast<(c * EPC) % 16, EPC>(acc[t], vq[t][(c * EPC) / 16], kv);
      };
      for_each_index(chunk, std::make_integer_sequence<int, CH>{});
      if (r0 + lane < L) {
#pragma unroll
        for (int t = 0; t < GT; ++t)
          scores[int64_t(h0 + t) * s.total_kv + kv0 + r0 + lane] = acc[t] + 0.0f;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// ------------------------------------------------------------------ head sum (Section 2.4 Eq. 5)
// summed[kv0 + j] = sum over query heads, ascending and starting from +0, of the pooled score of
// candidate j (the window clipped to the candidates): one thread per position, so the shared
// selection ranks one pre-summed row per sequence instead of walking every head inside the top-k.
__global__ __launch_bounds__(256) void head_sum_kernel(const float* __restrict__ scores,
                                                       const int32_t* __restrict__ cu_kv,
                                                       const int32_t* __restrict__ cu_k, int32_t total_kv,
                                                       int32_t pool_w, int32_t forced_tail, int32_t n_heads,
                                                       float* __restrict__ summed DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  const int b = blockIdx.y;
  if (cu_k[b + 1] == cu_k[b]) return;
  const int kv0 = cu_kv[b];
  const int L = cu_kv[b + 1] - kv0 - forced_tail;   // candidates
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= L) return;
  const int half = pool_w >> 1;
  const int lo = max(0, j - half), hi = min(L - 1, j + half);
  float acc = 0.0f;
  for (int hh = 0; hh < n_heads; ++hh) {
    const float* __restrict__ src = scores + int64_t(hh) * total_kv + kv0;
    float val = src[lo];
    for (int t = lo + 1; t <= hi; ++t) val = fmaxf(val, src[t]);
    acc = acc + val;
  }
  summed[kv0 + j] = acc;
}

// ------------------------------------------------------------------ top-k
#ifndef DLLM_TOPK_THREADS
#define DLLM_TOPK_THREADS 512
#endif
constexpr int kTopkThreads = DLLM_TOPK_THREADS;

__device__ __forceinline__ uint32_t order_key(float f) {
  // monotone map fp32 -> uint32 (larger float, larger key); +0 and -0 were already merged
  const uint32_t u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

// forced_tail: the last forced_tail positions of the sequence are kept without being ranked (the
// active block's own rows, Section 2.3 Eq. 4); the other kept rows are chosen among the positions
// before them.  head_sum: `scores` is the row of sums over the query heads (Section 2.4 Eq. 5,
// head_sum_kernel; pooling already applied, so pool_w is 1), ranked once per sequence and written to
// all n_heads heads; the grid then has one workgroup per sequence.
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k,
    int32_t total_kv, int32_t total_k, int32_t pool_w, int32_t lpad, int32_t forced_tail, int32_t head_sum,
    int32_t n_heads, int32_t* __restrict__ idx_out DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  extern __shared__ uint32_t dyn[];
  __shared__ uint32_t hist[256];
  // The leading byte of a score (sign and seven exponent bits) takes only a handful of values, and LDS
  // atomics of one instruction that hit one bank are served one after the other.  The first pass
  // therefore counts into 16 copies of the histogram, chosen by lane, that lie in 16 different banks.
  constexpr int kCopies = 16;
  __shared__ uint32_t hist0[256 * kCopies];
  __shared__ uint32_t wave_tot[kTopkThreads / 64];
  __shared__ uint32_t sh_prefix, sh_k;

  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int o0 = cu_k[b], kb_all = cu_k[b + 1] - o0;
  if (kb_all == 0) return;
  const int kv0 = cu_kv[b];
  const int L = cu_kv[b + 1] - kv0 - forced_tail;   // candidates: the positions before the forced ones
  const int kb = kb_all - forced_tail;              // kept among the candidates
  if (kb < 0 || L < kb) return;   // a precondition of the call is broken (fewer kept rows than forced ones, or more
                                  // than there are candidates): write nothing rather than outside this list
  const int h_first = head_sum ? 0 : h, h_last = head_sum ? n_heads : h + 1;   // heads that receive this list
  uint32_t* keys = dyn;

  // forced positions close the (ascending) list
  for (int t = tid; t < forced_tail; t += kTopkThreads)
    for (int hh = h_first; hh < h_last; ++hh) idx_out[int64_t(hh) * total_k + o0 + kb + t] = L + t;
  if (kb <= 0) return;

  // (pooled) score of every candidate -> order-preserving key.  With head_sum the scores are the
  // pre-summed (and pre-pooled) row of the sequence, ranked like one head's plain scores.
  float* raw = reinterpret_cast<float*>(dyn + lpad);
  const int half = pool_w >> 1;
  const bool plain = pool_w == 1;
  const float* __restrict__ src = scores + int64_t(head_sum ? 0 : h) * total_kv + kv0;
  if (plain) {
    // eight independent loads per thread in flight, then the keys; the histogram of the leading byte
    // (the first radix pass) is taken on the way
    for (int t = tid; t < 256 * kCopies; t += kTopkThreads) hist0[t] = 0;
    __syncthreads();
    for (int j0 = tid; j0 < L; j0 += 8 * kTopkThreads) {
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = j0 + u * kTopkThreads;
        x[u] = src[min(j, L - 1)];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = j0 + u * kTopkThreads;
        if (j < L) {
          const uint32_t key = order_key(x[u]);
          keys[j] = key;
          atomicAdd(&hist0[(key >> 24) * kCopies + (tid & (kCopies - 1))], 1u);
        }
      }
    }
  } else {
    for (int j0 = tid; j0 < L; j0 += 8 * kTopkThreads) {   // eight independent loads per thread in flight
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = src[min(j0 + u * kTopkThreads, L - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (j0 + u * kTopkThreads < L) raw[j0 + u * kTopkThreads] = x[u];
    }
    __syncthreads();
    for (int j = tid; j < L; j += kTopkThreads) {
      const int lo = max(0, j - half), hi = min(L - 1, j + half);
      float val = raw[lo];
      for (int t = lo + 1; t <= hi; ++t) val = fmaxf(val, raw[t]);
      keys[j] = order_key(val);
    }
  }
  __syncthreads();

  // radix select, most significant byte first: the kk-th largest among keys matching `prefix`
  uint32_t prefix = 0;
  uint32_t kk = uint32_t(kb);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (pass == 0) {
      if (!plain) {   // (the plain path counted while it built the keys)
        for (int t = tid; t < 256 * kCopies; t += kTopkThreads) hist0[t] = 0;
        __syncthreads();
        for (int j = tid; j < L; j += kTopkThreads)
          atomicAdd(&hist0[(keys[j] >> 24) * kCopies + (tid & (kCopies - 1))], 1u);
      }
      __syncthreads();
      if (tid < 256) {
        uint32_t t = 0;
#pragma unroll
        for (int c = 0; c < kCopies; ++c) t += hist0[tid * kCopies + c];
        hist[tid] = t;
      }
      __syncthreads();
    } else {   // later digits are spread evenly: one histogram, and no folding, is cheaper
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int j = tid; j < L; j += kTopkThreads) {
        const uint32_t key = keys[j];
        if ((key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
    }
    if (tid < 64) {
      uint32_t c[4], t = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) { c[i] = hist[255 - (4 * tid + i)]; t += c[i]; }
      uint32_t run = wave_inclusive_sum(t) - t;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (run < kk && kk <= run + c[i]) {
          sh_prefix = (prefix << 8) | uint32_t(255 - (4 * tid + i));
          sh_k = kk - run;
        }
        run += c[i];
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    kk = sh_k;
  }
  const uint32_t thr = prefix;   // key of the k-th largest
  const uint32_t need_eq = kk;   // how many keys equal to it are kept (lowest positions first)

  // ordered compaction: thread t owns positions [t*C, (t+1)*C); C odd keeps LDS reads conflict-free
  int C = (L + kTopkThreads - 1) / kTopkThreads;
  C |= 1;
  const int j0 = min(L, tid * C), j1 = min(L, j0 + C);
  // which of this thread's positions hold a key above / equal to the threshold (bit j - j0), when
  // they fit 64 bits: the emit loop then visits the kept positions only
  uint32_t gt = 0, eq = 0;
  uint64_t gt_bits = 0, eq_bits = 0;
  const bool masks = C <= 64;
  for (int j = j0; j < j1; ++j) {
    const uint32_t key = keys[j];
    gt += key > thr;
    eq += key == thr;
    if (masks) {
      gt_bits |= uint64_t(key > thr) << (j - j0);
      eq_bits |= uint64_t(key == thr) << (j - j0);
    }
  }
  uint32_t packed = gt | (eq << 16);   // both < 2^15
  const uint32_t incl = wave_inclusive_sum(packed);
  const int lane = tid & 63, wave = tid >> 6;
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t before = incl - packed;
  for (int w = 0; w < wave; ++w) before += wave_tot[w];
  uint32_t gt_before = before & 0xffffu, eq_before = before >> 16;
  // (both counters advance by selects, not in branches: with an increment in either arm of a branch the
  // compiler keeps the pair in scratch memory and indexes it, and a kernel that needs scratch starts its
  // waves more slowly)
  auto emit = [&](int j, bool above) {
    const uint32_t slot = gt_before + (above ? min(eq_before, need_eq) : eq_before);
    const bool keep = above || eq_before < need_eq;
    gt_before += above ? 1u : 0u;
    eq_before += above ? 0u : 1u;
    if (keep)
      for (int hh = h_first; hh < h_last; ++hh) idx_out[int64_t(hh) * total_k + o0 + slot] = j;
  };
  if (masks) {
    for (uint64_t m = gt_bits | eq_bits; m != 0; m &= m - 1) {
      const int t = __builtin_ctzll(m);
      emit(j0 + t, (gt_bits >> t) & 1);
    }
  } else {
    for (int j = j0; j < j1; ++j) {
      const uint32_t key = keys[j];
      if (key >= thr) emit(j, key > thr);
    }
  }
}

// Lists of up to R * T candidates: the same selection by a workgroup of T threads with the keys held in
// registers (thread t owns positions t, t + T, ...), so that no pass re-reads them from LDS.  Every wave scans
// the histogram of a pass for itself (the chosen digit is the same in all of them), which leaves one
// barrier per pass; the four histograms are cleared once, before the scores arrive.  The ordered
// compaction counts kept rows per (round, wave) with ballots, and every wave takes the prefix sums of
// those counts itself.  Positions past the end of the list hold key 0, the smallest: they are not counted
// in the first pass, and wherever later passes count them (in digit 0) they stand below every real key
// and, among equal keys, behind every real position, so they change neither the threshold nor the list.
template <int R, int T>
__global__ __launch_bounds__(T) void topk_reg_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k,
    int32_t total_kv, int32_t total_k, int32_t pool_w, int32_t forced_tail, int32_t head_sum, int32_t n_heads,
    int32_t* __restrict__ idx_out DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int kCopies = 16, kWaves = T / 64;
  constexpr int E = R * kWaves / 64;   // (round, wave) counts per lane in the final scan
  static_assert(T >= 256 && R * kWaves % 64 == 0 && (E == 1 || E == 2), "one or two counts per lane");
  extern __shared__ uint32_t dyn[];   // pooled selection only: the raw scores of the list
  __shared__ __align__(16) uint32_t hist0[256 * kCopies];   // first pass, bank-separated copies (see topk_kernel)
  __shared__ __align__(16) uint32_t hist[4][256];           // [0]: the folded first pass
  __shared__ uint32_t counts[R * kWaves];

  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int o0 = cu_k[b], kb_all = cu_k[b + 1] - o0;
  if (kb_all == 0) return;
  const int kv0 = cu_kv[b];
  const int L = cu_kv[b + 1] - kv0 - forced_tail;
  const int kb = kb_all - forced_tail;
  if (kb < 0 || L < kb) return;   // broken precondition (see topk_kernel): write nothing
  const int h_first = head_sum ? 0 : h, h_last = head_sum ? n_heads : h + 1;
  for (int t = tid; t < forced_tail; t += T)
    for (int hh = h_first; hh < h_last; ++hh) idx_out[int64_t(hh) * total_k + o0 + kb + t] = L + t;
  if (kb <= 0) return;

  const float* __restrict__ src = scores + int64_t(head_sum ? 0 : h) * total_kv + kv0;
  for (int t = tid; t < 256 * kCopies; t += T) hist0[t] = 0;
  for (int t = tid; t < 3 * 256; t += T) (&hist[1][0])[t] = 0;

  uint32_t key[R];
  float x[R];
#pragma unroll
  for (int u = 0; u < R; ++u)
    if (u * T < L) x[u] = src[min(tid + u * T, L - 1)];
  if (pool_w != 1) {
    float* raw = reinterpret_cast<float*>(dyn);
    const int half = pool_w >> 1;
#pragma unroll
    for (int u = 0; u < R; ++u)
      if (tid + u * T < L) raw[tid + u * T] = x[u];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const int j = tid + u * T;
      if (j < L) {
        const int lo = max(0, j - half), hi = min(L - 1, j + half);
        float val = raw[lo];
        for (int t = lo + 1; t <= hi; ++t) val = fmaxf(val, raw[t]);
        x[u] = val;
      }
    }
  } else {
    __syncthreads();   // histograms cleared
  }
#pragma unroll
  for (int u = 0; u < R; ++u) {
    key[u] = 0;
    if (tid + u * T < L) {
      key[u] = order_key(x[u]);
      atomicAdd(&hist0[(key[u] >> 24) * kCopies + (tid & (kCopies - 1))], 1u);
    }
  }
  __syncthreads();
  if (tid < 256) {
    const uint4* c4 = reinterpret_cast<const uint4*>(hist0 + tid * kCopies);
    uint32_t t = 0;
#pragma unroll
    for (int c = 0; c < kCopies / 4; ++c) {
      const uint4 v = c4[c];
      t += v.x + v.y + v.z + v.w;
    }
    hist[0][tid] = t;
  }
  __syncthreads();

  // the digit (bin) that holds the kk-th largest of the keys counted in hrow, found by every wave
  uint32_t prefix = 0, kk = uint32_t(kb);
  auto pick = [&](const uint32_t* hrow) {
    const uint4 v = *reinterpret_cast<const uint4*>(hrow + 252 - 4 * lane);
    const uint32_t c[4] = {v.w, v.z, v.y, v.x};   // bins 255 - 4 lane - i, descending
    const uint32_t t = c[0] + c[1] + c[2] + c[3];
    uint32_t run = wave_inclusive_sum(t) - t;
    uint32_t bin = 0, knew = 0;
    bool found = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (run < kk && kk <= run + c[i]) {
        found = true;
        bin = uint32_t(255 - (4 * lane + i));
        knew = kk - run;
      }
      run += c[i];
    }
    const uint64_t m = __ballot(found);   // one lane, since 1 <= kk <= number of keys counted
    const int owner = m ? __builtin_ctzll(m) : 0;
    prefix = (prefix << 8) | uint32_t(__builtin_amdgcn_readlane(int(bin), owner));
    kk = uint32_t(__builtin_amdgcn_readlane(int(knew), owner));
  };
  pick(hist[0]);
#pragma unroll
  for (int pass = 1; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
#pragma unroll
    for (int u = 0; u < R; ++u)
      if ((key[u] >> (shift + 8)) == prefix)
        atomicAdd(&hist[pass][(key[u] >> shift) & 255u], 1u);
    __syncthreads();
    pick(hist[pass]);
  }
  const uint32_t thr = prefix, need_eq = kk;

  // ordered compaction: kept rows before round u of this wave, as (above | equal << 16)
#pragma unroll
  for (int u = 0; u < R; ++u) {
    const uint64_t bg = __ballot(key[u] > thr), be = __ballot(key[u] == thr);
    const uint32_t c = uint32_t(__builtin_popcountll(bg)) | (uint32_t(__builtin_popcountll(be)) << 16);
    if (lane == 0) counts[u * kWaves + wave] = c;
  }
  __syncthreads();
  uint32_t c0 = counts[lane * E], c1 = E == 2 ? counts[lane * E + 1] : 0u;
  const uint32_t excl = wave_inclusive_sum(c0 + c1) - (c0 + c1);
  int32_t* __restrict__ out = idx_out + int64_t(h_first) * total_k + o0;
#pragma unroll
  for (int u = 0; u < R; ++u) {
    if (u * T >= L) break;
    const int e = u * kWaves + wave;
    uint32_t base = uint32_t(__builtin_amdgcn_readlane(int(excl), e / E));
    if (E == 2 && (e & 1)) base += uint32_t(__builtin_amdgcn_readlane(int(c0), e / E));
    const bool gt = key[u] > thr, eq = key[u] == thr;
    const uint64_t bg = __ballot(gt), be = __ballot(eq);
    const uint32_t gt_before =
        (base & 0xffffu) + __builtin_amdgcn_mbcnt_hi(uint32_t(bg >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(bg), 0u));
    // a key above the threshold goes behind the kept rows before it; without a key equal to the
    // threshold in this wave's round (the usual case) that is all there is to do
    uint32_t slot = gt_before + min(base >> 16, need_eq);
    bool keep = gt;
    if (be != 0) {
      const uint32_t eq_before =
          (base >> 16) + __builtin_amdgcn_mbcnt_hi(uint32_t(be >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(be), 0u));
      slot = gt_before + (gt ? min(eq_before, need_eq) : eq_before);
      keep = gt || (eq && eq_before < need_eq);
    }
    if (keep) {
      out[slot] = tid + u * T;
      for (int hh = h_first + 1; hh < h_last; ++hh) out[int64_t(hh - h_first) * total_k + slot] = tid + u * T;
    }
  }
}

// ------------------------------------------------------------------ scores and top-k in one workgroup
// One workgroup per (sequence, KV head) walks the head's whole K column once, keeps the keys of its
// GT query heads in registers (one key per lane, tile and head) and ranks them there: the scores never
// travel to HBM and back and the lists need no second launch.  Lists of up to kFusedWords * 64
// positions; the arithmetic, the tie rule and the output order are those of the kernels above.
//
// Ranking is a radix select over digits of 10, 11 and 11 bits.  The first histogram is counted while
// the column streams in (its atomics hide under the memory waits); the other two count only the keys
// that share the digits found so far, and the third is skipped for a head whose threshold bin holds
// kept keys only.  Each head's histogram is scanned by one wave, in two levels (a lane sums a run of
// bins, the owner's run is then looked at one bin per lane).  Compaction goes through a bitmap of the
// kept positions (see there).
// With a pooling window the keys are max-pooled in the registers once the column is in (see there); the
// first histogram is then counted afterwards, in the open.
constexpr int kFusedWords = 128;   // 64-row tiles per list at most (8192 positions): W waves of kFusedWords / W tiles
// Eight waves of 16 tiles for every group size.  (Four waves of 32 tiles for one or two query heads per
// KV head, so that two workgroups share a compute unit and one's start-up and ranking run under the
// other's streaming, measured 2-10 % slower on every batch tried.)
template <int GT> constexpr int fused_waves() { return 8; }
template <int N> struct KeyVec { typedef __attribute__((ext_vector_type(N))) uint32_t type; };
constexpr int kBinsA = 1024, kBinsB = 2048;   // digits: key >> 22, (key >> 11) & 2047, key & 2047

template <int ES, int D, int GT>
struct FusedLds {   // byte offsets inside the workgroup's dynamic LDS
  static constexpr int W = fused_waves<GT>();
  static constexpr size_t stage = size_t(W) * 64 * D * ES;            // the waves' tiles while streaming
  static constexpr size_t hist_bc = size_t(GT) * 2 * kBinsB * 4;                // afterwards: second and third histograms
  static constexpr size_t kept = size_t(GT) * kFusedWords * 64 * 4;                 // at the end: the kept positions [GT][8192]
  static constexpr size_t region0 = stage > hist_bc ? (stage > kept ? stage : kept) : (hist_bc > kept ? hist_bc : kept);
  static constexpr size_t off_a = region0;                                      // first histogram [GT][kBinsA]
  static constexpr size_t off_counts = off_a + size_t(GT) * kBinsA * 4;         // two bitmaps [GT][waves * tiles] of 64 bits, [2][waves] totals
  static constexpr size_t off_res = off_counts + size_t(GT) * kFusedWords * 16 + 2 * 8 * 4;   // [GT][4]
  static constexpr size_t off_sums = off_res + size_t(GT) * 16;                 // [GT][D]
  static constexpr size_t bytes = off_sums + size_t(GT) * D * 4;
};

// The bin that holds the kth-largest of the keys counted in hrow[0 .. NB) (bins descend from NB - 1), the
// rank of that key inside the bin and the bin's count: {bin, rank, count}, the same in every lane.
template <int NB>
__device__ __forceinline__ uint3 pick_bin(const uint32_t* hrow, uint32_t kth, int lane) {
  constexpr int BPL = NB / 64;   // bins per lane; lane 0 owns the highest
  static_assert(BPL % 4 == 0 && BPL <= 64, "runs of whole 16-byte words, one bin per lane in the second level");
  const uint32_t* run_lo = hrow + NB - BPL * (lane + 1);
  uint32_t tot = 0;
#pragma unroll
  for (int i = 0; i < BPL / 4; ++i) {
    const uint4 v = *reinterpret_cast<const uint4*>(run_lo + 4 * i);
    tot += v.x + v.y + v.z + v.w;
  }
  const uint32_t incl = wave_inclusive_sum(tot);
  const uint64_t m1 = __ballot(incl - tot < kth && kth <= incl);
  const int owner = m1 ? __builtin_ctzll(m1) : 0;
  const uint32_t above = uint32_t(__builtin_amdgcn_readlane(int(incl - tot), owner));
  const int top = NB - BPL * owner - 1;   // the owner's highest bin
  const uint32_t c = lane < BPL ? hrow[top - lane] : 0u;
  const uint32_t incl2 = wave_inclusive_sum(c) + above;
  const uint64_t m2 = __ballot(incl2 - c < kth && kth <= incl2);
  const int j = m2 ? __builtin_ctzll(m2) : 0;
  return make_uint3(uint32_t(top - j), kth - uint32_t(__builtin_amdgcn_readlane(int(incl2 - c), j)),
                    uint32_t(__builtin_amdgcn_readlane(int(c), j)));
}

// v[lane u] = x (x the same in all lanes).  A select, not v_writelane_b32: x usually comes straight from
// a vector compare, and a lane write that reads a compare's result in the next instruction was seen
// to pick up the previous compare's.
__device__ __forceinline__ void set_lane(uint32_t& v, uint32_t x, int u) { v = int(threadIdx.x & 63) == u ? x : v; }

template <int ES, int D, int GT>
__global__ __launch_bounds__(fused_waves<GT>() * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void select_fused_kernel(
    const char* __restrict__ k, const char* __restrict__ q, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k, int32_t total_k, int32_t forced_tail,
    int32_t pool_w, int32_t ranked, int32_t* __restrict__ idx_out, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int ROWB = D * ES, CH = ROWB / 16, EPC = 16 / ES, W = fused_waves<GT>(), NT = kFusedWords / W, T = W * 64;
  static_assert(NT <= 32, "a wave's tile masks are collected one per lane, its keys in one register vector per head");
  static_assert(GT <= W, "one wave scans one head's histogram");
  using Lds = FusedLds<ES, D, GT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  v4u* mine_all = reinterpret_cast<v4u*>(lds);
  uint32_t* hist_b = reinterpret_cast<uint32_t*>(lds);            // [GT][kBinsB], once streaming is over
  uint32_t* hist_c = hist_b + GT * kBinsB;                        // [GT][kBinsB]
  uint32_t* hist_a = reinterpret_cast<uint32_t*>(lds + Lds::off_a);
  uint32_t* res = reinterpret_cast<uint32_t*>(lds + Lds::off_res);
  float* sums = reinterpret_cast<float*>(lds + Lds::off_sums);

  // Which sequence: slot blockIdx.x / hkv.  When the workgroups run in several rounds (`ranked`, batches
  // of up to 64 sequences) the slots go down the sequences by length, longest first: workgroups start in
  // the order of their numbers, so the compute units that come free first pick up the longest lists
  // left and the rounds end level whatever the mix of lengths.
  int b = blockIdx.x / s.hkv;
  int ck0, ck1, kv0, kv1, q0, q1;
  if (ranked) {
    const int ln = threadIdx.x & 63, i = min(ln, s.batch - 1);
    const int a0 = cu_k[i], a1 = cu_k[i + 1], b0 = cu_kv[i], b1 = cu_kv[i + 1], c0 = cu_q[i], c1 = cu_q[i + 1];
    const int mine = ln < s.batch ? (a1 == a0 ? -1 : b1 - b0) : -2;   // (a sequence that is not scored has no length)
    int rank = 0;
    for (int j = 0; j < s.batch; ++j) {
      const int other = __builtin_amdgcn_readlane(mine, j);
      rank += (other > mine) || (other == mine && j < ln);
    }
    const uint64_t hit = __ballot(ln < s.batch && rank == b);   // exactly one lane: the ranks are a permutation
    b = hit ? __builtin_ctzll(hit) : 0;
    ck0 = __builtin_amdgcn_readlane(a0, b); ck1 = __builtin_amdgcn_readlane(a1, b);
    kv0 = __builtin_amdgcn_readlane(b0, b); kv1 = __builtin_amdgcn_readlane(b1, b);
    q0 = __builtin_amdgcn_readlane(c0, b); q1 = __builtin_amdgcn_readlane(c1, b);
  } else {
    ck0 = cu_k[b]; ck1 = cu_k[b + 1]; kv0 = cu_kv[b]; kv1 = cu_kv[b + 1]; q0 = cu_q[b]; q1 = cu_q[b + 1];
    asm volatile("" : "+s"(ck0), "+s"(ck1), "+s"(kv0), "+s"(kv1), "+s"(q0), "+s"(q1));
  }
  const int g = (blockIdx.x + b) % s.hkv;   // (rotation: see score_kernel)
  if (ck1 == ck0) return;
  const int L = kv1 - kv0, Lc = L - forced_tail, kb = ck1 - ck0 - forced_tail;
  if (kb < 0 || Lc < kb) return;   // broken precondition (see topk_kernel): write nothing
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int32_t* __restrict__ out = idx_out + int64_t(g * GT) * total_k + ck0;
  for (int t = tid; t < forced_tail; t += T)
#pragma unroll
    for (int hh = 0; hh < GT; ++hh) out[int64_t(hh) * total_k + kb + t] = Lc + t;
  if (kb <= 0) return;

  const int nt = (Lc + 63) >> 6, tpw = (nt + W - 1) / W;   // tpw <= NT: the host checked the longest list
  const int first = wave * tpw * 64;
  const int ntiles = max(0, min(min(tpw, NT), nt - wave * tpw));
  const char* base = k + (int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head) * ES + (lane % CH) * 16;
  const int64_t row_pitch = s.kv_tok * ES;
  v4u* mine = mine_all + wave * 64 * CH;
  const int sw = swz<CH>(lane);
  v4u regs[CH];
  auto fetch = [&](int r0) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int row = min(r0 + (i * 64 + lane) / CH, L - 1);
      regs[i] = load_once(base + row * row_pitch);
    }
  };
  if (ntiles > 0) fetch(first);

  for (int t = tid; t < GT * kBinsA; t += T) hist_a[t] = 0;
  {   // block sums of this KV head's query heads, ascending rows (as in score_kernel)
    const int nq = q1 - q0;
    const int64_t qpitch = s.q_tok * ES;
    auto widen = [](const char* p) -> float {
      if constexpr (ES == 2)
        return __uint_as_float(uint32_t(*reinterpret_cast<const uint16_t*>(p)) << 16);
      else
        return *reinterpret_cast<const float*>(p);
    };
    for (int e = tid; e < GT * D; e += T) {
      const char* p = q + (int64_t(q0) * s.q_tok + int64_t(g * GT + e / D) * s.q_head + e % D) * ES;
      float a = 0.0f;
      int i = 0;
      for (; i + 32 <= nq; i += 32) {
        float x[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) x[j] = widen(p + (i + j) * qpitch);
#pragma unroll
        for (int j = 0; j < 32; ++j) a = a + x[j];
      }
      for (; i < nq; ++i) a = a + widen(p + i * qpitch);
      sums[e] = a;
    }
    __syncthreads();
  }
  constexpr int NQ = D / 16;
  float vq[GT][NQ];
  {
    const float* qs = sums + (lane & 15);
#pragma unroll
    for (int t = 0; t < GT; ++t)
#pragma unroll
      for (int i = 0; i < NQ; ++i) vq[t][i] = qs[t * D + 16 * i];
  }

  const int half = pool_w >> 1;   // pooling window (Section 4.5 Eq. 6): positions p - half .. p + half, clipped to the candidates
  // key of tile u for head t in k<t>[u]; 0, below every real key, where there is no position
  // (four named vectors: an array of them is not kept in registers)
  typedef typename KeyVec<NT>::type keyvec;
  keyvec k0 = keyvec(0u), k1 = k0, k2 = k0, k3 = k0;
  for (int it = 0; it < ntiles; ++it) {
    const int r0 = first + it * 64;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int f = i * 64 + lane, row = f / CH, c = f % CH;
      mine[row * CH + (c ^ swz<CH>(row))] = regs[i];
    }
    if (it + 1 < ntiles) fetch(r0 + 64);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float acc[GT];
#pragma unroll
    for (int t = 0; t < GT; ++t) acc[t] = 0.0f;
    auto chunk = [&](auto cc) {
      constexpr int c = decltype(cc)::value;
      const v4u x = mine[lane * CH + (c ^ sw)];
      float kv[EPC];
      if constexpr (ES == 2) {
        kv[0] = bf16_lo(x.x); kv[1] = bf16_hi(x.x); kv[2] = bf16_lo(x.y); kv[3] = bf16_hi(x.y);
        kv[4] = bf16_lo(x.z); kv[5] = bf16_hi(x.z); kv[6] = bf16_lo(x.w); kv[7] = bf16_hi(x.w);
      } else {
        kv[0] = __uint_as_float(x.x); kv[1] = __uint_as_float(x.y);
        kv[2] = __uint_as_float(x.z); kv[3] = __uint_as_float(x.w);
      }
#pragma unroll
      for (int t = 0; t < GT; ++t) acc[t] = fma_row_bcast<(c * EPC) % 16, EPC>(acc[t], vq[t][(c * EPC) / 16], kv);
    };
    for_each_index(chunk, std::make_integer_sequence<int, CH>{});
    const bool valid = r0 + lane < Lc;
    uint32_t key[GT];
#pragma unroll
    for (int t = 0; t < GT; ++t) {
      key[t] = valid ? order_key(acc[t] + 0.0f) : 0u;
      if (valid && half == 0) atomicAdd(&hist_a[t * kBinsA + (key[t] >> 22)], 1u);   // (pooled keys are counted once they exist)
    }
    k0[it] = key[0];
    if constexpr (GT > 1) k1[it] = key[1];
    if constexpr (GT > 2) { k2[it] = key[2]; k3[it] = key[3]; }
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();   // every wave is done with its staging tile: the space now holds the later histograms
  {
    uint4* z = reinterpret_cast<uint4*>(hist_b);
    for (int t = tid; t < GT * 2 * kBinsB / 4; t += T) z[t] = make_uint4(0, 0, 0, 0);
  }
  uint32_t key[GT][NT];
#pragma unroll
  for (int u = 0; u < NT; ++u) {
    key[0][u] = k0[u];
    if constexpr (GT > 1) key[1][u] = k1[u];
    if constexpr (GT > 2) { key[2][u] = k2[u]; key[3][u] = k3[u]; }
  }

  if (half > 0) {
    // Max-pool the keys over the window (the key map is monotone, so this pools the scores).  A wave's
    // positions are consecutive, 64 per tile, so a neighbour is the next lane, across a tile edge the
    // next tile's first or the previous tile's last lane, and across a wave's edge a key of the
    // neighbouring wave: every wave leaves its first and its last tile in LDS for that.  The window is
    // built one position at a time: the keys moved on by one more lane per step, to either side, and
    // the running maximum.  Positions past the candidates hold key 0 and get it back at the end.
    uint32_t* edge = reinterpret_cast<uint32_t*>(lds + Lds::hist_bc);   // [GT][W][first | last][64]
    static_assert(Lds::hist_bc + size_t(GT) * W * 128 * 4 <= Lds::region0, "the waves' edge tiles fit beside the histograms");
    const int last_u = max(ntiles - 1, 0);
    edge[((0 * W + wave) * 2 + 0) * 64 + lane] = k0[0];
    edge[((0 * W + wave) * 2 + 1) * 64 + lane] = k0[last_u];
    if constexpr (GT > 1) {
      edge[((1 * W + wave) * 2 + 0) * 64 + lane] = k1[0];
      edge[((1 * W + wave) * 2 + 1) * 64 + lane] = k1[last_u];
    }
    if constexpr (GT > 2) {
      edge[((2 * W + wave) * 2 + 0) * 64 + lane] = k2[0];
      edge[((2 * W + wave) * 2 + 1) * 64 + lane] = k2[last_u];
      edge[((3 * W + wave) * 2 + 0) * 64 + lane] = k3[0];
      edge[((3 * W + wave) * 2 + 1) * 64 + lane] = k3[last_u];
    }
    __syncthreads();
    // (a wave with tiles has a full run before it; the wave after it may have none: its tiles then hold key 0)
    const bool has_prev = wave > 0 && ntiles > 0, has_next = wave + 1 < W && ntiles > 0;
#pragma unroll
    for (int t = 0; t < GT; ++t) {
      const uint32_t* prev_last = edge + ((t * W + max(wave - 1, 0)) * 2 + 1) * 64;
      const uint32_t* next_first = edge + ((t * W + min(wave + 1, W - 1)) * 2 + 0) * 64;
      uint32_t run[NT], best[NT];
#pragma unroll
      for (int u = 0; u < NT; ++u) run[u] = best[u] = key[t][u];
      // (rotations by one lane, then the lane at the tile's edge takes the neighbouring tile's rotated
      // value: no scalar register between two vector instructions)
      for (int sh = 1; sh <= half; ++sh) {   // keys of positions p - sh
        const uint32_t from_prev = has_prev ? prev_last[64 - sh] : 0u;
        uint32_t rot = uint32_t(__builtin_amdgcn_update_dpp(0, int(run[NT - 1]), 0x13c, 0xf, 0xf, false));   // wave_ror:1
#pragma unroll
        for (int u = NT - 1; u >= 0; --u) {
          const uint32_t below = u > 0 ? uint32_t(__builtin_amdgcn_update_dpp(0, int(run[u - 1]), 0x13c, 0xf, 0xf, false)) : from_prev;
          run[u] = lane == 0 ? below : rot;   // (lane 0 of the rotated tile below holds that tile's lane 63)
          best[u] = max(best[u], run[u]);
          rot = below;
        }
      }
#pragma unroll
      for (int u = 0; u < NT; ++u) run[u] = key[t][u];
      for (int sh = 1; sh <= half; ++sh) {   // keys of positions p + sh
        const uint32_t from_next = has_next ? next_first[sh - 1] : 0u;
        uint32_t rot = uint32_t(__builtin_amdgcn_update_dpp(0, int(run[0]), 0x134, 0xf, 0xf, false));   // wave_rol:1
#pragma unroll
        for (int u = 0; u < NT; ++u) {
          // the tile after this one: the next register, or the next wave's first tile after this wave's last
          uint32_t above = 0;
          if (u + 1 < NT) above = uint32_t(__builtin_amdgcn_update_dpp(0, int(run[u + 1]), 0x134, 0xf, 0xf, false));
          run[u] = lane == 63 ? (u + 1 == ntiles ? from_next : above) : rot;
          best[u] = max(best[u], run[u]);
          rot = above;
        }
      }
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        const bool valid = u < ntiles && first + u * 64 + lane < Lc;
        key[t][u] = valid ? best[u] : 0u;
        if (valid) atomicAdd(&hist_a[t * kBinsA + (key[t][u] >> 22)], 1u);
      }
    }
    __syncthreads();
  }

  // wave w < GT scans the histogram of head w and leaves {bin, rank, count} for all
  auto scan_and_share = [&](const uint32_t* h, auto nb, uint32_t kth) {
    constexpr int NB = decltype(nb)::value;
    if (wave < GT) {
      const uint3 r = pick_bin<NB>(h + wave * NB, kth, lane);
      if (lane == 0) { res[4 * wave] = r.x; res[4 * wave + 1] = r.y; res[4 * wave + 2] = r.z; }
    }
    __syncthreads();
  };
  // a value every lane read from the same LDS word, as a scalar
  auto shared = [](uint32_t x) { return uint32_t(__builtin_amdgcn_readfirstlane(int(x))); };
  const int my_head = wave % GT;
  uint32_t prefix[GT], kk[GT], tot_eq[GT];
  scan_and_share(hist_a, std::integral_constant<int, kBinsA>{}, uint32_t(kb));   // (its barrier also covers the clearing above)
  uint32_t my_kk = res[4 * my_head + 1];   // kk[my_head], read by address: indexing the register array would go through memory
#pragma unroll
  for (int t = 0; t < GT; ++t) { prefix[t] = shared(res[4 * t]); kk[t] = shared(res[4 * t + 1]); }
#pragma unroll
  for (int t = 0; t < GT; ++t)
#pragma unroll
    for (int u = 0; u < NT; ++u)
      if ((key[t][u] >> 22) == prefix[t]) atomicAdd(&hist_b[t * kBinsB + ((key[t][u] >> 11) & (kBinsB - 1))], 1u);
  __syncthreads();
  scan_and_share(hist_b, std::integral_constant<int, kBinsB>{}, my_kk);
  // A head whose threshold bin holds nothing but kept keys is settled after 21 bits: every key from
  // the bin's lowest value on is kept, whatever the last digit of the k-th largest is.  (Likely when the
  // bins are as thinly filled as here, two thousand of them for the keys of one first-level bin.)
  my_kk = res[4 * my_head + 1];
  const bool my_settled = res[4 * my_head + 2] == my_kk && res[4 * my_head] != 0;
  bool settled[GT], all_settled = true;
#pragma unroll
  for (int t = 0; t < GT; ++t) {
    prefix[t] = (prefix[t] << 11) | shared(res[4 * t]);
    kk[t] = shared(res[4 * t + 1]);
    settled[t] = shared(res[4 * t + 2]) == kk[t] && prefix[t] != 0;
    all_settled = all_settled && settled[t];
  }
  if (!all_settled) {   // (the same in every thread)
#pragma unroll
    for (int t = 0; t < GT; ++t)
      if (!settled[t]) {
#pragma unroll
        for (int u = 0; u < NT; ++u)
          if ((key[t][u] >> 11) == prefix[t]) atomicAdd(&hist_c[t * kBinsB + (key[t][u] & (kBinsB - 1))], 1u);
      }
    __syncthreads();
    if (wave < GT && !my_settled) {
      const uint3 r = pick_bin<kBinsB>(hist_c + wave * kBinsB, my_kk, lane);
      if (lane == 0) { res[4 * wave] = r.x; res[4 * wave + 1] = r.y; res[4 * wave + 2] = r.z; }
    }
    __syncthreads();
  }
#pragma unroll
  for (int t = 0; t < GT; ++t) {
    if (settled[t]) {
      prefix[t] = prefix[t] << 11;   // the lowest key of the bin: all keys from here on are kept
      kk[t] = tot_eq[t] = 1;         // (read below as "every key equal to the threshold is kept")
    } else {
      prefix[t] = (prefix[t] << 11) | shared(res[4 * t]);   // key of the k-th largest
      kk[t] = shared(res[4 * t + 1]);                       // how many keys equal to it are kept (lowest positions first)
      tot_eq[t] = shared(res[4 * t + 2]);
    }
  }

  // Compaction.  A ballot over a tile is the tile's 64 bits of the head's keep-bitmap, so each wave
  // leaves one word per tile in LDS.  Then the workgroup is dealt out anew, one thread per word (two
  // waves per head): a prefix sum over the words' population counts gives every word its first slot,
  // the thread walks the set bits of its word and writes their positions into LDS, and the finished
  // lists go out in whole lines.  Keys equal to the threshold have a bitmap of their own, used only
  // when not all of them are kept (scores that tie exactly): a word then keeps its first few equal
  // keys, as many as the rule "lower position first" leaves for it.
  static_assert(GT * kFusedWords <= T && W <= 8, "one thread per tile of each head; the waves' totals fit wave_tot");
  constexpr int kWords = kFusedWords;   // tiles, and so bitmap words, per head
  uint64_t* bitmap = reinterpret_cast<uint64_t*>(lds + Lds::off_counts);   // [GT][kWords] keys above the threshold
  uint64_t* bitmap_eq = bitmap + GT * kWords;                              // [GT][kWords] keys equal to it
  uint32_t* wave_tot = reinterpret_cast<uint32_t*>(bitmap_eq + GT * kWords);   // [2][W]
  constexpr int kKeptPerHead = W * NT * 64;
  int32_t* kept = reinterpret_cast<int32_t*>(lds);   // [GT][kKeptPerHead], in the histograms' space
  bool ties = false;
#pragma unroll
  for (int t = 0; t < GT; ++t) {
    const bool all_eq = kk[t] == tot_eq[t];
    const uint32_t thr = all_eq ? prefix[t] - 1 : prefix[t];   // (a threshold key is never 0)
    ties = ties || !all_eq;
    uint32_t mlo = 0, mhi = 0;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      const uint64_t bg = __ballot(key[t][u] > thr);
      set_lane(mlo, uint32_t(bg), u);
      set_lane(mhi, uint32_t(bg >> 32), u);
    }
    if (lane < ntiles) bitmap[t * kWords + wave * tpw + lane] = uint64_t(mlo) | (uint64_t(mhi) << 32);
    if (!all_eq) {
      uint32_t elo = 0, ehi = 0;
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        const uint64_t be = __ballot(key[t][u] == thr);
        set_lane(elo, uint32_t(be), u);
        set_lane(ehi, uint32_t(be >> 32), u);
      }
      if (lane < ntiles) bitmap_eq[t * kWords + wave * tpw + lane] = uint64_t(elo) | (uint64_t(ehi) << 32);
      if (tid == 0) res[4 * t + 3] = kk[t];
    } else if (tid == 0) {
      res[4 * t + 3] = 0;
    }
  }
  __syncthreads();
  const int th = wave >> 1, word = tid & 127;   // this thread's head and tile from here on
  const bool live = th < GT && word < nt;
  // exclusive prefix of x over the 128 threads of a head (two waves), through wave_tot[which]
  auto head_prefix = [&](uint32_t x, int which) {
    const uint32_t incl = wave_inclusive_sum(x);
    if (lane == 63) wave_tot[which * W + wave] = incl;
    __syncthreads();
    return incl - x + ((wave & 1) ? wave_tot[which * W + wave - 1] : 0u);
  };
  uint64_t m = live ? bitmap[th * kWords + word] : 0ull;
  if (ties) {   // (the same in every thread)
    const uint32_t need_eq = live ? res[4 * th + 3] : 0u;
    uint64_t e = (live && need_eq != 0) ? bitmap_eq[th * kWords + word] : 0ull;
    const uint32_t ce = uint32_t(__builtin_popcountll(e));
    const uint32_t eq_before = head_prefix(ce, 1);
    const uint32_t allowed = need_eq > eq_before ? min(ce, need_eq - eq_before) : 0u;
    for (uint32_t c = ce; c > allowed; --c) e &= ~(1ull << (63 - __builtin_clzll(e)));   // drop the highest
    m |= e;
  }
  uint32_t slot = head_prefix(uint32_t(__builtin_popcountll(m)), 0);
  {
    int32_t* __restrict__ o = kept + th * kKeptPerHead;
    const int p0 = word * 64;
    uint32_t half = uint32_t(m);
    for (; half != 0; half &= half - 1) o[slot++] = p0 + __builtin_ctz(half);
    half = uint32_t(m >> 32);
    for (; half != 0; half &= half - 1) o[slot++] = p0 + 32 + __builtin_ctz(half);
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < GT; ++t)
    for (int i = tid; i < kb; i += T) out[int64_t(t) * total_k + i] = kept[t * kKeptPerHead + i];
}

// ------------------------------------------------------------------ host side
SelectPlan plan_select(const Shape& s) {
  SelectPlan p;
  p.off_scores = 0;
  p.off_summed = align256(size_t(s.hq) * size_t(s.total_kv) * sizeof(float));   // one row of head sums (Eq. 5)
  p.bytes = p.off_summed + align256(size_t(s.total_kv) * sizeof(float));
  return p;
}

template <int ES, int D>
static hipError_t launch_score(const Shape& s, const void* k, const void* q, const int32_t* cu_q,
                               const int32_t* cu_kv, const int32_t* cu_k, float* scores, hipStream_t st) {
  // Tiles per wave, once there are about four workgroups per compute unit: two, or four when a tile is
  // scored for four or more query heads (measured on the benchmark workloads with launches back to
  // back: one tile costs the GQA case 20 %, two cost it 10 %, four cost the one-head case 3 %).
  const int64_t wg_tiles = int64_t(s.total_kv) * s.hkv / kScoreRowsPerBlock;
  const int tpw_max = s.group >= 4 ? 4 : 2;
  int tpw = int(wg_tiles / 1024);
  tpw = tpw < 1 ? 1 : (tpw > tpw_max ? tpw_max : tpw);
  const int rows_per_block = kScoreRowsPerBlock * tpw;
  dim3 grid(s.hkv, (s.max_kv + rows_per_block - 1) / rows_per_block, s.batch);
  dim3 block(kScoreWaves * 64);
  const char *kp = static_cast<const char*>(k), *qp = static_cast<const char*>(q);
  const size_t sums_bytes = size_t(s.group) * D * sizeof(float);   // dynamic LDS beside the 64 * 2*D-byte tiles
  auto launch = [&](auto kernel) -> hipError_t {
    const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, int(sums_bytes));
    if (ea != hipSuccess) return ea;
    kernel<<<grid, block, sums_bytes, st>>>(kp, qp, cu_q, cu_kv, cu_k, scores, tpw, s DLLM_CHECK_PASS);
    return hipGetLastError();
  };
  if (s.group % 4 == 0) return launch(score_kernel<ES, D, 4>);
  if (s.group % 2 == 0) return launch(score_kernel<ES, D, 2>);
  return launch(score_kernel<ES, D, 1>);
}

static std::atomic<int32_t> g_select_form{DLLM_SELECT_FORM_AUTO};
int32_t set_select_form(int32_t form) {
  if (form != DLLM_SELECT_FORM_AUTO && form != DLLM_SELECT_FORM_TWO_LAUNCHES && form != DLLM_SELECT_FORM_ONE_LAUNCH)
    return -1;
  return g_select_form.exchange(form);
}

// Shapes select_fused_kernel can take.
static bool fused_can(const Shape& s, dllm_dtype dt, int32_t pool_w, int32_t head_sum) {
  (void)pool_w;   // (any window the call accepts)
  if (head_sum) return false;
  if (s.group != 1 && s.group != 2 && s.group != 4) return false;
  if (s.d * (dt == DLLM_BF16 ? 2 : 4) > 256) return false;
  return s.max_kv <= kFusedWords * 64;
}
// ... and where it pays (measured on batches of equal lists, 1 to 4 query heads per KV head, lists of
// 2048 to 8192): each (sequence, KV head) pair is one workgroup that takes most of a compute unit's
// LDS, so the pairs run in rounds of one per compute unit.  The form wins by 5 to 30 % when the last
// round is mostly full, three quarters of the compute units in a single round, four fifths when there
// are several, and loses up to 2x when a few pairs leave most of the chip idle.  Lists of very
// different lengths make the rounds uneven, so the batch must also be fairly even (mean length at least
// 3/4 of the longest).  Walking the sequences longest first (see the kernel) makes up for most of that
// when there are several rounds, but not more: on 16 sequences of 770 to 3411 positions the two forms
// then tie (54.9 against 55.9 us in one harness, 56.3 against 54.9 us in the other; 56.2 us in batch
// order), so such batches keep two launches.
static int compute_units() {
  static std::atomic<int> cached{0};
  int n = cached.load();
  if (n > 0) return n;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  cached.store(n);
  return n;
}
static bool fused_pays(const Shape& s) {
  // a call this small is launch latency and nothing else: one launch instead of two (7.9 against 9.4 us on
  // one sequence of 256 positions with four heads; at 1024 positions and 32 heads two launches win again)
  if (int64_t(s.total_kv) * s.hkv <= 4096) return true;
  const int64_t pairs = int64_t(s.batch) * s.hkv, cus = compute_units();
  const int64_t rounds = (pairs + cus - 1) / cus;
  const bool full = rounds == 1 ? 4 * pairs >= 3 * cus : 5 * pairs >= 4 * rounds * cus;
  const bool even = 4 * int64_t(s.total_kv) >= 3 * int64_t(s.batch) * s.max_kv;
  return full && even;
}

template <int ES, int D>
static hipError_t launch_fused(const Shape& s, const void* k, const void* q, const int32_t* cu_q,
                               const int32_t* cu_kv, const int32_t* cu_k, int32_t total_k, int32_t forced_tail,
                               int32_t pool_w, int32_t* idx_out, hipStream_t st) {
  const char *kp = static_cast<const char*>(k), *qp = static_cast<const char*>(q);
  auto launch = [&](auto kernel, size_t lds, int waves) -> hipError_t {
    const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (ea != hipSuccess) return ea;
    const int32_t ranked = s.batch <= 64 && int64_t(s.batch) * s.hkv > compute_units() ? 1 : 0;
    kernel<<<dim3(s.batch * s.hkv), dim3(waves * 64), lds, st>>>(kp, qp, cu_q, cu_kv, cu_k, total_k, forced_tail,
                                                                      pool_w, ranked, idx_out, s DLLM_CHECK_PASS);
    return hipGetLastError();
  };
  if (s.group == 4) return launch(select_fused_kernel<ES, D, 4>, FusedLds<ES, D, 4>::bytes, fused_waves<4>());
  if (s.group == 2) return launch(select_fused_kernel<ES, D, 2>, FusedLds<ES, D, 2>::bytes, fused_waves<2>());
  return launch(select_fused_kernel<ES, D, 1>, FusedLds<ES, D, 1>::bytes, fused_waves<1>());
}

int32_t select_form_of(const Shape& s, dllm_dtype dt, int32_t pool_w, int32_t head_sum) {
  const int32_t form = g_select_form.load();
  const bool one = form != DLLM_SELECT_FORM_TWO_LAUNCHES && fused_can(s, dt, pool_w, head_sum) &&
                   (form == DLLM_SELECT_FORM_ONE_LAUNCH || fused_pays(s));
  return one ? DLLM_SELECT_FORM_ONE_LAUNCH : DLLM_SELECT_FORM_TWO_LAUNCHES;
}

hipError_t launch_select(const Shape& s, dllm_dtype dt, const void* q, const void* k, const int32_t* cu_q,
                         const int32_t* cu_kv, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                         int32_t pool_w, int32_t forced_tail, int32_t head_sum, int32_t* idx_out, void* ws,
                         hipStream_t st) {
  (void)max_k;
  if (select_form_of(s, dt, pool_w, head_sum) == DLLM_SELECT_FORM_ONE_LAUNCH)
    return dt == DLLM_BF16 ? (s.d == 128 ? launch_fused<2, 128>(s, k, q, cu_q, cu_kv, cu_k, total_k, forced_tail, pool_w, idx_out, st)
                                         : launch_fused<2, 64>(s, k, q, cu_q, cu_kv, cu_k, total_k, forced_tail, pool_w, idx_out, st))
                           : launch_fused<4, 64>(s, k, q, cu_q, cu_kv, cu_k, total_k, forced_tail, pool_w, idx_out, st);
  const SelectPlan p = plan_select(s);
  float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_scores);
  hipError_t e;
  if (dt == DLLM_BF16)
    e = s.d == 128 ? launch_score<2, 128>(s, k, q, cu_q, cu_kv, cu_k, scores, st)
                   : launch_score<2, 64>(s, k, q, cu_q, cu_kv, cu_k, scores, st);
  else
    e = s.d == 128 ? launch_score<4, 128>(s, k, q, cu_q, cu_kv, cu_k, scores, st)
                   : launch_score<4, 64>(s, k, q, cu_q, cu_kv, cu_k, scores, st);
  if (e != hipSuccess) return e;

  const float* ranked = scores;
  if (head_sum) {   // sum (pooled) scores over the heads first; the top-k then ranks one plain row per sequence
    float* summed = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_summed);
    head_sum_kernel<<<dim3((s.max_kv + 255) / 256, s.batch), 256, 0, st>>>(scores, cu_kv, cu_k, s.total_kv, pool_w,
                                                                           forced_tail, s.hq, summed DLLM_CHECK_PASS);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    ranked = summed;
    pool_w = 1;
  }
  const dim3 grid(head_sum ? 1 : s.hq, s.batch);
  const int32_t lpad = (s.max_kv + 63) & ~63;
  if (s.max_kv <= 8 * kTopkThreads) {
    // Keys in registers.  (Sixteen keys per thread for lists of up to 8192 measured slower than the
    // kernel below on the mixed workload, 20.5 against 18.1 us, although each workgroup took less time:
    // they did not all run at once.  Thirty-two per thread in four waves took 25 us.)
    topk_reg_kernel<8, kTopkThreads><<<grid, kTopkThreads, pool_w == 1 ? 0 : size_t(lpad) * 4, st>>>(
        ranked, cu_kv, cu_k, s.total_kv, total_k, pool_w, forced_tail, head_sum, s.hq, idx_out DLLM_CHECK_PASS);
    return hipGetLastError();
  }
  const size_t lds = size_t(lpad) * 4 * (pool_w == 1 ? 1 : 2);
  if (lds > 64 * 1024) {   // beyond the default dynamic-LDS limit: raise it for this kernel on this device
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(topk_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (e != hipSuccess) return e;
  }
  topk_kernel<<<grid, kTopkThreads, lds, st>>>(
      ranked, cu_kv, cu_k, s.total_kv, total_k, pool_w, lpad, forced_tail, head_sum, s.hq, idx_out DLLM_CHECK_PASS);
  return hipGetLastError();
}

}  // namespace dllm
