// Refresh-phase attention (Section 2.3, Eq. 3): dense bidirectional softmax attention, bf16 inputs,
// fp32 softmax state and accumulators, on the gfx950 matrix cores.  This path is a dense
// contraction (4*Lq*Lkv*D flop per head against O(L*D) bytes), so it is bound by MFMA throughput.
//
// Shape of the kernel
//   - A workgroup is four waves, one per SIMD, and owns 256 query rows of one (sequence, head); a wave
//     owns 64 of them as two blocks of 32.  Every K operand (ds_read_b128) and every V^T operand
//     (ds_read_b64_tr_b16) fetched from LDS feeds two MFMAs, one per block, which halves the LDS
//     operand traffic per flop, and the two blocks give the wave independent work to interleave.
//   - K/V tiles of 64 keys go from global memory straight into LDS (global_load_lds, 16 bytes per
//     lane), two tiles ahead of their use, into rings of four tiles each (128 KB at D = 128); one
//     workgroup barrier per tile.  LDS tiles are XOR-swizzled by row; since the LDS side of such a load
//     is lane-contiguous, the swizzle is applied to the global chunk each lane fetches.
//   - Keys are walked in steps of 32 with a three-deep software pipeline.  Iteration j issues
//         S^T(j+1) = K(j+1) Q^T          16 MFMAs (D = 128), A by ds_read_b128 one iteration ahead
//         P(j)     = exp2(S(j) z - m z)   vector work on the scores of the previous iteration
//         O^T     += V(j-1)^T P(j-1)^T    16 MFMAs, A by ds_read_b64_tr_b16 in the same iteration
//     so the matrix work of an iteration does not depend on its vector work and the issue order can
//     alternate them freely (one MFMA, then a few vector and LDS instructions, and so on).
//   - Q is not pre-scaled (rounding the scaled queries to bf16 again costs 2e-2 of output accuracy at
//     logits around 20): scores leave the matrix core raw, and one fused multiply-add per score,
//     s * z - m * z with z = softmax_scale * log2(e), makes them base-2 logits relative to the running
//     maximum m.
//   - m is raised lazily (only when a score exceeds it by more than 2^8, so probabilities may exceed 1
//     until then) behind one uniform branch per iteration.  When it is raised after iteration j, the
//     row sums are rescaled at once; the output accumulators, which still have to take P(j) V(j) at the
//     old scale during iteration j+1, are rescaled one iteration later.
//   - The loop is unrolled over one turn of the rings (eight steps), so every LDS address is a register
//     fixed before the loop plus an immediate offset.
#include <algorithm>
#include <type_traits>
#include <utility>

#include "attn_tile.h"
#include "attend_dense_step.inc"

namespace dllm {

constexpr int kDenseK = 64;          // keys per LDS tile
constexpr int kDenseRing = 4;        // K tiles, and V tiles, resident in LDS
constexpr int kDenseWaves = 4;       // waves per workgroup
constexpr int kDenseQB = 2;          // 32-query blocks per wave
constexpr int kDenseRows = kDenseWaves * kDenseQB * 32;   // query rows per workgroup
constexpr float kLazyStep = 8.0f;    // log2 of the growth that forces a rescale

typedef __attribute__((ext_vector_type(16))) int i32x16;

// The state a wave carries through the key loop, bound to the registers the step text of
// attend_dense_step.inc names.
//   a[0 : 16*2*NDB)          acc   O^T accumulators [qb][db][16]
//   a[.. +  4*2*NT)          q     Q^T operands [qb][t][4]
//   v[96:127], v[128:159]    st_a, st_b   raw scores of two consecutive steps, [qb][16]
//   v[160:175], v[176:191]   pb_a, pb_b   packed probabilities of two consecutive steps, [qb][u][4]
//   v[192 : 192 + 4*NT)      kop   K operands of the next score chain, [t][4]
//   v[80:95]                 addr  LDS byte addresses: K operand [t], then V^T operand [rd][db] from +8
//   a[.. + 16*2)             ls    row-sum blocks [qb][16] (only row 0 is used)
//   v72 .. v75               nmz[2] (= -m z per block), mx[2] (lane maxima of the newest scores)
//   v[76:79], v[224:255]     scratch of a step (logits in flight, V^T operand buffers)
// C++ code may read and write the v-register variables between steps like any others, and may write q;
// the accumulators are only ever handed from one assembly block to the next (this compiler cannot take
// single elements out of an a-register tuple that an assembly block has written), so clearing,
// rescaling and reading them are assembly blocks too.
template <int D>
struct DenseState;

// What the first step of a tile needs to request the tile two ahead: the tile's first K and V row
// (wave-uniform), the byte offset of each of this lane's 16-byte chunks from there, and the LDS address
// of this wave's slice of a load round.
template <int NLD>
struct DenseTileLoad {
  const char *k, *v;
  uint32_t off[NLD];
  uint32_t wave_lds;
};

#define DLLM_DENSE_SCRATCH                                                                                        \
  "v76", "v77", "v78", "v79", "v224", "v225", "v226", "v227", "v228", "v229", "v230", "v231", "v232", "v233", "v234", \
      "v235", "v236", "v237", "v238", "v239", "v240", "v241", "v242", "v243", "v244", "v245", "v246", "v247", "v248", \
      "v249", "v250", "v251", "v252", "v253", "v254", "v255"
#define DLLM_R16(k, x) "=v"(x[16 * (k) + 0]), "=v"(x[16 * (k) + 1]), "=v"(x[16 * (k) + 2]), "=v"(x[16 * (k) + 3]), \
      "=v"(x[16 * (k) + 4]), "=v"(x[16 * (k) + 5]), "=v"(x[16 * (k) + 6]), "=v"(x[16 * (k) + 7]),                  \
      "=v"(x[16 * (k) + 8]), "=v"(x[16 * (k) + 9]), "=v"(x[16 * (k) + 10]), "=v"(x[16 * (k) + 11]),               \
      "=v"(x[16 * (k) + 12]), "=v"(x[16 * (k) + 13]), "=v"(x[16 * (k) + 14]), "=v"(x[16 * (k) + 15])

// Row sums are taken on the matrix cores: one more accumulator block per query block (ls) takes P^T times
// a matrix whose first row is ones (the operand `ones`: lanes 0 and 32 hold eight bf16 ones, the others
// zeros), so row 0 of that block (register 0 of lanes 0..31) is the sum of the bf16 probabilities of the
// lane's query -- the same values the P V product multiplies, added in fp32 like its terms.  The vector
// form (unpack each packed pair with a shift and a mask, two adds) costs four vector instructions per pair
// of scores, a third of the step's vector work; v_dot2c_f32_bf16 does it in one but runs on the matrix
// pipe and holds back the MFMAs (+18 cycles per MFMA), and summing the unrounded values is off by up to
// 2^-8 of a row that one key rules.  Measured: 2 % of the launch.
#define DLLM_LS_OUT_128 "={a[192:207]}"(ls[0]), "={a[208:223]}"(ls[1])
#define DLLM_LS_OUT_64 "={a[96:111]}"(ls[0]), "={a[112:127]}"(ls[1])
#define DLLM_LS_TIED(a, b) a(ls[0]), b(ls[1])

template <>
struct DenseState<128> {
  static constexpr int kAcc = 128;   // accumulator registers
  f32x16 acc[8], q[4], st_a[2], st_b[2], kop[2], pb_a, pb_b;
  f32x16 ls[2];   // row sums (a-registers behind the queries, see above)
  v4u ones;
  float nmz[2], mx[2];   // v72, v73 (= -m z per block); v74, v75 (lane maxima of the newest scores)
  i32x16 addr;
#define DLLM_ACC_OUT                                                                                          \
  "={a[0:15]}"(acc[0]), "={a[16:31]}"(acc[1]), "={a[32:47]}"(acc[2]), "={a[48:63]}"(acc[3]),                  \
      "={a[64:79]}"(acc[4]), "={a[80:95]}"(acc[5]), "={a[96:111]}"(acc[6]), "={a[112:127]}"(acc[7])
#define DLLM_ACC_TIED "0"(acc[0]), "1"(acc[1]), "2"(acc[2]), "3"(acc[3]), "4"(acc[4]), "5"(acc[5]), "6"(acc[6]), "7"(acc[7])
#define DLLM_ACC_IN                                                                                           \
  "{a[0:15]}"(acc[0]), "{a[16:31]}"(acc[1]), "{a[32:47]}"(acc[2]), "{a[48:63]}"(acc[3]), "{a[64:79]}"(acc[4]), \
      "{a[80:95]}"(acc[5]), "{a[96:111]}"(acc[6]), "{a[112:127]}"(acc[7])
#define DLLM_Q_IN "{a[128:143]}"(q[0]), "{a[144:159]}"(q[1]), "{a[160:175]}"(q[2]), "{a[176:191]}"(q[3])
  template <bool AB, int KOFF, int VOFF0, int VOFF1, int LK, int LV>
  __device__ __forceinline__ void step(float zs, const DenseTileLoad<4>& tl, uint64_t& grow) {
    if constexpr (AB)
      asm volatile(DLLM_DENSE_STEP_128_AB
                   : DLLM_ACC_OUT, "={v[128:143]}"(st_b[0]), "={v[144:159]}"(st_b[1]), "={v[160:175]}"(pb_a),
                     "={v[192:207]}"(kop[0]), "={v[208:223]}"(kop[1]), DLLM_LS_OUT_128, "={v74}"(mx[0]),
                     "={v75}"(mx[1]), [grow] "=s"(grow)
                   : DLLM_ACC_TIED, "11"(kop[0]), "12"(kop[1]), DLLM_LS_TIED("13", "14"), [ones] "v"(ones), "{v72}"(nmz[0]), "{v73}"(nmz[1]), DLLM_Q_IN, "{v[96:111]}"(st_a[0]),
                     "{v[112:127]}"(st_a[1]), "{v[176:191]}"(pb_b), "{v[80:95]}"(addr), [zs] "s"(zs), [lazy] "s"(kLazyStep),
                     [koff] "n"(KOFF), [voff0] "n"(VOFF0), [voff1] "n"(VOFF1), [kt] "s"(tl.k), [vt] "s"(tl.v),
                     [lo0] "v"(tl.off[0]), [lo1] "v"(tl.off[1]), [lo2] "v"(tl.off[2]), [lo3] "v"(tl.off[3]),
                     [wl] "s"(tl.wave_lds), [lk] "n"(LK), [lv] "n"(LV)
                   : "memory", "m0", "scc", DLLM_DENSE_SCRATCH);
    else
      asm volatile(DLLM_DENSE_STEP_128_BA
                   : DLLM_ACC_OUT, "={v[96:111]}"(st_a[0]), "={v[112:127]}"(st_a[1]), "={v[176:191]}"(pb_b),
                     "={v[192:207]}"(kop[0]), "={v[208:223]}"(kop[1]), DLLM_LS_OUT_128, "={v74}"(mx[0]),
                     "={v75}"(mx[1]), [grow] "=s"(grow)
                   : DLLM_ACC_TIED, "11"(kop[0]), "12"(kop[1]), DLLM_LS_TIED("13", "14"), [ones] "v"(ones), "{v72}"(nmz[0]), "{v73}"(nmz[1]), DLLM_Q_IN, "{v[128:143]}"(st_b[0]),
                     "{v[144:159]}"(st_b[1]), "{v[160:175]}"(pb_a), "{v[80:95]}"(addr), [zs] "s"(zs), [lazy] "s"(kLazyStep),
                     [koff] "n"(KOFF), [voff0] "n"(VOFF0), [voff1] "n"(VOFF1)
                   : "memory", DLLM_DENSE_SCRATCH);
  }
  // the closing P V product, with the probabilities of pb_a (A) or pb_b; `ad`: addr with the V row
  // offset added to the V^T operand addresses (it is not a compile-time constant here)
  template <bool A>
  __device__ __forceinline__ void tail(i32x16 ad) {
    if constexpr (A)
      asm volatile(DLLM_DENSE_TAIL_128_A
                   : DLLM_ACC_OUT, DLLM_LS_OUT_128
                   : DLLM_ACC_TIED, DLLM_LS_TIED("8", "9"), [ones] "v"(ones), "{v[160:175]}"(pb_a), "{v[80:95]}"(ad), [voff0] "n"(0), [voff1] "n"(16 * 256)
                   : "memory", DLLM_DENSE_SCRATCH);
    else
      asm volatile(DLLM_DENSE_TAIL_128_B
                   : DLLM_ACC_OUT, DLLM_LS_OUT_128
                   : DLLM_ACC_TIED, DLLM_LS_TIED("8", "9"), [ones] "v"(ones), "{v[176:191]}"(pb_b), "{v[80:95]}"(ad), [voff0] "n"(0), [voff1] "n"(16 * 256)
                   : "memory", DLLM_DENSE_SCRATCH);
  }
  // S^T(0) into st_a from the K operands in kop
  __device__ __forceinline__ void score0() {
    asm volatile(DLLM_DENSE_SCORE0_128
                 : "={v[96:111]}"(st_a[0]), "={v[112:127]}"(st_a[1])
                 : "{v[192:207]}"(kop[0]), "{v[208:223]}"(kop[1]), DLLM_Q_IN);
  }
  __device__ __forceinline__ void row_sums(float& l0, float& l1) {
    asm volatile("s_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 %0, a192\n\tv_accvgpr_read_b32 %1, a208"
                 : "=v"(l0), "=v"(l1) : "{a[192:207]}"(ls[0]), "{a[208:223]}"(ls[1]));
  }
  __device__ __forceinline__ void acc_clear() { asm volatile(DLLM_DENSE_ACC_INIT_128 : DLLM_ACC_OUT, DLLM_LS_OUT_128); }
  // acc[qb] *= al[qb]; waits out the matrix pipe first (results may be read only 12 wait states after the
  // MFMA was issued, and nothing but software enforces it)
  __device__ __forceinline__ void acc_scale(float al0, float al1) {
    asm volatile(DLLM_DENSE_ACC_SCALE_128 : DLLM_ACC_OUT, DLLM_LS_OUT_128 : DLLM_ACC_TIED, DLLM_LS_TIED("8", "9"), [al0] "v"(al0), [al1] "v"(al1) : DLLM_DENSE_SCRATCH);
  }
  // all accumulators of block qb, head_dim block db, after the matrix pipe has drained
  __device__ __forceinline__ void acc_read(float (&x)[kAcc]) {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    asm volatile(DLLM_DENSE_ACC_READ_0 : DLLM_R16(0, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_1 : DLLM_R16(1, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_2 : DLLM_R16(2, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_3 : DLLM_R16(3, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_4 : DLLM_R16(4, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_5 : DLLM_R16(5, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_6 : DLLM_R16(6, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_7 : DLLM_R16(7, x) : DLLM_ACC_IN);
  }
#undef DLLM_ACC_OUT
#undef DLLM_ACC_TIED
#undef DLLM_ACC_IN
#undef DLLM_Q_IN
  // element access (indices are compile-time constants after unrolling)
  __device__ __forceinline__ float q_get(int qb, int t, int c) const { return q[2 * qb + t / 4][4 * (t % 4) + c]; }
  __device__ __forceinline__ void q_set(int qb, int t, int c, float x) { q[2 * qb + t / 4][4 * (t % 4) + c] = x; }
  __device__ __forceinline__ float kop_get(int t, int c) const { return kop[t / 4][4 * (t % 4) + c]; }
  __device__ __forceinline__ void kop_set(int t, int c, float x) { kop[t / 4][4 * (t % 4) + c] = x; }
};

template <>
struct DenseState<64> {
  static constexpr int kAcc = 64;
  f32x16 acc[4], q[2], st_a[2], st_b[2], kop[1], pb_a, pb_b;
  f32x16 ls[2];   // row sums (a-registers behind the queries, see above)
  v4u ones;
  float nmz[2], mx[2];   // v72, v73 (= -m z per block); v74, v75 (lane maxima of the newest scores)
  i32x16 addr;
#define DLLM_ACC_OUT "={a[0:15]}"(acc[0]), "={a[16:31]}"(acc[1]), "={a[32:47]}"(acc[2]), "={a[48:63]}"(acc[3])
#define DLLM_ACC_TIED "0"(acc[0]), "1"(acc[1]), "2"(acc[2]), "3"(acc[3])
#define DLLM_ACC_IN "{a[0:15]}"(acc[0]), "{a[16:31]}"(acc[1]), "{a[32:47]}"(acc[2]), "{a[48:63]}"(acc[3])
#define DLLM_Q_IN "{a[64:79]}"(q[0]), "{a[80:95]}"(q[1])
  template <bool AB, int KOFF, int VOFF0, int VOFF1, int LK, int LV>
  __device__ __forceinline__ void step(float zs, const DenseTileLoad<2>& tl, uint64_t& grow) {
    if constexpr (AB)
      asm volatile(DLLM_DENSE_STEP_64_AB
                   : DLLM_ACC_OUT, "={v[128:143]}"(st_b[0]), "={v[144:159]}"(st_b[1]), "={v[160:175]}"(pb_a),
                     "={v[192:207]}"(kop[0]), DLLM_LS_OUT_64, "={v74}"(mx[0]),
                     "={v75}"(mx[1]), [grow] "=s"(grow)
                   : DLLM_ACC_TIED, "7"(kop[0]), DLLM_LS_TIED("8", "9"), [ones] "v"(ones), "{v72}"(nmz[0]), "{v73}"(nmz[1]), DLLM_Q_IN, "{v[96:111]}"(st_a[0]), "{v[112:127]}"(st_a[1]),
                     "{v[176:191]}"(pb_b), "{v[80:95]}"(addr), [zs] "s"(zs), [lazy] "s"(kLazyStep), [koff] "n"(KOFF), [voff0] "n"(VOFF0),
                     [voff1] "n"(VOFF1), [kt] "s"(tl.k), [vt] "s"(tl.v), [lo0] "v"(tl.off[0]), [lo1] "v"(tl.off[1]),
                     [wl] "s"(tl.wave_lds), [lk] "n"(LK), [lv] "n"(LV)
                   : "memory", "m0", "scc", DLLM_DENSE_SCRATCH);
    else
      asm volatile(DLLM_DENSE_STEP_64_BA
                   : DLLM_ACC_OUT, "={v[96:111]}"(st_a[0]), "={v[112:127]}"(st_a[1]), "={v[176:191]}"(pb_b),
                     "={v[192:207]}"(kop[0]), DLLM_LS_OUT_64, "={v74}"(mx[0]),
                     "={v75}"(mx[1]), [grow] "=s"(grow)
                   : DLLM_ACC_TIED, "7"(kop[0]), DLLM_LS_TIED("8", "9"), [ones] "v"(ones), "{v72}"(nmz[0]), "{v73}"(nmz[1]), DLLM_Q_IN, "{v[128:143]}"(st_b[0]), "{v[144:159]}"(st_b[1]),
                     "{v[160:175]}"(pb_a), "{v[80:95]}"(addr), [zs] "s"(zs), [lazy] "s"(kLazyStep), [koff] "n"(KOFF), [voff0] "n"(VOFF0),
                     [voff1] "n"(VOFF1)
                   : "memory", DLLM_DENSE_SCRATCH);
  }
  template <bool A>
  __device__ __forceinline__ void tail(i32x16 ad) {
    if constexpr (A)
      asm volatile(DLLM_DENSE_TAIL_64_A
                   : DLLM_ACC_OUT, DLLM_LS_OUT_64
                   : DLLM_ACC_TIED, DLLM_LS_TIED("4", "5"), [ones] "v"(ones), "{v[160:175]}"(pb_a), "{v[80:95]}"(ad), [voff0] "n"(0), [voff1] "n"(16 * 128)
                   : "memory", DLLM_DENSE_SCRATCH);
    else
      asm volatile(DLLM_DENSE_TAIL_64_B
                   : DLLM_ACC_OUT, DLLM_LS_OUT_64
                   : DLLM_ACC_TIED, DLLM_LS_TIED("4", "5"), [ones] "v"(ones), "{v[176:191]}"(pb_b), "{v[80:95]}"(ad), [voff0] "n"(0), [voff1] "n"(16 * 128)
                   : "memory", DLLM_DENSE_SCRATCH);
  }
  __device__ __forceinline__ void score0() {
    asm volatile(DLLM_DENSE_SCORE0_64
                 : "={v[96:111]}"(st_a[0]), "={v[112:127]}"(st_a[1])
                 : "{v[192:207]}"(kop[0]), DLLM_Q_IN);
  }
  __device__ __forceinline__ void row_sums(float& l0, float& l1) {
    asm volatile("s_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 %0, a96\n\tv_accvgpr_read_b32 %1, a112"
                 : "=v"(l0), "=v"(l1) : "{a[96:111]}"(ls[0]), "{a[112:127]}"(ls[1]));
  }
  __device__ __forceinline__ void acc_clear() { asm volatile(DLLM_DENSE_ACC_INIT_64 : DLLM_ACC_OUT, DLLM_LS_OUT_64); }
  __device__ __forceinline__ void acc_scale(float al0, float al1) {
    asm volatile(DLLM_DENSE_ACC_SCALE_64 : DLLM_ACC_OUT, DLLM_LS_OUT_64 : DLLM_ACC_TIED, DLLM_LS_TIED("4", "5"), [al0] "v"(al0), [al1] "v"(al1) : DLLM_DENSE_SCRATCH);
  }
  __device__ __forceinline__ void acc_read(float (&x)[kAcc]) {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    asm volatile(DLLM_DENSE_ACC_READ_0 : DLLM_R16(0, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_1 : DLLM_R16(1, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_2 : DLLM_R16(2, x) : DLLM_ACC_IN);
    asm volatile(DLLM_DENSE_ACC_READ_3 : DLLM_R16(3, x) : DLLM_ACC_IN);
  }
#undef DLLM_ACC_OUT
#undef DLLM_ACC_TIED
#undef DLLM_ACC_IN
#undef DLLM_Q_IN
  __device__ __forceinline__ float q_get(int qb, int t, int c) const { return q[qb][4 * t + c]; }
  __device__ __forceinline__ void q_set(int qb, int t, int c, float x) { q[qb][4 * t + c] = x; }
  __device__ __forceinline__ float kop_get(int t, int c) const { return kop[0][4 * t + c]; }
  __device__ __forceinline__ void kop_set(int t, int c, float x) { kop[0][4 * t + c] = x; }
};

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ... in order
template <typename F, int... C>
__device__ __forceinline__ void for_each_round(F& f, std::integer_sequence<int, C...>) {
  (f(std::integral_constant<int, C>{}), ...);
}

// which: 1 = only sequences flagged dense in seq_mode; 2 = every sequence
template <int D>
__global__ __launch_bounds__(kDenseWaves * 64, 1) void attend_dense_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const uint8_t* __restrict__ seq_mode,
    int which, uint16_t* __restrict__ o, Shape s DLLM_CHECK_PARAM) {
  DLLM_CHECK_EXIT();
  constexpr int NQB = kDenseQB;
  constexpr int CH = D / 8;
  constexpr int ROWB = 2 * D;
  constexpr int TILEB = kDenseK * ROWB;
  constexpr int VBASE = kDenseRing * TILEB;      // V ring follows the K ring
  constexpr int NTHREADS = kDenseWaves * 64;
  constexpr int NLD = kDenseK * CH / NTHREADS;   // 16-byte loads per lane, tile and tensor
  constexpr int NT = D / 16;
  constexpr int NDB = D / 32;
  constexpr int ROUND = 2 * kDenseRing;          // steps in one turn of the rings
  static_assert(NLD >= 1 && kDenseK * CH % NTHREADS == 0, "tile does not split evenly over the threads");
  static_assert(kDenseRing * TILEB <= 65536, "ring offsets must fit the 16-bit LDS offset field");

  __shared__ __attribute__((aligned(16))) char smem[2 * kDenseRing * TILEB];   // K ring, V ring

  // Which query tile of which (sequence, head) this workgroup takes.
  //
  // Batches of up to 64 sequences are launched as a one-dimensional grid with just enough workgroups for the
  // query tiles the batch can have (the host bounds their number from total_q), and every workgroup finds
  // its tile itself: lane i looks at sequence i, a prefix sum over the tiles of the sequences that are
  // attended densely places the workgroup.  A mixed batch then starts no workgroups for its sparse
  // sequences, and a ragged one none for the query tiles short sequences do not have (an empty workgroup
  // holds a whole compute unit until it has found out that it is empty).  Larger batches use the
  // three-dimensional grid (query tile, head, sequence) with an early exit.
  //
  // Workgroups are handed to the eight XCDs round-robin by launch order, and each XCD has its own L2.
  // The numbering is such that the workgroups that stream the same K/V -- the query tiles of the query
  // heads that share one KV head of one sequence -- land on one XCD (launch ids equal modulo 8) and
  // share its L2, while consecutive (sequence, KV head) pairs go to different XCDs.
  int qtile, h, b, q0, nq, kv0, L;
  if (gridDim.y == 1 && gridDim.z == 1) {
    const int lane0 = threadIdx.x & 63;
    int my_q0 = 0, my_nq = 0, my_kv0 = 0, my_L = 0, my_tiles = 0;
    if (lane0 < s.batch) {
      my_q0 = cu_q[lane0];
      my_nq = cu_q[lane0 + 1] - my_q0;
      my_kv0 = cu_kv[lane0];
      my_L = cu_kv[lane0 + 1] - my_kv0;
      const bool dense = which == 2 || (seq_mode != nullptr && seq_mode[lane0] == DLLM_SEQ_DENSE);
      my_tiles = dense ? (my_nq + kDenseRows - 1) / kDenseRows : 0;
    }
    const int incl = int(wave_inclusive_sum(uint32_t(my_tiles)));
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const int n = blockIdx.x;
    int place;   // position of the tile in (sequence, tile) order, times what follows
    uint64_t m;
    if ((s.hkv & 7) == 0) {
      // XCD x = n % 8 takes KV heads x, x + 8, ...; within the XCD: sequence, KV head, query head of its group, tile
      const int per_seq = s.group * (s.hkv >> 3);
      place = n >> 3;
      if (place >= total * per_seq) return;
      m = __builtin_amdgcn_ballot_w64(incl * per_seq > place);
      b = __builtin_ctzll(m);
      const int tb = __builtin_amdgcn_readlane(my_tiles, b);
      const int rem = place - (__builtin_amdgcn_readlane(incl, b) - tb) * per_seq;
      const int per_head_group = tb * s.group;
      const int kvh = (rem / per_head_group) * 8 + (n & 7), r = rem % per_head_group;
      qtile = r % tb;
      h = kvh * s.group + r / tb;
    } else {
      place = n / s.hq;
      h = n % s.hq;
      if (place >= total) return;
      m = __builtin_amdgcn_ballot_w64(incl > place);
      b = __builtin_ctzll(m);
      qtile = place - (__builtin_amdgcn_readlane(incl, b) - __builtin_amdgcn_readlane(my_tiles, b));
    }
    q0 = __builtin_amdgcn_readlane(my_q0, b);
    nq = __builtin_amdgcn_readlane(my_nq, b);
    kv0 = __builtin_amdgcn_readlane(my_kv0, b);
    L = __builtin_amdgcn_readlane(my_L, b);
  } else {
    const int nx = gridDim.x, units = s.hkv * gridDim.z;
    const int n = blockIdx.x + nx * (blockIdx.y + gridDim.y * blockIdx.z);
    qtile = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    if ((units & 7) == 0) {
      const int per_unit = s.group * nx;
      const int j = n >> 3;   // position in this XCD's own launch sequence
      const int r = j % per_unit, unit = (j / per_unit) * 8 + (n & 7);
      qtile = r % nx;
      h = (unit % s.hkv) * s.group + r / nx;
      b = unit / s.hkv;
    }
    if (which == 1 && !(seq_mode != nullptr && seq_mode[b] == DLLM_SEQ_DENSE)) return;
    q0 = cu_q[b];
    nq = cu_q[b + 1] - q0;
    kv0 = cu_kv[b];
    L = cu_kv[b + 1] - kv0;
  }
  const int qbase = qtile * kDenseRows;
  if (qbase >= nq) return;
  const int g = h / s.group;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = lane & 31, hf = lane >> 5;
#ifdef DLLM_DENSE_STAMPS
  // timing experiments only: every workgroup leaves shader-clock counts in its own first output row
  // (and stores no outputs): [0] entry, [1] loop start, [2] loop end, [3] end, [4..11] cycles spent in
  // steps at ring position R, [12] slowest step, [13] number of steps over 3000 cycles
  const uint64_t rt_entry = __builtin_amdgcn_s_memrealtime();   // 100 MHz
  uint64_t t_entry = __builtin_readcyclecounter(), t_loop0 = 0, t_prev = 0, by_r[8] = {0, 0, 0, 0, 0, 0, 0, 0},
           t_max = 0, n_slow = 0, t_part = 0, parts[4] = {0, 0, 0, 0};
#define DLLM_STAMP_PART(i)                                   \
  {                                                          \
    const uint64_t t_now = __builtin_readcyclecounter();     \
    if (i > 0) parts[i] += t_now - t_part;                   \
    t_part = t_now;                                          \
  }
#define DLLM_STAMP_LOOP_START() t_loop0 = t_prev = __builtin_readcyclecounter()
#if DLLM_DENSE_STAMPS < 2
#define DLLM_STAMP_STEP(R)
#else
#define DLLM_STAMP_STEP(R)                                  \
  {                                                         \
    const uint64_t t_now = __builtin_readcyclecounter();    \
    const uint64_t dt = t_now - t_prev;                     \
    by_r[R] += dt;                                          \
    t_max = dt > t_max ? dt : t_max;                        \
    n_slow += dt > 3000 ? 1 : 0;                            \
    t_prev = t_now;                                         \
  }
#endif
#else
#define DLLM_STAMP_LOOP_START()
#define DLLM_STAMP_STEP(R)
#endif

  if (L == 0) {   // nothing to attend to: zeros
    for (int e = tid; e < kDenseRows * D; e += NTHREADS) {
      const int r = qbase + e / D;
      if (r < nq) o[(int64_t(q0 + r) * s.hq + h) * D + e % D] = 0;
    }
    return;
  }

  const char* kbase = reinterpret_cast<const char*>(k + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const char* vbase = reinterpret_cast<const char*>(v + int64_t(kv0) * s.kv_tok + int64_t(g) * s.kv_head);
  const int64_t pitch = s.kv_tok * 2;

  DenseState<D> w;
  // LDS addresses, fixed for the whole pass; ring slot, 32-key half and 16-key quarter are immediates
  {
    KAddr<D> kaddr;
    kaddr.init(lane);
    VtAddr<D> vaddr;
    vaddr.init(lane);
#pragma unroll
    for (int i = 0; i < 16; ++i) w.addr[i] = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) w.addr[t] = kaddr.off(t);
#pragma unroll
    for (int rd = 0; rd < 2; ++rd)
#pragma unroll
      for (int db = 0; db < NDB; ++db) w.addr[8 + NDB * rd + db] = VBASE + vaddr.off(rd, db);
  }
  // Global side of the tile loads: this lane's chunk f = i * NTHREADS + tid of a tile lands at LDS
  // byte 16 * f, i.e. row f / CH, chunk slot f % CH, and must hold chunk (slot ^ swizzle(row)) of
  // that row.  Rows past the end of the sequence re-read its last row (their keys are masked).
  uint32_t ld_off[NLD];   // byte offset of the chunk from the tile's first row (fits: checked on the host)
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * NTHREADS + tid, row = f / CH;
    ld_off[i] = uint32_t(row) * uint32_t(pitch) + uint32_t(((f % CH) ^ tile_swz<D>(row)) << 4);
  }
  // the same for the last tile when the sequence ends inside it: rows past the end re-read the last row
  const int ntiles = (L + kDenseK - 1) / kDenseK;
  uint32_t ld_off_last[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int f = i * NTHREADS + tid, row = min(f / CH, L - 1 - (ntiles - 1) * kDenseK);
    ld_off_last[i] = uint32_t(row) * uint32_t(pitch) + uint32_t(((f % CH) ^ tile_swz<D>(f / CH)) << 4);
  }
  // this wave's slice of each load round, as an LDS byte address
  const uint32_t wave_lds = __builtin_amdgcn_readfirstlane(lds_addr(smem) + wave * 64 * 16);
  auto load_tile = [&](const char* base, int tile, auto lds_off) __attribute__((always_inline)) {
    constexpr int kLdsOff = decltype(lds_off)::value;
    const int t0 = tile * kDenseK;
    if (t0 + kDenseK <= L) {   // whole tile inside the sequence: uniform tile address + fixed lane offsets
      const char* tbase = base + int64_t(t0) * pitch;
      auto round = [&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        load16_to_lds<kLdsOff + i * NTHREADS * 16>(tbase, ld_off[i], wave_lds);
      };
      for_each_round(round, std::make_integer_sequence<int, NLD>{});
    } else {
      auto round = [&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        const int f = i * NTHREADS + tid, r = f / CH;
        const int row = min(t0 + r, L - 1);
        load16_to_lds<kLdsOff + i * NTHREADS * 16>(base + row * pitch + (((f % CH) ^ tile_swz<D>(r)) << 4),
                                                   wave_lds);
      };
      for_each_round(round, std::make_integer_sequence<int, NLD>{});
    }
  };
#define DLLM_IC(x) std::integral_constant<int, (x)> {}

  // the first tiles are requested before anything else, so their latency overlaps the Q loads
  const int rem = L % 32;
  const int nsteps = L / 32 + (rem ? 1 : 0);
  load_tile(kbase, 0, DLLM_IC(0));
  load_tile(vbase, 0, DLLM_IC(VBASE));
  if (ntiles > 1) {
    load_tile(kbase, 1, DLLM_IC(TILEB));
    load_tile(vbase, 1, DLLM_IC(VBASE + TILEB));
  }
#ifdef DLLM_DENSE_FILL_RING   // timing experiments only: all four ring slots filled once (tiles 0..3)
  if (ntiles > 3) {
    load_tile(kbase, 2, DLLM_IC(2 * TILEB));
    load_tile(vbase, 2, DLLM_IC(VBASE + 2 * TILEB));
    load_tile(kbase, 3, DLLM_IC(3 * TILEB));
    load_tile(vbase, 3, DLLM_IC(VBASE + 3 * TILEB));
  }
#endif
  // Iteration 0 multiplies an all-zero P with the second half of ring slot 3 of V (the step "before
  // the first"): clear it, so that no stale NaN pattern meets the zeros.  Tile 3 lands there later.
  {
    constexpr int kHalf = 32 * ROWB;
    for (int e = tid * 16; e < kHalf; e += NTHREADS * 16)
      *reinterpret_cast<v4u*>(smem + VBASE + 3 * TILEB + kHalf + e) = v4u{0u, 0u, 0u, 0u};
  }

  // Q^T operands: lane (col = query, hf) holds Q[query][16t + 8hf .. +8) for every step t, as given
  const float zscale = s.scale * kLog2e;   // > 0; scores * zscale are base-2 logits
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const uint16_t* qp = q + int64_t(q0 + qi) * s.q_tok + int64_t(h) * s.q_head;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      v4u x = v4u{0u, 0u, 0u, 0u};
      if (qi < nq) x = *reinterpret_cast<const v4u*>(qp + 16 * t + 8 * hf);
      w.q_set(qb, t, 0, __uint_as_float(x.x));
      w.q_set(qb, t, 1, __uint_as_float(x.y));
      w.q_set(qb, t, 2, __uint_as_float(x.z));
      w.q_set(qb, t, 3, __uint_as_float(x.w));
    }
  }
  // per query (lane pair l, l ^ 32): -m * z for the running maximum m of the raw scores (w.nmz), the factor
  // the accumulators (outputs and row sums) still have to take, and the accumulators
  float palpha[NQB];
  bool pending = false;   // some palpha != 1 (uniform)
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    palpha[qb] = 1.0f;
  }
  {
    const uint32_t one2 = (lane & 31) == 0 ? 0x3f803f80u : 0u;
    w.ones = v4u{one2, one2, one2, one2};
  }
  w.acc_clear();
#pragma unroll
  for (int i = 0; i < 16; ++i) w.pb_a[i] = w.pb_b[i] = 0.0f;

  // A operands of one step's score chain: rows = 32 keys at byte offset `koff` of the K ring
  auto k_operands = [&](int koff) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const v4u x = *reinterpret_cast<const v4u*>(smem + w.addr[t] + koff);
      w.kop_set(t, 0, __uint_as_float(x.x));
      w.kop_set(t, 1, __uint_as_float(x.y));
      w.kop_set(t, 2, __uint_as_float(x.z));
      w.kop_set(t, 3, __uint_as_float(x.w));
    }
  };
  auto mask_tail = [&](f32x16 (&st)[NQB], int nvalid) __attribute__((always_inline)) {   // keys past the end get no weight
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = 8 * (i / 4) + 4 * hf + (i % 4);
        if (key >= nvalid) st[qb][i] = -INFINITY;
      }
  };
  // largest score of a step per lane (a query's scores sit in the lane pair l, l ^ 32)
  auto lane_max = [&](const f32x16& st) __attribute__((always_inline)) -> float {
    float mx = fmaxf(st[0], st[1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) mx = fmaxf(fmaxf(mx, st[i]), st[i + 1]);
    return mx;
  };
  // What the first step of each tile needs to request the tile two ahead (see the step text).  Past
  // the last tile the last one is requested again, into a ring slot nobody reads any more.
  const int64_t tile_bytes = int64_t(kDenseK) * pitch;
  const bool last_whole = ntiles * kDenseK == L;
  const int load_idx = min(2, ntiles - 1);   // tile the first tile boundary requests
  DenseTileLoad<NLD> tl;
  tl.k = kbase + load_idx * tile_bytes;
  tl.v = vbase + load_idx * tile_bytes;
  tl.wave_lds = wave_lds;
#pragma unroll
  for (int i = 0; i < NLD; ++i) tl.off[i] = (load_idx == ntiles - 1 && !last_whole) ? ld_off_last[i] : ld_off[i];

  wait_tile_loads();
  __syncthreads();

  // scores of step 0, its maxima outright (they may be negative)
  k_operands(0);
  w.score0();
  if (nsteps == 1 && rem) mask_tail(w.st_a, rem);
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) w.nmz[qb] = -(max_across_halves(lane_max(w.st_a[qb])) * zscale);
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int i = 0; i < 16; ++i) w.st_b[qb][i] = 0.0f;
  k_operands(32 * ROWB);   // step 1 (stale LDS if there is none; then unused)

  // Iteration j at position R = j % ROUND of the ring turn, which fixes every LDS offset.  Between two
  // steps the common path is a handful of scalar instructions and one branch; everything else (the end
  // of the sequence, the ragged last step, a running maximum to raise, accumulators that still owe a
  // factor) sits behind that branch.
  // Between two steps the common path is one test and, after the first step of a tile, the advance of
  // the tile pointers; everything else (the end of the sequence, the ragged last step, a running
  // maximum to raise, accumulators that still owe a factor) sits behind that test.  `special` is
  // set while something other than a grown score asks for the careful path: accumulators that owe a
  // factor, or the last steps of the sequence (from one ring turn before the end).
  int j = 0;        // steps done
  int jb = 0;       // steps done at the start of the current ring turn
  uint32_t special = 0;   // (kept wave-uniform in a scalar register)
  int64_t advance = load_idx < ntiles - 1 ? tile_bytes : 0;   // what the tile pointers move by after a tile's first step; 0 once they reached the last tile
  DLLM_STAMP_LOOP_START();
  // one step at ring position R (the text, with every offset it needs)
#define DLLM_RUN_STEP(R, grow)                                                                                  \
  w.template step<(R) % 2 == 0, ((((R) + 2) % ROUND) / 2) * TILEB + (((R) + 2) % 2) * 32 * ROWB,                 \
                  ((((R) + ROUND - 1) % ROUND) / 2) * TILEB + (((R) + ROUND - 1) % 2) * 32 * ROWB,               \
                  ((((R) + ROUND - 1) % ROUND) / 2) * TILEB + (((R) + ROUND - 1) % 2) * 32 * ROWB + 16 * ROWB,   \
                  (((R) / 2 + 2) % kDenseRing) * TILEB, VBASE + (((R) / 2 + 2) % kDenseRing) * TILEB>(zscale, tl, grow)
  // what may need doing after step number j - 1 (at ring position R); true when the sequence is finished
  auto careful = [&](auto rc, uint64_t grow) __attribute__((always_inline)) -> bool {
    constexpr int R = decltype(rc)::value;
    if (pending) {   // hand the accumulators the factor they still owe
      w.acc_scale(palpha[0], palpha[1]);
      palpha[0] = palpha[1] = 1.0f;
      pending = false;
    }
    if (j >= nsteps) return true;
    // tile requests near the end: the pointers stop at the last tile, whose rows may end early
    const int next_load = min((j + 1) / 2 + 2, ntiles - 1);   // tile the next boundary requests
    advance = next_load < ntiles - 1 ? tile_bytes : 0;
    tl.k = kbase + next_load * tile_bytes;
    tl.v = vbase + next_load * tile_bytes;
#pragma unroll
    for (int i = 0; i < NLD; ++i) tl.off[i] = (next_load == ntiles - 1 && !last_whole) ? ld_off_last[i] : ld_off[i];
    const bool ragged = rem != 0 && j + 1 == nsteps;
    if (ragged || grow != 0) {
      // Mask the ragged last step and raise the running maxima for the scores of step j.  Keys past the
      // end were scored from copies of the last row (the tile loads clamp the row), so they carry that
      // row's score and the lane maxima need no second look after masking.
      if (ragged) {
        if constexpr (R % 2 == 0) mask_tail(w.st_b, rem);
        else mask_tail(w.st_a, rem);
      }
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float mz_old = -w.nmz[qb];
        const float mz_new = fmaxf(mz_old, max_across_halves(w.mx[qb]) * zscale);
        const float alpha = __builtin_amdgcn_exp2f(mz_old - mz_new);
        palpha[qb] = alpha;
        w.nmz[qb] = -mz_new;
      }
      pending = true;
    }
    special = __builtin_amdgcn_readfirstlane((pending || j + 2 * ROUND > nsteps) ? 1u : 0u);
    return false;
  };
#define DLLM_STEP(R)                                         \
  {                                                          \
    uint64_t grow;                                           \
    DLLM_RUN_STEP(R, grow);                                  \
    DLLM_STAMP_STEP(R);                                      \
    if ((R) % 2 == 0) {                                      \
      tl.k += advance;                                       \
      tl.v += advance;                                       \
    }                                                        \
    if (__builtin_expect((uint32_t(grow) | uint32_t(grow >> 32) | special) != 0, 0)) { \
      j = jb + (R) + 1;                                      \
      if (careful(DLLM_IC(R), grow)) break;                  \
    }                                                        \
  }
  for (;;) {
    special = __builtin_amdgcn_readfirstlane((pending || jb + 2 * ROUND > nsteps) ? 1u : 0u);
    DLLM_STEP(0)
    DLLM_STEP(1)
    DLLM_STEP(2)
    DLLM_STEP(3)
    DLLM_STEP(4)
    DLLM_STEP(5)
    DLLM_STEP(6)
    DLLM_STEP(7)
    jb += ROUND;
  }
  // the last step's P V product: its probabilities are in pb_a after an odd number of steps, else in pb_b
  {
    const int last = nsteps - 1;
    const int voff = ((last >> 1) % kDenseRing) * TILEB + (last & 1) * 32 * ROWB;
    i32x16 ad = w.addr;
#pragma unroll
    for (int i = 8; i < 16; ++i) ad[i] += voff;
    if (nsteps & 1) w.template tail<true>(ad);
    else w.template tail<false>(ad);
  }
#ifdef DLLM_DENSE_STAMPS
  const uint64_t t_loop1 = __builtin_readcyclecounter();
#endif
  float accv[DenseState<D>::kAcc];   // [qb][db][16]
  w.acc_read(accv);
#ifdef DLLM_DENSE_STAMPS
  if (tid == 0) {
    uint64_t* dst = reinterpret_cast<uint64_t*>(o + (int64_t(q0 + qbase) * s.hq + h) * D);
    dst[0] = t_entry; dst[1] = t_loop0; dst[2] = t_loop1; dst[3] = __builtin_readcyclecounter();
    for (int r = 0; r < 8; ++r) dst[4 + r] = by_r[r];
    dst[12] = t_max; dst[13] = n_slow;
    dst[14] = parts[1]; dst[15] = parts[2]; dst[16] = parts[3];   // load wait, barrier, load issue: sums over the tiles
    dst[17] = rt_entry; dst[18] = __builtin_amdgcn_s_memrealtime();
    dst[19] = (uint64_t(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11))) << 32) | __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
  }
  return;   // the counts sit where outputs would go
#endif
  float lrow[NQB];
  w.row_sums(lrow[0], lrow[1]);   // lanes 0..31: the query's sum; lanes 32..63: row 4 of the block, zero
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qbase + (wave * NQB + qb) * 32 + col;
    const float l = sum_across_halves(lrow[qb]);
    if (qi < nq) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        uint16_t* op = o + (int64_t(q0 + qi) * s.hq + h) * D + db * 32 + 4 * hf;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          v2u w2;
          const float* a = accv + 16 * (NDB * qb + db) + 4 * i4;
          w2.x = cvt_pk_bf16(a[0] * inv, a[1] * inv);
          w2.y = cvt_pk_bf16(a[2] * inv, a[3] * inv);
          *reinterpret_cast<v2u*>(op + 8 * i4) = w2;
        }
      }
    }
  }
}

hipError_t launch_attend_dense_bf16(const Shape& s, const void* q, const void* k, const void* v,
                                    const int32_t* cu_q, const int32_t* cu_kv, const uint8_t* seq_mode, int which,
                                    void* o, hipStream_t st) {
  if (s.max_q == 0) return hipSuccess;   // no sequence has a query: nothing to write
  const int64_t nx = (s.max_q + kDenseRows - 1) / kDenseRows;
  dim3 grid(unsigned(nx), s.hq, s.batch);
  if (s.batch <= 64) {
    // the workgroups place themselves (see the kernel): as many as the batch can have query tiles, times the heads
    const int64_t tiles = std::min<int64_t>(int64_t(s.total_q) / kDenseRows + s.batch, nx * s.batch);
    if (tiles * s.hq < (int64_t(1) << 31)) grid = dim3(unsigned(tiles * s.hq), 1, 1);
  }
  const uint16_t *qh = static_cast<const uint16_t*>(q), *kh = static_cast<const uint16_t*>(k),
                 *vh = static_cast<const uint16_t*>(v);
  if (s.d == 128)
    attend_dense_bf16_kernel<128><<<grid, kDenseWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, seq_mode, which,
                                                                     static_cast<uint16_t*>(o), s DLLM_CHECK_PASS);
  else
    attend_dense_bf16_kernel<64><<<grid, kDenseWaves * 64, 0, st>>>(qh, kh, vh, cu_q, cu_kv, seq_mode, which,
                                                                    static_cast<uint16_t*>(o), s DLLM_CHECK_PASS);
  return hipGetLastError();
}

}  // namespace dllm
