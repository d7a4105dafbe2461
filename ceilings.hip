// Measured ceilings of one MI355X for the two rooflines this library is held to.  Stand-alone
// program (no part of the library): prints what a plain kernel achieves for
//   (a) streaming reads from HBM, no reuse between launches (each launch reads another 512 MiB
//       window of a 6 GiB buffer, so neither L2 nor the 256 MB memory-side cache helps), once with a
//       grid-stride loop and once with a contiguous span per workgroup and non-temporal loads,
//   (b) gathers of 256-byte rows at an 8 KiB token stride, 32 heads active, kept rows random at
//       33 % density and ascending -- the access pattern of Reuse-phase attention,
//   (c) back-to-back v_mfma_f32_32x32x16_bf16 with independent accumulators on every SIMD of the chip, with
//       operands that are all zero, all 1.0, or random normal bf16: the rate and the shader clock the chip
//       holds depend on how many operand bits toggle, because the board's power limit sets the clock,
//   (d) the same MFMA stream (random normal operands) with the other work of a dense attention step beside
//       it: exp / fma / convert vector instructions, LDS reads of 0.5 KB per MFMA, both, and idle slots.
//   (e) what writing a little costs a streaming read: 2048 waves that stay, each walking twelve 64-row tiles of a
//       256-byte column of a [196608 tokens][8 heads][128] bf16 tensor through LDS (the score pass of selection on
//       the grouped-query workload, without its arithmetic), alone, and with the four fp32 score rows per tile
//       written as they are produced or all at the end of the wave's run (6 % of the bytes read).
// All indices are generated on the host and are in bounds by construction; every LDS read stays inside the
// 64 KB array the kernel declares.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      exit(1);                                                                  \
    }                                                                           \
  } while (0)

__global__ __launch_bounds__(256) void stream_read(const uint4* __restrict__ p, size_t n16, unsigned* out) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
    acc.z ^= a.z ^ b.z ^ c.z ^ d.z; acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;   // keeps the loads alive
}

// each workgroup reads one contiguous span, eight non-temporal 16-byte loads per lane in flight
typedef __attribute__((ext_vector_type(4))) unsigned int v4u;
__global__ __launch_bounds__(256) void stream_read_spans(const v4u* __restrict__ p, size_t n16, unsigned* out) {
  const size_t per_block = n16 / gridDim.x;
  const v4u* q = p + (size_t)blockIdx.x * per_block;
  v4u acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i + 7 * 256 < per_block; i += 8 * 256) {
    v4u r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = __builtin_nontemporal_load(q + i + j * 256);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= r[j];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;
}

// wave -> (head, list of rows); NL 16-byte loads per lane in flight, four rows per load instruction
template <int NL>
__global__ __launch_bounds__(256) void gather_rows(const char* __restrict__ base, const int* __restrict__ rows,
                                                   int rows_per_wave, long pitch, unsigned* __restrict__ out) {
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  const int* my = rows + (long)wave * rows_per_wave;
  const char* b = base + (wave & 31) * 256 + (lane & 15) * 16;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (int i = 0; i < rows_per_wave; i += 4 * NL) {
    uint4 r[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) r[j] = *reinterpret_cast<const uint4*>(b + (long)my[i + 4 * j + (lane >> 4)] * pitch);
#pragma unroll
    for (int j = 0; j < NL; ++j) { acc.x ^= r[j].x; acc.y ^= r[j].y; acc.z ^= r[j].z; acc.w ^= r[j].w; }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[wave] = 1;
}

__device__ unsigned hash32(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }
// roughly normal (sum of four uniforms, unit variance)
__device__ float rnd_normal(unsigned seed) {
  float a = 0;
  for (int i = 0; i < 4; ++i) a += (hash32(seed * 4 + i) >> 8) * (1.0f / 16777216.0f) - 0.5f;
  return a * 1.73f;
}
__device__ unsigned rnd_bf16_pair(unsigned seed) {
  return (__float_as_uint(rnd_normal(seed)) >> 16) | (__float_as_uint(rnd_normal(seed + 0x9e3779b9u)) & 0xffff0000u);
}

// (c) eight MFMAs with different operands over four accumulators; mode 0: zeros, 1: all 1.0, 2: random normal
__global__ __launch_bounds__(256, 1) void mfma_by_data(float* out, int iters, int mode, unsigned long long* clk) {
  v4u a[8], b[8];
  const unsigned id = blockIdx.x * 256 + threadIdx.x;
  for (int i = 0; i < 8; ++i)
    for (int c = 0; c < 4; ++c) {
      a[i][c] = mode == 0 ? 0u : mode == 1 ? 0x3f803f80u : rnd_bf16_pair(id * 64 + i * 8 + c);
      b[i][c] = mode == 0 ? 0u : mode == 1 ? 0x3f803f80u : rnd_bf16_pair(id * 64 + i * 8 + 4 + c + 7777777u);
    }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[i]),
                                                          acc[i & 3], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float s = 0.0f;
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += acc[j][i];
  out[id] = s;
  if (id == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

// (d) instruction mixes around the same eight MFMAs, written as assembly so that the mix is exactly what is
// listed.  Registers: v40..v99 random operands, v100..v127 results of the side work, a0..a63 accumulators.
#define REP4(x) x x x x
#define CLOBV "v100","v101","v102","v103","v104","v105","v106","v107","v108","v109","v110","v111","v112","v113","v114","v115","v116","v117","v118","v119","v120","v121","v122","v123","v124","v125","v126","v127"
#define MFA(n, a, b) "v_mfma_f32_32x32x16_bf16 a[" #n "], v[" #a "], v[" #b "], a[" #n "]\n\t"
#define M0 MFA(0:15, 40:43, 72:75)
#define M1 MFA(16:31, 44:47, 76:79)
#define M2 MFA(32:47, 48:51, 80:83)
#define M3 MFA(48:63, 52:55, 84:87)
#define M4 MFA(0:15, 56:59, 88:91)
#define M5 MFA(16:31, 60:63, 92:95)
#define M6 MFA(32:47, 64:67, 96:99)
#define M7 MFA(48:63, 68:71, 72:75)
#define VX "v_fma_f32 v100, v40, v72, v101\n\tv_exp_f32_e32 v102, v41\n\tv_fma_f32 v103, v42, v73, v104\n\tv_cvt_pk_bf16_f32 v105, v43, v44\n\t"
#define DK "ds_read_b128 v[108:111], %0\n\t"
#define DV "ds_read_b64_tr_b16 v[112:113], %1\n\tds_read_b64_tr_b16 v[114:115], %1 offset:2048\n\t"
#define IDLE "s_nop 7\n\ts_nop 7\n\t"

template <int MODE>
__global__ __launch_bounds__(256, 1) void mfma_mix(float* out, int iters, unsigned long long* clk) {
  __shared__ char lds[65536];
  const unsigned id = blockIdx.x * 256 + threadIdx.x;
  const int lane = threadIdx.x & 63;
  for (int e = threadIdx.x; e < 16384; e += 256) reinterpret_cast<unsigned*>(lds)[e] = rnd_bf16_pair(e * 977 + blockIdx.x);
  __syncthreads();
  // byte addresses inside lds[]: at most 3*4096 + 63*16 + 15 and 3*8192 + 3*512 + 15*8 + 2048 + 7
  const int addr = lane * 16 + (threadIdx.x >> 6) * 4096, addr_tr = (lane >> 4) * 512 + (lane & 15) * 8 + (threadIdx.x >> 6) * 8192;
#define SETV(r) asm volatile("v_mov_b32 v" #r ", %0" :: "v"(rnd_bf16_pair(id * 64 + r)));
  SETV(40) SETV(41) SETV(42) SETV(43) SETV(44) SETV(45) SETV(46) SETV(47) SETV(48) SETV(49) SETV(50) SETV(51) SETV(52) SETV(53) SETV(54) SETV(55)
  SETV(56) SETV(57) SETV(58) SETV(59) SETV(60) SETV(61) SETV(62) SETV(63) SETV(64) SETV(65) SETV(66) SETV(67) SETV(68) SETV(69) SETV(70) SETV(71)
  SETV(72) SETV(73) SETV(74) SETV(75) SETV(76) SETV(77) SETV(78) SETV(79) SETV(80) SETV(81) SETV(82) SETV(83) SETV(84) SETV(85) SETV(86) SETV(87)
  SETV(88) SETV(89) SETV(90) SETV(91) SETV(92) SETV(93) SETV(94) SETV(95) SETV(96) SETV(97) SETV(98) SETV(99)
#define ZA(n) asm volatile("v_accvgpr_write_b32 a" #n ", 0");
  ZA(0) ZA(1) ZA(2) ZA(3) ZA(4) ZA(5) ZA(6) ZA(7) ZA(8) ZA(9) ZA(10) ZA(11) ZA(12) ZA(13) ZA(14) ZA(15) ZA(16) ZA(17) ZA(18) ZA(19) ZA(20) ZA(21) ZA(22) ZA(23) ZA(24) ZA(25) ZA(26) ZA(27) ZA(28) ZA(29) ZA(30) ZA(31)
  ZA(32) ZA(33) ZA(34) ZA(35) ZA(36) ZA(37) ZA(38) ZA(39) ZA(40) ZA(41) ZA(42) ZA(43) ZA(44) ZA(45) ZA(46) ZA(47) ZA(48) ZA(49) ZA(50) ZA(51) ZA(52) ZA(53) ZA(54) ZA(55) ZA(56) ZA(57) ZA(58) ZA(59) ZA(60) ZA(61) ZA(62) ZA(63)
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    if constexpr (MODE == 0) asm volatile(M0 M1 M2 M3 M4 M5 M6 M7 :: "v"(addr), "v"(addr_tr) : CLOBV);
    if constexpr (MODE == 1) asm volatile(M0 VX M1 VX M2 VX M3 VX M4 VX M5 VX M6 VX M7 VX :: "v"(addr), "v"(addr_tr) : CLOBV);
    if constexpr (MODE == 2) asm volatile(M0 DK M1 DV M2 M3 DK M4 DV M5 M6 M7 "s_waitcnt lgkmcnt(0)\n\t" :: "v"(addr), "v"(addr_tr) : CLOBV);
    if constexpr (MODE == 3) asm volatile(M0 VX DK M1 VX DV M2 VX M3 VX DK M4 VX DV M5 VX M6 VX M7 VX "s_waitcnt lgkmcnt(0)\n\t" :: "v"(addr), "v"(addr_tr) : CLOBV);
    if constexpr (MODE == 4) asm volatile(M0 IDLE M1 IDLE M2 IDLE M3 IDLE M4 IDLE M5 IDLE M6 IDLE M7 IDLE :: "v"(addr), "v"(addr_tr) : CLOBV);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float s;
  asm volatile("s_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 %0, a0" : "=v"(s));   // MFMA results need 12+ wait states before a read
  out[id] = s;
  if (id == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}


// (e) WMODE 0: reads only; 1: four 256-byte rows of a [32][196608] fp32 matrix per tile; 2: the wave's 12 KB at the end
template <int WMODE>
__global__ __launch_bounds__(256, 2) void column_walk(const char* __restrict__ k, float* __restrict__ sc, unsigned* out) {
  __shared__ v4u tile[4][64 * 16];
  __shared__ float keep[WMODE == 2 ? 4 : 1][WMODE == 2 ? 12 * 256 : 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int w = blockIdx.x * 4 + wave, g = w & 7, run = w >> 3;   // 2048 waves: 256 runs of 768 rows x 8 heads
  const char* base = k + (size_t)run * 768 * 2048 + g * 256 + (lane & 15) * 16;
  v4u acc = {0, 0, 0, 0}, r[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) r[i] = __builtin_nontemporal_load((const v4u*)(base + (size_t)(i * 4 + (lane >> 4)) * 2048));
#pragma unroll 1
  for (int t = 0; t < 12; ++t) {
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[wave][(i * 4 + (lane >> 4)) * 16 + ((lane & 15) ^ ((i * 4 + (lane >> 4)) & 15))] = r[i];
    if (t + 1 < 12) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        r[i] = __builtin_nontemporal_load((const v4u*)(base + (size_t)((t + 1) * 64 + i * 4 + (lane >> 4)) * 2048));
    }
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const v4u x = tile[wave][lane * 16 + (lane & 15)];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    acc ^= x;
    const float v[4] = {__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
    if (WMODE == 1) {
#pragma unroll
      for (int h = 0; h < 4; ++h) sc[(size_t)(g * 4 + h) * 196608 + (size_t)run * 768 + t * 64 + lane] = v[h];
    } else if (WMODE == 2) {
#pragma unroll
      for (int h = 0; h < 4; ++h) keep[wave][t * 256 + h * 64 + lane] = v[h];
    }
  }
  if (WMODE == 2) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    for (int e = lane * 4; e < 3072; e += 256) *(v4u*)(sc + (size_t)w * 3072 + e) = *(const v4u*)(&keep[wave][e]);
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;
}

struct MfmaRun { double tflops, cycles_per_mfma, mhz; };
template <class Launch>
MfmaRun time_mfma(Launch launch, unsigned long long* d_clk, hipEvent_t a, hipEvent_t b) {
  const int iters = 20000;
  launch(iters);                                   // bring the clock to its steady state
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a));
  for (int r = 0; r < 5; ++r) launch(iters);
  CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b)); ms /= 5;
  unsigned long long clk[2]; CK(hipMemcpy(clk, d_clk, 16, hipMemcpyDeviceToHost));
  const double flops = 256.0 * 4 * iters * 8 * 2.0 * 32 * 32 * 16;
  return {flops / ms / 1e9, (double)clk[0] / ((double)iters * 8), (double)clk[0] / ((double)clk[1] / 100.0)};
}

int main() {
  const long pitch = 8192;                 // token stride of a 32-head x 128 bf16 K or V tensor
  const long tokens_total = 786432;        // 6 GiB
  const long win_tokens = 65536;           // 512 MiB window per launch
  const int nwin = (int)(tokens_total / win_tokens);
  char* d_buf; CK(hipMalloc(&d_buf, tokens_total * pitch)); CK(hipMemset(d_buf, 1, tokens_total * pitch));
  unsigned* d_out; CK(hipMalloc(&d_out, 1 << 22));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));

  {  // (a)
    float tot = 0; int reps = 0;
    for (int w = 0; w < nwin; ++w) {
      CK(hipEventRecord(a));
      stream_read<<<2048, 256>>>((const uint4*)(d_buf + (long)w * win_tokens * pitch), win_tokens * pitch / 16, d_out);
      CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
      float ms; CK(hipEventElapsedTime(&ms, a, b));
      if (w >= 2) { tot += ms; ++reps; }
    }
    printf("stream_read (grid-stride loop): %.1f us per 512 MiB -> %.0f GB/s\n", tot / reps * 1e3, 536.870912 / (tot / reps));
    tot = 0; reps = 0;
    for (int w = 0; w < nwin; ++w) {
      CK(hipEventRecord(a));
      stream_read_spans<<<8192, 256>>>((const v4u*)(d_buf + (long)w * win_tokens * pitch), win_tokens * pitch / 16, d_out);
      CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
      float ms; CK(hipEventElapsedTime(&ms, a, b));
      if (w >= 2) { tot += ms; ++reps; }
    }
    printf("stream_read (contiguous span per workgroup, non-temporal loads): %.1f us per 512 MiB -> %.0f GB/s\n", tot / reps * 1e3,
           536.870912 / (tot / reps));
  }
  {  // (b)
    std::mt19937 rng(7);
    const int nwaves = 4096, kept_per_head = 21504, waves_per_head = nwaves / 32;
    const int rows_per_wave = kept_per_head / waves_per_head / 128 * 128;
    std::vector<int> rows((size_t)nwaves * rows_per_wave), perm(win_tokens);
    for (int h = 0; h < 32; ++h) {
      for (int i = 0; i < win_tokens; ++i) perm[i] = i;
      std::shuffle(perm.begin(), perm.end(), rng);
      std::vector<int> kept(perm.begin(), perm.begin() + waves_per_head * rows_per_wave);
      std::sort(kept.begin(), kept.end());
      for (int j = 0; j < waves_per_head; ++j)
        std::copy(kept.begin() + (size_t)j * rows_per_wave, kept.begin() + (size_t)(j + 1) * rows_per_wave,
                  rows.begin() + (size_t)(j * 32 + h) * rows_per_wave);
    }
    int* d_rows; CK(hipMalloc(&d_rows, rows.size() * 4));
    CK(hipMemcpy(d_rows, rows.data(), rows.size() * 4, hipMemcpyHostToDevice));
    const double mb = (double)nwaves * rows_per_wave * 256 / 1e6;
    float tot = 0; int reps = 0;
    for (int w = 0; w < nwin; ++w) {
      CK(hipEventRecord(a));
      gather_rows<16><<<nwaves / 4, 256>>>(d_buf + (long)w * win_tokens * pitch, d_rows, rows_per_wave, pitch, d_out);
      CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
      float ms; CK(hipEventElapsedTime(&ms, a, b));
      if (w >= 2) { tot += ms; ++reps; }
    }
    printf("gather_rows (256 B rows, 33 %% kept, 16 loads in flight per lane): %.1f us for %.0f MB -> %.0f GB/s\n",
           tot / reps * 1e3, mb, mb / (tot / reps));
  }
  {  // (e)
    const size_t tensor = (size_t)196608 * 2048;   // 402.7 MB; three copies in turn, so that no launch finds its rows cached
    float* d_sc; CK(hipMalloc(&d_sc, (size_t)3 * 32 * 196608 * 4));
    const char* names[] = {"reads only", "+ 4 score rows of 256 B per tile", "+ the wave's 12 KB of scores at the end"};
    for (int mode = 0; mode < 3; ++mode) {
      float tot = 0; int reps = 0;
      for (int it = 0; it < 12; ++it) {
        const char* src = d_buf + (size_t)(it % 3) * tensor;
        float* dst = d_sc + (size_t)(it % 3) * 32 * 196608;
        CK(hipEventRecord(a));
        if (mode == 0) column_walk<0><<<512, 256>>>(src, dst, d_out);
        if (mode == 1) column_walk<1><<<512, 256>>>(src, dst, d_out);
        if (mode == 2) column_walk<2><<<512, 256>>>(src, dst, d_out);
        CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
        float ms; CK(hipEventElapsedTime(&ms, a, b));
        if (it >= 3) { tot += ms; ++reps; }
      }
      printf("column walk of 402.7 MB through LDS, %-40s: %.1f us -> %.0f GB/s read\n", names[mode], tot / reps * 1e3,
             tensor / 1e6 / (tot / reps));
    }
  }
  {  // (c), (d)
    float* d_f; unsigned long long* d_clk;
    CK(hipMalloc(&d_f, 256 * 256 * 4)); CK(hipMalloc(&d_clk, 16));
    const char* data[] = {"all zero", "all 1.0", "random normal"};
    for (int mode = 0; mode < 3; ++mode) {
      const MfmaRun r = time_mfma([&](int it) { mfma_by_data<<<256, 256>>>(d_f, it, mode, d_clk); }, d_clk, a, b);
      printf("mfma bf16 32x32x16, 1 wave per SIMD, operands %-14s: %5.0f TFLOP/s at %4.0f MHz shader clock, %.1f cycles per MFMA\n",
             data[mode], r.tflops, r.mhz, r.cycles_per_mfma);
    }
    const char* mix[] = {"nothing else", "fma, exp, fma, cvt_pk per MFMA", "0.5 KB of LDS reads per MFMA",
                         "vector work and LDS reads", "16 idle cycles per MFMA"};
    MfmaRun r[5];
    r[0] = time_mfma([&](int it) { mfma_mix<0><<<256, 256>>>(d_f, it, d_clk); }, d_clk, a, b);
    r[1] = time_mfma([&](int it) { mfma_mix<1><<<256, 256>>>(d_f, it, d_clk); }, d_clk, a, b);
    r[2] = time_mfma([&](int it) { mfma_mix<2><<<256, 256>>>(d_f, it, d_clk); }, d_clk, a, b);
    r[3] = time_mfma([&](int it) { mfma_mix<3><<<256, 256>>>(d_f, it, d_clk); }, d_clk, a, b);
    r[4] = time_mfma([&](int it) { mfma_mix<4><<<256, 256>>>(d_f, it, d_clk); }, d_clk, a, b);
    for (int m = 0; m < 5; ++m)
      printf("mfma (random normal operands) + %-32s: %5.0f TFLOP/s at %4.0f MHz shader clock, %.1f cycles per MFMA\n", mix[m],
             r[m].tflops, r[m].mhz, r[m].cycles_per_mfma);
  }
  return 0;
}
