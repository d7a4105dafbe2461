// Measured ceilings of one MI355X for the two rooflines this library is held to.  Stand-alone
// program (no part of the library): prints what a plain kernel achieves for
//   (a) streaming reads from HBM, no reuse between launches (each launch reads another 512 MiB
//       window of a 6 GiB buffer, so neither L2 nor the 256 MB memory-side cache helps), once with a
//       grid-stride loop and once with a contiguous span per workgroup and non-temporal loads,
//   (b) gathers of 256-byte rows at an 8 KiB token stride, 32 heads active, kept rows random at
//       33 % density and ascending -- the access pattern of Reuse-phase attention,
//   (c) back-to-back v_mfma_f32_32x32x16_bf16 with independent accumulators, with the shader clock
//       it sustains.
// All indices are generated on the host and are in bounds by construction.
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

__global__ __launch_bounds__(256) void mfma_loop(float* out, unsigned long long* clk, int iters) {
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x % 3); b[e] = (__bf16)(float)(threadIdx.x % 5); }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float s = 0.0f;
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += acc[j][i];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
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
  {  // (c)
    float* d_f; unsigned long long* d_clk;
    CK(hipMalloc(&d_f, 512 * 256 * 4)); CK(hipMalloc(&d_clk, 16));
    const int iters = 20000, blocks = 256;
    mfma_loop<<<blocks, 256>>>(d_f, d_clk, 1000);
    CK(hipEventRecord(a));
    mfma_loop<<<blocks, 256>>>(d_f, d_clk, iters);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    unsigned long long clk[2]; CK(hipMemcpy(clk, d_clk, 16, hipMemcpyDeviceToHost));
    const double flops = (double)blocks * 4 * iters * 4 * 2.0 * 32 * 32 * 16;
    printf("mfma_loop (bf16 32x32x16, 4 accumulators, 1 wave per SIMD): %.0f TFLOP/s at %.0f MHz shader clock, %.1f cycles per MFMA\n",
           flops / ms / 1e9, (double)clk[0] / ((double)clk[1] / 100.0), (double)clk[0] / ((double)iters * 4));
  }
  return 0;
}
