// Building blocks shared by the two bf16 attention kernels (gfx950): LDS tile layout, matrix-core
// operand fetches and the softmax helpers.
//
// Tile layout in LDS: rows of D bf16 (ROWB = 2*D bytes), row-major, with the 16-byte chunks of a row
// permuted by an XOR that depends on the row.  The permutation is chosen so that
//   - a ds_read_b128 by 16 lanes holding 16 consecutive rows (the K operand fetch) and
//   - a ds_read_b64_tr_b16 by a wave covering 8 consecutive rows x 64 bytes (the V^T operand fetch)
// both spread evenly over the 16-byte bank groups.
//
// Matrix-core shapes (v_mfma_f32_32x32x16_bf16, D = A*B + C with A 32x16, B 16x32):
//   A operand  lane l holds row (l % 32), contraction slots 8*(l / 32) .. +7
//   B operand  lane l holds column (l % 32), the same contraction slots
//   C/D        lane l, register i holds row 8*(i/4) + 4*(l/32) + i%4, column l % 32
// S^T = K Q^T puts keys on rows and queries on columns, so a query's softmax statistics live in
// one lane pair (l, l ^ 32) and the S^T accumulators are, unchanged, the B operand of O^T = V^T P^T:
// contraction slot s of lane half hf is key 16u + 8*(s/4) + 4*hf + s%4 of the 32-key block.
#pragma once
#include "common.h"

namespace dllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr float kLog2e = 1.4426950408889634f;

// XOR applied to the chunk index of `row`; depends on row & 15 only
template <int D>
__device__ __forceinline__ int tile_swz(int row) {
  if constexpr (D == 128) {
    const int r = row & 15;
    return ((r & 3) << 2) | (r >> 2);
  } else {
    const int x = (row >> 1) & 7;
    return ((x & 1) << 2) | (x >> 1);
  }
}

// byte offset of 16-byte chunk `chunk` of `row` inside a tile
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ tile_swz<D>(row)) << 4);
}

__device__ __forceinline__ f32x16 mfma_bf16(v4u a, v4u b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// sum of the two bf16 halves of `packed`, added to acc (fp32)
__device__ __forceinline__ float add_pair_bf16(uint32_t packed, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), ones, acc, false);
}

// max of x over the lane pair (l, l ^ 32)
__device__ __forceinline__ float max_across_halves(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element (i % 4) of the four
// 8-byte pieces addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4 of the group.
__device__ __forceinline__ v2u lds_read_tr16(const char* p) {
  const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(__attribute__((address_space(3))) void*)p);
  return __builtin_bit_cast(v2u, r);
}

// 16 bytes per lane from global memory straight into LDS (no register in between).  The LDS side is
// lane-contiguous: lane l's bytes land at LDS byte address lds_wave_base + 16 * l, and lds_wave_base
// must be the same in every lane of the wave.  Written as inline assembly on purpose: the compiler
// then does not know that LDS is being written behind its back and does not make the next LDS read
// wait for the load (it cannot tell ring slots apart and would wait for all of them).  The caller
// therefore owns the ordering: wait_tile_loads() and then a workgroup barrier before any lane reads
// what was loaded.  These loads count in vmcnt like any vector memory load.
__device__ __forceinline__ void load16_to_lds(const void* src, uint32_t lds_wave_base) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off"
      :
      : "v"(src), "s"(lds_wave_base)
      : "memory", "m0");
}
// Same, with the global address given as a wave-uniform base plus a 32-bit per-lane byte offset (no
// vector arithmetic on 64-bit addresses).
__device__ __forceinline__ void load16_to_lds(const void* uniform_base, uint32_t lane_off, uint32_t lds_wave_base) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(lane_off), "s"(uniform_base), "s"(lds_wave_base)
      : "memory", "m0");
}
// The same two with the LDS address given as a base that stays in one scalar register plus a
// compile-time byte offset, added on the way into m0 (so that an unrolled loop does not keep one
// scalar register per LDS destination).
template <int kLdsOff>
__device__ __forceinline__ void load16_to_lds(const void* src, uint32_t lds_wave_base) {
  asm volatile(
      "s_add_u32 m0, %1, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off"
      :
      : "v"(src), "s"(lds_wave_base), "n"(kLdsOff)
      : "memory", "m0", "scc");
}
template <int kLdsOff>
__device__ __forceinline__ void load16_to_lds(const void* uniform_base, uint32_t lane_off, uint32_t lds_wave_base) {
  asm volatile(
      "s_add_u32 m0, %2, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(lane_off), "s"(uniform_base), "s"(lds_wave_base), "n"(kLdsOff)
      : "memory", "m0", "scc");
}
// Four bytes per lane: lane l's dword lands at LDS byte address lds_wave_base + 4 * l.
__device__ __forceinline__ void load4_to_lds(const void* src, uint32_t lds_wave_base) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %0, off"
      :
      : "v"(src), "s"(lds_wave_base)
      : "memory", "m0");
}
// Waits until every load16_to_lds / load4_to_lds this wave has issued has written its LDS bytes.
__device__ __forceinline__ void wait_tile_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// LDS byte address of a pointer into a __shared__ array
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return uint32_t(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void*)p));
}

// Per-lane byte offsets for fetching the V^T operand (32 head_dim rows x 16 keys) of one 16-key step
// out of a row-major V tile.  The first read returns the keys of contraction slots 0..3
// (key 4*hf + j of the step), the second those of slots 4..7 (8 + 4*hf + j).  base[rd] is for
// head_dim block 0 of the step starting at tile row 0; block db flips chunk bits (XOR with db << 6,
// the swizzle being an XOR too) and other steps add 16 * n * ROWB.
template <int D>
struct VtAddr {
  int base[2];
  __device__ __forceinline__ void init(int lane) {
    const int hf = lane >> 5, sl = lane & 15, dhalf = (lane >> 4) & 1;
    const int d0 = 16 * dhalf + 4 * (sl & 3);
#pragma unroll
    for (int rd = 0; rd < 2; ++rd) base[rd] = tile_off<D>(8 * rd + 4 * hf + (sl >> 2), d0 >> 3) + (d0 & 7) * 2;
  }
  __device__ __forceinline__ int off(int rd, int db) const { return base[rd] ^ (db << 6); }
};

// K operand offsets: lane (col, hf) reads chunk 2t + hf of tile row col; step t flips bit t << 5
template <int D>
struct KAddr {
  int base;
  __device__ __forceinline__ void init(int lane) { base = tile_off<D>(lane & 31, lane >> 5); }
  __device__ __forceinline__ int off(int t) const { return base ^ (t << 5); }
};

}  // namespace dllm
