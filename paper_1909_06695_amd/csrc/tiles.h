// LDS tile staging shared by the MFMA kernels: 64-element (128-byte) rows of bf16 with an
// XOR swizzle of the 16-byte chunks, filled from row-form (k contiguous) or column-form
// (row contiguous, transposed in registers) global tiles.
#pragma once
#include "common.h"

namespace ouro {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// 16-byte chunk c (8 bf16 along k) of tile row `row` lives at chunk c ^ swz(row) of that
// row's 128 bytes: conflict-free for the per-row operand reads and for the transposing
// writes alike.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// Row-form operand: element (row, k) at src[row*ld + k] (k contiguous).
template <int ROWS, int NT>
__device__ __forceinline__ void load_rowform(const bf16_t* __restrict__ src, int ld, int row0, int rmax,
                                             int k0, int kend, int tid, uint4* reg) {
  constexpr int PER = ROWS * 8 / NT;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    int c = tid + i * NT;
    int row = c >> 3, kc = c & 7;
    int gr = row0 + row, gk = k0 + kc * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (gr < rmax && gk < kend) v = *reinterpret_cast<const uint4*>(src + (size_t)gr * ld + gk);
    reg[i] = v;
  }
}
template <int ROWS, int NT>
__device__ __forceinline__ void store_rowform(uint4* lds, int tid, const uint4* reg) {
  constexpr int PER = ROWS * 8 / NT;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    int c = tid + i * NT;
    int row = c >> 3, kc = c & 7;
    lds[row * 8 + (kc ^ swz(row))] = reg[i];
  }
}
// Column-form operand: element (row, k) at src[k*ld + row] (row contiguous).  A thread
// takes a 4(k) x 8(row) block: four 16-byte loads, transposed in registers into eight
// 8-byte pieces (4 consecutive k for one row each).
template <int ROWS, int NT>
__device__ __forceinline__ void load_colform(const bf16_t* __restrict__ src, int ld, int row0, int rmax,
                                             int k0, int kend, int tid, uint4* reg) {
  constexpr int NBLK = 16 * (ROWS / 8);
  constexpr int PER = (NBLK + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    int blk = tid + i * NT;
    if (NBLK % NT != 0 && blk >= NBLK) break;
    int rb = blk % (ROWS / 8), kb = blk / (ROWS / 8);
    int gr = row0 + rb * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      int gk = k0 + kb * 4 + kk;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (gr < rmax && gk < kend) v = *reinterpret_cast<const uint4*>(src + (size_t)gk * ld + gr);
      reg[i * 4 + kk] = v;
    }
  }
}
template <int ROWS, int NT>
__device__ __forceinline__ void store_colform(uint4* lds, int tid, const uint4* reg) {
  constexpr int NBLK = 16 * (ROWS / 8);
  constexpr int PER = (NBLK + NT - 1) / NT;
  uint2* l2 = reinterpret_cast<uint2*>(lds);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    int blk = tid + i * NT;
    if (NBLK % NT != 0 && blk >= NBLK) break;
    int rb = blk % (ROWS / 8), kb = blk / (ROWS / 8);
    const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&reg[i * 4 + 0]);
    const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&reg[i * 4 + 1]);
    const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&reg[i * 4 + 2]);
    const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&reg[i * 4 + 3]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {           // dword j holds rows 2j (low half) and 2j+1 (high half)
      uint2 even, odd;
      even.x = (w0[j] & 0xffffu) | (w1[j] << 16);
      even.y = (w2[j] & 0xffffu) | (w3[j] << 16);
      odd.x = (w0[j] >> 16) | (w1[j] & 0xffff0000u);
      odd.y = (w2[j] >> 16) | (w3[j] & 0xffff0000u);
      int r0 = rb * 8 + 2 * j, r1 = r0 + 1;
      int kc = kb >> 1, half = kb & 1;
      l2[(r0 * 8 + (kc ^ swz(r0))) * 2 + half] = even;
      l2[(r1 * 8 + (kc ^ swz(r1))) * 2 + half] = odd;
    }
  }
}


}  // namespace ouro
