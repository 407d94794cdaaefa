// Building blocks of the fused attention kernels (bf16, head size 64): parameters, LDS tile
// layout, direct global->LDS tile loads, fragment reads in row and accumulator order, and the
// workgroup -> (causal block, head, batch) decode.
#pragma once
#include "common.h"
#include "tiles.h"

namespace ouro {

struct FaParams {
  int B, H, T, S, Mv;
  const bf16_t* q; int ldq;
  const bf16_t* k; int ldk;
  const bf16_t* v; int ldv;
  bf16_t* o; int ldo;
  float* lse;
  float scale, scale_log2;
  const bf16_t* d_o; int lddo;
  bf16_t* dq; int lddq;
  bf16_t* dk; int lddk;
  bf16_t* dv; int lddv;
  float* D;
  float* lse2;
  // relative-position variant (Transformer-XL): per-head biases u, vb [H, 64], projected
  // distance table r [S, ldr] (row = distance), and their fp32 gradients
  const bf16_t* u; const bf16_t* vb;
  const bf16_t* r; int ldr;
  float* du; float* dvb; float* dr;
  // what the relative-position dQ kernel leaves for the contractions that give dK, dV and dr
  bf16_t *pt, *dst, *qu, *qv, *dop;
  int t_ld;
};

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int TILE_BYTES = 64 * 128;
constexpr int NSTAGE = 3;

// Chunk swizzle of a tile row (128-byte rows: two rows per 256-byte bank window).  A 16-byte row
// read serves 16 consecutive rows per cycle at one chunk index: the eight rows of each parity
// need eight different swizzle values, so the value is a bijection of row bits 1-3.  A
// transposed read serves four consecutive rows per cycle, each over four adjacent chunks: the
// two rows of each parity need different chunk groups of four, so swizzle bit 2 is row bit 1.
// (SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE of the attention kernels: 25-40 % with a swizzle of
// row bits 0-2 only, whose rows r and r+8 collide in the row reads.)
__device__ __forceinline__ int swza(int row) { return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1); }

template <int N>
__device__ __forceinline__ void fa_wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));   // also all LDS operations
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 t) { return *reinterpret_cast<bf16x8*>(&t); }

// Direct load of rows [row0, row0+64) x 64 features of src into an LDS tile (4 waves, two
// 1 KiB wave-loads each).  Rows past rmax-1 repeat the last valid row; callers mask them.
__device__ __forceinline__ void dma_tile(const bf16_t* src, int ld, int row0, int rmax, char* tile, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int j = wave * 2 + i;
    const int row = 8 * j + (lane >> 3);
    const int c = (lane & 7) ^ swza(row);
    const int gr = min(row0 + row, rmax - 1);
    __builtin_amdgcn_global_load_lds((gbl_void*)(src + (size_t)gr * ld + 8 * c), (lds_void*)(tile + j * 1024), 16, 0, 0);
  }
}
// 64 floats src[i0 .. i0+63] (index clamped to n-1) into LDS, one dword per lane.
__device__ __forceinline__ void dma_floats(const float* src, int i0, int n, char* dst, int lane) {
  const int i = min(i0 + lane, n - 1);
  __builtin_amdgcn_global_load_lds((gbl_void*)(src + i), (lds_void*)dst, 4, 0, 0);
}

// operand whose contraction index is the feature: row = r0 + lane%32, features 16*ks + 8*(lane/32) ..+7
__device__ __forceinline__ bf16x8 read_rows(const char* tile, int r0, int ks, int lane) {
  const int row = r0 + (lane & 31);
  const int c = 2 * ks + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(tile + row * 128 + ((c ^ swza(row)) << 4));
}
// operand whose contraction index is the tile row, in accumulator order: lane owns feature
// f0 + lane%32; elements 0..3 = tile rows k0 + 4*(lane/32) + (0..3), elements 4..7 = rows
// k0 + 8 + 4*(lane/32) + (0..3).  Two transpose reads (each 16-lane group gathers a
// 4-row x 16-feature block).
__device__ __forceinline__ bf16x8 read_rows_t(const char* tile, int f0, int k0, int lane) {
  const int g4 = lane >> 4, i = lane & 15;
  const int f = f0 + 16 * (g4 & 1) + 4 * (i & 3);
  const int ka = k0 + 4 * (g4 >> 1) + (i >> 2);
  const int kb = ka + 8;
  const char* a0 = tile + ka * 128 + (((f >> 3) ^ swza(ka)) << 4) + ((f & 7) << 1);
  const char* a1 = tile + kb * 128 + (((f >> 3) ^ swza(kb)) << 4) + ((f & 7) << 1);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)a0);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)a1);
  union { struct { s16x4 l, h; } p; bf16x8 v; } u;
  u.p.l = lo; u.p.h = hi;
  return u.v;
}
__device__ __forceinline__ bf16x8 pack_acc(const f32x16& a, int sub) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)a[8 * sub + e];
  return r;
}
// accumulator tile (rows = feature 32*dt + 8g + 4*h32 + j, column = lane's query/key) -> global row
__device__ __forceinline__ void store_acc_row(bf16_t* dst, const f32x16 (&acc)[2], float mul, int h32) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      union { bf16_t h[4]; uint2 u; } cv;
#pragma unroll
      for (int j = 0; j < 4; ++j) cv.h[j] = (bf16_t)(acc[dt][4 * g + j] * mul);
      *reinterpret_cast<uint2*>(dst + 32 * dt + 8 * g + 4 * h32) = cv.u;
    }
}


// Workgroup -> (block along the causal axis, head, batch).  Causal work per block grows
// linearly along the axis, consecutive workgroup ids go to consecutive XCDs, and within an
// XCD workgroups are placed on compute units in id order.  So ids are decoded such that every
// XCD gets every block index equally often and the second half of an XCD's workgroups runs
// through the blocks in the opposite order: the two workgroups that share a compute unit
// then carry complementary loads.  `rank` counts from the heaviest block (0) to the lightest.
__device__ __forceinline__ void fa_decode_block(int& rank, int& head, int& b) {
  const int gx = gridDim.x, groups = gridDim.y * gridDim.z;
  int grp;
  if ((groups & 7) == 0 && ((groups >> 3) & 1) == 0) {
    const int lin = blockIdx.x + gx * (blockIdx.y + gridDim.y * blockIdx.z);
    const int xcd = lin & 7, slot = lin >> 3, per = (gx * groups) >> 3;
    rank = slot % gx;
    grp = xcd + 8 * (slot / gx);
    if (slot >= (per >> 1)) rank = gx - 1 - rank;
  } else {
    rank = blockIdx.x;
    grp = blockIdx.y + gridDim.y * blockIdx.z;
  }
  head = grp % gridDim.y;
  b = grp / gridDim.y;
}


inline FaParams fa_params(const AttnDesc& a) {
  FaParams p;
  p.B = a.B; p.H = a.H; p.T = a.T; p.S = a.S; p.Mv = a.Mv;
  p.q = (const bf16_t*)a.q; p.ldq = a.ldq; p.k = (const bf16_t*)a.k; p.ldk = a.ldk;
  p.v = (const bf16_t*)a.v; p.ldv = a.ldv; p.o = (bf16_t*)a.o; p.ldo = a.ldo; p.lse = a.lse;
  p.scale = a.scale; p.scale_log2 = a.scale * 1.4426950408889634f;
  p.d_o = (const bf16_t*)a.d_o; p.lddo = a.lddo; p.dq = (bf16_t*)a.dq; p.lddq = a.lddq;
  p.dk = (bf16_t*)a.dk; p.lddk = a.lddk; p.dv = (bf16_t*)a.dv; p.lddv = a.lddv;
  p.D = a.scratch;
  p.lse2 = a.scratch ? a.scratch + (size_t)a.B * a.H * a.T : nullptr;
  p.u = (const bf16_t*)a.u; p.vb = (const bf16_t*)a.vb; p.r = (const bf16_t*)a.r; p.ldr = a.ldr;
  p.du = a.du; p.dvb = a.dvb; p.dr = a.dr;
  p.pt = p.dst = p.qu = p.qv = p.dop = nullptr; p.t_ld = 0;
  return p;
}

}  // namespace ouro
