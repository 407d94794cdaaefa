// bf16 MFMA contraction kernel with a multi-stage LDS ring filled by direct global->LDS
// loads (16 bytes per lane, no register staging), so several K-tiles are in flight while
// the matrix cores work on the current one.  Operands whose contraction index is the slow
// dimension in memory are kept in their natural layout in LDS and transposed at read time
// with the LDS transpose-read instruction.
//
// LDS layouts (per stage, BK = 64):
//   row-form operand (k contiguous):  [rows][64 k], 128-byte rows, 16-byte chunk c of row r
//     stored at chunk c ^ swz(r);
//   column-form operand (row index contiguous): [64 k][ROWS], chunk c of k-row k stored at
//     chunk c ^ colswz(k).  One transpose-read serves 32 lanes per cycle: four k-rows times eight
//     8-byte pieces that span four chunks of each k-row.  K-rows of 256 bytes or more start at the
//     same bank, so the four k-rows get four disjoint chunk groups (XOR with 0, 4, 8, 12); k-rows
//     of 128 bytes (ROWS = 64) alternate between the two halves of the banks, and the two k-rows
//     of a half get the two chunk groups of that row (XOR with 0 or 4).  (Measured with
//     SQ_LDS_BANK_CONFLICT: none left; an XOR with 0, 2, 4, 6 had every second cycle in conflict.)
// A direct load writes lane i's 16 bytes to (wave-uniform base) + 16*i, so the swizzle is
// applied by choosing which global chunk each lane fetches.
#include "gemm_common.h"

namespace ouro {

typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int ROWS>
__device__ __forceinline__ int colswz(int k) {
  static_assert(ROWS == 64 || ROWS % 128 == 0, "column-form tiles are 64 or a multiple of 128 rows wide");
  return ROWS >= 128 ? ((k & 3) << 2) : (((k >> 1) & 1) << 2);
}
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

// Wait until at most N vector-memory operations are outstanding and every LDS operation of
// this wave has completed.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

// One operand's share of a K-tile.  ROWS = tile extent along m (or n); NW = waves per
// workgroup; COL = column-form.  Every wave-load moves 1 KiB.
template <int ROWS, int NW, bool COL>
struct OperandTile {
  static constexpr int BYTES = ROWS * 128;                 // per stage
  static constexpr int NLOAD = BYTES / 1024;               // wave-loads per tile
  static constexpr int PER = NLOAD / NW;                   // per wave
  static_assert(NLOAD % NW == 0, "tile loads must divide over the waves");
  static constexpr int CPR = COL ? ROWS / 8 : 8;           // 16-byte chunks per LDS row
  static constexpr int RPL = 64 / CPR;                     // LDS rows per wave-load

  // Global element offset (without the K-tile term) of the chunk lane `lane` fetches in
  // wave-load j.  rmax: valid extent along the row index (clamped: out-of-range rows only
  // feed outputs that are never stored).
  __device__ static __forceinline__ size_t src_offset(int j, int lane, int row0, int rmax, int ld) {
    const int lr = j * RPL + lane / CPR;                   // LDS row
    const int pc = lane % CPR;                             // physical chunk
    if (!COL) {
      const int c = pc ^ swz(lr);
      const int gr = min(row0 + lr, rmax - 1);
      return (size_t)gr * ld + 8 * c;                      // + k0
    } else {
      const int c = pc ^ colswz<ROWS>(lr);
      const int gm = min(row0 + 8 * c, rmax - 8);
      return (size_t)lr * ld + gm;                         // + k0 * ld
    }
  }
};

// A/B fragment of substep ks for the 32-row tile starting at row t0 (row-form).
__device__ __forceinline__ bf16x8 frag_row(const char* tile, int t0, int ks, int lane) {
  const int row = t0 + (lane & 31);
  const int c = 2 * ks + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(tile + row * 128 + ((c ^ swz(row)) << 4));
}
// Same fragment from a column-form tile [64 k][ROWS]: two transpose reads of 4 k each.
template <int ROWS>
__device__ __forceinline__ bf16x8 frag_col(const char* tile, int t0, int ks, int lane) {
  const int g4 = lane >> 4, i = lane & 15;
  const int k = 16 * ks + 8 * (g4 >> 1) + (i >> 2);
  const int m = t0 + 16 * (g4 & 1) + 4 * (i & 3);
  const char* a = tile + k * (ROWS * 2) + (((m >> 3) ^ colswz<ROWS>(k)) << 4) + ((m & 7) << 1);
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)a);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 4 * (ROWS * 2)));
  union { struct { s16x4 l, h; } p; bf16x8 v; } u;
  u.p.l = lo; u.p.h = hi;
  return u.v;
}

// Which output tile and K range a workgroup takes.  Workgroups go to the 8 XCDs round-robin, and
// each XCD has its own L2: the grid index is turned into (XCD, position in that XCD's share)
// and the XCD's share is a contiguous run of work items, ordered so that the workgroups in
// flight together share operand tiles through that L2:
//  - with split K the K range is the slowest index, so an XCD works inside one K range (or
//    few) instead of streaming every range at once; tiles are numbered along M first when B
//    is the larger operand (neighbours then share the B tile), else along N;
//  - without split K and with tilesM a multiple of 8 an XCD owns a band of tilesM/8 tile rows
//    and walks it in groups of 8 tile columns (tilesN a multiple of 8), rows fastest: the 32 to 64 tiles in flight
//    cover (band x 8 columns), so both operands' tiles are re-used from L2 instead of one
//    operand being re-streamed for every tile row.
__device__ __forceinline__ void tile_of_block(const GemmParams& p, int BM, int BN, int bid, int nb, int& m0, int& n0, int& kbeg) {
  {
    int q = nb >> 3, r = nb & 7, x = bid & 7, idx = bid >> 3;
    if (p.band) {
      const int mb = p.tilesM >> 3, per = mb * 8;            // tile rows per XCD, tiles per full group
      const int g = idx / per, w = idx - g * per;
      m0 = (x * mb + w % mb) * BM;
      n0 = (g * 8 + w / mb) * BN;
      kbeg = 0;
      return;
    }
    bid = x * q + min(x, r) + idx;
  }
  const int kz = bid / p.ntiles;
  const int tile = bid - kz * p.ntiles;
  m0 = (p.mfast ? tile % p.tilesM : tile / p.tilesN) * BM;
  n0 = (p.mfast ? tile / p.tilesM : tile % p.tilesN) * BN;
  kbeg = kz * p.kchunk;
}

// The product this workgroup belongs to, of a batch laid over blockIdx.y and blockIdx.z.
__device__ __forceinline__ void batch_offsets(GemmParams& p) {
  int z = blockIdx.z;
  if (z >= p.bz1) { z -= p.bz1; p.A = p.A2; p.B = p.B2; p.C = p.C2; p.alpha = p.alpha2; }
  p.A = reinterpret_cast<const char*>(p.A) + blockIdx.y * p.bAy + z * p.bAz;
  p.B = reinterpret_cast<const char*>(p.B) + blockIdx.y * p.bBy + z * p.bBz;
  p.C = reinterpret_cast<char*>(p.C) + blockIdx.y * p.bCy + z * p.bCz;
  if (p.res32) p.res32 = reinterpret_cast<const float*>(reinterpret_cast<const char*>(p.res32) + blockIdx.y * p.bCy + z * p.bCz);
}

// One workgroup's share of a product: work item `bid` of `nb` (see tile_of_block).
template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S>
__device__ __forceinline__ void gemm_dlds_body(const GemmParams& p, int bid, int nb, uint4* smem) {
  constexpr int BK = 64;
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  using TileA = OperandTile<BM, NW, TA>;
  using TileB = OperandTile<BN, NW, !TB>;
  constexpr int STAGE = TileA::BYTES + TileB::BYTES;
  constexpr int LPT = TileA::PER + TileB::PER;             // loads per thread per K-tile
  static_assert((S - 1) * LPT < 64, "too many loads in flight for vmcnt");
  char* lds = reinterpret_cast<char*>(smem);
  const bf16_t* A = reinterpret_cast<const bf16_t*>(p.A);
  const bf16_t* B = reinterpret_cast<const bf16_t*>(p.B);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: kept in a scalar register
  const int wm = wave / WN, wn = wave % WN;
  int m0, n0, kbeg;
  tile_of_block(p, BM, BN, bid, nb, m0, n0, kbeg);
  if (kbeg >= p.K) return;                                  // a work item past the last K range (grouped launches round up)
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nk = (kend - kbeg) / BK;                        // launcher guarantees exact tiles

  // per-load byte offsets from the operand base (32-bit: the launcher keeps operands under
  // 2 GiB); the K-tile term is a uniform add at issue time
  uint32_t oa[TileA::PER], ob[TileB::PER];
#pragma unroll
  for (int i = 0; i < TileA::PER; ++i)
    oa[i] = (uint32_t)(2 * (TileA::src_offset(wave + i * NW, lane, m0, p.M, p.lda) + (TA ? (size_t)kbeg * p.lda : (size_t)kbeg)));
#pragma unroll
  for (int i = 0; i < TileB::PER; ++i)
    ob[i] = (uint32_t)(2 * (TileB::src_offset(wave + i * NW, lane, n0, p.N, p.ldb) + (TB ? (size_t)kbeg : (size_t)kbeg * p.ldb)));
  const uint32_t stepA = 2u * (TA ? (uint32_t)BK * p.lda : (uint32_t)BK);
  const uint32_t stepB = 2u * (TB ? (uint32_t)BK : (uint32_t)BK * p.ldb);
  const char* Ab = reinterpret_cast<const char*>(A);
  const char* Bb = reinterpret_cast<const char*>(B);

  // `slot` (the ring stage) is a compile-time value at every call, so LDS addresses are a lane
  // term plus an immediate offset
  auto issue = [&](int kt, char* st) __attribute__((always_inline)) {
    const uint32_t ka = (uint32_t)kt * stepA, kb = (uint32_t)kt * stepB;
#pragma unroll
    for (int i = 0; i < TileA::PER; ++i)
      __builtin_amdgcn_global_load_lds((gbl_void*)(Ab + (oa[i] + ka)), (lds_void*)(st + (wave + i * NW) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < TileB::PER; ++i)
      __builtin_amdgcn_global_load_lds((gbl_void*)(Bb + (ob[i] + kb)),
                                       (lds_void*)(st + TileA::BYTES + (wave + i * NW) * 1024), 16, 0, 0);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < nk) issue(s, lds + s * STAGE);

  // One K-tile: wait for it, refill the stage read last, multiply.  The stage that is filled and
  // the stage that is read are distinct `__restrict__` objects of this call: without that the
  // compiler cannot tell a transposing LDS read from the target of the loads just issued and
  // drains them (s_waitcnt vmcnt(0)) before the first fragment read, which takes the ring's
  // prefetch distance to zero.  What orders the fill of a stage and its reads is the explicit
  // wait and barrier below.
  auto step = [&](int kt, char* __restrict__ fill, const char* __restrict__ sa) __attribute__((always_inline)) {
    // tile kt has landed once at most the loads of the younger tiles are outstanding
    if (kt + S - 1 <= nk) wait_vmcnt<(S - 2) * LPT>();
    else wait_vmcnt<0>();
    // plain hardware barrier: a fenced barrier would drain the younger tiles' loads too.
    // Before it every wave has waited for its own share of tile kt and for its LDS reads of
    // tile kt-1; after it tile kt is complete in LDS and stage (kt-1)%S may be refilled.
    __builtin_amdgcn_s_barrier();
    if (kt + S - 1 < nk) issue(kt + S - 1, fill);
    const char* sb = sa + TileA::BYTES;
    if constexpr (TM * TN <= 2) {
      // small wave tiles: every fragment of the K-tile is requested up front (48 registers) and
      // the matrix instructions start as the fragments arrive, so a wave meets the LDS latency
      // once per K-tile
      bf16x8 af[4][TM], bfr[4][TN];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[ks][i] = TA ? frag_col<BM>(sa, wm * (TM * 32) + i * 32, ks, lane) : frag_row(sa, wm * (TM * 32) + i * 32, ks, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[ks][j] = TB ? frag_row(sb, wn * (TN * 32) + j * 32, ks, lane) : frag_col<BN>(sb, wn * (TN * 32) + j * 32, ks, lane);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
      // keep the requests ahead of the matrix instructions
      constexpr int NRD = 4 * ((TA ? 2 : 1) * TM + (TB ? 1 : 2) * TN);
      __builtin_amdgcn_sched_group_barrier(0x100, NRD, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4 * TM * TN, 0);
    } else {
    // fragments of substep ks+1 are fetched before the matrix instructions of substep ks
    // are issued, so LDS latency hides behind the matrix pipe even with one wave per SIMD
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
      af[0][i] = TA ? frag_col<BM>(sa, wm * (TM * 32) + i * 32, 0, lane) : frag_row(sa, wm * (TM * 32) + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      bfr[0][j] = TB ? frag_row(sb, wn * (TN * 32) + j * 32, 0, lane) : frag_col<BN>(sb, wn * (TN * 32) + j * 32, 0, lane);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      if (ks < 3) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[nxt][i] = TA ? frag_col<BM>(sa, wm * (TM * 32) + i * 32, ks + 1, lane)
                          : frag_row(sa, wm * (TM * 32) + i * 32, ks + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[nxt][j] = TB ? frag_row(sb, wn * (TN * 32) + j * 32, ks + 1, lane)
                           : frag_col<BN>(sb, wn * (TN * 32) + j * 32, ks + 1, lane);
      }
      // the requests of substep ks+1 stay ahead of the matrix instructions of substep ks
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bfr[cur][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    }
  };
  // the K loop goes round the ring once per trip
  for (int kt = 0; kt < nk; kt += S) {
#pragma unroll
    for (int slot = 0; slot < S; ++slot)
      if (kt + slot < nk) step(kt + slot, lds + ((slot + S - 1) % S) * STAGE, lds + slot * STAGE);
  }
  __syncthreads();                                          // operand reads done: LDS reusable
  mfma_epilogue<TM, TN>(p, acc, smem, m0 + wm * (TM * 32), n0 + wn * (TN * 32), lane, wave);
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S>
__global__ __launch_bounds__(WM * WN * 64) void gemm_dlds_kernel(GemmParams p) {
  extern __shared__ uint4 smem[];
  batch_offsets(p);
  gemm_dlds_body<BM, BN, WM, WN, TA, TB, S>(p, blockIdx.x, gridDim.x, smem);
}

// Several products in one launch (weight gradients of a layer: small outputs, long contractions).
// Product i owns the work items [first[i], first[i+1]), a multiple of 8 each so that the low bits
// of a work item still name its XCD.  With all of them in flight together every workgroup can take a
// long K range and the grid still fills the chip in whole rounds, which no product does alone.
struct GemmGroupParams {
  int n;
  int first[GEMM_GROUP_MAX + 1];
  GemmParams p[GEMM_GROUP_MAX];
};
static_assert(sizeof(GemmGroupParams) <= 4096, "kernel arguments are limited to 4 KiB");
template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S>
__global__ __launch_bounds__(WM * WN * 64) void gemm_dlds_group_kernel(GemmGroupParams g) {
  extern __shared__ uint4 smem[];
  const int bid = blockIdx.x;
  int i = 0;
  while (i + 1 < g.n && bid >= g.first[i + 1]) ++i;
  gemm_dlds_body<BM, BN, WM, WN, TA, TB, S>(g.p[i], bid - g.first[i], g.first[i + 1] - g.first[i], smem);
}

// Same ring, deeper software pipeline: the fragments of a whole K-tile live in registers and
// are refilled for K-tile kt+1 right behind the matrix instructions of K-tile kt that last
// used them, so an LDS read has a full K-tile of matrix work to hide behind.  Stage kt+1 is
// being read while kt computes, so S >= 3 and S-2 stages are in flight from memory.
template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S>
__global__ __launch_bounds__(WM * WN * 64) void gemm_pipe_kernel(GemmParams p) {
  constexpr int BK = 64;
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  using TileA = OperandTile<BM, NW, TA>;
  using TileB = OperandTile<BN, NW, !TB>;
  constexpr int STAGE = TileA::BYTES + TileB::BYTES;
  constexpr int LPT = TileA::PER + TileB::PER;
  static_assert(S >= 3, "one stage is read while another computes");
  static_assert((S - 2) * LPT < 64, "too many loads in flight for vmcnt");
  extern __shared__ uint4 smem[];
  char* lds = reinterpret_cast<char*>(smem);
  batch_offsets(p);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: kept in a scalar register
  const int wm = wave / WN, wn = wave % WN;
  int m0, n0, kbeg;
  tile_of_block(p, BM, BN, blockIdx.x, gridDim.x, m0, n0, kbeg);
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nk = (kend - kbeg) / BK;

  uint32_t oa[TileA::PER], ob[TileB::PER];
#pragma unroll
  for (int i = 0; i < TileA::PER; ++i)
    oa[i] = (uint32_t)(2 * (TileA::src_offset(wave + i * NW, lane, m0, p.M, p.lda) + (TA ? (size_t)kbeg * p.lda : (size_t)kbeg)));
#pragma unroll
  for (int i = 0; i < TileB::PER; ++i)
    ob[i] = (uint32_t)(2 * (TileB::src_offset(wave + i * NW, lane, n0, p.N, p.ldb) + (TB ? (size_t)kbeg : (size_t)kbeg * p.ldb)));
  const uint32_t stepA = 2u * (TA ? (uint32_t)BK * p.lda : (uint32_t)BK);
  const uint32_t stepB = 2u * (TB ? (uint32_t)BK : (uint32_t)BK * p.ldb);
  const char* Ab = reinterpret_cast<const char*>(p.A);
  const char* Bb = reinterpret_cast<const char*>(p.B);

  // `slot` (the ring stage) is a compile-time value at every call: LDS addresses are a lane term
  // plus an immediate offset
  auto issue = [&](int kt, char* st) __attribute__((always_inline)) {
    const uint32_t ka = (uint32_t)kt * stepA, kb = (uint32_t)kt * stepB;
#pragma unroll
    for (int i = 0; i < TileA::PER; ++i)
      __builtin_amdgcn_global_load_lds((gbl_void*)(Ab + (oa[i] + ka)), (lds_void*)(st + (wave + i * NW) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < TileB::PER; ++i)
      __builtin_amdgcn_global_load_lds((gbl_void*)(Bb + (ob[i] + kb)),
                                       (lds_void*)(st + TileA::BYTES + (wave + i * NW) * 1024), 16, 0, 0);
  };
  bf16x8 af[4][TM], bfr[4][TN];
  auto fetch = [&](const char* sa, int ks) __attribute__((always_inline)) {
    const char* sb = sa + TileA::BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      af[ks][i] = TA ? frag_col<BM>(sa, wm * (TM * 32) + i * 32, ks, lane) : frag_row(sa, wm * (TM * 32) + i * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      bfr[ks][j] = TB ? frag_row(sb, wn * (TN * 32) + j * 32, ks, lane) : frag_col<BN>(sb, wn * (TN * 32) + j * 32, ks, lane);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // tiles 0 .. S-2 on their way; tile 0 into registers
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < nk) issue(s, lds + s * STAGE);
  if (nk >= S - 1) wait_vmcnt<(S - 2) * LPT>();
  else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) fetch(lds, ks);

  // `fill` and `next` (the stage refilled and the stage read) are distinct objects of a call, see
  // gemm_dlds_body
  auto step = [&](int kt, char* __restrict__ fill, const char* __restrict__ next) __attribute__((always_inline)) {
    // tile kt+1 has landed once only the loads of tiles kt+2 .. kt+S-2 are outstanding
    if (kt + S - 1 <= nk) wait_vmcnt<(S - 3) * LPT>();
    else wait_vmcnt<0>();
    // After this barrier tile kt+1 is complete in LDS, and every wave has issued the matrix
    // instructions of tile kt-1, which consumed the last reads of stage (kt-1)%S: refill it.
    __builtin_amdgcn_s_barrier();
    if (kt + S - 1 < nk) issue(kt + S - 1, fill);
    const bool more = kt + 1 < nk;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (more) fetch(next, ks);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // the K loop goes round the ring once per trip
  for (int kt = 0; kt < nk; kt += S) {
#pragma unroll
    for (int slot = 0; slot < S; ++slot)
      if (kt + slot < nk) step(kt + slot, lds + ((slot + S - 1) % S) * STAGE, lds + ((slot + 1) % S) * STAGE);
  }
  __syncthreads();                                          // operand reads done: LDS reusable
  mfma_epilogue<TM, TN>(p, acc, smem, m0 + wm * (TM * 32), n0 + wn * (TN * 32), lane, wave);
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S, bool PIPE>
struct KernelOf {
  static auto get() { return gemm_dlds_kernel<BM, BN, WM, WN, TA, TB, S>; }
};
template <int BM, int BN, int WM, int WN, bool TA, bool TB, int S>
struct KernelOf<BM, BN, WM, WN, TA, TB, S, true> {
  static auto get() { return gemm_pipe_kernel<BM, BN, WM, WN, TA, TB, S>; }
};

template <int BM, int BN, int WM, int WN, int S, bool PIPE>
hipError_t launch_dlds_cfg_impl(hipStream_t s, GemmParams& p, int transA, int transB, int splits) {
  constexpr size_t smem_main = (size_t)S * (BM + BN) * 128;
  constexpr size_t smem_epi = (size_t)WM * WN * epilogue_stage_floats<BN / WN / 32>() * sizeof(float);
  constexpr size_t smem = smem_main > smem_epi ? smem_main : smem_epi;
  p.tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  p.ntiles = p.tilesM * p.tilesN;
  p.mfast = splits > 1 && p.N > p.M;
  p.band = splits == 1 && p.tilesM % 8 == 0 && p.tilesN % 8 == 0 && p.tilesN > 8;
  dim3 grid(p.ntiles * splits, p.by, p.bz), block(WM * WN * 64);
#define OURO_LAUNCH(TA_, TB_)                                                                    \
  do {                                                                                           \
    static bool attr_done = false;                                                               \
    auto kern = KernelOf<BM, BN, WM, WN, TA_, TB_, S, PIPE>::get();                              \
    if (!attr_done) {                                                                            \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                    \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
      if (e != hipSuccess) return e;                                                             \
      attr_done = true;                                                                          \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, smem, s, p);                                           \
  } while (0)
  if (!transA && !transB) OURO_LAUNCH(false, false);
  else if (!transA && transB) OURO_LAUNCH(false, true);
  else if (transA && !transB) OURO_LAUNCH(true, false);
  else OURO_LAUNCH(true, true);
#undef OURO_LAUNCH
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int S>
hipError_t launch_dlds_cfg(hipStream_t s, GemmParams& p, int transA, int transB, int splits) {
  return launch_dlds_cfg_impl<BM, BN, WM, WN, S, false>(s, p, transA, transB, splits);
}
template <int BM, int BN, int WM, int WN, int S>
hipError_t launch_pipe_cfg(hipStream_t s, GemmParams& p, int transA, int transB, int splits) {
  return launch_dlds_cfg_impl<BM, BN, WM, WN, S, true>(s, p, transA, transB, splits);
}

// Products ps[0..n) (kchunk set, accumulate form) in one launch of the 128x128 kernel.
hipError_t launch_gemm_dlds_group(hipStream_t s, GemmParams* ps, int n, int transA, int transB) {
  constexpr int BM = 128, BN = 128, WM = 2, WN = 4, S = 2;
  constexpr size_t smem_main = (size_t)S * (BM + BN) * 128;
  constexpr size_t smem_epi = (size_t)WM * WN * epilogue_stage_floats<BN / WN / 32>() * sizeof(float);
  constexpr size_t smem = smem_main > smem_epi ? smem_main : smem_epi;
  if (n < 1 || n > GEMM_GROUP_MAX) return hipErrorInvalidValue;
  GemmGroupParams g;
  g.n = n;
  g.first[0] = 0;
  for (int i = 0; i < n; ++i) {
    GemmParams& p = ps[i];
    p.tilesM = (p.M + BM - 1) / BM;
    p.tilesN = (p.N + BN - 1) / BN;
    p.ntiles = p.tilesM * p.tilesN;
    const int splits = (p.K + p.kchunk - 1) / p.kchunk;
    p.mfast = p.N > p.M;                                    // neighbours share the larger operand's tile (two equal 1024 x 4096 products, one K range: 173 -> 150 us)
    p.band = 0;
    g.p[i] = p;
    g.first[i + 1] = g.first[i] + (p.ntiles * splits + 7) / 8 * 8;
  }
  for (int i = n; i < GEMM_GROUP_MAX; ++i) { g.p[i] = ps[0]; g.first[i + 1] = g.first[n]; }
  dim3 grid(g.first[n]), block(WM * WN * 64);
#define OURO_LAUNCH(TA_, TB_)                                                                    \
  do {                                                                                           \
    static bool attr_done = false;                                                               \
    auto kern = gemm_dlds_group_kernel<BM, BN, WM, WN, TA_, TB_, S>;                             \
    if (!attr_done) {                                                                            \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                    \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
      if (e != hipSuccess) return e;                                                             \
      attr_done = true;                                                                          \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, smem, s, g);                                           \
  } while (0)
  if (transA && !transB) OURO_LAUNCH(true, false);
  else return hipErrorInvalidValue;
#undef OURO_LAUNCH
  return hipGetLastError();
}

hipError_t launch_gemm_dlds(hipStream_t s, GemmParams& p, int transA, int transB, int splits, int cfg) {
  switch (cfg) {
    case GEMM_TILE_128x128: return launch_dlds_cfg<128, 128, 2, 4, 2>(s, p, transA, transB, splits);
    case GEMM_TILE_128x64: return launch_dlds_cfg<128, 64, 4, 1, 2>(s, p, transA, transB, splits);
    case GEMM_TILE_PIPE128: return launch_pipe_cfg<128, 128, 2, 4, 4>(s, p, transA, transB, splits);
    case GEMM_TILE_256x256: return launch_dlds_cfg<256, 256, 2, 4, 2>(s, p, transA, transB, splits);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace ouro
