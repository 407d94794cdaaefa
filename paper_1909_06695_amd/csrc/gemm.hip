// Dense contractions of the training step: a bf16 MFMA kernel (LDS double-buffered,
// XOR-swizzled tiles, 32x32x16 matrix instructions, 64-wide wavefronts) and a plain
// bounds-checked tiled kernel for fp32 operands and shapes the MFMA kernel does not take.
#include "gemm_common.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>

namespace ouro {

// ------------------------------------------------------------------ plain tiled kernel
template <typename T, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_plain_kernel(GemmParams p) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const T* A = reinterpret_cast<const T*>(p.A);
  const T* B = reinterpret_cast<const T*>(p.B);
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int e = tid + i * 256;                 // 0..1023
      int mm, kk;
      if (TA) { mm = e % BM; kk = e / BM; } else { kk = e % BK; mm = e / BK; }
      int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < p.M && gk < kend) v = to_f32(TA ? A[(size_t)gk * p.lda + gm] : A[(size_t)gm * p.lda + gk]);
      As[kk][mm] = v;
      int nn, kb;
      if (TB) { kb = e % BK; nn = e / BK; } else { nn = e % BN; kb = e / BN; }
      int gn = n0 + nn; gk = k0 + kb;
      v = 0.f;
      if (gn < p.N && gk < kend) v = to_f32(TB ? B[(size_t)gn * p.ldb + gk] : B[(size_t)gk * p.ldb + gn]);
      Bs[kb][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < p.M && n < p.N) epilogue_store<T>(p, m, n, acc[i][j]);
    }
}

// ------------------------------------------------------------------------- MFMA kernel
template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmParams p) {
  constexpr int BK = 64;
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int STAGE = (BM + BN) * 8;                      // uint4 per stage
  constexpr int RA = TA ? (16 * (BM / 8) / NT) * 4 : BM * 8 / NT;
  constexpr int RB = TB ? BN * 8 / NT : (16 * (BN / 8) / NT) * 4;
  extern __shared__ uint4 smem[];
  const bf16_t* A = reinterpret_cast<const bf16_t*>(p.A);
  const bf16_t* B = reinterpret_cast<const bf16_t*>(p.B);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // spread consecutive tiles of one matrix band over one XCD (blocks go round-robin
  // over the 8 XCDs, each with its own L2)
  int bid = blockIdx.x;
  {
    int nb = gridDim.x, q = nb >> 3, r = nb & 7, x = bid & 7, idx = bid >> 3;
    bid = x * q + min(x, r) + idx;
  }
  const int m0 = (bid / p.tilesN) * BM, n0 = (bid % p.tilesN) * BN;
  const int kbeg = blockIdx.z * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nk = (kend - kbeg + BK - 1) / BK;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[RA], rb[RB];
  auto gload = [&](int kt) {
    int k0 = kbeg + kt * BK;
    if (TA) load_colform<BM, NT>(A, p.lda, m0, p.M, k0, kend, tid, ra);
    else load_rowform<BM, NT>(A, p.lda, m0, p.M, k0, kend, tid, ra);
    if (TB) load_rowform<BN, NT>(B, p.ldb, n0, p.N, k0, kend, tid, rb);
    else load_colform<BN, NT>(B, p.ldb, n0, p.N, k0, kend, tid, rb);
  };
  auto sstore = [&](int stage) {
    uint4* sa = smem + stage * STAGE;
    uint4* sb = sa + BM * 8;
    if (TA) store_colform<BM, NT>(sa, tid, ra); else store_rowform<BM, NT>(sa, tid, ra);
    if (TB) store_rowform<BN, NT>(sb, tid, rb); else store_colform<BN, NT>(sb, tid, rb);
  };

  if (nk > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) gload(kt + 1);
    const uint4* sa = smem + (kt & 1) * STAGE;
    const uint4* sb = sa + BM * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[TM], bfr[TN];
      const int c = ks * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int row = wm * (TM * 32) + i * 32 + (lane & 31);
        uint4 t = sa[row * 8 + (c ^ swz(row))];
        af[i] = *reinterpret_cast<bf16x8*>(&t);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int row = wn * (TN * 32) + j * 32 + (lane & 31);
        uint4 t = sb[row * 8 + (c ^ swz(row))];
        bfr[j] = *reinterpret_cast<bf16x8*>(&t);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) sstore((kt + 1) & 1);
    __syncthreads();
  }

  mfma_epilogue<TM, TN>(p, acc, smem, m0 + wm * (TM * 32), n0 + wn * (TN * 32), lane, wave);
}

// ----------------------------------------------------------------------------- launch
hipError_t launch_gemm_dlds(hipStream_t s, GemmParams& p, int transA, int transB, int splits, int cfg);
hipError_t launch_gemm_dlds_group(hipStream_t s, GemmParams* ps, int n, int transA, int transB);
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bool gemm_uses_mfma(int dtype, const GemmDesc& g) {
  if (dtype != 1) return false;
  if (!aligned16(g.A) || !aligned16(g.B)) return false;
  if ((g.lda & 7) || (g.ldb & 7)) return false;
  if (g.transA ? (g.M & 7) : (g.K & 7)) return false;
  if (g.transB ? (g.K & 7) : (g.N & 7)) return false;
  if (g.M < 32 || g.N < 32 || g.K < 32) return false;
  return true;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_mfma_cfg(hipStream_t s, GemmParams& p, int transA, int transB, int splits) {
  constexpr size_t smem_main = 2 * (size_t)(BM + BN) * 8 * sizeof(uint4);
  constexpr size_t smem_epi = (size_t)WM * WN * epilogue_stage_floats<BN / WN / 32>() * sizeof(float);
  constexpr size_t smem = smem_main > smem_epi ? smem_main : smem_epi;
  int tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  dim3 grid(tilesM * p.tilesN, 1, splits), block(WM * WN * 64);
#define OURO_LAUNCH(TA_, TB_)                                                                   \
  do {                                                                                          \
    static bool attr_done = false;                                                              \
    auto kern = gemm_mfma_kernel<BM, BN, WM, WN, TA_, TB_>;                                     \
    if (!attr_done) {                                                                           \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                   \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);\
      if (e != hipSuccess) return e;                                                            \
      attr_done = true;                                                                         \
    }                                                                                           \
    hipLaunchKernelGGL(kern, grid, block, smem, s, p);                                          \
  } while (0)
  if (!transA && !transB) OURO_LAUNCH(false, false);
  else if (!transA && transB) OURO_LAUNCH(false, true);
  else if (transA && !transB) OURO_LAUNCH(true, false);
  else OURO_LAUNCH(true, true);
#undef OURO_LAUNCH
  return hipGetLastError();
}

hipError_t launch_gemm(hipStream_t s, int dtype, const GemmDesc& g, int force_generic) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  GemmParams p;
  p.A = g.A; p.B = g.B; p.C = g.C;
  p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
  p.out_fp32 = g.out_fp32; p.accumulate = g.accumulate;
  p.bias = g.bias; p.residual = g.residual; p.ldr = g.ldr;
  p.res32 = g.res32; p.ldr32 = g.ldr32; p.ln_mean = g.ln_mean; p.ln_rstd = g.ln_rstd; p.ln_g = g.ln_g; p.ln_b = g.ln_b;
  if (g.res32 && (g.residual || g.accumulate || (g.ln_mean && !(g.ln_rstd && g.ln_g && g.ln_b)))) return hipErrorInvalidValue;
  p.epilogue = g.epilogue; p.Z = g.Z; p.ldz = g.ldz; p.alpha = g.alpha;
  p.drop = g.drop;
  p.kchunk = g.K; p.tilesN = 0; p.vec_epi = 0;
  if (g.accumulate && (!g.out_fp32 || g.bias || g.residual || g.epilogue != EPI_NONE)) return hipErrorInvalidValue;
  // a batch of products: over the grid's y and z in the direct-to-LDS kernels, else one launch each
  const int by = std::max(1, g.by), bz = std::max(1, g.bz);
  const size_t esz = dtype == 1 ? 2 : 4, csz = g.out_fp32 ? 4 : esz;
  const int grids = g.C2 ? 2 : 1;
  if (g.C2 && (!g.A2 || !g.B2)) return hipErrorInvalidValue;
  p.by = by; p.bz = bz * grids; p.bz1 = bz;
  p.A2 = g.A2; p.B2 = g.B2; p.C2 = g.C2; p.alpha2 = g.alpha2;
  p.bAy = g.sAy * (long long)esz; p.bAz = g.sAz * (long long)esz;
  p.bBy = g.sBy * (long long)esz; p.bBz = g.sBz * (long long)esz;
  p.bCy = g.sCy * (long long)csz; p.bCz = g.sCz * (long long)csz;
  if (by * bz * grids > 1) {
    if (g.bias || g.residual || g.epilogue != EPI_NONE || g.drop.on) return hipErrorInvalidValue;
    if (g.res32 && (!g.out_fp32 || g.ln_mean || g.C2)) return hipErrorInvalidValue;
    const size_t bA = 2 * (size_t)(g.transA ? g.K : g.M) * g.lda, bB = 2 * (size_t)(g.transB ? g.N : g.K) * g.ldb;
    const bool in_grid = force_generic != 1 && gemm_uses_mfma(dtype, g) && (g.K % 64) == 0 && bA < (1ull << 31) && bB < (1ull << 31) &&
                         !((p.bAy | p.bAz | p.bBy | p.bBz | p.bCy | p.bCz) & 15) &&
                         (!g.C2 || (aligned16(g.A2) && aligned16(g.B2) && aligned16(g.C2) == aligned16(g.C)));
    if (!in_grid) {
      for (int w = 0; w < grids; ++w)
        for (int z = 0; z < bz; ++z)
          for (int y = 0; y < by; ++y) {
            GemmDesc h = g;
            h.by = h.bz = 0; h.A2 = h.B2 = nullptr; h.C2 = nullptr;
            h.A = (const char*)(w ? g.A2 : g.A) + y * p.bAy + z * p.bAz;
            h.B = (const char*)(w ? g.B2 : g.B) + y * p.bBy + z * p.bBz;
            h.C = (char*)(w ? g.C2 : g.C) + y * p.bCy + z * p.bCz;
            if (g.res32) h.res32 = reinterpret_cast<const float*>(reinterpret_cast<const char*>(g.res32) + y * p.bCy + z * p.bCz);
            if (w) h.alpha = g.alpha2;
            hipError_t e = launch_gemm(s, dtype, h, force_generic);
            if (e != hipSuccess) return e;
          }
      return hipSuccess;
    }
  }

  if (force_generic != 1 && gemm_uses_mfma(dtype, g)) {
    const int oe = g.out_fp32 ? 3 : 7;   // ldc granularity for 16-byte row chunks
    p.vec_epi = aligned16(g.C) && !(g.ldc & oe) && (!g.residual || (aligned16(g.residual) && !(g.ldr & 7))) &&
                (!g.res32 || (aligned16(g.res32) && !(g.ldr32 & 3))) &&
                (g.epilogue == EPI_NONE || (aligned16(g.Z) && !(g.ldz & 7)));
    int cfg = force_generic >= 2 ? force_generic : -1;
    if (cfg < 0) {
      // 128x128 tiles (8 waves, two workgroups per CU) when they fill the chip at least twice
      // over; with one tile per CU and a long contraction the register-prefetch kernel with its
      // four-stage ring; otherwise, and for the split-K weight gradients, 128x64 tiles, which
      // put more workgroups on every compute unit
      const int t128 = ((g.M + 127) / 128) * ((g.N + 127) / 128);
      const int t256 = ((g.M + 255) / 256) * ((g.N + 255) / 256);
      // 256x256 tiles halve the operand bytes per flop; they pay once there are several per CU
      // (the logits) or one per CU with a long contraction (dV_o)
      if (!g.accumulate && (t256 >= 1024 || (t256 >= 256 && g.K >= 4096))) cfg = GEMM_TILE_256x256;
      else if (g.accumulate && t128 >= 192) cfg = GEMM_TILE_128x128;   // split-K with two workgroups per CU
      else if (g.accumulate || t128 <= 384) cfg = (!g.accumulate && (long)t128 * by * bz * grids <= 256 && g.K >= 1024 && g.K <= 8192) ? GEMM_TILE_PIPE128 : GEMM_TILE_128x64;
      else cfg = GEMM_TILE_128x128;
    }
    const size_t bytesA = 2 * (size_t)(g.transA ? g.K : g.M) * g.lda, bytesB = 2 * (size_t)(g.transB ? g.N : g.K) * g.ldb;
    // direct global->LDS loads need whole 64-wide K tiles and 32-bit operand offsets
    const bool direct_ok = (g.K % 64) == 0 && bytesA < (1ull << 31) && bytesB < (1ull << 31);
    // 256x256 tiles run one workgroup per CU, so a launch takes whole rounds of 256 tiles.  A
    // few tile rows beyond the last full round would cost a whole round more (dV_o of a
    // 50257-word vocabulary: 788 tiles, 3.08 rounds): those rows go out as a second, split-K
    // launch that adds into the zeroed rows of the fp32 result.
    if (cfg == GEMM_TILE_256x256 && force_generic == 0 && direct_ok && g.out_fp32 && !g.accumulate && !g.bias && !g.residual &&
        !g.res32 && g.epilogue == EPI_NONE && !g.drop.on && by * bz * grids == 1 && g.ldc == g.N && g.K >= 2048) {
      const int tn = (g.N + 255) / 256;
      if (tn <= 256 && 256 % tn == 0) {
        const int rows_round = 256 / tn * 256;
        const int main = g.M / rows_round * rows_round, tail = g.M - main;
        if (main > 0 && tail > 0 && ((tail + 255) / 256) * tn <= 64) {
          GemmDesc a = g;
          a.M = main;
          hipError_t e = launch_gemm(s, dtype, a, 0);
          if (e != hipSuccess) return e;
          GemmDesc b = g;
          b.M = tail;
          b.A = reinterpret_cast<const char*>(g.A) + 2 * (g.transA ? (size_t)main : (size_t)main * g.lda);
          b.C = reinterpret_cast<float*>(g.C) + (size_t)main * g.ldc;
          b.accumulate = 1;
          e = launch_fill_zero(s, b.C, (size_t)tail * g.ldc * 4);
          if (e != hipSuccess) return e;
          return launch_gemm(s, dtype, b, 0);
        }
      }
    }
    int splits = 1;
    bool modelled = false;
    if (g.accumulate && force_generic < 2 && direct_ok && g.K >= 512) {
      modelled = true;
      // Split-K launch: tile shape and number of K ranges together, so that the grid fills the
      // chip in whole rounds.  Cost of a candidate in units of (tile area x K-tiles) per CU:
      // rounds x workgroups per CU x tile area x (K-tiles per workgroup + fixed cost) / rate,
      // the fixed cost (ring fill, atomic epilogue) taken as 6 K-tiles, the rate of the 128x64
      // tiles as 0.8 of the 128x128 ones (more operand bytes per flop).
      double best = 1e30;
      for (int c = 0; c < 2; ++c) {
        const int bm = 128, bn = c ? 64 : 128, per_cu = c ? 3 : 2;
        const long tiles = (long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn) * by * bz * grids;
        const int max_s = std::min(16, g.K / 256);
        for (int sp = 1; sp <= max_s; ++sp) {
          const int kc = ((g.K + sp - 1) / sp + 63) / 64 * 64;
          const int real = (g.K + kc - 1) / kc;
          if (real != sp) continue;
          const long rounds = (tiles * sp + 256L * per_cu - 1) / (256L * per_cu);
          const double cost = (double)rounds * per_cu * bm * bn * (kc / 64 + 6) / (c ? 0.8 : 1.0);
          if (cost < best) { best = cost; cfg = c ? GEMM_TILE_128x64 : GEMM_TILE_128x128; splits = sp; }
        }
      }
    }
    if (!direct_ok) cfg = GEMM_TILE_STAGED128;
    if (cfg < GEMM_TILE_STAGED128 || cfg > GEMM_TILE_256x256) return hipErrorInvalidValue;
    const int BM = cfg == GEMM_TILE_256x256 ? 256 : 128, BN = cfg == GEMM_TILE_128x64 ? 64 : BM;
    int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * by * bz * grids;
    if (g.accumulate && !modelled && tiles < 384 && g.K >= 512) {
      splits = (512 + tiles - 1) / tiles;
      int maxs = g.K / 256;
      if (splits > maxs) splits = maxs;
      if (splits < 1) splits = 1;
    }
    int kchunk = (g.K + splits - 1) / splits;
    kchunk = (kchunk + 63) / 64 * 64;
    splits = (g.K + kchunk - 1) / kchunk;
    p.kchunk = kchunk;
    if (cfg != GEMM_TILE_STAGED128) return launch_gemm_dlds(s, p, g.transA, g.transB, splits, cfg);
    return launch_mfma_cfg<128, 128, 2, 2>(s, p, g.transA, g.transB, splits);
  }

  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64, 1), block(256);
#define OURO_PLAIN(T_)                                                                        \
  do {                                                                                        \
    if (!g.transA && !g.transB) hipLaunchKernelGGL((gemm_plain_kernel<T_, false, false>), grid, block, 0, s, p); \
    else if (!g.transA && g.transB) hipLaunchKernelGGL((gemm_plain_kernel<T_, false, true>), grid, block, 0, s, p); \
    else if (g.transA && !g.transB) hipLaunchKernelGGL((gemm_plain_kernel<T_, true, false>), grid, block, 0, s, p); \
    else hipLaunchKernelGGL((gemm_plain_kernel<T_, true, true>), grid, block, 0, s, p);       \
  } while (0)
  if (dtype == 1) OURO_PLAIN(bf16_t); else OURO_PLAIN(float);
#undef OURO_PLAIN
  return hipGetLastError();
}

hipError_t launch_gemm_group(hipStream_t s, int dtype, const GemmDesc* g, int n, bool* grouped) {
  if (grouped) *grouped = false;
  if (n < 1 || n > GEMM_GROUP_MAX) return hipErrorInvalidValue;
  // products that do not admit the grouped kernel go by themselves
  GemmDesc in[GEMM_GROUP_MAX];
  int ni = 0;
  for (int i = 0; i < n; ++i) {
    const GemmDesc& d = g[i];
    const size_t bA = 2 * (size_t)d.K * d.lda, bB = 2 * (size_t)d.K * d.ldb;
    const bool ok = dtype == 1 && d.transA == 1 && d.transB == 0 && d.accumulate && d.out_fp32 && !d.bias && !d.residual &&
                    !d.res32 && d.epilogue == EPI_NONE && !d.drop.on && d.by <= 1 && d.bz <= 1 && !d.C2 && d.M > 0 && d.N > 0 &&
                    gemm_uses_mfma(dtype, d) && (d.K % 64) == 0 && d.K >= 512 && bA < (1ull << 31) && bB < (1ull << 31);
    if (ok) { in[ni++] = d; continue; }
    hipError_t e = launch_gemm(s, dtype, d, 0);
    if (e != hipSuccess) return e;
  }
  if (ni == 0) return hipSuccess;
  if (ni == 1) return launch_gemm(s, dtype, in[0], 0);
  g = in; n = ni;
  // One K-range length for all products: whole rounds of workgroups (two per CU) times the K-tiles
  // of a workgroup plus its fixed cost (ring fill, atomic epilogue: 6 K-tiles), as in launch_gemm.
  int kmax = 0;
  for (int i = 0; i < n; ++i) kmax = std::max(kmax, g[i].K);
  double best = 1e30;
  int kchunk = kmax;
  for (int kc = 256; kc <= kmax; kc += 64) {
    long wgs = 0;
    for (int i = 0; i < n; ++i)
      wgs += (long)((g[i].M + 127) / 128) * ((g[i].N + 127) / 128) * ((g[i].K + kc - 1) / kc);
    const long rounds = (wgs + 511) / 512;
    const double cost = (double)rounds * (kc / 64 + 6);
    if (cost < best - 1e-9) { best = cost; kchunk = kc; }
  }
  GemmParams ps[GEMM_GROUP_MAX];
  for (int i = 0; i < n; ++i) {
    const GemmDesc& d = g[i];
    GemmParams& p = ps[i];
    memset(&p, 0, sizeof p);
    p.A = d.A; p.B = d.B; p.C = d.C;
    p.M = d.M; p.N = d.N; p.K = d.K; p.lda = d.lda; p.ldb = d.ldb; p.ldc = d.ldc;
    p.out_fp32 = 1; p.accumulate = 1; p.epilogue = EPI_NONE; p.alpha = d.alpha;
    p.by = p.bz = p.bz1 = 1;
    // every product splits into ranges of the same length, rounded so that the last is not a sliver
    const int splits = (d.K + kchunk - 1) / kchunk;
    p.kchunk = ((d.K + splits - 1) / splits + 63) / 64 * 64;
  }
  if (grouped) *grouped = true;
  return launch_gemm_dlds_group(s, ps, n, 1, 0);
}

}  // namespace ouro
