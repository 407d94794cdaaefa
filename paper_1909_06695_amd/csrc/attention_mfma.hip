// Fused causal attention on the matrix cores (bf16, head size 64, no relative term).
//
// All three kernels keep the softmax row index in the lane: the score tile is produced
// transposed (keys x queries in the forward and dQ kernels, queries x keys in the dK/dV
// kernel), so a lane owns one query (or key) column and row statistics need a single
// cross-half shuffle.  The probabilities feed the next matrix instruction straight from
// the accumulator registers: the contraction index may be enumerated in any order as long
// as both operands agree, so the other operand is fetched in the accumulator's own row
// order and nothing is exchanged between lanes.
//
// K / V / Q / dO tiles (64 rows x 64 features) go global -> LDS with direct 16-byte loads
// into a three-stage ring, one copy per tile: products that contract over the feature
// index read rows (16 bytes per lane); products that contract over the row index read the
// same tile with the LDS transpose-read instruction.  Online softmax in base 2; the
// log-sum-exp is saved for the backward kernels.
#include "attention_tiles.h"

#include <algorithm>

namespace ouro {

// ------------------------------------------------------------------------------ forward
// grid (ceil(T/128), H, B); 4 waves x 32 queries; key blocks of 64.
// The forward kernel runs four waves per SIMD (four workgroups per CU): it fits 128 registers, and
// a two-stage K/V ring (32 KB) leaves room for four workgroups in LDS.  The kernel is a chain of
// matrix instructions, softmax arithmetic and matrix instructions again per key block, so what
// it needs is other waves to run meanwhile, not a deeper ring: 46 -> 35 us at T = 1024, 8 x 16 heads.
// The dQ kernel works through one 32-key sub-tile at a time so that it fits three waves per SIMD
// (76 -> 69 us); the dK/dV kernel needs 190 registers without spilling and stays at two.
constexpr int FWD_NSTAGE = 2;
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void fa_fwd_kernel(FaParams p) {
  __shared__ __attribute__((aligned(16))) char lds[FWD_NSTAGE * 2 * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  int rank, head, b;
  fa_decode_block(rank, head, b);
  const int qblk = gridDim.x - 1 - rank;                  // the last query block has the longest rows
  const int q0 = qblk * 128 + wave * 32, qi = q0 + l32;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (qi < p.T) t = *reinterpret_cast<const uint4*>(qb + (size_t)qi * p.ldq + 16 * ks + 8 * h32);
    qf[ks] = as_bf16x8(t);
  }
  const int wg_last_q = min(p.T, qblk * 128 + 128) - 1;
  const int kend = min(p.S, p.Mv + wg_last_q + 1);
  const int nkb = (kend + 63) / 64;
  const bool wave_on = q0 < p.T;
  const int wave_kmax = p.Mv + min(p.T - 1, q0 + 31);
  f32x16 oacc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % FWD_NSTAGE) * (2 * TILE_BYTES);
    dma_tile(kb, p.ldk, jb * 64, p.S, st, wave, lane);
    dma_tile(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane);
  };
  constexpr int LPT = 4;                                   // loads per thread per stage
#pragma unroll
  for (int s = 0; s < FWD_NSTAGE - 1; ++s)
    if (s < nkb) issue(s);
  for (int jb = 0; jb < nkb; ++jb) {
    if (jb + FWD_NSTAGE - 1 <= nkb) fa_wait_vmcnt<(FWD_NSTAGE - 2) * LPT>();
    else fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // unfenced: younger tiles' loads stay in flight
    if (jb + FWD_NSTAGE - 1 < nkb) issue(jb + FWD_NSTAGE - 1);
    const char* sK = lds + (jb % FWD_NSTAGE) * (2 * TILE_BYTES);
    const char* sV = sK + TILE_BYTES;
    if (wave_on && jb * 64 <= wave_kmax) {
      // keys 32..63 of a diagonal block are masked for every query of some waves: skip them
      const int nkt = (jb * 64 + 32 <= wave_kmax) ? 2 : 1;
      // no element of the block is masked when its last key is visible to the wave's first query
      const bool edge = jb * 64 + 63 > p.Mv + q0 || jb * 64 + 63 >= p.S || q0 + 31 >= p.T;
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kt, ks, lane), qf[ks], s[kt], 0, 0, 0);
        }
      }
      float mloc = -INFINITY;                              // of the raw scores (the scale is positive)
      if (edge) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
          if (kt < nkt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int key = jb * 64 + 32 * kt + 8 * (r >> 2) + 4 * h32 + (r & 3);
              bool vis = key <= p.Mv + qi && key < p.S && qi < p.T;
              float val = vis ? s[kt][r] : -INFINITY;
              s[kt][r] = val;
              mloc = fmaxf(mloc, val);
            }
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[kt][r]);
      }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64)) * p.scale_log2;
      // The reference maximum only moves when a row's maximum grows by more than 2^8: any
      // reference gives the same quotient, and probabilities up to 2^8 are harmless in fp32
      // and bf16, so most blocks skip the rescaling of the output accumulator.
      const bool grow = mloc > m + 8.f;
      if (__any(grow)) {
        const float m_new = grow ? mloc : m;
        const float alpha = grow ? __builtin_amdgcn_exp2f(m - m_new) : 1.f;
        l *= alpha;
        m = m_new;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
      }
      const float neg_m = (m == -INFINITY) ? 0.f : -m;
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float pv = __builtin_amdgcn_exp2f(fmaf(s[kt][r], p.scale_log2, neg_m));
            s[kt][r] = pv;
            lsum += pv;
          }
        }
      lsum += __shfl_xor(lsum, 32, 64);
      l += lsum;
#pragma unroll
      for (int ks2 = 0; ks2 < 4; ++ks2) {
        const int kt = ks2 >> 1, sub = ks2 & 1;
        if (kt < nkt) {
          bf16x8 pb = pack_acc(s[kt], sub);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sV, 32 * dt, 32 * kt + 16 * sub, lane), pb, oacc[dt], 0, 0, 0);
        }
      }
    }
  }
  if (qi < p.T) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
    store_acc_row(p.o + ((size_t)b * p.T + qi) * p.ldo + head * 64, oacc, inv, h32);
    if (h32 == 0) p.lse[((size_t)b * p.H + head) * p.T + qi] = (m + log2f(l)) * 0.6931471805599453f;
  }
}

// ------------------------------------------------------------------------ dK, dV kernel
// grid (ceil(ceil(S/128) / 2), H, B); 4 waves x 32 keys; query blocks of 64: S = Q K^T and dP = dO V^T
// read Q / dO rows, dV^T += dO^T P and dK^T += Q^T dS read the same tiles transposed.
constexpr int DKV_STAGE = 2 * TILE_BYTES + 1024;   // Q, dO, lse[64], D[64], two spare lines
// two workgroups per compute unit (256 registers per lane)
template <bool PAIR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void fa_bwd_dkv_kernel(FaParams p) {
  __shared__ __attribute__((aligned(16))) char lds[NSTAGE * DKV_STAGE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  int first, head, b;                                     // key block 0 sees every query: the heaviest
  if (PAIR) { first = blockIdx.x; head = blockIdx.y; b = blockIdx.z; }
  else fa_decode_block(first, head, b);
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* dob = p.d_o + (size_t)b * p.T * p.lddo + head * 64;
  const bf16_t* kbp = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vbp = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const float* lseb = p.lse2 + ((size_t)b * p.H + head) * p.T;
  const float* Db = p.D + ((size_t)b * p.H + head) * p.T;
  // Key block k sees the queries from 128 k - Mv on, so its work falls linearly with k.  Where
  // the launch still fills the chip that way (PAIR), a workgroup takes block k and then block
  // (last - k), and every workgroup has the same amount of work: with one block each the resident
  // waves per SIMD averaged 1.1 of 2 over the launch, the slots of the light blocks standing empty
  // while the heavy ones finished (T = 1024, 8 x 16 heads: 77 -> 62 us).
  const int nkblk = (p.S + 127) / 128;
  for (int pass = 0; pass < (PAIR ? 2 : 1); ++pass) {
  const int kblk = pass == 0 ? first : nkblk - 1 - first;
  if (pass == 1) {
    if (kblk <= first) break;                             // odd count: the middle block has no partner
    fa_wait_vmcnt<0>();                                   // the first block's stores and loads are done,
    __syncthreads();                                      // ... and every wave is past its last LDS read
  }
  const int kb0 = kblk * 128 + wave * 32, key = kb0 + l32;
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t0 = make_uint4(0, 0, 0, 0), t1 = t0;
    if (key < p.S) {
      t0 = *reinterpret_cast<const uint4*>(kbp + (size_t)key * p.ldk + 16 * ks + 8 * h32);
      t1 = *reinterpret_cast<const uint4*>(vbp + (size_t)key * p.ldv + 16 * ks + 8 * h32);
    }
    kf[ks] = as_bf16x8(t0);
    vf[ks] = as_bf16x8(t1);
  }
  f32x16 dkT[2], dvT[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkT[dt][r] = 0.f; dvT[dt][r] = 0.f; }
  // first query block that sees the workgroup's first key: i >= key - Mv
  const int ib0 = max(0, kblk * 128 - p.Mv) / 64;
  const int nib = (p.T + 63) / 64;
  const int nit = nib - ib0;
  const bool wave_on = kb0 < p.S;
  auto issue = [&](int it) __attribute__((always_inline)) {
    char* st = lds + (it % NSTAGE) * DKV_STAGE;
    const int i0 = (ib0 + it) * 64;
    dma_tile(qb, p.ldq, i0, p.T, st, wave, lane);
    dma_tile(dob, p.lddo, i0, p.T, st + TILE_BYTES, wave, lane);
    // waves 0/1 fetch lse / D; waves 2/3 repeat them into spare lines so that every wave
    // has the same number of loads in flight
    dma_floats((wave & 1) ? Db : lseb, i0, p.T, st + 2 * TILE_BYTES + wave * 256, lane);
  };
  constexpr int LPT = 5;
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nit) issue(s);
  for (int it = 0; it < nit; ++it) {
    if (it + NSTAGE - 1 <= nit) fa_wait_vmcnt<(NSTAGE - 2) * LPT>();
    else fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // unfenced: younger tiles' loads stay in flight
    if (it + NSTAGE - 1 < nit) issue(it + NSTAGE - 1);
    const int ib = ib0 + it;
    const char* sQ = lds + (it % NSTAGE) * DKV_STAGE;
    const char* sdO = sQ + TILE_BYTES;
    const float* sl = reinterpret_cast<const float*>(sQ + 2 * TILE_BYTES);
    const float* sD = sl + 64;
    if (wave_on && p.Mv + ib * 64 + 63 >= kb0) {
      // queries 0..31 of a diagonal block see none of some waves' keys: skip them
      const int qt0 = (p.Mv + ib * 64 + 31 >= kb0) ? 0 : 1;
      // nothing is masked when the block's first query sees the wave's last key
      const bool edge = kb0 + 31 > p.Mv + ib * 64 || ib * 64 + 63 >= p.T || kb0 + 31 >= p.S;
      // one 32-query sub-tile at a time: scores and dP of a single sub-tile are live
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        if (qt >= qt0) {
          f32x16 s, dp;
#pragma unroll
          for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sQ, 32 * qt, ks, lane), kf[ks], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sdO, 32 * qt, ks, lane), vf[ks], dp, 0, 0, 0);
          }
          // P = exp2(s * scale * log2 e - lse2); dS = P (dP - D); the factor `scale` of dS is
          // applied once, to the finished dK.  Two copies of the loop: the test for masked
          // elements stays out of the blocks the diagonal does not cross.
          if (edge) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int ql0 = 32 * qt + 8 * g + 4 * h32;
              const float4 l4 = *reinterpret_cast<const float4*>(sl + ql0);
              const float4 d4 = *reinterpret_cast<const float4*>(sD + ql0);
              const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int r = 4 * g + j;
                const int qi = ib * 64 + ql0 + j;
                const bool vis = key <= p.Mv + qi && qi < p.T && key < p.S;
                const float pv = vis ? __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lv[j])) : 0.f;
                s[r] = pv;
                dp[r] = pv * (dp[r] - dv4[j]);
              }
            }
          } else {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int ql0 = 32 * qt + 8 * g + 4 * h32;
              const float4 l4 = *reinterpret_cast<const float4*>(sl + ql0);
              const float4 d4 = *reinterpret_cast<const float4*>(sD + ql0);
              const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const int r = 4 * g + j;
                const float pv = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lv[j]));
                s[r] = pv;
                dp[r] = pv * (dp[r] - dv4[j]);
              }
            }
          }
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) {
            bf16x8 pb = pack_acc(s, sub);
            bf16x8 dsb = pack_acc(dp, sub);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
              dvT[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sdO, 32 * dt, 32 * qt + 16 * sub, lane), pb, dvT[dt], 0, 0, 0);
              dkT[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sQ, 32 * dt, 32 * qt + 16 * sub, lane), dsb, dkT[dt], 0, 0, 0);
            }
          }
        }
      }
    }
  }
  if (key < p.S) {
    store_acc_row(p.dk + ((size_t)b * p.S + key) * p.lddk + head * 64, dkT, p.scale, h32);
    store_acc_row(p.dv + ((size_t)b * p.S + key) * p.lddv + head * 64, dvT, 1.f, h32);
  }
  }
}

// ---------------------------------------------------------------------------- dQ kernel
// grid (ceil(ceil(T/128) / 2), H, B); 4 waves x 32 queries; key blocks of 64: S^T = K Q^T and
// dP^T = V dO^T read K / V rows, dQ^T += K^T dS^T reads the K tile transposed.
template <bool PAIR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void fa_bwd_dq_kernel(FaParams p) {
  __shared__ __attribute__((aligned(16))) char lds[NSTAGE * 2 * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  int rank, head, b;                                      // rank 0: the last query block, the heaviest
  if (PAIR) { rank = blockIdx.x; head = blockIdx.y; b = blockIdx.z; }
  else fa_decode_block(rank, head, b);
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* dob = p.d_o + (size_t)b * p.T * p.lddo + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  // the work of query block q grows linearly with q: with PAIR a workgroup takes block
  // (last - rank) and then block rank, so that all workgroups of the launch carry the same load
  // (see the dK/dV kernel; 59 -> 53 us)
  const int nqblk = (p.T + 127) / 128;
  for (int pass = 0; pass < (PAIR ? 2 : 1); ++pass) {
  const int qblk = pass == 0 ? nqblk - 1 - rank : rank;
  if (pass == 1) {
    if (qblk >= nqblk - 1 - rank) break;                  // odd count: the middle block has no partner
    fa_wait_vmcnt<0>();                                   // the first block's stores and loads are done,
    __syncthreads();                                      // ... and every wave is past its last LDS read
  }
  const int q0 = qblk * 128 + wave * 32, qi = q0 + l32;
  bf16x8 qf[4], dof[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t0 = make_uint4(0, 0, 0, 0), t1 = t0;
    if (qi < p.T) {
      t0 = *reinterpret_cast<const uint4*>(qb + (size_t)qi * p.ldq + 16 * ks + 8 * h32);
      t1 = *reinterpret_cast<const uint4*>(dob + (size_t)qi * p.lddo + 16 * ks + 8 * h32);
    }
    qf[ks] = as_bf16x8(t0);
    dof[ks] = as_bf16x8(t1);
  }
  // D = sum_c dO[i,c] O[i,c] and the base-2 log-sum-exp of the lane's query; both are also
  // left in the scratch arrays for the dK/dV kernel, which runs after this one
  float lse_q = 0.f, D_q = 0.f;
  {
    const bf16_t* ob = p.o + (size_t)b * p.T * p.ldo + head * 64;
    float part = 0.f;
    if (qi < p.T) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8 of = as_bf16x8(*reinterpret_cast<const uint4*>(ob + (size_t)qi * p.ldo + 16 * ks + 8 * h32));
#pragma unroll
        for (int e = 0; e < 8; ++e) part += (float)of[e] * (float)dof[ks][e];
      }
    }
    D_q = part + __shfl_xor(part, 32, 64);
    if (qi < p.T) {
      const size_t r = ((size_t)b * p.H + head) * p.T + qi;
      lse_q = p.lse[r] * 1.4426950408889634f;
      if (h32 == 0) { p.D[r] = D_q; p.lse2[r] = lse_q; }
    }
  }
  const int wg_last_q = min(p.T, qblk * 128 + 128) - 1;
  const int kend = min(p.S, p.Mv + wg_last_q + 1);
  const int nkb = (kend + 63) / 64;
  const bool wave_on = q0 < p.T;
  const int wave_kmax = p.Mv + min(p.T - 1, q0 + 31);
  f32x16 dqT[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqT[dt][r] = 0.f;
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % NSTAGE) * (2 * TILE_BYTES);
    dma_tile(kb, p.ldk, jb * 64, p.S, st, wave, lane);
    dma_tile(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane);
  };
  constexpr int LPT = 4;
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nkb) issue(s);
  for (int jb = 0; jb < nkb; ++jb) {
    if (jb + NSTAGE - 1 <= nkb) fa_wait_vmcnt<(NSTAGE - 2) * LPT>();
    else fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // unfenced: younger tiles' loads stay in flight
    if (jb + NSTAGE - 1 < nkb) issue(jb + NSTAGE - 1);
    const char* sK = lds + (jb % NSTAGE) * (2 * TILE_BYTES);
    const char* sV = sK + TILE_BYTES;
    if (wave_on && jb * 64 <= wave_kmax) {
      const int nkt = (jb * 64 + 32 <= wave_kmax) ? 2 : 1;
      const bool edge = jb * 64 + 63 > p.Mv + q0 || jb * 64 + 63 >= p.S || q0 + 31 >= p.T;
      // one 32-key sub-tile at a time: scores and dP of a single sub-tile are live, which keeps
      // the kernel at three waves per SIMD
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        if (kt < nkt) {
          f32x16 s, dp;
#pragma unroll
          for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kt, ks, lane), qf[ks], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sV, 32 * kt, ks, lane), dof[ks], dp, 0, 0, 0);
          }
          // dS without its factor `scale`, which the finished dQ takes once.  Two copies of the
          // loop: the test for masked elements stays out of the blocks the diagonal does not cross.
          if (edge) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = jb * 64 + 32 * kt + 8 * (r >> 2) + 4 * h32 + (r & 3);
              const bool vis = key <= p.Mv + qi && key < p.S && qi < p.T;
              const float pv = vis ? __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lse_q)) : 0.f;
              dp[r] = pv * (dp[r] - D_q);
            }
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float pv = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lse_q));
              dp[r] = pv * (dp[r] - D_q);
            }
          }
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) {
            bf16x8 dsb = pack_acc(dp, sub);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
              dqT[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sK, 32 * dt, 32 * kt + 16 * sub, lane), dsb, dqT[dt], 0, 0, 0);
          }
        }
      }
    }
  }
  if (qi < p.T) store_acc_row(p.dq + ((size_t)b * p.T + qi) * p.lddq + head * 64, dqT, p.scale, h32);
  }
}

// ----------------------------------------------------------------------------- dispatch
static inline bool al16(const void* x) { return (reinterpret_cast<uintptr_t>(x) & 15) == 0; }

bool attn_mfma_ok(int dtype, const AttnDesc& a) {
  if (dtype != 1 || a.dh != 64 || a.rel) return false;
  if ((a.ldq | a.ldk | a.ldv | a.ldo) & 7) return false;
  if (!al16(a.q) || !al16(a.k) || !al16(a.v) || !al16(a.o)) return false;
  if (a.d_o) {
    if ((a.lddo | a.lddq | a.lddk | a.lddv) & 7) return false;
    if (!al16(a.d_o) || !al16(a.dq) || !al16(a.dk) || !al16(a.dv)) return false;
  }
  return true;
}

hipError_t launch_attn_fwd_mfma(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  dim3 grid((a.T + 127) / 128, a.H, a.B), block(256);
  hipLaunchKernelGGL(fa_fwd_kernel, grid, block, 0, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  // two blocks of the causal axis per workgroup where that still leaves two workgroups per compute unit
  const int nq = (a.T + 127) / 128, nk = (a.S + 127) / 128;
  const bool pair = (long)((std::min(nq, nk) + 1) / 2) * a.H * a.B >= 512;
  // the dQ kernel also produces the row sums D and the base-2 log-sum-exp the dK/dV kernel reads
  if (pair) hipLaunchKernelGGL(fa_bwd_dq_kernel<true>, dim3((nq + 1) / 2, a.H, a.B), dim3(256), 0, s, p);
  else hipLaunchKernelGGL(fa_bwd_dq_kernel<false>, dim3(nq, a.H, a.B), dim3(256), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (pair) hipLaunchKernelGGL(fa_bwd_dkv_kernel<true>, dim3((nk + 1) / 2, a.H, a.B), dim3(256), 0, s, p);
  else hipLaunchKernelGGL(fa_bwd_dkv_kernel<false>, dim3(nk, a.H, a.B), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace ouro
