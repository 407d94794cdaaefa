// Fused causal attention with the Transformer-XL relative-position term on the matrix cores
// (bf16, head size 64):  score(i, j) = (q_i + u) . k_j + (q_i + v) . r_{Mv + i - j}.
//
// The content term is the plain kernel's product with q + u in place of q.  The position term
// of a 32-query x 64-key block only involves the 95 distances Mv + i - j of the block: the
// product of those rows of r with q + v is one more matrix product, and the element the score
// (i, j) needs sits on the diagonal Mv + i - j of it.  A lane owns a query (forward and dQ
// kernels), so that diagonal runs through the lane's own column: the product goes through a
// per-wave LDS patch and comes back shifted, and dS takes the same way back for dQ.
//
// dK and dV have no attention kernel of their own: the dQ kernel, which holds the probabilities
// P and dS of every visible pair anyway, leaves P^T and dS^T (key as row) in the workspace, and
// dV = P^T dO, dK = scale dS^T (Q + u) are contractions on the contraction kernels (one product
// per (head, batch)); dr is gathered from dS^T along its diagonals by fa_xl_dr_kernel.  A kernel
// that owns keys would have to rotate the position product across lanes element by element and
// add dr atomically from every (batch, key block): that took 418 us per layer at 16 x 16 heads,
// T = M = 384.
#include "attention_tiles.h"

#include <algorithm>

namespace ouro {

constexpr int XL_RWIN = 192;                         // rows of r a workgroup needs per block
constexpr int XL_STAGE = 2 * TILE_BYTES + XL_RWIN * 128;   // K, V, r window
constexpr int XL_NSTAGE = 2;
constexpr int XL8_LD = 34;                           // floats per patch row (33: 218 us in the dQ kernel, 32: 227, 34: 214)
constexpr int XL8_PATCH = 64 * XL8_LD * 4;           // bytes per wave
constexpr int XL_LDS_Q8 = XL_NSTAGE * XL_STAGE + 8 * XL8_PATCH;

// One wave's share (8 rows) of a direct load of 64 rows x 64 features into an LDS tile; the row
// index is clamped to [0 or -inf, rmax-1].
__device__ __forceinline__ void dma_tile8(const bf16_t* src, int ld, int row0, int rmax, char* tile, int wave, int lane, bool clamp_low) {
  const int row = 8 * wave + (lane >> 3);
  const int c = (lane & 7) ^ swza(row);
  int gr = min(row0 + row, rmax - 1);
  if (clamp_low) gr = max(0, gr);
  __builtin_amdgcn_global_load_lds((gbl_void*)(src + (size_t)gr * ld + 8 * c), (lds_void*)(tile + wave * 1024), 16, 0, 0);
}

// q + bias for the lane's fragment features (fp32 add, rounded to bf16 once)
__device__ __forceinline__ bf16x8 add_bias(bf16x8 q, const bf16_t* bias8) {
  bf16x8 b = as_bf16x8(*reinterpret_cast<const uint4*>(bias8)), r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)((float)q[e] + (float)b[e]);
  return r;
}

// row of the accumulator element r of the lane's half: 8*(r/4) + 4*half + r%4
__device__ __forceinline__ constexpr int acc_row(int r, int h32) { return 8 * (r >> 2) + 4 * h32 + (r & 3); }

// Position term of a 32-key sub-tile for a wave whose lanes own queries: rows [rrow0, +64) of
// the r window times (q + v), written to the wave's patch as patch[rho][query].  Key kk of the
// sub-tile and the lane's query meet at patch row 31 + lane%32 - kk.
__device__ __forceinline__ void xl_position_product(const char* sR, int rrow0, const bf16x8 (&qvf)[4], float* patch, int lane) {
  const int h32 = lane >> 5, l32 = lane & 31;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sR, rrow0 + 32 * t, ks, lane), qvf[ks], acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) patch[(32 * t + acc_row(r, h32)) * XL8_LD + l32] = acc[r];
  }
}

// Forward kernel: workgroup -> (query block, head, batch), longest rows first over the whole launch: the
// dispatcher hands out workgroups in linear id order, so all workgroups of the last query block
// (the most keys) start first and the lighter blocks fill the slots as they free up.
__device__ __forceinline__ void xl_decode_block(int& qblk, int& head, int& b) {
  const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int per = gridDim.y * gridDim.z;
  const int rest = lin % per;
  qblk = gridDim.x - 1 - lin / per;
  head = rest % gridDim.y;
  b = rest / gridDim.y;
}

// Both kernels below: grid (ceil(T/128), H, B); 8 waves = (4 groups of 32 queries) x (the two
// 32-key halves of a 64-key block), waves w and w + 4 (one query group) on one SIMD; one
// workgroup per CU, so two waves per SIMD (with four waves owning whole 64-key blocks, one per
// SIMD, the forward pass took 93 us and the dQ kernel 266 us per layer at 16 x 16 heads,
// T = M = 384; in this form 89 and 214).  A wave's patch holds the 63 distances of its 32 x 32
// sub-tile (64 rows).  Stages hold K, V and the r window of the 128 queries; every wave issues
// one 1 KiB load per tile.

// ------------------------------------------------------------------------------ forward
// The two key halves of a query group keep their own running maximum, sum and output; the
// second half hands its state to the first through LDS at the end.
__global__ __launch_bounds__(512) void fa_xl_fwd_kernel(FaParams p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  const int qg = wave & 3, kh = wave >> 2;
  int qblk, head, b;
  xl_decode_block(qblk, head, b);
  const int Q0 = qblk * 128, q0 = Q0 + qg * 32, qi = q0 + l32;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const bf16_t* rb = p.r + head * 64;
  float* patch = reinterpret_cast<float*>(lds + XL_NSTAGE * XL_STAGE + wave * XL8_PATCH);
  bf16x8 quf[4], qvf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (qi < p.T) t = *reinterpret_cast<const uint4*>(qb + (size_t)qi * p.ldq + 16 * ks + 8 * h32);
    quf[ks] = add_bias(as_bf16x8(t), p.u + head * 64 + 16 * ks + 8 * h32);
    qvf[ks] = add_bias(as_bf16x8(t), p.vb + head * 64 + 16 * ks + 8 * h32);
  }
  const int wg_last_q = min(p.T, Q0 + 128) - 1;
  const int kend = min(p.S, p.Mv + wg_last_q + 1);
  const int nkb = (kend + 63) / 64;
  const bool wave_on = q0 < p.T;
  const int wave_kmax = p.Mv + min(p.T - 1, q0 + 31);
  const int rrow0 = 32 * qg + 32 * (1 - kh);                // window row of the wave's patch row 0
  f32x16 oacc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % XL_NSTAGE) * XL_STAGE;
    dma_tile8(kb, p.ldk, jb * 64, p.S, st, wave, lane, false);
    dma_tile8(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane, false);
    const int d0 = p.Mv + Q0 - jb * 64 - 63;              // distance of window row 0
#pragma unroll
    for (int t = 0; t < 3; ++t) dma_tile8(rb, p.ldr, d0 + 64 * t, p.S, st + 2 * TILE_BYTES + t * TILE_BYTES, wave, lane, true);
  };
  issue(0);
  for (int jb = 0; jb < nkb; ++jb) {
    fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (jb + 1 < nkb) issue(jb + 1);
    const char* sK = lds + (jb % XL_NSTAGE) * XL_STAGE;
    const char* sV = sK + TILE_BYTES;
    const char* sR = sK + 2 * TILE_BYTES;
    const int key0 = jb * 64 + 32 * kh;                     // first key of the wave's sub-tile
    if (wave_on && key0 <= wave_kmax) {
      const bool edge = key0 + 31 > p.Mv + q0 || key0 + 31 >= p.S || q0 + 31 >= p.T;
      xl_position_product(sR, rrow0, qvf, patch, lane);
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kh, ks, lane), quf[ks], s, 0, 0, 0);
      __builtin_amdgcn_wave_barrier();
      const float* cell0 = patch + (31 + l32 - 4 * h32) * XL8_LD + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] += cell0[-(8 * (r >> 2) + (r & 3)) * XL8_LD];
      __builtin_amdgcn_wave_barrier();
      float mloc = -INFINITY;
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + acc_row(r, h32);
          const bool vis = key <= p.Mv + qi && key < p.S && qi < p.T;
          s[r] = vis ? s[r] : -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[r]);
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64)) * p.scale_log2;
      const bool grow = mloc > m + 8.f;                    // lazy reference maximum, as in the plain kernel
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
      for (int r = 0; r < 16; ++r) {
        s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, neg_m));
        lsum += s[r];
      }
      lsum += __shfl_xor(lsum, 32, 64);
      l += lsum;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        bf16x8 pb = pack_acc(s, sub);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sV, 32 * dt, 32 * kh + 16 * sub, lane), pb, oacc[dt], 0, 0, 0);
      }
    }
  }
  // merge the two key halves: state of the second through its patch (34 floats per lane)
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) patch[(16 * dt + r) * 64 + lane] = oacc[dt][r];
    patch[32 * 64 + lane] = m;
    patch[33 * 64 + lane] = l;
  }
  __syncthreads();
  if (kh == 0 && qi < p.T) {
    const float* other = reinterpret_cast<const float*>(lds + XL_NSTAGE * XL_STAGE + (wave + 4) * XL8_PATCH);
    const float m1 = other[32 * 64 + lane], l1 = other[33 * 64 + lane];
    const float mm = fmaxf(m, m1);
    const float a0 = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mm);
    const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - mm);
    l = l * a0 + l1 * a1;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] = oacc[dt][r] * a0 + other[(16 * dt + r) * 64 + lane] * a1;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    store_acc_row(p.o + ((size_t)b * p.T + qi) * p.ldo + head * 64, oacc, inv, h32);
    if (h32 == 0) p.lse[((size_t)b * p.H + head) * p.T + qi] = (mm + log2f(l)) * 0.6931471805599453f;
  }
}


// ---------------------------------------------------------------------------- dQ kernel
// The two key halves of a query group add their dQ through LDS at the end.  Besides dQ the
// kernel produces the gradients of the two biases (du = sum over queries of the content half of
// dq, dvb = that of the position half) and leaves what the gradients of k, v and r are
// contractions of:
//   pt  [B, H, S, t_ld]   P^T, probabilities with the key as row, bf16 (dV = P^T dO)
//   dst [B, H, S, t_ld]   dS^T, likewise (dK = scale dS^T (Q + u); dr: fa_xl_dr_kernel)
//   qu, qv, dop [B, t_ld, H * 64]   q + u, q + v, dO with rows padded to t_ld
// t_ld = T rounded up to 64; a cell of pt / dst is addressed by a 32-bit byte offset within its
// (batch, head) matrix, so S * t_ld * 2 < 2^32 (attn_xl_ok).  Every (query, key) cell in a
// computed 32-key sub-tile is written (masked cells as zero); cells outside (keys no query of
// the wave sees, rows i >= T) are never written and must be zero from the caller (they are the
// same cells for the same Mv).
__global__ __launch_bounds__(512) void fa_xl_dq_kernel(FaParams p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  const int qg = wave & 3, kh = wave >> 2;                  // waves w and w + 4 share a SIMD
  // (the launch-wide heaviest-first order of the forward kernel measured 10 % slower here: the three
  // query blocks of a (batch, head) then write their parts of P^T and dS^T far apart in time)
  const int qblk = gridDim.x - 1 - blockIdx.x;
  const int head = blockIdx.y, b = blockIdx.z;
  const int Q0 = qblk * 128, q0 = Q0 + qg * 32, qi = q0 + l32;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* dob = p.d_o + (size_t)b * p.T * p.lddo + head * 64;
  const bf16_t* ob = p.o + (size_t)b * p.T * p.ldo + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const bf16_t* rb = p.r + head * 64;
  float* patch = reinterpret_cast<float*>(lds + XL_NSTAGE * XL_STAGE + wave * XL8_PATCH);
  bf16x8 quf[4], qvf[4], dof[4];
  float part = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t0 = make_uint4(0, 0, 0, 0), t1 = t0, t2 = t0;
    if (qi < p.T) {
      t0 = *reinterpret_cast<const uint4*>(qb + (size_t)qi * p.ldq + 16 * ks + 8 * h32);
      t1 = *reinterpret_cast<const uint4*>(dob + (size_t)qi * p.lddo + 16 * ks + 8 * h32);
      t2 = *reinterpret_cast<const uint4*>(ob + (size_t)qi * p.ldo + 16 * ks + 8 * h32);
    }
    quf[ks] = add_bias(as_bf16x8(t0), p.u + head * 64 + 16 * ks + 8 * h32);
    qvf[ks] = add_bias(as_bf16x8(t0), p.vb + head * 64 + 16 * ks + 8 * h32);
    dof[ks] = as_bf16x8(t1);
    if (qi < p.T && kh == 0) {
      const size_t at = ((size_t)b * p.t_ld + qi) * (p.H * 64) + head * 64 + 16 * ks + 8 * h32;
      *reinterpret_cast<bf16x8*>(p.qu + at) = quf[ks];
      *reinterpret_cast<bf16x8*>(p.qv + at) = qvf[ks];
      *reinterpret_cast<bf16x8*>(p.dop + at) = dof[ks];
    }
    const bf16x8 of = as_bf16x8(t2);
#pragma unroll
    for (int e = 0; e < 8; ++e) part += (float)of[e] * (float)dof[ks][e];
  }
  const float D_q = part + __shfl_xor(part, 32, 64);
  float lse_q = 0.f;
  if (qi < p.T) lse_q = p.lse[((size_t)b * p.H + head) * p.T + qi] * 1.4426950408889634f;
  // this (batch, head)'s P^T and dS^T (uniform bases; a cell's offset fits 32 bits)
  bf16_t* ptb = p.pt + ((size_t)b * p.H + head) * p.S * p.t_ld;
  bf16_t* dstb = p.dst + ((size_t)b * p.H + head) * p.S * p.t_ld;
  const int wg_last_q = min(p.T, Q0 + 128) - 1;
  const int kend = min(p.S, p.Mv + wg_last_q + 1);
  const int nkb = (kend + 63) / 64;
  const bool wave_on = q0 < p.T;
  const int wave_kmax = p.Mv + min(p.T - 1, q0 + 31);
  const int rrow0 = 32 * qg + 32 * (1 - kh);                // window row of the wave's patch row 0
  f32x16 dqa[2], dqb[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dqa[dt][r] = 0.f; dqb[dt][r] = 0.f; }
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % XL_NSTAGE) * XL_STAGE;
    dma_tile8(kb, p.ldk, jb * 64, p.S, st, wave, lane, false);
    dma_tile8(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane, false);
    const int d0 = p.Mv + Q0 - jb * 64 - 63;
#pragma unroll
    for (int t = 0; t < 3; ++t) dma_tile8(rb, p.ldr, d0 + 64 * t, p.S, st + 2 * TILE_BYTES + t * TILE_BYTES, wave, lane, true);
  };
  issue(0);
  for (int jb = 0; jb < nkb; ++jb) {
    fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (jb + 1 < nkb) issue(jb + 1);
    const char* sK = lds + (jb % XL_NSTAGE) * XL_STAGE;
    const char* sV = sK + TILE_BYTES;
    const char* sR = sK + 2 * TILE_BYTES;
    const int key0 = jb * 64 + 32 * kh;                     // first key of the wave's sub-tile
    if (wave_on && key0 <= wave_kmax) {
      const bool edge = key0 + 31 > p.Mv + q0 || key0 + 31 >= p.S || q0 + 31 >= p.T;
      xl_position_product(sR, rrow0, qvf, patch, lane);
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kh, ks, lane), quf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sV, 32 * kh, ks, lane), dof[ks], dp, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
      // key kk of the sub-tile and the lane's query meet at patch row 31 + l32 - kk: the lane
      // takes its position terms from there, forms P and dS, and puts dS (without its factor
      // `scale`: the finished gradients take it once) back in the same cells
      float* cell0 = patch + (31 + l32 - 4 * h32) * XL8_LD + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] += cell0[-(8 * (r >> 2) + (r & 3)) * XL8_LD];
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + acc_row(r, h32);
          const bool vis = key <= p.Mv + qi && key < p.S && qi < p.T;
          s[r] = vis ? __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lse_q)) : 0.f;
          dp[r] = s[r] * (dp[r] - D_q);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], p.scale_log2, -lse_q));
          dp[r] = s[r] * (dp[r] - D_q);
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) cell0[-(8 * (r >> 2) + (r & 3)) * XL8_LD] = dp[r];
      // bf16 once: the rounded dS feeds dQ below and, with P, goes to the workspace
      bf16x8 pb[2], dsb[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) { pb[sub] = pack_acc(s, sub); dsb[sub] = pack_acc(dp, sub); }
      const unsigned at0 = ((unsigned)(key0 + 4 * h32) * (unsigned)p.t_ld + (unsigned)qi) * 2u;   // byte offset
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (key0 + acc_row(r, h32) < p.S && qi < p.T) {
            const unsigned at = at0 + (unsigned)(8 * (r >> 2) + (r & 3)) * (unsigned)p.t_ld * 2u;
            *reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(ptb) + at) = pb[r >> 3][r & 7];
            *reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(dstb) + at) = dsb[r >> 3][r & 7];
          }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned at = at0 + (unsigned)(8 * (r >> 2) + (r & 3)) * (unsigned)p.t_ld * 2u;
          *reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(ptb) + at) = pb[r >> 3][r & 7];
          *reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(dstb) + at) = dsb[r >> 3][r & 7];
        }
      }
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
          dqa[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sK, 32 * dt, 32 * kh + 16 * sub, lane), dsb[sub], dqa[dt], 0, 0, 0);
      __builtin_amdgcn_wave_barrier();
      // rows of the patch that hold a gradient: 0 <= 31 + l32 - rho < 32
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16 g;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rho = 32 * t + acc_row(r, h32);
          const int kk = 31 + l32 - rho;
          const float v = patch[rho * XL8_LD + l32];
          g[r] = (kk >= 0 && kk < 32) ? v : 0.f;
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          bf16x8 gb = pack_acc(g, sub);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
            dqb[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sR, 32 * dt, rrow0 + 32 * t + 16 * sub, lane), gb, dqb[dt], 0, 0, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  // bias gradients: sums over the wave's queries (lanes of a half), one atomic per feature
  if (wave_on) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float a = dqa[dt][r], c = dqb[dt][r];
#pragma unroll
        for (int m = 1; m < 32; m <<= 1) { a += __shfl_xor(a, m, 64); c += __shfl_xor(c, m, 64); }
        if (l32 == 0) {
          const int f = head * 64 + 32 * dt + acc_row(r, h32);
          unsafeAtomicAdd(p.du + f, a * p.scale);
          unsafeAtomicAdd(p.dvb + f, c * p.scale);
        }
      }
  }
  // dQ: the second key half hands its sum to the first through its (own) patch
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) patch[(16 * dt + r) * 64 + lane] = dqa[dt][r] + dqb[dt][r];
  }
  __syncthreads();
  if (kh == 0 && qi < p.T) {
    const float* other = reinterpret_cast<const float*>(lds + XL_NSTAGE * XL_STAGE + (wave + 4) * XL8_PATCH);
    f32x16 sum[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[dt][r] = dqa[dt][r] + dqb[dt][r] + other[(16 * dt + r) * 64 + lane];
    store_acc_row(p.dq + ((size_t)b * p.T + qi) * p.lddq + head * 64, sum, p.scale, h32);
  }
}


// ------------------------------------------------------------------------------ dr kernel
// dr[delta, f] += scale * sum over (b, i) of dS(b, i, j = Mv + i - delta) * (q + v)(b, i, f), from
// the dS^T the dQ kernel left (key as row).  grid (ceil(S/64) distance blocks, H, batch groups);
// 4 waves: wave = (32 of the 64 distances) x (32 of the 64 features).  Per (batch, 64 queries)
// the cells that meet the block's distances lie in 127 key rows of dS^T; they are staged in LDS
// with rows of 33 dwords, so that the lanes of a fragment read, which walk a diagonal (next
// distance = previous key row, same query column), fall on 32 different banks.  Rows outside
// [0, S) are staged as zeros.  The fragment's eight contraction slots hold the queries
// 8 (e / 4) + 4 half + e % 4 of a 16-query step, the order of the transposing LDS read that
// fetches the (q + v) operand.
constexpr int DR_LD = 132;                               // bytes per staged row
constexpr int DR_STAGE = 128 * DR_LD + TILE_BYTES;       // dS^T rows + the (q + v) tile
constexpr int XL_LDS_DR = 2 * DR_STAGE;

__global__ __launch_bounds__(256) void fa_xl_dr_kernel(FaParams p, int bpw) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), h32 = lane >> 5, l32 = lane & 31;
  const int D0 = blockIdx.x * 64, head = blockIdx.y;
  const int b0 = blockIdx.z * bpw, nb = min(p.B, b0 + bpw) - b0;
  const int wd = wave & 1, wf = wave >> 1;
  const int HD = p.H * 64;
  const int nib = (p.T + 63) / 64;
  const int ib_lo = max(0, D0 - p.Mv) / 64;              // first query block with a key at these distances
  const int nper = nib - ib_lo;
  const int nit = nb * nper;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  uint4 stage[4];
  auto fetch = [&](int it) __attribute__((always_inline)) {
    const int b = b0 + it / nper, i0 = (ib_lo + it % nper) * 64;
    const int jbase = p.Mv + i0 - D0 - 63;
    const bf16_t* src = p.dst + ((size_t)b * p.H + head) * p.S * p.t_ld + i0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = tid + 256 * q, r = c >> 3, cc = c & 7, j = jbase + r;
      stage[q] = make_uint4(0, 0, 0, 0);
      if (j >= 0 && j < p.S) stage[q] = *reinterpret_cast<const uint4*>(src + (size_t)j * p.t_ld + 8 * cc);
    }
    dma_tile(p.qv + (size_t)b * p.t_ld * HD + head * 64, HD, i0, p.t_ld, lds + (it & 1) * DR_STAGE + 128 * DR_LD, wave, lane);
  };
  auto put = [&](int it) __attribute__((always_inline)) {
    char* sT = lds + (it & 1) * DR_STAGE;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = tid + 256 * q, r = c >> 3, cc = c & 7;
      uint32_t* d = reinterpret_cast<uint32_t*>(sT + r * DR_LD + cc * 16);
      d[0] = stage[q].x; d[1] = stage[q].y; d[2] = stage[q].z; d[3] = stage[q].w;
    }
  };
  if (nit > 0) { fetch(0); put(0); }
  for (int it = 0; it < nit; ++it) {
    fa_wait_vmcnt<0>();                                   // this iteration's (q + v) tile has landed
    __syncthreads();                                      // ... and every wave's share of the staged rows is written
    if (it + 1 < nit) fetch(it + 1);
    const char* sT = lds + (it & 1) * DR_STAGE;
    const char* sQ = sT + 128 * DR_LD;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      union { uint16_t h[8]; bf16x8 v; } a;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int qq = 16 * ks + 8 * (e >> 2) + 4 * h32 + (e & 3);
        const int row = qq - (32 * wd + l32) + 63;
        a.h[e] = *reinterpret_cast<const uint16_t*>(sT + row * DR_LD + qq * 2);
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, read_rows_t(sQ, 32 * wf, 16 * ks, lane), acc, 0, 0, 0);
    }
    if (it + 1 < nit) put(it + 1);                         // the other buffer: last read before the barrier above
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int delta = D0 + 32 * wd + acc_row(r, h32);
    if (delta < p.S && nit > 0) unsafeAtomicAdd(p.dr + (size_t)delta * HD + head * 64 + 32 * wf + l32, acc[r] * p.scale);
  }
}

// ----------------------------------------------------------------------------- dispatch
static inline bool xl_al16(const void* x) { return (reinterpret_cast<uintptr_t>(x) & 15) == 0; }

bool attn_xl_ok(int dtype, const AttnDesc& a) {
  if (dtype != 1 || a.dh != 64 || !a.rel) return false;
  if ((a.ldq | a.ldk | a.ldv | a.ldo | a.ldr) & 7) return false;
  if (!xl_al16(a.q) || !xl_al16(a.k) || !xl_al16(a.v) || !xl_al16(a.o) || !xl_al16(a.r) || !xl_al16(a.u) || !xl_al16(a.vb)) return false;
  if (a.d_o) {
    if ((a.lddo | a.lddq | a.lddk | a.lddv) & 7) return false;
    if (!xl_al16(a.d_o) || !xl_al16(a.dq) || !xl_al16(a.dk) || !xl_al16(a.dv)) return false;
    if ((size_t)a.S * ((a.T + 63) / 64 * 64) * 2 >= ((size_t)1 << 32)) return false;   // 32-bit offsets into P^T, dS^T
  }
  return true;
}

hipError_t launch_attn_fwd_xl(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_xl_fwd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, XL_LDS_Q8);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid((a.T + 127) / 128, a.H, a.B), block(512);
  hipLaunchKernelGGL(fa_xl_fwd_kernel, grid, block, XL_LDS_Q8, s, p);
  return hipGetLastError();
}

// Workspace of the backward pass in floats: two [B, H, S, t_ld] bf16 arrays (see
// fa_xl_dq_kernel) and three [B, t_ld, H * 64] ones.
size_t attn_bwd_xl_scratch_floats(int B, int H, int T, int S) {
  const size_t t_ld = (size_t)(T + 63) / 64 * 64;
  return (2 * (size_t)B * H * S * t_ld + 3 * (size_t)B * t_ld * H * 64) / 2;
}

hipError_t launch_attn_bwd_xl(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_xl_dq_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, XL_LDS_Q8);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int t_ld = (a.T + 63) / 64 * 64, HD = a.H * 64;
  const size_t nmat = (size_t)a.B * a.H * a.S * t_ld, npad = (size_t)a.B * t_ld * HD;
  bf16_t* w = reinterpret_cast<bf16_t*>(a.scratch);
  p.t_ld = t_ld;
  p.pt = w; p.dst = w + nmat;
  p.qu = w + 2 * nmat; p.qv = p.qu + npad; p.dop = p.qv + npad;
  // cells the kernel never writes must read as zero in the contractions below
  if (!a.scratch_clean) {
    hipError_t e = launch_fill_zero(s, w, (2 * nmat + 3 * npad) * 2);
    if (e != hipSuccess) return e;
  }
  // du, dvb and dr are accumulated into (the caller zeroes them)
  hipLaunchKernelGGL(fa_xl_dq_kernel, dim3((a.T + 127) / 128, a.H, a.B), dim3(512), XL_LDS_Q8, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // dV[b, :, h] = P^T dO ; dK[b, :, h] = scale dS^T (Q + u): one product per (head, batch)
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.M = a.S; g.N = 64; g.K = t_ld; g.lda = t_ld; g.ldb = HD; g.transA = 0; g.transB = 0;
  g.by = a.H; g.bz = a.B;
  g.sAy = (long long)a.S * t_ld; g.sAz = (long long)a.H * a.S * t_ld;
  g.sBy = 64; g.sBz = (long long)t_ld * HD;
  g.sCy = 64;
  g.A = p.pt; g.B = p.dop; g.C = a.dv; g.ldc = a.lddv; g.sCz = (long long)a.S * a.lddv; g.alpha = 1.f;
  if (a.lddk == a.lddv) {          // both grids in one launch
    g.A2 = p.dst; g.B2 = p.qu; g.C2 = a.dk; g.alpha2 = a.scale;
    e = launch_gemm(s, 1, g, 0);
    if (e != hipSuccess) return e;
  } else {
    e = launch_gemm(s, 1, g, 0);
    if (e != hipSuccess) return e;
    g.A = p.dst; g.B = p.qu; g.C = a.dk; g.ldc = a.lddk; g.sCz = (long long)a.S * a.lddk; g.alpha = a.scale;
    e = launch_gemm(s, 1, g, 0);
    if (e != hipSuccess) return e;
  }
  // dr += scale sum over (b, i) of dS at distance delta times (q + v): about 768 workgroups
  const int ndb = (a.S + 63) / 64;
  const int bpw = std::max(1, (int)((long long)a.B * ndb * a.H / 768));
  hipLaunchKernelGGL(fa_xl_dr_kernel, dim3(ndb, a.H, (a.B + bpw - 1) / bpw), dim3(256), XL_LDS_DR, s, p, bpw);
  return hipGetLastError();
}

}  // namespace ouro
