// Fused causal attention with the Transformer-XL relative-position term on the matrix cores
// (bf16, head size 64):  score(i, j) = (q_i + u) . k_j + (q_i + v) . r_{Mv + i - j}.
//
// The content term is the plain kernel's product with q + u in place of q.  The position term
// of a 32-query x 64-key block only involves the 95 distances Mv + i - j of the block: the
// product of those rows of r with q + v is one more matrix product, and the element the score
// (i, j) needs sits on the diagonal Mv + i - j of it.  Where a lane owns a query (forward and
// dQ kernels) that diagonal runs through the lane's own column, so the product goes through a
// per-wave LDS patch and comes back shifted; where a lane owns a key (dK/dV kernel) the
// diagonal is a rotation of lanes within a register, done with lane shuffles.  The gradient
// of r takes the same way back.
#include "attention_tiles.h"

namespace ouro {

constexpr int XL_RWIN = 192;                         // rows of r a workgroup needs per block
constexpr int XL_STAGE = 2 * TILE_BYTES + XL_RWIN * 128;   // K, V, r window
constexpr int XL_NSTAGE = 2;
constexpr int XL_PATCH_LD = 33;                      // floats per patch row (32 queries + pad)
constexpr int XL_PATCH = 96 * XL_PATCH_LD * 4;       // bytes per wave
constexpr int XL_LDS_Q = XL_NSTAGE * XL_STAGE + 4 * XL_PATCH;

// Direct load of 64 rows (row index clamped to [0, rmax-1]) x 64 features into an LDS tile.
__device__ __forceinline__ void dma_tile_clamped(const bf16_t* src, int ld, int row0, int rmax, char* tile, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int j = wave * 2 + i;
    const int row = 8 * j + (lane >> 3);
    const int c = (lane & 7) ^ swza(row);
    const int gr = max(0, min(row0 + row, rmax - 1));
    __builtin_amdgcn_global_load_lds((gbl_void*)(src + (size_t)gr * ld + 8 * c), (lds_void*)(tile + j * 1024), 16, 0, 0);
  }
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

// Position term of a block for a wave whose lanes own queries: acc2 = rows [32*wave, +96) of
// the r window times (q + v), written to the wave's patch as patch[rho][query].
__device__ __forceinline__ void xl_position_product(const char* sR, const bf16x8 (&qvf)[4], float* patch, int wave, int lane) {
  const int h32 = lane >> 5, l32 = lane & 31;
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sR, 32 * wave + 32 * t, ks, lane), qvf[ks], acc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) patch[(32 * t + acc_row(r, h32)) * XL_PATCH_LD + l32] = acc[r];
  }
  __builtin_amdgcn_wave_barrier();
}

// ------------------------------------------------------------------------------ forward
// grid (ceil(T/128), H, B); 4 waves x 32 queries; key blocks of 64; one workgroup per CU.
__global__ __launch_bounds__(256) void fa_xl_fwd_kernel(FaParams p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h32 = lane >> 5, l32 = lane & 31;
  const int qblk = gridDim.x - 1 - blockIdx.x;            // longest rows first
  const int head = blockIdx.y, b = blockIdx.z;
  const int Q0 = qblk * 128, q0 = Q0 + wave * 32, qi = q0 + l32;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const bf16_t* rb = p.r + head * 64;
  float* patch = reinterpret_cast<float*>(lds + XL_NSTAGE * XL_STAGE + wave * XL_PATCH);
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
  f32x16 oacc[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % XL_NSTAGE) * XL_STAGE;
    dma_tile(kb, p.ldk, jb * 64, p.S, st, wave, lane);
    dma_tile(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane);
    const int d0 = p.Mv + Q0 - jb * 64 - 63;              // distance of window row 0
#pragma unroll
    for (int t = 0; t < 3; ++t) dma_tile_clamped(rb, p.ldr, d0 + 64 * t, p.S, st + 2 * TILE_BYTES + t * TILE_BYTES, wave, lane);
  };
  issue(0);
  for (int jb = 0; jb < nkb; ++jb) {
    fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (jb + 1 < nkb) issue(jb + 1);
    const char* sK = lds + (jb % XL_NSTAGE) * XL_STAGE;
    const char* sV = sK + TILE_BYTES;
    const char* sR = sK + 2 * TILE_BYTES;
    if (wave_on && jb * 64 <= wave_kmax) {
      const int nkt = (jb * 64 + 32 <= wave_kmax) ? 2 : 1;
      const bool edge = jb * 64 + 63 > p.Mv + q0 || jb * 64 + 63 >= p.S || q0 + 31 >= p.T;
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kt, ks, lane), quf[ks], s[kt], 0, 0, 0);
        }
      }
      // position term: key kk of the block and the lane's query meet at patch row 63 + l32 - kk
      xl_position_product(sR, qvf, patch, wave, lane);
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = 32 * kt + acc_row(r, h32);
            s[kt][r] += patch[(63 + l32 - kk) * XL_PATCH_LD + l32];
          }
        }
      __builtin_amdgcn_wave_barrier();
      float mloc = -INFINITY;
      if (edge) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
          if (kt < nkt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int key = jb * 64 + 32 * kt + acc_row(r, h32);
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


// ---------------------------------------------------------------------------- dQ kernel
// grid (ceil(T/128), H, B); 4 waves x 32 queries; key blocks of 64.  Besides dQ it produces
// the row sums D and the base-2 log-sum-exp for the dK/dV kernel, and the gradients of the
// two biases: du = sum over queries of the content half of dq, dvb = that of the position half.
__global__ __launch_bounds__(256) void fa_xl_dq_kernel(FaParams p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h32 = lane >> 5, l32 = lane & 31;
  const int qblk = gridDim.x - 1 - blockIdx.x;
  const int head = blockIdx.y, b = blockIdx.z;
  const int Q0 = qblk * 128, q0 = Q0 + wave * 32, qi = q0 + l32;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* dob = p.d_o + (size_t)b * p.T * p.lddo + head * 64;
  const bf16_t* ob = p.o + (size_t)b * p.T * p.ldo + head * 64;
  const bf16_t* kb = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vb = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const bf16_t* rb = p.r + head * 64;
  float* patch = reinterpret_cast<float*>(lds + XL_NSTAGE * XL_STAGE + wave * XL_PATCH);
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
    const bf16x8 of = as_bf16x8(t2);
#pragma unroll
    for (int e = 0; e < 8; ++e) part += (float)of[e] * (float)dof[ks][e];
  }
  const float D_q = part + __shfl_xor(part, 32, 64);
  float lse_q = 0.f;
  if (qi < p.T) {
    const size_t rix = ((size_t)b * p.H + head) * p.T + qi;
    lse_q = p.lse[rix] * 1.4426950408889634f;
    if (h32 == 0) { p.D[rix] = D_q; p.lse2[rix] = lse_q; }
  }
  const int wg_last_q = min(p.T, Q0 + 128) - 1;
  const int kend = min(p.S, p.Mv + wg_last_q + 1);
  const int nkb = (kend + 63) / 64;
  const bool wave_on = q0 < p.T;
  const int wave_kmax = p.Mv + min(p.T - 1, q0 + 31);
  f32x16 dqa[2], dqb[2];                                   // content / position halves of dQ^T
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dqa[dt][r] = 0.f; dqb[dt][r] = 0.f; }
  auto issue = [&](int jb) __attribute__((always_inline)) {
    char* st = lds + (jb % XL_NSTAGE) * XL_STAGE;
    dma_tile(kb, p.ldk, jb * 64, p.S, st, wave, lane);
    dma_tile(vb, p.ldv, jb * 64, p.S, st + TILE_BYTES, wave, lane);
    const int d0 = p.Mv + Q0 - jb * 64 - 63;
#pragma unroll
    for (int t = 0; t < 3; ++t) dma_tile_clamped(rb, p.ldr, d0 + 64 * t, p.S, st + 2 * TILE_BYTES + t * TILE_BYTES, wave, lane);
  };
  issue(0);
  for (int jb = 0; jb < nkb; ++jb) {
    fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (jb + 1 < nkb) issue(jb + 1);
    const char* sK = lds + (jb % XL_NSTAGE) * XL_STAGE;
    const char* sV = sK + TILE_BYTES;
    const char* sR = sK + 2 * TILE_BYTES;
    if (wave_on && jb * 64 <= wave_kmax) {
      const int nkt = (jb * 64 + 32 <= wave_kmax) ? 2 : 1;
      const bool edge = jb * 64 + 63 > p.Mv + q0 || jb * 64 + 63 >= p.S || q0 + 31 >= p.T;
      f32x16 s[2], dp[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) { s[kt][r] = 0.f; dp[kt][r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sK, 32 * kt, ks, lane), quf[ks], s[kt], 0, 0, 0);
            dp[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sV, 32 * kt, ks, lane), dof[ks], dp[kt], 0, 0, 0);
          }
        }
      }
      xl_position_product(sR, qvf, patch, wave, lane);
      // dS without its factor `scale`, which the finished gradients take once
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = 32 * kt + acc_row(r, h32);
            const float sc = s[kt][r] + patch[(63 + l32 - kk) * XL_PATCH_LD + l32];
            float pv = __builtin_amdgcn_exp2f(fmaf(sc, p.scale_log2, -lse_q));
            if (edge) {
              const int key = jb * 64 + kk;
              const bool vis = key <= p.Mv + qi && key < p.S && qi < p.T;
              pv = vis ? pv : 0.f;
            }
            dp[kt][r] = pv * (dp[kt][r] - D_q);
          }
        }
      __builtin_amdgcn_wave_barrier();
      // the same diagonal backwards: dS goes into the patch at its distance row
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        if (kt < nkt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = 32 * kt + acc_row(r, h32);
            patch[(63 + l32 - kk) * XL_PATCH_LD + l32] = dp[kt][r];
          }
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int ks2 = 0; ks2 < 4; ++ks2) {
        const int kt = ks2 >> 1, sub = ks2 & 1;
        if (kt < nkt) {
          bf16x8 dsb = pack_acc(dp[kt], sub);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
            dqa[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sK, 32 * dt, 32 * kt + 16 * sub, lane), dsb, dqa[dt], 0, 0, 0);
        }
      }
      // rows of the patch that hold a gradient: 0 <= 63 + l32 - rho < 32 * nkt
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        f32x16 g;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rho = 32 * t + acc_row(r, h32);
          const int kk = 63 + l32 - rho;
          const float v = patch[rho * XL_PATCH_LD + l32];
          g[r] = (kk >= 0 && kk < 32 * nkt) ? v : 0.f;
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          bf16x8 gb = pack_acc(g, sub);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
            dqb[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sR, 32 * dt, 32 * wave + 32 * t + 16 * sub, lane), gb, dqb[dt], 0, 0, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  if (qi < p.T) {
    f32x16 sum[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[dt][r] = dqa[dt][r] + dqb[dt][r];
    store_acc_row(p.dq + ((size_t)b * p.T + qi) * p.lddq + head * 64, sum, p.scale, h32);
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
}


// ------------------------------------------------------------------------ dK, dV, dr kernel
// grid (ceil(S/128), H, B); 4 waves x 32 keys (a lane owns a key); query blocks of 64.
// Scores are queries (registers) x keys (lanes).  The position product q . r_delta is computed
// as queries x distances (lanes); the score (i, j) takes the element of row i at distance
// lane 31 + a - l32 (a = i mod 32, l32 = the key's lane), i.e. a rotation of lanes within the
// register, split over two 32-wide distance tiles.  v . r_delta is a per-distance-lane scalar
// added before the rotation; u . k_j a per-key scalar.  dS goes the same way back into the
// distance layout; dr (distances x features, so that lanes run along features) is added
// atomically to the fp32 table: the window of distances moves with every query block.
constexpr int XL_KV_STAGE = 2 * TILE_BYTES + 1024 + XL_RWIN * 128;   // Q, dO, lse2/D lines, r window
constexpr int XL_LDS_KV = XL_NSTAGE * XL_KV_STAGE;

__device__ __forceinline__ bf16x8 add_scalar(bf16x8 q, float c) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)((float)q[e] + c);
  return r;
}

__global__ __launch_bounds__(256) void fa_xl_dkv_kernel(FaParams p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h32 = lane >> 5, l32 = lane & 31;
  const int kblk = blockIdx.x;                            // key block 0 sees every query: longest first
  const int head = blockIdx.y, b = blockIdx.z;
  const int K0 = kblk * 128, kb0 = K0 + wave * 32, key = kb0 + l32;
  const int HD = p.H * 64;
  const bf16_t* qb = p.q + (size_t)b * p.T * p.ldq + head * 64;
  const bf16_t* dob = p.d_o + (size_t)b * p.T * p.lddo + head * 64;
  const bf16_t* kbp = p.k + (size_t)b * p.S * p.ldk + head * 64;
  const bf16_t* vbp = p.v + (size_t)b * p.S * p.ldv + head * 64;
  const bf16_t* rb = p.r + head * 64;
  const float* lseb = p.lse2 + ((size_t)b * p.H + head) * p.T;
  const float* Db = p.D + ((size_t)b * p.H + head) * p.T;
  bf16x8 kf[4], vf[4];
  float uk = 0.f;                                          // u . k_j, this lane's half of the features
  float vbl[4][8];                                         // v bias at the lane's fragment features
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 t0 = make_uint4(0, 0, 0, 0), t1 = t0;
    if (key < p.S) {
      t0 = *reinterpret_cast<const uint4*>(kbp + (size_t)key * p.ldk + 16 * ks + 8 * h32);
      t1 = *reinterpret_cast<const uint4*>(vbp + (size_t)key * p.ldv + 16 * ks + 8 * h32);
    }
    kf[ks] = as_bf16x8(t0);
    vf[ks] = as_bf16x8(t1);
    const bf16x8 uf = as_bf16x8(*reinterpret_cast<const uint4*>(p.u + head * 64 + 16 * ks + 8 * h32));
    const bf16x8 vbf = as_bf16x8(*reinterpret_cast<const uint4*>(p.vb + head * 64 + 16 * ks + 8 * h32));
#pragma unroll
    for (int e = 0; e < 8; ++e) { uk += (float)kf[ks][e] * (float)uf[e]; vbl[ks][e] = (float)vbf[e]; }
  }
  uk += __shfl_xor(uk, 32, 64);
  // v bias at the features this lane owns as an operand column (feature = 32 dt + l32)
  const float v_f[2] = {(float)p.vb[head * 64 + l32], (float)p.vb[head * 64 + 32 + l32]};
  f32x16 dkT[2], dvT[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkT[dt][r] = 0.f; dvT[dt][r] = 0.f; }
  float tsum = 0.f;                                        // sum over queries of dS(i, key), this half's rows
  f32x16 carry[2];                                         // dr tile that the next query block continues
  bool have_carry = false;
  const int ib0 = max(0, K0 - p.Mv) / 64;
  const int nib = (p.T + 63) / 64;
  const int nit = nib - ib0;
  const bool wave_on = kb0 < p.S;
  auto issue = [&](int it) __attribute__((always_inline)) {
    char* st = lds + (it % XL_NSTAGE) * XL_KV_STAGE;
    const int i0 = (ib0 + it) * 64;
    dma_tile(qb, p.ldq, i0, p.T, st, wave, lane);
    dma_tile(dob, p.lddo, i0, p.T, st + TILE_BYTES, wave, lane);
    dma_floats((wave & 1) ? Db : lseb, i0, p.T, st + 2 * TILE_BYTES + wave * 256, lane);
    const int d0 = p.Mv + i0 - K0 - 127;                   // distance of window row 0
#pragma unroll
    for (int t = 0; t < 3; ++t)
      dma_tile_clamped(rb, p.ldr, d0 + 64 * t, p.S, st + 2 * TILE_BYTES + 1024 + t * TILE_BYTES, wave, lane);
  };
  issue(0);
  for (int it = 0; it < nit; ++it) {
    fa_wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (it + 1 < nit) issue(it + 1);
    const int ib = ib0 + it;
    const char* sQ = lds + (it % XL_NSTAGE) * XL_KV_STAGE;
    const char* sdO = sQ + TILE_BYTES;
    const float* sl = reinterpret_cast<const float*>(sQ + 2 * TILE_BYTES);
    const float* sD = sl + 64;
    const char* sR = sQ + 2 * TILE_BYTES + 1024;
    const int wrow = 96 - 32 * wave;                       // the wave's 96 window rows start here
    const int dmin = p.Mv + ib * 64 - kb0 - 31;            // distance of the wave's window row 0
    if (wave_on && p.Mv + ib * 64 + 63 >= kb0) {
      const int qt0 = (p.Mv + ib * 64 + 31 >= kb0) ? 0 : 1;
      const bool edge = kb0 + 31 > p.Mv + ib * 64 || ib * 64 + 63 >= p.T || kb0 + 31 >= p.S;
      // distance fragments (lane = distance) and v . r_delta
      bf16x8 rf[3][4];
      float vr[3];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        float a = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          rf[t][ks] = read_rows(sR, wrow + 32 * t, ks, lane);
#pragma unroll
          for (int e = 0; e < 8; ++e) a += (float)rf[t][ks][e] * vbl[ks][e];
        }
        vr[t] = a + __shfl_xor(a, 32, 64);
      }
      f32x16 s[2], dp[2];
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        if (qt >= qt0) {
          f32x16 pos[2];
          bf16x8 qa[4];
#pragma unroll
          for (int r = 0; r < 16; ++r) { s[qt][r] = 0.f; dp[qt][r] = 0.f; pos[0][r] = 0.f; pos[1][r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            qa[ks] = read_rows(sQ, 32 * qt, ks, lane);
            s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], kf[ks], s[qt], 0, 0, 0);
            dp[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows(sdO, 32 * qt, ks, lane), vf[ks], dp[qt], 0, 0, 0);
            pos[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], rf[qt][ks], pos[0], 0, 0, 0);
            pos[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], rf[qt + 1][ks], pos[1], 0, 0, 0);
          }
          // rotate the position term into the key lanes and finish the score
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int a = acc_row(r, h32);
            const float x0 = pos[0][r] + vr[qt], x1 = pos[1][r] + vr[qt + 1];
            const float g0 = __shfl(x0, 32 * h32 + ((a + 31 - l32) & 31), 64);
            const float g1 = __shfl(x1, 32 * h32 + ((a - 1 - l32) & 31), 64);
            s[qt][r] += uk + (l32 >= a ? g0 : g1);
          }
        }
      }
      // P = exp2(s * scale * log2 e - lse2); dS = P (dP - D), without its factor `scale`
#pragma unroll
      for (int qt = 0; qt < 2; ++qt)
        if (qt >= qt0) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int ql0 = 32 * qt + 8 * g + 4 * h32;
            const float4 l4 = *reinterpret_cast<const float4*>(sl + ql0);
            const float4 d4 = *reinterpret_cast<const float4*>(sD + ql0);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int r = 4 * g + j;
              float pv = __builtin_amdgcn_exp2f(fmaf(s[qt][r], p.scale_log2, -lv[j]));
              if (edge) {
                const int qi = ib * 64 + ql0 + j;
                const bool vis = key <= p.Mv + qi && qi < p.T && key < p.S;
                pv = vis ? pv : 0.f;
              }
              s[qt][r] = pv;
              dp[qt][r] = pv * (dp[qt][r] - dv4[j]);
              tsum += dp[qt][r];
            }
          }
        }
#pragma unroll
      for (int ks2 = 0; ks2 < 4; ++ks2) {
        const int qt = ks2 >> 1, sub = ks2 & 1;
        if (qt >= qt0) {
          bf16x8 pb = pack_acc(s[qt], sub);
          bf16x8 dsb = pack_acc(dp[qt], sub);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) {
            dvT[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sdO, 32 * dt, 32 * qt + 16 * sub, lane), pb, dvT[dt], 0, 0, 0);
            dkT[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_rows_t(sQ, 32 * dt, 32 * qt + 16 * sub, lane), dsb, dkT[dt], 0, 0, 0);
          }
        }
      }
      // dS back into the distance layout (same rotation reversed), then dr = dS_delta^T (q + v).
      // The window moves up by 64 distances per query block, so this block's tile 2 is the
      // next block's tile 0: it stays in registers and only tiles 0 and 1 go to memory.
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        f32x16 dr[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) dr[dt][r] = (t == 0 && have_carry) ? carry[dt][r] : 0.f;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const int qt = t - tt;                           // query tile whose rotation lands in tile t
          if (qt >= 0 && qt < 2 && qt >= qt0) {
            f32x16 g;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int a = acc_row(r, h32);
              const int src = tt == 0 ? a + 31 - l32 : a - 1 - l32;     // key lane that holds dS(i, delta)
              const float v = __shfl(dp[qt][r], 32 * h32 + (src & 31), 64);
              g[r] = (src >= 0 && src < 32) ? v : 0.f;
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
              bf16x8 gb = pack_acc(g, sub);
#pragma unroll
              for (int dt = 0; dt < 2; ++dt) {
                bf16x8 qT = add_scalar(read_rows_t(sQ, 32 * dt, 32 * qt + 16 * sub, lane), v_f[dt]);
                dr[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gb, qT, dr[dt], 0, 0, 0);
              }
            }
          }
        }
        if (t == 2 && it + 1 < nit) {
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) carry[dt] = dr[dt];
        } else {
          // rows = distances dmin + 32 t + acc_row, lanes = features 32 dt + l32
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int delta = dmin + 32 * t + acc_row(r, h32);
              if (delta >= 0 && delta < p.S) unsafeAtomicAdd(p.dr + (size_t)delta * HD + head * 64 + 32 * dt + l32, dr[dt][r] * p.scale);
            }
        }
      }
      have_carry = it + 1 < nit;
    }
  }
  if (key < p.S) {
    // dk = sum_i dS(i, key) (q_i + u): the u part from the per-key sum of dS
    const float tj = tsum + __shfl_xor(tsum, 32, 64);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float uf = (float)p.u[head * 64 + 32 * dt + acc_row(r, h32)];
        dkT[dt][r] += uf * tj;
      }
    store_acc_row(p.dk + ((size_t)b * p.S + key) * p.lddk + head * 64, dkT, p.scale, h32);
    store_acc_row(p.dv + ((size_t)b * p.S + key) * p.lddv + head * 64, dvT, 1.f, h32);
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
  }
  return true;
}

hipError_t launch_attn_fwd_xl(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_xl_fwd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, XL_LDS_Q);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid((a.T + 127) / 128, a.H, a.B), block(256);
  hipLaunchKernelGGL(fa_xl_fwd_kernel, grid, block, XL_LDS_Q, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_xl(hipStream_t s, const AttnDesc& a) {
  FaParams p = fa_params(a);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_xl_dq_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, XL_LDS_Q);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(fa_xl_dkv_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, XL_LDS_KV);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // du, dvb and dr are accumulated into (the caller zeroes them)
  hipLaunchKernelGGL(fa_xl_dq_kernel, dim3((a.T + 127) / 128, a.H, a.B), dim3(256), XL_LDS_Q, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fa_xl_dkv_kernel, dim3((a.S + 127) / 128, a.H, a.B), dim3(256), XL_LDS_KV, s, p);
  return hipGetLastError();
}

}  // namespace ouro
