// Parameters and epilogues shared by the contraction kernels.
#pragma once
#include "common.h"
#include "tiles.h"

namespace ouro {

struct GemmParams {
  const void* A; const void* B; void* C;
  int M, N, K, lda, ldb, ldc;
  int out_fp32, accumulate;
  const float* bias;
  const void* residual; int ldr;
  const float* res32; int ldr32;
  const float* ln_mean; const float* ln_rstd; const float* ln_g; const float* ln_b;
  int epilogue;
  void* Z; int ldz;
  float alpha;
  int kchunk;      // K range per blockIdx.z
  int tilesN;      // tiles along N (MFMA kernel)
  int tilesM, ntiles, mfast, band;   // direct-to-LDS kernels: see tile_of_block
  int vec_epi;     // 1: C, Z, residual allow 16-byte row-chunk accesses (MFMA kernel)
  int by, bz, bz1;                          // bz1: blockIdx.z from here on belongs to the second grid of products
  const void* A2; const void* B2; void* C2; float alpha2;
  long long bAy, bAz, bBy, bBz, bCy, bCz;   // byte strides of a batch of products over blockIdx.y, blockIdx.z (direct-to-LDS kernels)
  DropDesc drop;
};

template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmParams& p, int m, int n, float acc) {
  float v = acc * p.alpha;
  if (p.accumulate) {
    unsafeAtomicAdd(reinterpret_cast<float*>(p.C) + (size_t)m * p.ldc + n, v);
    return;
  }
  if (p.bias) v += p.bias[n];
  if (p.drop.on) v *= drop_factor(p.drop, (uint64_t)m * p.drop.ld + n);
  if (p.epilogue == EPI_GELU) {
    reinterpret_cast<T*>(p.Z)[(size_t)m * p.ldz + n] = from_f32<T>(v);
    v = gelu_f(v);
  } else if (p.epilogue == EPI_GELUGRAD) {
    v *= gelu_grad_f(to_f32(reinterpret_cast<const T*>(p.Z)[(size_t)m * p.ldz + n]));
  }
  if (p.residual) v += to_f32(reinterpret_cast<const T*>(p.residual)[(size_t)m * p.ldr + n]);
  if (p.res32) {
    float r = p.res32[(size_t)m * p.ldr32 + n];
    if (p.ln_mean) r = (r - p.ln_mean[m]) * p.ln_rstd[m] * p.ln_g[n] + p.ln_b[n];
    v += r;
  }
  if (p.out_fp32) reinterpret_cast<float*>(p.C)[(size_t)m * p.ldc + n] = v;
  else reinterpret_cast<T*>(p.C)[(size_t)m * p.ldc + n] = from_f32<T>(v);
}


// Eight consecutive columns n..n+7 of row m (bf16 operands), all in range and 16-byte
// addressable: the same epilogue as epilogue_store with 16-byte accesses.
__device__ __forceinline__ void epilogue_store8(const GemmParams& p, int m, int n, const float* acc) {
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = acc[e] * p.alpha;
  if (p.bias) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += p.bias[n + e];
  }
  if (p.drop.on) {
    const uint64_t i0 = (uint64_t)m * p.drop.ld + n;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= drop_factor(p.drop, i0 + e);
  }
  if (p.epilogue == EPI_GELU) {
    union { bf16_t h[8]; uint4 u; } z;
#pragma unroll
    for (int e = 0; e < 8; ++e) { z.h[e] = (bf16_t)v[e]; v[e] = gelu_f(v[e]); }
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(p.Z) + (size_t)m * p.ldz + n) = z.u;
  } else if (p.epilogue == EPI_GELUGRAD) {
    union { bf16_t h[8]; uint4 u; } z;
    z.u = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.Z) + (size_t)m * p.ldz + n);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f((float)z.h[e]);
  }
  if (p.residual) {
    union { bf16_t h[8]; uint4 u; } r;
    r.u = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.residual) + (size_t)m * p.ldr + n);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += (float)r.h[e];
  }
  if (p.res32) {
    const float4* rp = reinterpret_cast<const float4*>(p.res32 + (size_t)m * p.ldr32 + n);
    const float4 lo = rp[0], hi = rp[1];
    float r[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    if (p.ln_mean) {
      const float mu = p.ln_mean[m], rs = p.ln_rstd[m];
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = (r[e] - mu) * rs * p.ln_g[n + e] + p.ln_b[n + e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += r[e];
  }
  if (p.out_fp32) {
    float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(p.C) + (size_t)m * p.ldc + n);
    c[0] = make_float4(v[0], v[1], v[2], v[3]);
    c[1] = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    union { bf16_t h[8]; uint4 u; } o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.h[e] = (bf16_t)v[e];
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(p.C) + (size_t)m * p.ldc + n) = o.u;
  }
}

// Floats of LDS each wave needs for the staged epilogue (one row of TN 32x32 tiles).
template <int TN> constexpr int epilogue_stage_floats() { return TN * 32 * 36; }

// Writes a wave's TM x TN accumulator tiles (32x32 each; column = lane%32, row =
// 8*(r/4) + 4*(lane/32) + r%4) through the epilogue.  smem must be free for reuse (all
// waves past their last operand read).  m_w, n_w: first row / column of the wave's tiles.
// Split-K accumulation adds straight from the registers (128 contiguous bytes per
// instruction).  Otherwise each wave turns one row of tiles at a time through a private
// LDS patch (row stride 36 floats) so that a lane leaves with 8 consecutive columns of one
// output row: 16-byte loads of the residual / pre-activation, 16-byte stores of the result.
// Only the register dump is unrolled; the arithmetic runs in a rolled loop over the patch.
template <int TM, int TN>
__device__ __forceinline__ void mfma_epilogue(const GemmParams& p, f32x16 (&acc)[TM][TN], uint4* smem, int m_w, int n_w,
                                              int lane, int wave) {
  if (p.accumulate) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n_w + j * 32 + (lane & 31);
        const int mb = m_w + i * 32 + 4 * (lane >> 5);
        float* c = reinterpret_cast<float*>(p.C) + (size_t)mb * p.ldc + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dm = 8 * (r >> 2) + (r & 3);
          if (n < p.N && mb + dm < p.M) unsafeAtomicAdd(c + (size_t)dm * p.ldc, acc[i][j][r] * p.alpha);
        }
      }
    return;
  }
  float* stage = reinterpret_cast<float*>(smem) + wave * epilogue_stage_floats<TN>();
  const int h32 = lane >> 5, l32 = lane & 31;
  const int srow = lane >> 2, scol = (lane & 3) * 8;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[j * (32 * 36) + (8 * (r >> 2) + 4 * h32 + (r & 3)) * 36 + l32] = acc[i][j][r];
    __builtin_amdgcn_wave_barrier();
#pragma unroll 1
    for (int t = 0; t < 2 * TN; ++t) {
      const int j = t >> 1;
      const int row = (t & 1) * 16 + srow;
      const float* src = stage + j * (32 * 36) + row * 36 + scol;
      const int m = m_w + i * 32 + row;
      const int n = n_w + j * 32 + scol;
      if (m < p.M) {
        if (p.vec_epi && n + 8 <= p.N) {
          float4 lo = *reinterpret_cast<const float4*>(src);
          float4 hi = *reinterpret_cast<const float4*>(src + 4);
          const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          epilogue_store8(p, m, n, v);
        } else {
#pragma unroll 1
          for (int e = 0; e < 8; ++e)
            if (n + e < p.N) epilogue_store<bf16_t>(p, m, n + e, src[e]);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace ouro
