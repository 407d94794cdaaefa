// Bandwidth-bound kernels of the step: LayerNorm forward/backward, column sums (bias and
// LayerNorm parameter gradients), embedding gather / scatter-add, softmax cross-entropy
// rows, conversions, and the delayed SGD / Adam update.
#include "common.h"

#include <algorithm>

namespace ouro {

// 16-byte packs: 4 fp32 or 8 bf16
template <typename T> struct Pack { static constexpr int N = 16 / sizeof(T); };
template <typename T> __device__ __forceinline__ void load_pack(const T* p, float* out);
template <> __device__ __forceinline__ void load_pack<float>(const float* p, float* out) {
  float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <> __device__ __forceinline__ void load_pack<bf16_t>(const bf16_t* p, float* out) {
  uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
template <typename T> __device__ __forceinline__ void store_pack(T* p, const float* in);
template <> __device__ __forceinline__ void store_pack<float>(float* p, const float* in) {
  *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
}
template <> __device__ __forceinline__ void store_pack<bf16_t>(bf16_t* p, const float* in) {
  union { bf16_t h[8]; uint4 v; } u;
#pragma unroll
  for (int i = 0; i < 8; ++i) u.h[i] = (bf16_t)in[i];
  *reinterpret_cast<uint4*>(p) = u.v;
}

// N consecutive elements (N = 4 or 8) in 16-byte accesses: a group of 8 fp32 takes two of them
template <typename T, int N> __device__ __forceinline__ void load_n(const T* p, float* out) {
  if constexpr (sizeof(T) == 4 && N == 8) { load_pack<T>(p, out); load_pack<T>(p + 4, out + 4); }
  else { static_assert(Pack<T>::N == N, "group size"); load_pack<T>(p, out); }
}
template <typename T, int N> __device__ __forceinline__ void store_n(T* p, const float* in) {
  if constexpr (sizeof(T) == 4 && N == 8) { store_pack<T>(p, in); store_pack<T>(p + 4, in + 4); }
  else { static_assert(Pack<T>::N == N, "group size"); store_pack<T>(p, in); }
}
// Elements per lane group of a row kernel whose operands have the types A and B: 8 as soon as one
// of them is bf16 (its 16-byte pack), else 4.
template <typename A, typename B> struct Group { static constexpr int N = (sizeof(A) == 2 || sizeof(B) == 2) ? 8 : 4; };

// ------------------------------------------------------------------------ LayerNorm fwd
// One wavefront per row.  VEC: row held in registers as up to MAXI groups per lane.  TX: type of
// the rows read (the pre-normalisation sums: fp32 in bf16 models), TY: type of the rows written.
template <typename TX, typename TY, int MAXI>
__global__ __launch_bounds__(256) void ln_fwd_vec_kernel(const TX* __restrict__ x, const float* __restrict__ g,
                                                         const float* __restrict__ b, TY* __restrict__ y,
                                                         float* __restrict__ mean, float* __restrict__ rstd,
                                                         int rows, int d, int dn) {
  constexpr int N = Group<TX, TY>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nvec = d / N;
  float v[MAXI][N];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int vi = lane + 64 * i;
    if (vi < nvec) {
      load_n<TX, N>(x + (size_t)row * d + vi * N, v[i]);
#pragma unroll
      for (int e = 0; e < N; ++e) s += v[i][e];
    }
  }
  const float mu = wave_sum(s) / dn;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int vi = lane + 64 * i;
    if (vi < nvec) {
#pragma unroll
      for (int e = 0; e < N; ++e) { float t = v[i][e] - mu; q += vi * N + e < dn ? t * t : 0.f; }
    }
  }
  const float rs = rsqrtf(wave_sum(q) / dn + 1e-5f);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int vi = lane + 64 * i;
    if (vi < nvec) {
      float out[N];
#pragma unroll
      for (int e = 0; e < N; ++e) out[e] = (v[i][e] - mu) * rs * g[vi * N + e] + b[vi * N + e];
      store_n<TY, N>(y + (size_t)row * d + vi * N, out);
    }
  }
}

template <typename TX, typename TY>
__global__ __launch_bounds__(256) void ln_fwd_scalar_kernel(const TX* __restrict__ x, const float* __restrict__ g,
                                                            const float* __restrict__ b, TY* __restrict__ y,
                                                            float* __restrict__ mean, float* __restrict__ rstd,
                                                            int rows, int d, int dn) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const TX* xr = x + (size_t)row * d;
  float s = 0.f;
  for (int c = lane; c < dn; c += 64) s += to_f32(xr[c]);
  const float mu = wave_sum(s) / dn;
  float q = 0.f;
  for (int c = lane; c < dn; c += 64) { float t = to_f32(xr[c]) - mu; q += t * t; }
  const float rs = rsqrtf(wave_sum(q) / dn + 1e-5f);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  for (int c = lane; c < d; c += 64)
    y[(size_t)row * d + c] = from_f32<TY>((to_f32(xr[c]) - mu) * rs * g[c] + b[c]);
}

static inline bool ptr16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// dtype 0: fp32 rows in and out; 1: bf16 in and out; 2: fp32 rows in, bf16 rows out (bf16 models keep the
// sums that enter a LayerNorm in fp32).
hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, const void* x, const float* g, const float* b,
                                void* y, float* mean, float* rstd, int rows, int d, int dn) {
  if (rows <= 0) return hipSuccess;
  if (dn <= 0 || dn > d) dn = d;
  dim3 grid((rows + 3) / 4), block(256);
  const int grp = dtype == 0 ? 4 : 8;
  const bool vec = d % grp == 0 && d / grp <= 256 && ptr16(x) && ptr16(y);
  const int npl = (d / grp + 63) / 64;
#define OURO_LNF(TX_, TY_)                                                                                                                  \
  do {                                                                                                                                      \
    if (!vec) hipLaunchKernelGGL((ln_fwd_scalar_kernel<TX_, TY_>), grid, block, 0, s, (const TX_*)x, g, b, (TY_*)y, mean, rstd, rows, d, dn); \
    else if (npl <= 1) hipLaunchKernelGGL((ln_fwd_vec_kernel<TX_, TY_, 1>), grid, block, 0, s, (const TX_*)x, g, b, (TY_*)y, mean, rstd, rows, d, dn); \
    else if (npl <= 2) hipLaunchKernelGGL((ln_fwd_vec_kernel<TX_, TY_, 2>), grid, block, 0, s, (const TX_*)x, g, b, (TY_*)y, mean, rstd, rows, d, dn); \
    else hipLaunchKernelGGL((ln_fwd_vec_kernel<TX_, TY_, 4>), grid, block, 0, s, (const TX_*)x, g, b, (TY_*)y, mean, rstd, rows, d, dn);  \
  } while (0)
  if (dtype == 1) OURO_LNF(bf16_t, bf16_t);
  else if (dtype == 2) OURO_LNF(float, bf16_t);
  else OURO_LNF(float, float);
#undef OURO_LNF
  return hipGetLastError();
}

// ------------------------------------------------------------------------ LayerNorm bwd
// dx = rstd * (dyg - mean(dyg) - xhat * mean(dyg * xhat)), dyg = dy * g
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void ln_bwd_dx_kernel(const TI* __restrict__ dy, const TI* __restrict__ x,
                                                        const float* __restrict__ g, const float* __restrict__ mean,
                                                        const float* __restrict__ rstd, TO* __restrict__ dx,
                                                        int rows, int d, int dn) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const TI* xr = x + (size_t)row * d;
  const TI* dyr = dy + (size_t)row * d;
  const float mu = mean[row], rs = rstd[row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < d; c += 64) {
    float xh = (to_f32(xr[c]) - mu) * rs;
    float t = to_f32(dyr[c]) * g[c];
    s1 += t;
    s2 += t * xh;
  }
  s1 = wave_sum(s1) / dn;
  s2 = wave_sum(s2) / dn;
  for (int c = lane; c < d; c += 64) {
    float xh = (to_f32(xr[c]) - mu) * rs;
    float t = to_f32(dyr[c]) * g[c];
    dx[(size_t)row * d + c] = from_f32<TO>(c < dn ? rs * (t - s1 - xh * s2) : 0.f);
  }
}

// Column sums over a chunk of rows; 64 columns x 4 row lanes per block, then atomics.
// MODE 0: out0[c] += sum x[r,c].  MODE 1 (LayerNorm): out0[c] += sum dy*xhat, out1[c] += sum dy.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, int ldx, const T* __restrict__ x2,
                                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                                     float* __restrict__ out0, float* __restrict__ out1,
                                                     int rows, int cols, int rows_per_block) {
  __shared__ float red0[4][64];
  __shared__ float red1[4][64];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cx;
  const int rbeg = blockIdx.y * rows_per_block;
  const int rend = min(rows, rbeg + rows_per_block);
  float a0 = 0.f, a1 = 0.f;
  if (c < cols) {
    for (int r = rbeg + ry; r < rend; r += 4) {
      float v = to_f32(x[(size_t)r * ldx + c]);
      if (MODE == 0) {
        a0 += v;
      } else {
        float xh = (to_f32(x2[(size_t)r * ldx + c]) - mean[r]) * rstd[r];
        a0 += v * xh;
        a1 += v;
      }
    }
  }
  red0[ry][cx] = a0;
  red1[ry][cx] = a1;
  __syncthreads();
  if (ry == 0 && c < cols) {
    float t0 = red0[0][cx] + red0[1][cx] + red0[2][cx] + red0[3][cx];
    unsafeAtomicAdd(out0 + c, t0);
    if (MODE == 1) {
      float t1 = red1[0][cx] + red1[1][cx] + red1[2][cx] + red1[3][cx];
      unsafeAtomicAdd(out1 + c, t1);
    }
  }
}

// Vector path of the LayerNorm backward: one wavefront per row, rows strided over the grid;
// the row's packs stay in registers, dg / db partial sums are kept per lane over all the
// wave's rows, reduced over the block's four waves through LDS and added atomically once.
template <typename TI, typename TO, int MAXI, bool PARAMS>
__global__ __launch_bounds__(256) void ln_bwd_fused_kernel(const TI* __restrict__ dy, const TI* __restrict__ x,
                                                           const float* __restrict__ g, const float* __restrict__ mean,
                                                           const float* __restrict__ rstd, TO* __restrict__ dx,
                                                           float* __restrict__ dg, float* __restrict__ db, int rows, int d,
                                                           int dn, size_t copy_stride) {
  constexpr int N = Group<TI, TO>::N;
  extern __shared__ float red[];                 // [4][d]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nvec = d / N;
  float gl[MAXI][N], ag[MAXI][N], ab[MAXI][N];
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    int vi = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < N; ++e) {
      gl[i][e] = vi < nvec ? g[vi * N + e] : 0.f;
      ag[i][e] = 0.f;
      ab[i][e] = 0.f;
    }
  }
  // two rows per trip: their loads are issued together so one row's latency hides the other's
  const int rstep = gridDim.x * 4;
  for (int row0 = blockIdx.x * 4 + wave; row0 < rows; row0 += 2 * rstep) {
    float xh[2][MAXI][N], t[2][MAXI][N], mu[2], rs[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = row0 + u * rstep;
      if (row < rows) {
        mu[u] = mean[row]; rs[u] = rstd[row];
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
          int vi = lane + 64 * i;
          if (vi < nvec) {
            load_n<TI, N>(x + (size_t)row * d + vi * N, xh[u][i]);
            load_n<TI, N>(dy + (size_t)row * d + vi * N, t[u][i]);
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = row0 + u * rstep;
      if (row >= rows) continue;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        int vi = lane + 64 * i;
        if (vi < nvec) {
#pragma unroll
          for (int e = 0; e < N; ++e) {
            xh[u][i][e] = (xh[u][i][e] - mu[u]) * rs[u];
            if (PARAMS) {
              ag[i][e] += t[u][i][e] * xh[u][i][e];
              ab[i][e] += t[u][i][e];
            }
            t[u][i][e] *= gl[i][e];
            s1 += t[u][i][e];
            s2 += t[u][i][e] * xh[u][i][e];
          }
        }
      }
      s1 = wave_sum(s1) / dn;
      s2 = wave_sum(s2) / dn;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        int vi = lane + 64 * i;
        if (vi < nvec) {
          float out[N];
#pragma unroll
          for (int e = 0; e < N; ++e) out[e] = vi * N + e < dn ? rs[u] * (t[u][i][e] - s1 - xh[u][i][e] * s2) : 0.f;
          store_n<TO, N>(dx + (size_t)row * d + vi * N, out);
        }
      }
    }
  }
  if (!PARAMS) return;
  // every block adds d sums to the same d addresses; with copy_stride the adds of the blocks of
  // one XCD (blocks are dealt to the 8 XCDs in launch order) go to that XCD's own copy
  dg += (blockIdx.x & 7) * copy_stride;
  db += (blockIdx.x & 7) * copy_stride;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      int vi = lane + 64 * i;
      if (vi < nvec) {
#pragma unroll
        for (int e = 0; e < N; ++e) red[wave * d + vi * N + e] = pass ? ab[i][e] : ag[i][e];
      }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += 256)
      unsafeAtomicAdd((pass ? db : dg) + c, red[c] + red[d + c] + red[2 * d + c] + red[3 * d + c]);
    __syncthreads();
  }
}

// Vector column sum: a wave covers 64 packs of one row (1 KiB), the block's four waves take
// alternate rows; partial sums are reduced through LDS and added atomically.
template <typename T>
__global__ __launch_bounds__(256) void colsum_vec_kernel(const T* __restrict__ x, int ldx, float* __restrict__ out,
                                                         int rows, int rows_per_block, size_t copy_stride) {
  constexpr int N = Pack<T>::N;
  __shared__ float red[4][64 * N];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 64 + lane) * N;
  const int rbeg = blockIdx.y * rows_per_block;
  const int rend = min(rows, rbeg + rows_per_block);
  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;
  for (int r = rbeg + wave; r < rend; r += 4) {
    float v[N];
    load_pack<T>(x + (size_t)r * ldx + c0, v);
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < N; ++e) red[wave][lane * N + e] = acc[e];
  __syncthreads();
  out += ((blockIdx.x + gridDim.x * blockIdx.y) & 7) * copy_stride;     // the XCD's own copy (see ln_bwd_fused_kernel)
  for (int c = threadIdx.x; c < 64 * N; c += 256)
    unsafeAtomicAdd(out + blockIdx.x * 64 * N + c, red[0][c] + red[1][c] + red[2][c] + red[3][c]);
}

// Scale and shift gradients of LayerNorm as column sums: dg[c] += sum_r dy*xhat, db[c] += sum_r dy.
// A wave covers 64 packs of one row, the block's sixteen waves take alternate rows; the partial
// sums meet in LDS and leave as one atomic per column and block.  Adds to one address complete
// one after the other, so the grid has few, large blocks.
template <typename T, int N>
__global__ __launch_bounds__(1024) void ln_param_vec_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            float* __restrict__ dg, float* __restrict__ db, int rows, int d,
                                                            int rows_per_block) {
  constexpr int NWV = 16;
  extern __shared__ float red[];                 // [2][NWV][64 * N]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 64 + lane) * N;
  const bool live = c0 < d;
  const int rbeg = blockIdx.y * rows_per_block;
  const int rend = min(rows, rbeg + rows_per_block);
  float a0[N], a1[N];
#pragma unroll
  for (int e = 0; e < N; ++e) a0[e] = a1[e] = 0.f;
  if (live) {
    for (int r = rbeg + wave; r < rend; r += NWV) {
      float v[N], xv[N];
      load_n<T, N>(dy + (size_t)r * d + c0, v);
      load_n<T, N>(x + (size_t)r * d + c0, xv);
      const float mu = mean[r], rs = rstd[r];
#pragma unroll
      for (int e = 0; e < N; ++e) {
        a0[e] += v[e] * ((xv[e] - mu) * rs);
        a1[e] += v[e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < N; ++e) {
    red[(0 * NWV + wave) * 64 * N + lane * N + e] = a0[e];
    red[(1 * NWV + wave) * 64 * N + lane * N + e] = a1[e];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * 64 * N; c += 1024) {
    const int which = c / (64 * N), cc = c % (64 * N);
    const int col = blockIdx.x * 64 * N + cc;
    if (col < d) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < NWV; ++w) t += red[(which * NWV + w) * 64 * N + cc];
      unsafeAtomicAdd((which ? db : dg) + col, t);
    }
  }
}

static bool ln_vec_ok(int dtype, const void* dy, const void* x, int d) {
  const int grp = dtype == 0 ? 4 : 8;
  return d % grp == 0 && d / grp <= 256 && ptr16(dy) && ptr16(x);
}

// dtype 0: fp32 throughout; 1: bf16 throughout; 2: dy and x fp32, dx bf16 (bf16 models keep the
// gradients and sums on the normalised path in fp32).
// dg == nullptr: input gradient only (the parameter gradients then come from
// launch_layernorm_bwd_params, on any stream that sees dy and x).  fuse_params: dg and db (which
// must be zero or hold what is to be added to) are produced by the same kernel that writes dx.
// copy_stride: dg and db are the first of 8 copies that far apart (floats); a kernel that adds
// from many blocks spreads its adds over them by XCD and the caller sums the copies (0: one copy).
hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, const void* dy, const void* x, const float* g,
                                const float* mean, const float* rstd, void* dx, float* dg, float* db,
                                int rows, int d, int dn, bool fuse_params, size_t copy_stride) {
  if (rows <= 0) return hipSuccess;
  if (dn <= 0 || dn > d) dn = d;
  dim3 grid((rows + 3) / 4), block(256);
  bool fused = false;
  if (ln_vec_ok(dtype, dy, x, d) && ptr16(dx)) {
    const int grp = dtype == 0 ? 4 : 8;
    dim3 gf(std::min((rows + 3) / 4, 384));   // every block ends with 2 d atomic adds: 384 blocks measured best in the step (256, 512: +0.5 %)
    const int npl = (d / grp + 63) / 64;      // groups per lane
    fused = fuse_params && dg && db;
    const size_t smem = fused ? (size_t)4 * d * sizeof(float) : 0;
#define OURO_LNB2(TI_, TO_, MI_, PAR_) hipLaunchKernelGGL((ln_bwd_fused_kernel<TI_, TO_, MI_, PAR_>), gf, block, smem, s, (const TI_*)dy, (const TI_*)x, g, mean, rstd, (TO_*)dx, dg, db, rows, d, dn, copy_stride)
#define OURO_LNB(TI_, TO_)                                                                  \
  do {                                                                                      \
    if (fused) { if (npl <= 1) OURO_LNB2(TI_, TO_, 1, true); else if (npl <= 2) OURO_LNB2(TI_, TO_, 2, true); else OURO_LNB2(TI_, TO_, 4, true); } \
    else { if (npl <= 1) OURO_LNB2(TI_, TO_, 1, false); else if (npl <= 2) OURO_LNB2(TI_, TO_, 2, false); else OURO_LNB2(TI_, TO_, 4, false); }  \
  } while (0)
    if (dtype == 1) OURO_LNB(bf16_t, bf16_t);
    else if (dtype == 2) OURO_LNB(float, bf16_t);
    else OURO_LNB(float, float);
#undef OURO_LNB
#undef OURO_LNB2
  } else if (dtype == 1) {
    hipLaunchKernelGGL((ln_bwd_dx_kernel<bf16_t, bf16_t>), grid, block, 0, s, (const bf16_t*)dy, (const bf16_t*)x, g, mean, rstd, (bf16_t*)dx, rows, d, dn);
  } else if (dtype == 2) {
    hipLaunchKernelGGL((ln_bwd_dx_kernel<float, bf16_t>), grid, block, 0, s, (const float*)dy, (const float*)x, g, mean, rstd, (bf16_t*)dx, rows, d, dn);
  } else {
    hipLaunchKernelGGL((ln_bwd_dx_kernel<float, float>), grid, block, 0, s, (const float*)dy, (const float*)x, g, mean, rstd, (float*)dx, rows, d, dn);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !dg || fused) return e;
  return launch_layernorm_bwd_params(s, dtype, dy, x, mean, rstd, dg, db, rows, d);
}

// dtype as above (2: dy and x are fp32).
hipError_t launch_layernorm_bwd_params(hipStream_t s, int dtype, const void* dy, const void* x, const float* mean,
                                       const float* rstd, float* dg, float* db, int rows, int d) {
  if (rows <= 0) return hipSuccess;
  dim3 block(256);
  if (ln_vec_ok(dtype, dy, x, d)) {
    const int grp = dtype == 0 ? 4 : 8;
    const int gx = (d + 64 * grp - 1) / (64 * grp);
    const int rpb = 64;                          // four rows per wave
    dim3 grid(gx, (rows + rpb - 1) / rpb), blk(1024);
    const size_t smem = 2 * 16 * 64 * (size_t)grp * sizeof(float);
    if (dtype == 1) hipLaunchKernelGGL((ln_param_vec_kernel<bf16_t, 8>), grid, blk, smem, s, (const bf16_t*)dy, (const bf16_t*)x, mean, rstd, dg, db, rows, d, rpb);
    else if (dtype == 2) hipLaunchKernelGGL((ln_param_vec_kernel<float, 8>), grid, blk, smem, s, (const float*)dy, (const float*)x, mean, rstd, dg, db, rows, d, rpb);
    else hipLaunchKernelGGL((ln_param_vec_kernel<float, 4>), grid, blk, smem, s, (const float*)dy, (const float*)x, mean, rstd, dg, db, rows, d, rpb);
    return hipGetLastError();
  }
  const int rpb = 128;
  dim3 g2((d + 63) / 64, (rows + rpb - 1) / rpb);
  if (dtype == 1)
    hipLaunchKernelGGL((colsum_kernel<bf16_t, 1>), g2, block, 0, s, (const bf16_t*)dy, d, (const bf16_t*)x, mean, rstd, dg, db, rows, d, rpb);
  else
    hipLaunchKernelGGL((colsum_kernel<float, 1>), g2, block, 0, s, (const float*)dy, d, (const float*)x, mean, rstd, dg, db, rows, d, rpb);
  return hipGetLastError();
}

// One block per segment: sums the 8 copies, zeroes them, adds the sum to its place in dst.
__global__ __launch_bounds__(256) void sum_segments_kernel(const SumSegment* __restrict__ table, float* __restrict__ src,
                                                           size_t stride, float* __restrict__ dst) {
  const SumSegment sg = table[blockIdx.x];
  if (threadIdx.x >= sg.len) return;
  float t = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    float* p = src + c * stride + sg.src_off + threadIdx.x;
    t += *p;
    *p = 0.f;
  }
  dst[sg.dst_off + threadIdx.x] += t;
}
hipError_t launch_sum_segments(hipStream_t s, const SumSegment* table, int count, float* src, size_t stride, float* dst) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(sum_segments_kernel, dim3(count), dim3(256), 0, s, table, src, stride, dst);
  return hipGetLastError();
}

hipError_t launch_colsum(hipStream_t s, int dtype, const void* x, int ldx, float* out, int rows, int cols, size_t copy_stride) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  dim3 block(256);
  const int pack = dtype == 1 ? 8 : 4;
  if (cols % (64 * pack) == 0 && ldx % pack == 0 && ptr16(x)) {
    const int rpb = 64;
    dim3 grid(cols / (64 * pack), (rows + rpb - 1) / rpb);
    if (dtype == 1) hipLaunchKernelGGL(colsum_vec_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)x, ldx, out, rows, rpb, copy_stride);
    else hipLaunchKernelGGL(colsum_vec_kernel<float>, grid, block, 0, s, (const float*)x, ldx, out, rows, rpb, copy_stride);
    return hipGetLastError();
  }
  const int rpb = 128;
  dim3 grid((cols + 63) / 64, (rows + rpb - 1) / rpb);
  if (dtype == 1)
    hipLaunchKernelGGL((colsum_kernel<bf16_t, 0>), grid, block, 0, s, (const bf16_t*)x, ldx, (const bf16_t*)nullptr, nullptr, nullptr, out, nullptr, rows, cols, rpb);
  else
    hipLaunchKernelGGL((colsum_kernel<float, 0>), grid, block, 0, s, (const float*)x, ldx, (const float*)nullptr, nullptr, nullptr, out, nullptr, rows, cols, rpb);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- embedding
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ V,
                                                        const float* __restrict__ pe, T* __restrict__ h, int N, int T_,
                                                        int d, int vocab, float scale, int* flag, DropDesc drop) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const int id = tok[n];
  const bool ok = id >= 0 && id < vocab;
  if (!ok && lane == 0) atomicOr(flag, 1);
  const T* row = V + (size_t)(ok ? id : 0) * d;
  const float* per = pe ? pe + (size_t)(n % T_) * d : nullptr;
  for (int c = lane; c < d; c += 64) {
    float v = ok ? scale * to_f32(row[c]) : 0.f;
    if (per) v += per[c];
    if (drop.on) v *= drop_factor(drop, (uint64_t)n * drop.ld + c);
    h[(size_t)n * d + c] = from_f32<T>(v);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dh,
                                                        float* __restrict__ dVi, int N, int d, int vocab, float scale,
                                                        DropDesc drop) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const int id = tok[n];
  if (id < 0 || id >= vocab) return;
  for (int c = lane; c < d; c += 64) {
    float g = scale * to_f32(dh[(size_t)n * d + c]);
    if (drop.on) g *= drop_factor(drop, (uint64_t)n * drop.ld + c);
    unsafeAtomicAdd(dVi + (size_t)id * d + c, g);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void dropout_apply_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows,
                                                            int cols, int ld, DropDesc drop) {
  const size_t total = (size_t)rows * cols;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / cols, c = i % cols;
    dst[r * ld + c] = from_f32<T>(to_f32(src[r * ld + c]) * drop_factor(drop, (uint64_t)r * drop.ld + c));
  }
}

hipError_t launch_embed_fwd(hipStream_t s, int dtype, const int32_t* tok, const void* V, const float* pe,
                            void* h, int N, int T, int d, int vocab, float scale, int* flag, const DropDesc* drop) {
  dim3 grid((N + 3) / 4), block(256);
  DropDesc dd;
  memset(&dd, 0, sizeof dd);
  if (drop) dd = *drop;
  if (dtype == 1) hipLaunchKernelGGL(embed_fwd_kernel<bf16_t>, grid, block, 0, s, tok, (const bf16_t*)V, pe, (bf16_t*)h, N, T, d, vocab, scale, flag, dd);
  else hipLaunchKernelGGL(embed_fwd_kernel<float>, grid, block, 0, s, tok, (const float*)V, pe, (float*)h, N, T, d, vocab, scale, flag, dd);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void transpose_table_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                                              const TransposeEntry* __restrict__ tab, int entries) {
  __shared__ bf16_t tile[64][72];              // row stride 144 bytes: 16-byte aligned rows
  int e = 0;
  while (e + 1 < entries && tab[e + 1].tile0 <= (int)blockIdx.x) ++e;
  const TransposeEntry t = tab[e];
  const int tiles_c = (t.cols + 63) / 64;
  const int local = blockIdx.x - t.tile0;
  const int r0 = (local / tiles_c) * 64, c0 = (local % tiles_c) * 64;
  const bf16_t* a = src + t.off;
  bf16_t* b = dst + t.off;
  // 16-byte path: whole tile inside the matrix, rows of both layouts 16-byte aligned
  const bool vec = r0 + 64 <= t.rows && c0 + 64 <= t.cols && !(t.cols & 7) && !(t.ld_out & 7) && !(t.off & 7);
  if (vec) {
    const int q = threadIdx.x & 7, rr = threadIdx.x >> 3;          // 8 threads per 64-element row, 32 rows per pass
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int r = rr + 32 * pass;
      *reinterpret_cast<uint4*>(&tile[r][q * 8]) = *reinterpret_cast<const uint4*>(a + (size_t)(r0 + r) * t.cols + c0 + q * 8);
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int c = rr + 32 * pass;                                 // output row = input column
      union { bf16_t h[8]; uint4 v; } u;
#pragma unroll
      for (int i = 0; i < 8; ++i) u.h[i] = tile[q * 8 + i][c];
      *reinterpret_cast<uint4*>(b + (size_t)(c0 + c) * t.ld_out + r0 + q * 8) = u.v;
    }
    return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < t.rows && c < t.cols) tile[i][tx] = a[(size_t)r * t.cols + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < t.rows && c < t.cols) b[(size_t)c * t.ld_out + r] = tile[tx][i];
  }
}

hipError_t launch_transpose_table(hipStream_t s, const void* src, void* dst, const TransposeEntry* dev_tab, int entries, int tiles) {
  if (entries <= 0 || tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_table_kernel, dim3(tiles), dim3(256), 0, s, (const bf16_t*)src, (bf16_t*)dst, dev_tab, entries);
  return hipGetLastError();
}

hipError_t launch_dropout_apply(hipStream_t s, int dtype, const void* src, void* dst, int rows, int cols, int ld,
                                const DropDesc& drop) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const size_t total = (size_t)rows * cols;
  dim3 grid((unsigned)std::min<size_t>((total + 255) / 256, 4096)), block(256);
  if (dtype == 1) hipLaunchKernelGGL(dropout_apply_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)src, (bf16_t*)dst, rows, cols, ld, drop);
  else hipLaunchKernelGGL(dropout_apply_kernel<float>, grid, block, 0, s, (const float*)src, (float*)dst, rows, cols, ld, drop);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(hipStream_t s, int dtype, const int32_t* tok, const void* dh, float* dVi,
                            int N, int d, int vocab, float scale, const DropDesc* drop) {
  dim3 grid((N + 3) / 4), block(256);
  DropDesc dd;
  memset(&dd, 0, sizeof dd);
  if (drop) dd = *drop;
  if (dtype == 1) hipLaunchKernelGGL(embed_bwd_kernel<bf16_t>, grid, block, 0, s, tok, (const bf16_t*)dh, dVi, N, d, vocab, scale, dd);
  else hipLaunchKernelGGL(embed_bwd_kernel<float>, grid, block, 0, s, tok, (const float*)dh, dVi, N, d, vocab, scale, dd);
  return hipGetLastError();
}

// ------------------------------------------------------------------------ cross entropy
// One block per row of logits (type T): online (max, sum) over the vocabulary in 16-byte
// packs, then G = (softmax - onehot)/N written over the same positions (G may alias the
// logits: a thread overwrites only elements it alone reads in the second pass, and the
// target logit is fetched before the block-wide barrier).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void ce_rows_kernel(const T* __restrict__ logits, int ld,
                                                      const int32_t* __restrict__ tgt, T* __restrict__ G, int ldg,
                                                      float* __restrict__ lse_out, float* __restrict__ rowloss,
                                                      int N, int vocab, int* flag) {
  constexpr int P = Pack<T>::N;
  __shared__ float sm_m[4], sm_s[4];
  const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* row = logits + (size_t)n * ld;
  T* grow = G + (size_t)n * ldg;
  const int t = tgt[n];
  const bool ok = t >= 0 && t < vocab;
  const float tl = ok ? to_f32(row[t]) : 0.f;
  const int nvec = VEC ? vocab / P : 0;
  float m = -INFINITY, ssum = 0.f;
  auto upd = [&](float v) __attribute__((always_inline)) {
    if (v > m) { ssum = ssum * __expf(m - v) + 1.f; m = v; }
    else ssum += __expf(v - m);
  };
  for (int vi = tid; vi < nvec; vi += 256) {
    float v[P];
    load_pack<T>(row + vi * P, v);
#pragma unroll
    for (int e = 0; e < P; ++e) upd(v[e]);
  }
  for (int c = nvec * P + tid; c < vocab; c += 256) upd(to_f32(row[c]));
  float wm = wave_max(m);
  ssum = (m == -INFINITY) ? 0.f : ssum * __expf(m - wm);
  ssum = wave_sum(ssum);
  if (lane == 0) { sm_m[wave] = wm; sm_s[wave] = ssum; }
  __syncthreads();
  float bm = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) bs += sm_s[w] * __expf(sm_m[w] - bm);
  const float lse = bm + logf(bs);
  if (tid == 0) {
    lse_out[n] = lse;
    rowloss[n] = ok ? lse - tl : 0.f;
    if (!ok) atomicOr(flag, 2);
  }
  const float invN = 1.f / N;
  for (int vi = tid; vi < nvec; vi += 256) {
    float v[P];
    load_pack<T>(row + vi * P, v);
#pragma unroll
    for (int e = 0; e < P; ++e) {
      float gval = __expf(v[e] - lse);
      if (ok && vi * P + e == t) gval -= 1.f;
      v[e] = gval * invN;
    }
    store_pack<T>(grow + vi * P, v);
  }
  for (int c = nvec * P + tid; c < vocab; c += 256) {
    float gval = __expf(to_f32(row[c]) - lse);
    if (ok && c == t) gval -= 1.f;
    grow[c] = from_f32<T>(gval * invN);
  }
}

// The same for bf16 rows of up to NP * NT * 8 elements, 16-byte aligned: the row stays in
// registers (NP packs per thread, NT threads) between the passes, so the logits are read once.
template <int NP, int NT>
__global__ __launch_bounds__(NT) void ce_rows_cached_kernel(const bf16_t* __restrict__ logits, int ld,
                                                             const int32_t* __restrict__ tgt, bf16_t* __restrict__ G, int ldg,
                                                             float* __restrict__ lse_out, float* __restrict__ rowloss,
                                                             int N, int vocab, int* flag) {
  constexpr int NWV = NT / 64;
  __shared__ float sm_m[NWV], sm_s[NWV];
  const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bf16_t* row = logits + (size_t)n * ld;
  bf16_t* grow = G + (size_t)n * ldg;
  const int t = tgt[n];
  const bool ok = t >= 0 && t < vocab;
  const float tl = ok ? to_f32(row[t]) : 0.f;
  const int nvec = vocab / 8;
  uint4 buf[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int vi = tid + NT * i;
    buf[i] = vi < nvec ? *reinterpret_cast<const uint4*>(row + vi * 8) : make_uint4(0, 0, 0, 0);
  }
  auto unpack = [](const uint4& q, float* out) __attribute__((always_inline)) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      out[2 * k] = __uint_as_float(w[k] << 16);
      out[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
    }
  };
  // per-thread maximum first, then one exponential per element (no rescaling chain)
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NP; ++i)
    if (tid + NT * i < nvec) {
      float v[8];
      unpack(buf[i], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) m = fmaxf(m, v[e]);
    }
  for (int c = nvec * 8 + tid; c < vocab; c += NT) m = fmaxf(m, to_f32(row[c]));
  const float wm = wave_max(m);
  if (lane == 0) sm_m[wave] = wm;
  __syncthreads();
  float bm = sm_m[0];
#pragma unroll
  for (int w = 1; w < NWV; ++w) bm = fmaxf(bm, sm_m[w]);
  float ssum = 0.f;
#pragma unroll
  for (int i = 0; i < NP; ++i)
    if (tid + NT * i < nvec) {
      float v[8];
      unpack(buf[i], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) ssum += __expf(v[e] - bm);
    }
  for (int c = nvec * 8 + tid; c < vocab; c += NT) ssum += __expf(to_f32(row[c]) - bm);
  ssum = wave_sum(ssum);
  if (lane == 0) sm_s[wave] = ssum;
  __syncthreads();
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < NWV; ++w) bs += sm_s[w];
  const float lse = bm + logf(bs);
  if (tid == 0) {
    lse_out[n] = lse;
    rowloss[n] = ok ? lse - tl : 0.f;
    if (!ok) atomicOr(flag, 2);
  }
  const float invN = 1.f / N;
  // the scalar tail is read before anything of this row is overwritten by this thread only
  for (int c = nvec * 8 + tid; c < vocab; c += NT) {
    float gval = __expf(to_f32(row[c]) - lse);
    if (ok && c == t) gval -= 1.f;
    grow[c] = from_f32<bf16_t>(gval * invN);
  }
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int vi = tid + NT * i;
    if (vi < nvec) {
      float v[8];
      unpack(buf[i], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float gval = __expf(v[e] - lse);
        if (ok && vi * 8 + e == t) gval -= 1.f;
        v[e] = gval * invN;
      }
      store_pack<bf16_t>(grow + vi * 8, v);
    }
  }
}

hipError_t launch_ce_rows(hipStream_t s, int dtype, const void* logits, int ld, const int32_t* tgt,
                          void* G, int ldg, float* lse, float* rowloss, int N, int vocab, int* flag) {
  dim3 grid(N), block(256);
  const int pack = dtype == 1 ? 8 : 4;
  const bool vec = ld % pack == 0 && ldg % pack == 0 && ptr16(logits) && ptr16(G);
  if (dtype == 1 && vec && vocab <= 16 * 512 * 8) {
    if (vocab <= 16 * 256 * 8)
      hipLaunchKernelGGL((ce_rows_cached_kernel<16, 256>), grid, block, 0, s, (const bf16_t*)logits, ld, tgt, (bf16_t*)G, ldg, lse, rowloss, N, vocab, flag);
    else
      hipLaunchKernelGGL((ce_rows_cached_kernel<16, 512>), grid, dim3(512), 0, s, (const bf16_t*)logits, ld, tgt, (bf16_t*)G, ldg, lse, rowloss, N, vocab, flag);
  } else if (dtype == 1) {
    if (vec) hipLaunchKernelGGL((ce_rows_kernel<bf16_t, true>), grid, block, 0, s, (const bf16_t*)logits, ld, tgt, (bf16_t*)G, ldg, lse, rowloss, N, vocab, flag);
    else hipLaunchKernelGGL((ce_rows_kernel<bf16_t, false>), grid, block, 0, s, (const bf16_t*)logits, ld, tgt, (bf16_t*)G, ldg, lse, rowloss, N, vocab, flag);
  } else {
    if (vec) hipLaunchKernelGGL((ce_rows_kernel<float, true>), grid, block, 0, s, (const float*)logits, ld, tgt, (float*)G, ldg, lse, rowloss, N, vocab, flag);
    else hipLaunchKernelGGL((ce_rows_kernel<float, false>), grid, block, 0, s, (const float*)logits, ld, tgt, (float*)G, ldg, lse, rowloss, N, vocab, flag);
  }
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void sum_rows_kernel(const float* __restrict__ rowloss, int N, float* loss) {
  __shared__ float red[256];
  float a = 0.f;
  for (int i = threadIdx.x; i < N; i += 256) a += rowloss[i];
  red[threadIdx.x] = a;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = red[0] / N;
}

hipError_t launch_sum_rows(hipStream_t s, const float* rowloss, int N, float* loss) {
  hipLaunchKernelGGL(sum_rows_kernel, dim3(1), dim3(256), 0, s, rowloss, N, loss);
  return hipGetLastError();
}

// -------------------------------------------------------------------------- conversions
template <typename T>
__global__ void convert_kernel(T* dst, const float* src, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = from_f32<T>(src[i]);
}
template <typename T>
__global__ void to_f32_kernel(float* dst, const T* src, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = to_f32(src[i]);
}
__global__ void fill_zero_kernel(uint32_t* p, size_t nwords) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t n4 = nwords / 4;
  uint4* p4 = reinterpret_cast<uint4*>(p);
  for (size_t j = i; j < n4; j += stride) p4[j] = make_uint4(0, 0, 0, 0);
  for (size_t j = n4 * 4 + i; j < nwords; j += stride) p[j] = 0;
}
static inline unsigned grid_for(size_t n, unsigned per_block = 256, unsigned cap = 8192) {
  size_t g = (n + per_block - 1) / per_block;
  if (g > cap) g = cap;
  if (g < 1) g = 1;
  return (unsigned)g;
}
hipError_t launch_convert(hipStream_t s, int dtype_dst, void* dst, const float* src, size_t n) {
  if (n == 0) return hipSuccess;
  if (dtype_dst == 1) hipLaunchKernelGGL(convert_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, s, (bf16_t*)dst, src, n);
  else hipLaunchKernelGGL(convert_kernel<float>, dim3(grid_for(n)), dim3(256), 0, s, (float*)dst, src, n);
  return hipGetLastError();
}
hipError_t launch_to_f32(hipStream_t s, int dtype_src, float* dst, const void* src, size_t n) {
  if (n == 0) return hipSuccess;
  if (dtype_src == 1) hipLaunchKernelGGL(to_f32_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, s, dst, (const bf16_t*)src, n);
  else hipLaunchKernelGGL(to_f32_kernel<float>, dim3(grid_for(n)), dim3(256), 0, s, dst, (const float*)src, n);
  return hipGetLastError();
}
hipError_t launch_fill_zero(hipStream_t s, void* p, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  if ((bytes & 3) || (reinterpret_cast<uintptr_t>(p) & 15)) return hipErrorInvalidValue;
  size_t nwords = bytes / 4;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(nwords / 4 + 1)), dim3(256), 0, s, (uint32_t*)p, nwords);
  return hipGetLastError();
}

template <typename T>
__global__ void copy_rows_kernel(T* dst, size_t dst_bstride, size_t dst_off, const T* src, size_t src_bstride,
                                 size_t src_off, int rows, int d) {
  const int b = blockIdx.y;
  const size_t n = (size_t)rows * d;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[b * dst_bstride + dst_off + i] = src[b * src_bstride + src_off + i];
}
// The same copy in 16-byte pieces (all strides, offsets and the row block a multiple of 16 bytes).
__global__ void copy_rows_vec_kernel(uint4* dst, size_t dst_bstride, size_t dst_off, const uint4* src, size_t src_bstride,
                                     size_t src_off, size_t n) {
  const int b = blockIdx.y;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[b * dst_bstride + dst_off + i] = src[b * src_bstride + src_off + i];
}
hipError_t launch_copy_rows(hipStream_t s, int dtype, void* dst, size_t dst_bstride, size_t dst_off,
                            const void* src, size_t src_bstride, size_t src_off, int B, int rows, int d) {
  if (B <= 0 || rows <= 0) return hipSuccess;
  const size_t esz = dtype == 1 ? 2 : 4, per = 16 / esz, n = (size_t)rows * d;
  if (!((dst_bstride | dst_off | src_bstride | src_off | n) % per) && !((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15)) {
    dim3 grid(grid_for(n / per, 256, 1024), B), block(256);
    hipLaunchKernelGGL(copy_rows_vec_kernel, grid, block, 0, s, (uint4*)dst, dst_bstride / per, dst_off / per, (const uint4*)src,
                       src_bstride / per, src_off / per, n / per);
    return hipGetLastError();
  }
  dim3 grid(grid_for((size_t)rows * d, 256, 1024), B), block(256);
  if (dtype == 1) hipLaunchKernelGGL(copy_rows_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)dst, dst_bstride, dst_off, (const bf16_t*)src, src_bstride, src_off, rows, d);
  else hipLaunchKernelGGL(copy_rows_kernel<float>, grid, block, 0, s, (float*)dst, dst_bstride, dst_off, (const float*)src, src_bstride, src_off, rows, d);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------- update
// Algorithm 1: w -= lr*g.  Algorithm 2: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
// w -= lr * (m/bc1) / (sqrt(v/bc2) + eps).  16 bytes per lane per stream.
struct UpdParams {
  float* w; float* m; float* v; bf16_t* shadow;
  const float* g0; const float* g1; float s0, s1;
  size_t n; float lr, b1, b2, eps, bc1, bc2;
};
template <bool ADAM>
__device__ __forceinline__ float upd_one(float w, float g, float& m, float& v, const UpdParams& p) {
  if (!ADAM) return w - p.lr * g;
  m = p.b1 * m + (1.f - p.b1) * g;
  v = p.b2 * v + (1.f - p.b2) * g * g;
  float mh = m / p.bc1, vh = v / p.bc2;
  return w - p.lr * (mh / (sqrtf(vh) + p.eps));
}
// Streaming accesses of the update: every byte is touched once per iteration, so it is kept out of
// the caches' way (the bf16 copy, which the next forward pass reads, is stored normally).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float4* p) {
  f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store4(float4* p, float4 a) {
  f32x4_t v = {a.x, a.y, a.z, a.w};
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(p));
}
template <bool ADAM>
__global__ __launch_bounds__(256) void update_kernel(UpdParams p) {
  const size_t n4 = p.n / 4;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  // two 16-byte packs per trip and stream: all loads are issued before the arithmetic
  for (size_t j0 = i; j0 < n4; j0 += 2 * stride) {
    float4 w[2], g[2], m[2], v[2];
    bool on[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const size_t j = j0 + u * stride;
      on[u] = j < n4;
      g[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      m[u] = g[u]; v[u] = g[u]; w[u] = g[u];
      if (on[u]) {
        w[u] = nt_load4(reinterpret_cast<const float4*>(p.w) + j);
        if (p.g0) { float4 a = nt_load4(reinterpret_cast<const float4*>(p.g0) + j); g[u].x = p.s0 * a.x; g[u].y = p.s0 * a.y; g[u].z = p.s0 * a.z; g[u].w = p.s0 * a.w; }
        if (p.g1) { float4 a = nt_load4(reinterpret_cast<const float4*>(p.g1) + j); g[u].x += p.s1 * a.x; g[u].y += p.s1 * a.y; g[u].z += p.s1 * a.z; g[u].w += p.s1 * a.w; }
        if (ADAM) { m[u] = nt_load4(reinterpret_cast<const float4*>(p.m) + j); v[u] = nt_load4(reinterpret_cast<const float4*>(p.v) + j); }
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (!on[u]) continue;
      const size_t j = j0 + u * stride;
      w[u].x = upd_one<ADAM>(w[u].x, g[u].x, m[u].x, v[u].x, p);
      w[u].y = upd_one<ADAM>(w[u].y, g[u].y, m[u].y, v[u].y, p);
      w[u].z = upd_one<ADAM>(w[u].z, g[u].z, m[u].z, v[u].z, p);
      w[u].w = upd_one<ADAM>(w[u].w, g[u].w, m[u].w, v[u].w, p);
      nt_store4(reinterpret_cast<float4*>(p.w) + j, w[u]);
      if (ADAM) { nt_store4(reinterpret_cast<float4*>(p.m) + j, m[u]); nt_store4(reinterpret_cast<float4*>(p.v) + j, v[u]); }
      if (p.shadow) {
        union { bf16_t h[4]; uint2 q; } cv;
        cv.h[0] = (bf16_t)w[u].x; cv.h[1] = (bf16_t)w[u].y; cv.h[2] = (bf16_t)w[u].z; cv.h[3] = (bf16_t)w[u].w;
        reinterpret_cast<uint2*>(p.shadow)[j] = cv.q;
      }
    }
  }
  for (size_t j = n4 * 4 + i; j < p.n; j += stride) {
    float g = 0.f;
    if (p.g0) g = p.s0 * p.g0[j];
    if (p.g1) g += p.s1 * p.g1[j];
    float m = 0.f, v = 0.f;
    if (ADAM) { m = p.m[j]; v = p.v[j]; }
    float w = upd_one<ADAM>(p.w[j], g, m, v, p);
    p.w[j] = w;
    if (ADAM) { p.m[j] = m; p.v[j] = v; }
    if (p.shadow) p.shadow[j] = (bf16_t)w;
  }
}

hipError_t launch_update(hipStream_t s, const UpdateDesc& u) {
  if (u.n == 0) return hipSuccess;
  UpdParams p;
  p.w = u.w; p.m = u.m; p.v = u.v; p.shadow = u.shadow; p.g0 = u.g0; p.g1 = u.g1; p.s0 = u.gscale0; p.s1 = u.gscale1;
  p.n = u.n; p.lr = u.lr; p.b1 = u.beta1; p.b2 = u.beta2; p.eps = u.eps; p.bc1 = u.bc1; p.bc2 = u.bc2;
  dim3 grid(grid_for(u.n / 4 + 1, 256, 4096)), block(256);
  if (u.adam) hipLaunchKernelGGL(update_kernel<true>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(update_kernel<false>, grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace ouro
