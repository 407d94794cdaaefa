// Straightforward causal attention kernels (one wavefront per query row) for fp32
// operands, odd head sizes and the relative-position variant.  Slow but general; the
// MFMA kernels in attention_mfma.hip take the aligned bf16 cases.
#include "common.h"

#include <algorithm>

namespace ouro {

struct AttnParams {
  int B, H, T, S, dh, Mv;
  const void* q; int ldq;
  const void* k; int ldk;
  const void* v; int ldv;
  void* o; int ldo;
  float* lse;
  int rel;
  const void* u; const void* vb;
  const void* r; int ldr;
  float scale;
  const void* d_o; int lddo;
  void* dq; int lddq;
  void* dk; int lddk;
  void* dv; int lddv;
  float* dq_ac; float* dq_bd;     // fp32 [B*T, H*dh]: content / position halves of dq
  float* Dq;                      // fp32 [B, H, T]
  float* du; float* dvb; float* dr;
};

// shared: sc[S] | qu[dh] | qv[dh]
template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_plain_kernel(AttnParams p) {
  extern __shared__ float sm[];
  float* sc = sm;
  float* qu = sm + p.S;
  float* qv = qu + p.dh;
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const T* q = reinterpret_cast<const T*>(p.q) + ((size_t)b * p.T + i) * p.ldq + h * p.dh;
  const T* kb = reinterpret_cast<const T*>(p.k) + (size_t)b * p.S * p.ldk + h * p.dh;
  const T* vbase = reinterpret_cast<const T*>(p.v) + (size_t)b * p.S * p.ldv + h * p.dh;
  const T* rb = p.rel ? reinterpret_cast<const T*>(p.r) + h * p.dh : nullptr;
  for (int c = lane; c < p.dh; c += 64) {
    float qc = to_f32(q[c]);
    qu[c] = qc + (p.rel ? to_f32(reinterpret_cast<const T*>(p.u)[h * p.dh + c]) : 0.f);
    qv[c] = qc + (p.rel ? to_f32(reinterpret_cast<const T*>(p.vb)[h * p.dh + c]) : 0.f);
  }
  __syncthreads();
  const int nvis = p.Mv + i + 1;
  float mx = -INFINITY;
  for (int j = lane; j < nvis; j += 64) {
    const T* kj = kb + (size_t)j * p.ldk;
    float s = 0.f;
    for (int c = 0; c < p.dh; ++c) s = fmaf(qu[c], to_f32(kj[c]), s);
    if (p.rel) {
      const T* rj = rb + (size_t)(p.Mv + i - j) * p.ldr;
      for (int c = 0; c < p.dh; ++c) s = fmaf(qv[c], to_f32(rj[c]), s);
    }
    s *= p.scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < nvis; j += 64) {
    float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __syncthreads();
  if (lane == 0) p.lse[((size_t)b * p.H + h) * p.T + i] = mx + logf(sum);
  const float inv = 1.f / sum;
  T* o = reinterpret_cast<T*>(p.o) + ((size_t)b * p.T + i) * p.ldo + h * p.dh;
  for (int c = lane; c < p.dh; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < nvis; ++j) acc = fmaf(sc[j], to_f32(vbase[(size_t)j * p.ldv + c]), acc);
    o[c] = from_f32<T>(acc * inv);
  }
}

// ------------------------------------------------------------------------------ backward
// Three passes, none of which adds atomically per (query, key) pair:
//   attn_bwd_q_kernel   one wave per query: dq, the content / position halves of dq as fp32
//                       rows (their column sums are du and dvb) and D = sum_c dO*O;
//   attn_bwd_kv_kernel  one wave per key, lanes over the queries that see it: dk, dv;
//   attn_bwd_r_kernel   one wave per (head, distance), lanes over (batch, query): dr.
// The second and third pass recompute the probabilities from the saved log-sum-exp.
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_q_kernel(AttnParams p) {
  extern __shared__ float sm[];
  float* qu = sm;
  float* qv = qu + p.dh;
  float* dov = qv + p.dh;
  float* sds = dov + p.dh;        // scaled score gradients [S]
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const int HD = p.H * p.dh;
  const T* q = reinterpret_cast<const T*>(p.q) + ((size_t)b * p.T + i) * p.ldq + h * p.dh;
  const T* o = reinterpret_cast<const T*>(p.o) + ((size_t)b * p.T + i) * p.ldo + h * p.dh;
  const T* dop = reinterpret_cast<const T*>(p.d_o) + ((size_t)b * p.T + i) * p.lddo + h * p.dh;
  const T* kb = reinterpret_cast<const T*>(p.k) + (size_t)b * p.S * p.ldk + h * p.dh;
  const T* vbase = reinterpret_cast<const T*>(p.v) + (size_t)b * p.S * p.ldv + h * p.dh;
  const T* rb = p.rel ? reinterpret_cast<const T*>(p.r) + h * p.dh : nullptr;
  float dpart = 0.f;
  for (int c = lane; c < p.dh; c += 64) {
    float qc = to_f32(q[c]);
    qu[c] = qc + (p.rel ? to_f32(reinterpret_cast<const T*>(p.u)[h * p.dh + c]) : 0.f);
    qv[c] = qc + (p.rel ? to_f32(reinterpret_cast<const T*>(p.vb)[h * p.dh + c]) : 0.f);
    float d = to_f32(dop[c]);
    dov[c] = d;
    dpart += d * to_f32(o[c]);
  }
  const float D = wave_sum(dpart);
  __syncthreads();
  const size_t stat = ((size_t)b * p.H + h) * p.T + i;
  const float lse = p.lse[stat];
  if (lane == 0) p.Dq[stat] = D;
  const int nvis = p.Mv + i + 1;
  for (int j = lane; j < nvis; j += 64) {
    const T* kj = kb + (size_t)j * p.ldk;
    const T* vj = vbase + (size_t)j * p.ldv;
    float s = 0.f, dP = 0.f;
    for (int c = 0; c < p.dh; ++c) {
      s = fmaf(qu[c], to_f32(kj[c]), s);
      dP = fmaf(dov[c], to_f32(vj[c]), dP);
    }
    if (p.rel) {
      const T* rj = rb + (size_t)(p.Mv + i - j) * p.ldr;
      for (int c = 0; c < p.dh; ++c) s = fmaf(qv[c], to_f32(rj[c]), s);
    }
    sds[j] = expf(s * p.scale - lse) * (dP - D) * p.scale;
  }
  __syncthreads();
  T* dq = reinterpret_cast<T*>(p.dq) + ((size_t)b * p.T + i) * p.lddq + h * p.dh;
  for (int c = lane; c < p.dh; c += 64) {
    float ak = 0.f, ar = 0.f;
    for (int j = 0; j < nvis; ++j) {
      ak = fmaf(sds[j], to_f32(kb[(size_t)j * p.ldk + c]), ak);
      if (p.rel) ar = fmaf(sds[j], to_f32(rb[(size_t)(p.Mv + i - j) * p.ldr + c]), ar);
    }
    dq[c] = from_f32<T>(ak + ar);
    if (p.rel) {
      p.dq_ac[((size_t)b * p.T + i) * HD + h * p.dh + c] = ak;
      p.dq_bd[((size_t)b * p.T + i) * HD + h * p.dh + c] = ar;
    }
  }
}

// Row of dh elements (stride 1) into registers; DHP = dh rounded up to the template's width.
template <typename T, int DHP>
__device__ __forceinline__ void load_row(const T* src, int dh, bool vec, float (&dst)[DHP]) {
  if (vec) {        // dh is a multiple of the 16-byte pack and src is 16-byte aligned
    constexpr int N = 16 / sizeof(T);
#pragma unroll
    for (int c0 = 0; c0 < DHP; c0 += N) {
      if (c0 < dh) {
        if constexpr (sizeof(T) == 2) {
          uint4 w = *reinterpret_cast<const uint4*>(src + c0);
          const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            dst[c0 + 2 * e] = __uint_as_float(ww[e] << 16);
            dst[c0 + 2 * e + 1] = __uint_as_float(ww[e] & 0xffff0000u);
          }
        } else {
          float4 w = *reinterpret_cast<const float4*>(src + c0);
          dst[c0] = w.x; dst[c0 + 1] = w.y; dst[c0 + 2] = w.z; dst[c0 + 3] = w.w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < N; ++e) dst[c0 + e] = 0.f;
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < DHP; ++c) dst[c] = c < dh ? to_f32(src[c]) : 0.f;
  }
}

// shared: key row, value row and the two biases of the head; padding features are zero
template <typename T, int DHP>
__global__ __launch_bounds__(64) void attn_bwd_kv_kernel(AttnParams p, int vec) {
  __shared__ float kj[DHP], vj[DHP], ub[DHP], vbias[DHP];
  const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const T* krow = reinterpret_cast<const T*>(p.k) + ((size_t)b * p.S + j) * p.ldk + h * p.dh;
  const T* vrow = reinterpret_cast<const T*>(p.v) + ((size_t)b * p.S + j) * p.ldv + h * p.dh;
  for (int c = lane; c < DHP; c += 64) {
    const bool in = c < p.dh;
    kj[c] = in ? to_f32(krow[c]) : 0.f;
    vj[c] = in ? to_f32(vrow[c]) : 0.f;
    ub[c] = (in && p.rel) ? to_f32(reinterpret_cast<const T*>(p.u)[h * p.dh + c]) : 0.f;
    vbias[c] = (in && p.rel) ? to_f32(reinterpret_cast<const T*>(p.vb)[h * p.dh + c]) : 0.f;
  }
  __syncthreads();
  float dk[DHP], dv[DHP];
#pragma unroll
  for (int c = 0; c < DHP; ++c) { dk[c] = 0.f; dv[c] = 0.f; }
  const T* rb = p.rel ? reinterpret_cast<const T*>(p.r) + h * p.dh : nullptr;
  const int i0 = max(0, j - p.Mv);                         // first query that sees key j
  for (int i = i0 + lane; i < p.T; i += 64) {
    float q[DHP], g[DHP];
    load_row<T, DHP>(reinterpret_cast<const T*>(p.q) + ((size_t)b * p.T + i) * p.ldq + h * p.dh, p.dh, vec, q);
    load_row<T, DHP>(reinterpret_cast<const T*>(p.d_o) + ((size_t)b * p.T + i) * p.lddo + h * p.dh, p.dh, vec, g);
    float s = 0.f, dP = 0.f;
#pragma unroll
    for (int c = 0; c < DHP; ++c) {
      s = fmaf(q[c] + ub[c], kj[c], s);
      dP = fmaf(g[c], vj[c], dP);
    }
    if (p.rel) {
      float r[DHP];
      load_row<T, DHP>(rb + (size_t)(p.Mv + i - j) * p.ldr, p.dh, vec, r);
#pragma unroll
      for (int c = 0; c < DHP; ++c) s = fmaf(q[c] + vbias[c], r[c], s);
    }
    const size_t stat = ((size_t)b * p.H + h) * p.T + i;
    const float pj = expf(s * p.scale - p.lse[stat]);
    const float ds = pj * (dP - p.Dq[stat]) * p.scale;
#pragma unroll
    for (int c = 0; c < DHP; ++c) {
      dv[c] = fmaf(pj, g[c], dv[c]);
      dk[c] = fmaf(ds, q[c] + ub[c], dk[c]);
    }
  }
  T* dko = reinterpret_cast<T*>(p.dk) + ((size_t)b * p.S + j) * p.lddk + h * p.dh;
  T* dvo = reinterpret_cast<T*>(p.dv) + ((size_t)b * p.S + j) * p.lddv + h * p.dh;
#pragma unroll
  for (int c = 0; c < DHP; ++c) {
    const float a = wave_sum(dk[c]), bsum = wave_sum(dv[c]);
    if (lane == 0 && c < p.dh) { dko[c] = from_f32<T>(a); dvo[c] = from_f32<T>(bsum); }
  }
}

// dr[delta, h, :] = sum over (b, i) whose key j = Mv + i - delta exists of dS(b,i,j) * (q_i + v)
template <typename T, int DHP>
__global__ __launch_bounds__(64) void attn_bwd_r_kernel(AttnParams p, int vec) {
  __shared__ float rd[DHP], ub[DHP], vbias[DHP];
  const int delta = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const T* rrow = reinterpret_cast<const T*>(p.r) + (size_t)delta * p.ldr + h * p.dh;
  for (int c = lane; c < DHP; c += 64) {
    const bool in = c < p.dh;
    rd[c] = in ? to_f32(rrow[c]) : 0.f;
    ub[c] = in ? to_f32(reinterpret_cast<const T*>(p.u)[h * p.dh + c]) : 0.f;
    vbias[c] = in ? to_f32(reinterpret_cast<const T*>(p.vb)[h * p.dh + c]) : 0.f;
  }
  __syncthreads();
  float dr[DHP];
#pragma unroll
  for (int c = 0; c < DHP; ++c) dr[c] = 0.f;
  const int i0 = max(0, delta - p.Mv);                     // key Mv + i - delta >= 0
  const int ni = p.T - i0;                                 // queries at this distance per stream
  for (int t = lane; t < ni * p.B; t += 64) {
    const int b = t / ni, i = i0 + t % ni, j = p.Mv + i - delta;
    float q[DHP], g[DHP], kk[DHP], vv[DHP];
    load_row<T, DHP>(reinterpret_cast<const T*>(p.q) + ((size_t)b * p.T + i) * p.ldq + h * p.dh, p.dh, vec, q);
    load_row<T, DHP>(reinterpret_cast<const T*>(p.d_o) + ((size_t)b * p.T + i) * p.lddo + h * p.dh, p.dh, vec, g);
    load_row<T, DHP>(reinterpret_cast<const T*>(p.k) + ((size_t)b * p.S + j) * p.ldk + h * p.dh, p.dh, vec, kk);
    load_row<T, DHP>(reinterpret_cast<const T*>(p.v) + ((size_t)b * p.S + j) * p.ldv + h * p.dh, p.dh, vec, vv);
    float s = 0.f, dP = 0.f;
#pragma unroll
    for (int c = 0; c < DHP; ++c) {
      s = fmaf(q[c] + ub[c], kk[c], s);
      s = fmaf(q[c] + vbias[c], rd[c], s);
      dP = fmaf(g[c], vv[c], dP);
    }
    const size_t stat = ((size_t)b * p.H + h) * p.T + i;
    const float ds = expf(s * p.scale - p.lse[stat]) * (dP - p.Dq[stat]) * p.scale;
#pragma unroll
    for (int c = 0; c < DHP; ++c) dr[c] = fmaf(ds, q[c] + vbias[c], dr[c]);
  }
  float* out = p.dr + (size_t)delta * p.H * p.dh + h * p.dh;
#pragma unroll
  for (int c = 0; c < DHP; ++c) {
    const float a = wave_sum(dr[c]);
    if (lane == 0 && c < p.dh) out[c] = a;
  }
}

size_t attn_bwd_scratch_floats(int B, int H, int T, int S, int dh) {
  // general path: content / position halves of dq (fp32 rows) + D; MFMA path: D and base-2 lse
  return 2 * (size_t)B * S * H * dh + 2 * (size_t)B * H * T;
}

size_t attn_bwd_scratch_floats_any(int B, int H, int T, int S, int dh) {
  const size_t gen = attn_bwd_scratch_floats(B, H, T, S, dh);
  return dh == 64 ? std::max(gen, attn_bwd_xl_scratch_floats(B, H, T, S)) : gen;
}

static AttnParams to_params(const AttnDesc& a) {
  AttnParams p;
  p.B = a.B; p.H = a.H; p.T = a.T; p.S = a.S; p.dh = a.dh; p.Mv = a.Mv;
  p.q = a.q; p.ldq = a.ldq; p.k = a.k; p.ldk = a.ldk; p.v = a.v; p.ldv = a.ldv;
  p.o = a.o; p.ldo = a.ldo; p.lse = a.lse; p.rel = a.rel; p.u = a.u; p.vb = a.vb; p.r = a.r; p.ldr = a.ldr;
  p.scale = a.scale; p.d_o = a.d_o; p.lddo = a.lddo; p.dq = a.dq; p.lddq = a.lddq;
  p.dk = a.dk; p.lddk = a.lddk; p.dv = a.dv; p.lddv = a.lddv;
  p.dq_ac = nullptr; p.dq_bd = nullptr; p.Dq = nullptr; p.du = a.du; p.dvb = a.dvb; p.dr = a.dr;
  return p;
}

hipError_t launch_attn_fwd_plain(hipStream_t s, int dtype, const AttnDesc& a) {
  AttnParams p = to_params(a);
  dim3 grid(a.T, a.H, a.B), block(64);
  size_t smem = ((size_t)a.S + 2 * a.dh) * sizeof(float);
  if (smem > 60000) return hipErrorInvalidValue;
  if (dtype == 1) hipLaunchKernelGGL(attn_fwd_plain_kernel<bf16_t>, grid, block, smem, s, p);
  else hipLaunchKernelGGL(attn_fwd_plain_kernel<float>, grid, block, smem, s, p);
  return hipGetLastError();
}

static inline bool al16p(const void* x) { return (reinterpret_cast<uintptr_t>(x) & 15) == 0; }

hipError_t launch_attn_bwd_plain(hipStream_t s, int dtype, const AttnDesc& a) {
  if (a.dh > 128) return hipErrorInvalidValue;
  AttnParams p = to_params(a);
  const int HD = a.H * a.dh;
  const size_t nq = (size_t)a.B * a.T;
  p.dq_ac = a.scratch;
  p.dq_bd = a.scratch + nq * HD;
  p.Dq = a.scratch + 2 * (size_t)a.B * a.S * HD;
  {
    dim3 grid(a.T, a.H, a.B), block(64);
    size_t smem = ((size_t)a.S + 3 * a.dh) * sizeof(float);
    if (smem > 60000) return hipErrorInvalidValue;
    if (dtype == 1) hipLaunchKernelGGL(attn_bwd_q_kernel<bf16_t>, grid, block, smem, s, p);
    else hipLaunchKernelGGL(attn_bwd_q_kernel<float>, grid, block, smem, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // 16-byte row loads when every head slice of every operand row is aligned
  const int pack = dtype == 1 ? 8 : 4;
  const bool vec = a.dh % pack == 0 && al16p(a.q) && al16p(a.k) && al16p(a.v) && al16p(a.d_o) &&
                   !((a.ldq | a.ldk | a.ldv | a.lddo) % pack) && (!a.rel || (al16p(a.r) && !(a.ldr % pack)));
#define OURO_ATT(KERN, GRID)                                                                       \
  do {                                                                                            \
    if (dtype == 1) {                                                                             \
      if (a.dh <= 64) hipLaunchKernelGGL((KERN<bf16_t, 64>), GRID, dim3(64), 0, s, p, (int)vec);   \
      else hipLaunchKernelGGL((KERN<bf16_t, 128>), GRID, dim3(64), 0, s, p, (int)vec);             \
    } else {                                                                                      \
      if (a.dh <= 64) hipLaunchKernelGGL((KERN<float, 64>), GRID, dim3(64), 0, s, p, (int)vec);    \
      else hipLaunchKernelGGL((KERN<float, 128>), GRID, dim3(64), 0, s, p, (int)vec);              \
    }                                                                                             \
  } while (0)
  OURO_ATT(attn_bwd_kv_kernel, dim3(a.S, a.H, a.B));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.rel) {
    OURO_ATT(attn_bwd_r_kernel, dim3(a.S, a.H, 1));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // du, dvb: column sums over all queries of the two halves of dq (accumulated into)
    e = launch_colsum(s, 0, p.dq_ac, HD, a.du, (int)nq, HD);
    if (e != hipSuccess) return e;
    e = launch_colsum(s, 0, p.dq_bd, HD, a.dvb, (int)nq, HD);
  }
#undef OURO_ATT
  return e;
}

}  // namespace ouro
