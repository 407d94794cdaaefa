// Straightforward causal attention kernels (one wavefront per query row) for fp32
// operands, odd head sizes and the relative-position variant.  Slow but general; the
// MFMA kernels in attention_mfma.hip take the aligned bf16 cases.
#include "common.h"

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
  float* dk_acc; float* dv_acc;   // fp32 [B*S, H*dh]
  float* du; float* dvb; float* dr;
};

// shared: sc[S] | qu[dh] | qv[dh] | (bwd) dov[dh] | sds[S]
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

template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_plain_kernel(AttnParams p) {
  extern __shared__ float sm[];
  float* sp = sm;                 // probabilities
  float* qu = sm + p.S;
  float* qv = qu + p.dh;
  float* dov = qv + p.dh;
  float* sds = dov + p.dh;        // scaled score gradients
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
  const float lse = p.lse[((size_t)b * p.H + h) * p.T + i];
  const int nvis = p.Mv + i + 1;
  for (int j = lane; j < nvis; j += 64) {
    const T* kj = kb + (size_t)j * p.ldk;
    const T* vj = vbase + (size_t)j * p.ldv;
    float s = 0.f, dP = 0.f;
    for (int c = 0; c < p.dh; ++c) {
      s = fmaf(qu[c], to_f32(kj[c]), s);
      dP = fmaf(dov[c], to_f32(vj[c]), dP);
    }
    const T* rj = nullptr;
    if (p.rel) {
      rj = rb + (size_t)(p.Mv + i - j) * p.ldr;
      for (int c = 0; c < p.dh; ++c) s = fmaf(qv[c], to_f32(rj[c]), s);
    }
    float pj = expf(s * p.scale - lse);
    float ds = pj * (dP - D) * p.scale;
    sp[j] = pj;
    sds[j] = ds;
    float* dkj = p.dk_acc + ((size_t)b * p.S + j) * HD + h * p.dh;
    float* dvj = p.dv_acc + ((size_t)b * p.S + j) * HD + h * p.dh;
    for (int c = 0; c < p.dh; ++c) {
      unsafeAtomicAdd(dvj + c, pj * dov[c]);
      unsafeAtomicAdd(dkj + c, ds * qu[c]);
    }
    if (p.rel) {
      float* drj = p.dr + (size_t)(p.Mv + i - j) * HD + h * p.dh;
      for (int c = 0; c < p.dh; ++c) unsafeAtomicAdd(drj + c, ds * qv[c]);
    }
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
      unsafeAtomicAdd(p.du + h * p.dh + c, ak);
      unsafeAtomicAdd(p.dvb + h * p.dh + c, ar);
    }
  }
}

// dst[row, h*dh..] (type T, stride ld) = acc[row, :] (fp32 dense)
template <typename T>
__global__ void attn_acc_to_out_kernel(const float* acc, T* dst, int ld, size_t rows, int HD) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * HD) return;
  size_t row = idx / HD;
  int c = (int)(idx % HD);
  dst[row * ld + c] = from_f32<T>(acc[idx]);
}

size_t attn_bwd_scratch_floats(int B, int H, int T, int S, int dh) {
  (void)T;
  return 2 * (size_t)B * S * H * dh;
}

static AttnParams to_params(const AttnDesc& a) {
  AttnParams p;
  p.B = a.B; p.H = a.H; p.T = a.T; p.S = a.S; p.dh = a.dh; p.Mv = a.Mv;
  p.q = a.q; p.ldq = a.ldq; p.k = a.k; p.ldk = a.ldk; p.v = a.v; p.ldv = a.ldv;
  p.o = a.o; p.ldo = a.ldo; p.lse = a.lse; p.rel = a.rel; p.u = a.u; p.vb = a.vb; p.r = a.r; p.ldr = a.ldr;
  p.scale = a.scale; p.d_o = a.d_o; p.lddo = a.lddo; p.dq = a.dq; p.lddq = a.lddq;
  p.dk_acc = nullptr; p.dv_acc = nullptr; p.du = a.du; p.dvb = a.dvb; p.dr = a.dr;
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

hipError_t launch_attn_bwd_plain(hipStream_t s, int dtype, const AttnDesc& a) {
  AttnParams p = to_params(a);
  const int HD = a.H * a.dh;
  const size_t rows = (size_t)a.B * a.S;
  p.dk_acc = a.scratch;
  p.dv_acc = a.scratch + rows * HD;
  hipError_t e = launch_fill_zero(s, a.scratch, 2 * rows * HD * sizeof(float));
  if (e != hipSuccess) return e;
  dim3 grid(a.T, a.H, a.B), block(64);
  size_t smem = (2 * (size_t)a.S + 3 * a.dh) * sizeof(float);
  if (smem > 60000) return hipErrorInvalidValue;
  if (dtype == 1) hipLaunchKernelGGL(attn_bwd_plain_kernel<bf16_t>, grid, block, smem, s, p);
  else hipLaunchKernelGGL(attn_bwd_plain_kernel<float>, grid, block, smem, s, p);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  size_t n = rows * HD;
  dim3 g2((unsigned)((n + 255) / 256)), b2(256);
  if (dtype == 1) {
    hipLaunchKernelGGL(attn_acc_to_out_kernel<bf16_t>, g2, b2, 0, s, p.dk_acc, (bf16_t*)a.dk, a.lddk, rows, HD);
    hipLaunchKernelGGL(attn_acc_to_out_kernel<bf16_t>, g2, b2, 0, s, p.dv_acc, (bf16_t*)a.dv, a.lddv, rows, HD);
  } else {
    hipLaunchKernelGGL(attn_acc_to_out_kernel<float>, g2, b2, 0, s, p.dk_acc, (float*)a.dk, a.lddk, rows, HD);
    hipLaunchKernelGGL(attn_acc_to_out_kernel<float>, g2, b2, 0, s, p.dv_acc, (float*)a.dv, a.lddv, rows, HD);
  }
  return hipGetLastError();
}

}  // namespace ouro
