// Internal declarations shared by the HIP translation units of libouro (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

typedef __bf16 bf16_t;

namespace ouro {

// ----------------------------------------------------------------------------- helpers
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// erf by the rational-exponential form 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1/(1 + p|x|)
// (Abramowitz & Stegun 7.1.26, absolute error below 1.5e-7): a dozen instructions instead
// of the library routine's several dozen, which matters in the GEMM epilogues.
__device__ __forceinline__ float erf_fast(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float poly = fmaf(t, 1.061405429f, -1.453152027f);
  poly = fmaf(t, poly, 1.421413741f);
  poly = fmaf(t, poly, -0.284496736f);
  poly = fmaf(t, poly, 0.254829592f);
  const float r = 1.0f - poly * t * __expf(-ax * ax);
  return copysignf(r, x);
}
// erf-form GELU x*Phi(x) and its derivative Phi(x) + x*phi(x); erf to 1.5e-7 absolute (erf_fast)
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erf_fast(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  return 0.5f * (1.0f + erf_fast(x * 0.70710678118654752f)) + x * 0.3989422804014327f * __expf(-0.5f * x * x);
}

// --------------------------------------------------------------------------------- GEMM
// C[M,N] = op(A)[M,K] * op(B)[K,N], fp32 accumulation, then the epilogue
//   v = acc (+ bias[n]); EPI_GELU: Z[m,n] = v, v = gelu(v); EPI_GELUGRAD: v *= gelu'(Z[m,n]);
//   (+ residual[m,n]); store as T or fp32, or atomically add to fp32 C (split-K).
// transA == 0: A stored [M,K] (lda >= K); transA == 1: A stored [K,M] (lda >= M).
// transB == 0: B stored [K,N] (ldb >= N); transB == 1: B stored [N,K] (ldb >= K).
enum { EPI_NONE = 0, EPI_GELU = 1, EPI_GELUGRAD = 2 };
// Repeatable dropout (Section 5.2): element i of a tensor is kept iff the high 32 bits of output
// number i + stream*2^40 + 1 of the SplitMix64 sequence started at the seed are >= thresh; kept
// elements are scaled.  base = seed + gamma*(stream*2^40 + 1) is formed on the host.
struct DropDesc {
  int on;
  uint32_t thresh;       // floor(p * 2^32)
  float scale;           // 1 / (1 - p)
  uint64_t base;
  int ld;                // row length that turns (row, column) into the element index
};
inline DropDesc make_drop(float p, uint64_t seed, uint32_t stream, int ld) {
  DropDesc d;
  d.on = p > 0.f;
  d.thresh = (uint32_t)((double)p * 4294967296.0);
  d.scale = 1.f / (1.f - p);
  d.base = seed + 0x9E3779B97F4A7C15ull * (((uint64_t)stream << 40) + 1ull);
  d.ld = ld;
  return d;
}
__device__ __forceinline__ float drop_factor(const DropDesc& d, uint64_t idx) {
  uint64_t z = d.base + 0x9E3779B97F4A7C15ull * idx;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (uint32_t)(z >> 32) >= d.thresh ? d.scale : 0.f;
}

struct GemmDesc {
  const void* A; const void* B; void* C;
  int M, N, K, lda, ldb, ldc;
  int transA, transB;
  int out_fp32;          // C element type: 1 fp32, 0 same as inputs
  int accumulate;        // 1: C (fp32) += result (atomic, allows split-K); else overwrite
  const float* bias;     // [N] or null
  const void* residual;  // [M, ldr] element type T, or null
  int ldr;
  // fp32 residual instead (residual must be null): res32 [M, ldr32].  With ln_mean set the residual is
  // the LayerNorm of res32 recomputed in place, (res32[m,n] - ln_mean[m]) * ln_rstd[m] * ln_g[n] + ln_b[n]:
  // a block's input is the LayerNorm of the sum before it, and adding it back from that fp32 sum keeps
  // the bf16 rounding of the LayerNorm's stored output (the contraction operand) off the residual path.
  const float* res32; int ldr32;
  const float* ln_mean; const float* ln_rstd; const float* ln_g; const float* ln_b;
  int epilogue;
  void* Z; int ldz;      // EPI_GELU: written (type T); EPI_GELUGRAD: read (type T)
  float alpha;           // scales acc before the epilogue
  DropDesc drop;         // dropout on (alpha*acc + bias), before the residual; element index m*drop.ld + n
  // A grid of by x bz independent products of the same shape (0 or 1: a single one): product
  // (y, z) takes A + y*sAy + z*sAz, B + y*sBy + z*sBz and writes C + y*sCy + z*sCz (elements).
  // Only with plain epilogues (no bias, residual, Z, dropout), except res32 without the
  // LayerNorm terms on an fp32 output: it then follows C's batch strides (res32 == C adds in place).
  int by, bz;
  long long sAy, sAz, sBy, sBz, sCy, sCz;
  // A second grid of products of the same shape, strides and leading dimensions in the same
  // launch (C2 != null): A2, B2, C2 and alpha2 in place of A, B, C and alpha.  Two grids of short
  // products are bound by memory latency; side by side they keep twice as many loads in flight.
  const void* A2; const void* B2; void* C2; float alpha2;
};
// Most products one grouped launch takes (launch_gemm_group).
constexpr int GEMM_GROUP_MAX = 6;
// MFMA tile configurations (bf16): register-staged 128x128 (any K multiple of 8), and four
// direct-to-LDS kernels that need K % 64 == 0 and operands under 2 GiB.
enum { GEMM_TILE_STAGED128 = 10, GEMM_TILE_128x128 = 11, GEMM_TILE_128x64 = 12, GEMM_TILE_PIPE128 = 13, GEMM_TILE_256x256 = 14 };
// dtype 0: fp32 operands, 1: bf16 operands.  force_generic: 0 = automatic choice, 1 = the
// plain tiled kernel, GEMM_TILE_* = that MFMA configuration where the problem admits MFMA
// (a direct-to-LDS configuration falls back to the staged one when its conditions fail).
hipError_t launch_gemm(hipStream_t s, int dtype, const GemmDesc& g, int force_generic);
// n <= GEMM_GROUP_MAX accumulating products (fp32 C += alpha A^T B, plain epilogue, no batch) in one
// launch when all of them are bf16 with transA = 1, transB = 0 and admit the direct-to-LDS MFMA
// kernel; otherwise one launch_gemm each.  *grouped (optional) tells which it was.
hipError_t launch_gemm_group(hipStream_t s, int dtype, const GemmDesc* g, int n, bool* grouped = nullptr);
// true if launch_gemm would take the MFMA path for this problem
bool gemm_uses_mfma(int dtype, const GemmDesc& g);

// ---------------------------------------------------------------------------- attention
// q rows: (b*T + i), head h at columns [h*dh, (h+1)*dh) of a row of stride ldq elements.
// k, v rows: (b*S + j), S = Mv + T keys per stream; query i sits at position Mv + i and
// sees keys j <= Mv + i.  o like q.  lse [B,H,T] fp32 = log-sum-exp of the scaled scores.
// Relative variant (rel != 0): score = ((q+u_h).k_j + (q+vb_h).r_h[Mv+i-j]) * scale, with
// r rows indexed by distance (0..S-1), head h at columns [h*dh,..) of stride ldr.
struct AttnDesc {
  int B, H, T, S, dh, Mv;
  const void* q; int ldq;
  const void* k; int ldk;
  const void* v; int ldv;
  void* o; int ldo;
  float* lse;
  int rel;
  const void* u; const void* vb;   // [H, dh] element type T
  const void* r; int ldr;          // [S, H*dh] element type T
  float scale;
  // backward only
  const void* d_o; int lddo;       // gradient of o
  void* dq; int lddq;              // type T
  void* dk; int lddk;              // type T, rows b*S + j
  void* dv; int lddv;
  float* du; float* dvb;           // fp32 [H, dh], accumulated into (caller zeroes)
  float* dr;                       // fp32 [S, H*dh] dense, accumulated into (caller zeroes)
  float* scratch;                  // fp32 workspace, attn_bwd_scratch_floats() elements
  // relative-position MFMA path: the workspace's cells that the pass does not write are known to
  // be zero (the caller cleared it and every pass since ran with the same B, H, T, Mv); else it is cleared
  int scratch_clean;
};
// general kernels and the plain MFMA kernels / the relative-position MFMA path / the larger of the two
size_t attn_bwd_scratch_floats(int B, int H, int T, int S, int dh);
size_t attn_bwd_xl_scratch_floats(int B, int H, int T, int S);
size_t attn_bwd_scratch_floats_any(int B, int H, int T, int S, int dh);
// records msg as the calling thread's last error (ouro_last_error) and returns code
int set_error(int code, const char* msg);
hipError_t launch_attn_fwd(hipStream_t s, int dtype, const AttnDesc& a, int force_generic);
hipError_t launch_attn_bwd(hipStream_t s, int dtype, const AttnDesc& a, int force_generic);

// -------------------------------------------------------------------- row-wise kernels
// y = LN(x) * g + b over rows of d elements (biased variance, eps 1e-5); saves mean, rstd.
// Rows are d wide; the statistics run over the first dn columns (dn = 0: all d).  With dn < d the
// remaining columns are zero padding: they must hold zero scale and shift, and the input
// gradient is written as zero there.
// dtype of the LayerNorm launchers: 0 fp32 rows, 1 bf16 rows, 2 fp32 rows read (x, dy) and bf16 rows
// written (y, dx): the form bf16 models use, whose pre-normalisation sums and the gradients of the
// normalised rows stay in fp32 (they are the path every layer's rounding error travels along).
hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, const void* x, const float* g, const float* b,
                                void* y, float* mean, float* rstd, int rows, int d, int dn = 0);
// dx from dy, x, stats; dg/db (fp32) are accumulated into (caller zeroes). dg == nullptr: dx only.
// fuse_params: dg, db come from the kernel that writes dx (one pass over dy and x instead of two).
// copy_stride (floats, 0 = one copy): dg / db / out are the first of 8 copies that far apart.  Many
// blocks add to the same few addresses, and adds from different XCDs move the line from L2 to L2;
// the vector kernels therefore add into the copy of the XCD the block runs on (blocks are dealt to
// the 8 XCDs in launch order), and the caller sums the copies (launch_sum_segments).
hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, const void* dy, const void* x, const float* g,
                                const float* mean, const float* rstd, void* dx, float* dg, float* db,
                                int rows, int d, int dn = 0, bool fuse_params = false, size_t copy_stride = 0);
// dg[c] += sum_r dy*xhat, db[c] += sum_r dy alone (any stream that sees dy, x and the stats)
hipError_t launch_layernorm_bwd_params(hipStream_t s, int dtype, const void* dy, const void* x, const float* mean,
                                       const float* rstd, float* dg, float* db, int rows, int d);
// out[c] += sum over rows of x[r, c]  (fp32 accumulate into, caller zeroes)
hipError_t launch_colsum(hipStream_t s, int dtype, const void* x, int ldx, float* out, int rows, int cols, size_t copy_stride = 0);
// One piece of a gathered sum: dst[dst_off + i] += sum over 8 copies of src[c * stride + src_off + i], i < len <= 256
struct SumSegment { unsigned src_off, dst_off, len; };
// All pieces of a device table in one launch; the copies are left zero.
hipError_t launch_sum_segments(hipStream_t s, const SumSegment* table, int count, float* src, size_t stride, float* dst);
// h[n,:] = scale * V[tok[n],:] (+ pe[n % T,:]); ids outside [0,vocab) set *flag and give a zero row
// drop (optional): dropout on the sum, element index n*drop->ld + c
hipError_t launch_embed_fwd(hipStream_t s, int dtype, const int32_t* tok, const void* V, const float* pe,
                            void* h, int N, int T, int d, int vocab, float scale, int* flag,
                            const DropDesc* drop = nullptr);
// dVi[tok[n],:] += scale * dh[n,:]   (fp32 atomics; caller zeroes dVi); dtype: type of dh (1 bf16, else fp32)
hipError_t launch_embed_bwd(hipStream_t s, int dtype, const int32_t* tok, const void* dh, float* dVi,
                            int N, int d, int vocab, float scale, const DropDesc* drop = nullptr);
// One matrix of a parameter blob to be kept transposed as well: bf16 [rows, cols] at element offset
// off of src -> [cols, rows] with leading dimension ld_out at the same offset of dst.  tile0 is the
// running count of 64x64 tiles before this matrix (the launch covers all matrices of a table).
struct TransposeEntry { unsigned long long off; int rows, cols, ld_out, tile0; };
hipError_t launch_transpose_table(hipStream_t s, const void* src, void* dst, const TransposeEntry* dev_tab, int entries, int tiles);
// dst[r, c] = src[r, c] * mask(r*drop.ld + c) over rows x cols elements, both with row stride ld
hipError_t launch_dropout_apply(hipStream_t s, int dtype, const void* src, void* dst, int rows, int cols, int ld,
                                const DropDesc& drop);
// per row n of logits [N, ld] (type T): lse, rowloss = lse - logit[target]; G = (softmax - onehot)/N as T
// (G may alias logits: every element is read before it is overwritten by the same thread)
hipError_t launch_ce_rows(hipStream_t s, int dtype, const void* logits, int ld, const int32_t* tgt,
                          void* G, int ldg, float* lse, float* rowloss, int N, int vocab, int* flag);
// loss = sum(rowloss) (fixed order, one block)
hipError_t launch_sum_rows(hipStream_t s, const float* rowloss, int N, float* loss);
hipError_t launch_convert(hipStream_t s, int dtype_dst, void* dst, const float* src, size_t n);      // fp32 -> T
hipError_t launch_to_f32(hipStream_t s, int dtype_src, float* dst, const void* src, size_t n);       // T -> fp32
hipError_t launch_fill_zero(hipStream_t s, void* p, size_t bytes);                                   // bytes % 4 == 0
// strided row copy: dst[b, r, :] = src[b, r0 + r, :]; rows of d elements of type T
hipError_t launch_copy_rows(hipStream_t s, int dtype, void* dst, size_t dst_bstride, size_t dst_off,
                            const void* src, size_t src_bstride, size_t src_off, int B, int rows, int d);

// ------------------------------------------------------------------------------ update
// Algorithm 1 / Algorithm 2 on n elements.  g = gscale0*g0 + gscale1*g1 (null pointers
// count as zero).  Adam: bias corrections bc1 = 1-beta1^(t+1), bc2 = 1-beta2^(t+1).
// shadow (bf16) may be null.
struct UpdateDesc {
  float* w; float* m; float* v; bf16_t* shadow;
  const float* g0; const float* g1; float gscale0, gscale1;
  size_t n; int adam;
  float lr, beta1, beta2, eps, bc1, bc2;
};
hipError_t launch_update(hipStream_t s, const UpdateDesc& u);

}  // namespace ouro
