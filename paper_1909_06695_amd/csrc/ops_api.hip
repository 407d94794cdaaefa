// Single-kernel C entry points (per-kernel parity tests and micro-benchmarks).
#include "common.h"
#include "../../include/ouro.h"
#include "../../include/ouro_ops.h"

#include <cmath>
#include <cstdio>
#include <cstring>

using namespace ouro;

static int rc_of(hipError_t e) { return e == hipSuccess ? OURO_OK : OURO_E_HIP; }

static GemmDesc make_gemm(int transA, int transB, int M, int N, int K, float alpha, const void* A, int lda,
                          const void* B, int ldb, void* C, int ldc, int out_fp32, int accumulate, const float* bias,
                          const void* residual, int ldr, int epilogue, void* Z, int ldz) {
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.transA = transA; g.transB = transB; g.out_fp32 = out_fp32; g.accumulate = accumulate;
  g.bias = bias; g.residual = residual; g.ldr = ldr; g.epilogue = epilogue; g.Z = Z; g.ldz = ldz; g.alpha = alpha;
  return g;
}

extern "C" int ouro_op_gemm(void* stream, int dtype, int transA, int transB, int M, int N, int K, float alpha,
                            const void* A, int lda, const void* B, int ldb, void* C, int ldc, int out_fp32,
                            int accumulate, const float* bias, const void* residual, int ldr, int epilogue,
                            void* Z, int ldz, int force_generic) {
  if (!A || !B || !C || M < 0 || N < 0 || K < 0) return OURO_E_ARG;
  if ((epilogue == EPI_GELU || epilogue == EPI_GELUGRAD) && !Z) return OURO_E_ARG;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return OURO_E_ARG;
  GemmDesc g = make_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, C, ldc, out_fp32, accumulate, bias, residual, ldr, epilogue, Z, ldz);
  return rc_of(launch_gemm((hipStream_t)stream, dtype, g, force_generic));
}

extern "C" int ouro_op_gemm_batched(void* stream, int dtype, int transA, int transB, int M, int N, int K, float alpha,
                                    const void* A, int lda, const void* B, int ldb, void* C, int ldc, int out_fp32,
                                    int accumulate, int by, int bz, long long sAy, long long sAz, long long sBy,
                                    long long sBz, long long sCy, long long sCz, const void* A2, const void* B2,
                                    void* C2, float alpha2, int force_generic) {
  if (!A || !B || !C || M < 0 || N < 0 || K < 0 || by < 1 || bz < 1 || by > 65535 || bz > 32767) return OURO_E_ARG;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return OURO_E_ARG;
  if (C2 && (!A2 || !B2)) return OURO_E_ARG;
  if (accumulate < 0 || accumulate > 2 || (accumulate == 2 && (!out_fp32 || C2))) return OURO_E_ARG;
  GemmDesc g = make_gemm(transA, transB, M, N, K, alpha, A, lda, B, ldb, C, ldc, out_fp32, accumulate == 1, nullptr, nullptr, 0, EPI_NONE, nullptr, 0);
  if (accumulate == 2) { g.res32 = reinterpret_cast<const float*>(C); g.ldr32 = ldc; }   // every product adds to its own C in the epilogue
  g.by = by; g.bz = bz; g.sAy = sAy; g.sAz = sAz; g.sBy = sBy; g.sBz = sBz; g.sCy = sCy; g.sCz = sCz;
  g.A2 = A2; g.B2 = B2; g.C2 = C2; g.alpha2 = alpha2;
  return rc_of(launch_gemm((hipStream_t)stream, dtype, g, force_generic));
}

extern "C" int ouro_op_gemm_group(void* stream, int dtype, int n, const int* M, const int* N, const int* K,
                                  const void* const* A, const int* lda, const void* const* B, const int* ldb,
                                  float* const* C, const int* ldc, float alpha) {
  if (n < 1 || n > GEMM_GROUP_MAX || !M || !N || !K || !A || !lda || !B || !ldb || !C || !ldc) return OURO_E_ARG;
  GemmDesc g[GEMM_GROUP_MAX];
  for (int i = 0; i < n; ++i) {
    if (!A[i] || !B[i] || !C[i] || M[i] < 0 || N[i] < 0 || K[i] < 0 || lda[i] < M[i] || ldb[i] < N[i] || ldc[i] < N[i]) return OURO_E_ARG;
    g[i] = make_gemm(1, 0, M[i], N[i], K[i], alpha, A[i], lda[i], B[i], ldb[i], C[i], ldc[i], 1, 1, nullptr, nullptr, 0, EPI_NONE, nullptr, 0);
  }
  return rc_of(launch_gemm_group((hipStream_t)stream, dtype, g, n));
}

extern "C" int ouro_op_gemm_dropout(void* stream, int dtype, int transA, int transB, int M, int N, int K,
                                    const void* A, int lda, const void* B, int ldb, void* C, int ldc, const float* bias,
                                    const void* residual, int ldr, float p, uint64_t seed, uint32_t stream_id, int drop_ld,
                                    int force_generic) {
  if (!A || !B || !C || M < 0 || N < 0 || K < 0 || !(p >= 0.f && p < 1.f) || drop_ld < N) return OURO_E_ARG;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return OURO_E_ARG;
  GemmDesc g = make_gemm(transA, transB, M, N, K, 1.f, A, lda, B, ldb, C, ldc, 0, 0, bias, residual, ldr, EPI_NONE, nullptr, 0);
  g.drop = make_drop(p, seed, stream_id, drop_ld);
  return rc_of(launch_gemm((hipStream_t)stream, dtype, g, force_generic));
}

extern "C" int ouro_op_gemm_ln_residual(void* stream, int dtype, int transA, int transB, int M, int N, int K, const void* A,
                                        int lda, const void* B, int ldb, void* C, int ldc, int out_fp32, const float* bias,
                                        const float* res32, int ldr32, const float* mean, const float* rstd, const float* g,
                                        const float* b, int force_generic) {
  if (!A || !B || !C || !res32 || M < 0 || N < 0 || K < 0 || ldr32 < N) return OURO_E_ARG;
  if (mean && (!rstd || !g || !b)) return OURO_E_ARG;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return OURO_E_ARG;
  GemmDesc gd = make_gemm(transA, transB, M, N, K, 1.f, A, lda, B, ldb, C, ldc, out_fp32, 0, bias, nullptr, 0, EPI_NONE, nullptr, 0);
  gd.res32 = res32; gd.ldr32 = ldr32; gd.ln_mean = mean; gd.ln_rstd = rstd; gd.ln_g = g; gd.ln_b = b;
  return rc_of(launch_gemm((hipStream_t)stream, dtype, gd, force_generic));
}

extern "C" int ouro_op_dropout(void* stream, int dtype, const void* src, void* dst, int rows, int cols, int ld,
                               float p, uint64_t seed, uint32_t stream_id, int drop_ld) {
  if (!src || !dst || rows < 0 || cols < 0 || ld < cols || !(p >= 0.f && p < 1.f) || drop_ld < cols) return OURO_E_ARG;
  return rc_of(launch_dropout_apply((hipStream_t)stream, dtype, src, dst, rows, cols, ld, make_drop(p, seed, stream_id, drop_ld)));
}

extern "C" int ouro_op_gemm_uses_mfma(int dtype, int transA, int transB, int M, int N, int K, const void* A, int lda,
                                      const void* B, int ldb) {
  GemmDesc g = make_gemm(transA, transB, M, N, K, 1.f, A, lda, B, ldb, nullptr, N, 0, 0, nullptr, nullptr, 0, 0, nullptr, 0);
  return gemm_uses_mfma(dtype, g) ? 1 : 0;
}

static AttnDesc make_attn(int B, int H, int T, int S, int dh, int Mv, float scale, const void* q, int ldq, const void* k,
                          int ldk, const void* v, int ldv, void* o, int ldo, float* lse, int rel, const void* u,
                          const void* vb, const void* r, int ldr) {
  AttnDesc a;
  memset(&a, 0, sizeof a);
  a.B = B; a.H = H; a.T = T; a.S = S; a.dh = dh; a.Mv = Mv; a.scale = scale;
  a.q = q; a.ldq = ldq; a.k = k; a.ldk = ldk; a.v = v; a.ldv = ldv; a.o = o; a.ldo = ldo; a.lse = lse;
  a.rel = rel; a.u = u; a.vb = vb; a.r = r; a.ldr = ldr;
  return a;
}

extern "C" int ouro_op_attention_fwd(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv, float scale,
                                     const void* q, int ldq, const void* k, int ldk, const void* v, int ldv, void* o,
                                     int ldo, float* lse, int rel, const void* u, const void* vb, const void* r, int ldr,
                                     int force_generic) {
  if (!q || !k || !v || !o || !lse || S != Mv + T || B < 1 || H < 1 || T < 1 || dh < 1 || Mv < 0) return OURO_E_ARG;
  if (rel && (!u || !vb || !r)) return OURO_E_ARG;
  AttnDesc a = make_attn(B, H, T, S, dh, Mv, scale, q, ldq, k, ldk, v, ldv, o, ldo, lse, rel, u, vb, r, ldr);
  return rc_of(launch_attn_fwd((hipStream_t)stream, dtype, a, force_generic));
}

extern "C" size_t ouro_op_attention_bwd_scratch(int B, int H, int T, int S, int dh) {
  return attn_bwd_scratch_floats_any(B, H, T, S, dh);
}

extern "C" int ouro_op_attention_bwd(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv, float scale,
                                     const void* q, int ldq, const void* k, int ldk, const void* v, int ldv,
                                     const void* o, int ldo, const float* lse, const void* d_o, int lddo, void* dq,
                                     int lddq, void* dk, int lddk, void* dv, int lddv, int rel, const void* u,
                                     const void* vb, const void* r, int ldr, float* du, float* dvb, float* dr,
                                     float* scratch, int force_generic) {
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !scratch || S != Mv + T) return OURO_E_ARG;
  if (rel && (!u || !vb || !r || !du || !dvb || !dr)) return OURO_E_ARG;
  AttnDesc a = make_attn(B, H, T, S, dh, Mv, scale, q, ldq, k, ldk, v, ldv, const_cast<void*>(o), ldo,
                         const_cast<float*>(lse), rel, u, vb, r, ldr);
  a.d_o = d_o; a.lddo = lddo; a.dq = dq; a.lddq = lddq; a.dk = dk; a.lddk = lddk; a.dv = dv; a.lddv = lddv;
  a.du = du; a.dvb = dvb; a.dr = dr; a.scratch = scratch;
  hipStream_t s = (hipStream_t)stream;
  if (rel) {
    hipError_t e = launch_fill_zero(s, du, (size_t)H * dh * 4);
    if (e == hipSuccess) e = launch_fill_zero(s, dvb, (size_t)H * dh * 4);
    if (e == hipSuccess) e = launch_fill_zero(s, dr, (size_t)S * H * dh * 4);
    if (e != hipSuccess) return OURO_E_HIP;
  }
  return rc_of(launch_attn_bwd(s, dtype, a, force_generic));
}

// ---- attention backward for callers that cannot allocate: the workspace is a device array of the library
constexpr size_t NOALLOC_SCRATCH_FLOATS = (size_t)4 << 20;       // 16 MiB per GPU, held until the process ends
static __device__ __align__(256) float scratch[NOALLOC_SCRATCH_FLOATS];
constexpr int NOALLOC_MAX_DEVICES = 64;
static float* g_scratch_ptr[NOALLOC_MAX_DEVICES];                 // device address of `scratch` on each GPU (host-side table)

extern "C" int ouro_op_attention_bwd_noalloc(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv, float scale,
                                             const void* q, int ldq, const void* k, int ldk, const void* v, int ldv,
                                             const void* o, int ldo, const float* lse, const void* d_o, int lddo, void* dq,
                                             int lddq, void* dk, int lddk, void* dv, int lddv, int rel, const void* u,
                                             const void* vb, const void* r, int ldr, float* du, float* dvb, float* dr,
                                             int force_generic) {
  if (B < 1 || H < 1 || T < 1 || dh < 1 || Mv < 0 || S != Mv + T) return set_error(OURO_E_ARG, "attention_bwd_noalloc: bad sizes");
  const size_t need = rel ? attn_bwd_scratch_floats_any(B, H, T, S, dh) : attn_bwd_scratch_floats(B, H, T, S, dh);
  if (need > NOALLOC_SCRATCH_FLOATS) {
    char msg[200];
    snprintf(msg, sizeof msg, "attention_bwd_noalloc: needs %zu workspace floats, the built-in workspace holds %zu", need,
             NOALLOC_SCRATCH_FLOATS);
    return set_error(OURO_E_ARG, msg);
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES)
    return set_error(OURO_E_HIP, "attention_bwd_noalloc: no current device (or more than 64 devices)");
  if (!g_scratch_ptr[dev]) {
    // the array's name is a host-side stand-in: its address on the current device comes from the runtime
    float* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return set_error(OURO_E_HIP, "attention_bwd_noalloc: hipGetSymbolAddress failed");
    g_scratch_ptr[dev] = ptr;
  }
  float* ws = g_scratch_ptr[dev];
  // the array keeps the previous call's contents: start the part in use from zero (a fill kernel, not a memset
  // node, so that the call can be captured into a graph)
  if (launch_fill_zero((hipStream_t)stream, ws, need * sizeof(float)) != hipSuccess) return set_error(OURO_E_HIP, "attention_bwd_noalloc: clear failed");
  return ouro_op_attention_bwd(stream, dtype, B, H, T, S, dh, Mv, scale, q, ldq, k, ldk, v, ldv, o, ldo, lse, d_o, lddo, dq, lddq,
                               dk, lddk, dv, lddv, rel, u, vb, r, ldr, du, dvb, dr, ws, force_generic);
}

extern "C" int ouro_op_layernorm_fwd(void* stream, int dtype, const void* x, const float* g, const float* b, void* y,
                                     float* mean, float* rstd, int rows, int d, int dn) {
  if (!x || !g || !b || !y || !mean || !rstd || rows < 0 || d < 1 || dn < 0 || dn > d || dtype < 0 || dtype > 2) return OURO_E_ARG;
  return rc_of(launch_layernorm_fwd((hipStream_t)stream, dtype, x, g, b, y, mean, rstd, rows, d, dn));
}

extern "C" int ouro_op_layernorm_bwd(void* stream, int dtype, const void* dy, const void* x, const float* g,
                                     const float* mean, const float* rstd, void* dx, float* dg, float* db, int rows,
                                     int d, int dn) {
  if (!dy || !x || !g || !mean || !rstd || !dx || !dg || !db || rows < 0 || d < 1 || dn < 0 || dn > d || dtype < 0 || dtype > 2) return OURO_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (launch_fill_zero(s, dg, (size_t)d * 4) != hipSuccess || launch_fill_zero(s, db, (size_t)d * 4) != hipSuccess) return OURO_E_HIP;
  return rc_of(launch_layernorm_bwd(s, dtype, dy, x, g, mean, rstd, dx, dg, db, rows, d, dn, true));
}

extern "C" int ouro_op_colsum(void* stream, int dtype, const void* x, int ldx, float* out, int rows, int cols) {
  if (!x || !out || ldx < cols) return OURO_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (launch_fill_zero(s, out, (size_t)cols * 4) != hipSuccess) return OURO_E_HIP;
  return rc_of(launch_colsum(s, dtype, x, ldx, out, rows, cols));
}

extern "C" int ouro_op_embed_fwd(void* stream, int dtype, const int32_t* tok, const void* V, const float* pe, void* h,
                                 int N, int T, int d, int vocab, float scale, int* flag) {
  if (!tok || !V || !h || !flag || N < 0 || T < 1) return OURO_E_ARG;
  return rc_of(launch_embed_fwd((hipStream_t)stream, dtype, tok, V, pe, h, N, T, d, vocab, scale, flag));
}

extern "C" int ouro_op_embed_bwd(void* stream, int dtype, const int32_t* tok, const void* dh, float* dVi, int N, int d,
                                 int vocab, float scale) {
  if (!tok || !dh || !dVi) return OURO_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (launch_fill_zero(s, dVi, (size_t)vocab * d * 4) != hipSuccess) return OURO_E_HIP;
  return rc_of(launch_embed_bwd(s, dtype, tok, dh, dVi, N, d, vocab, scale));
}

extern "C" int ouro_op_softmax_ce(void* stream, int dtype, const void* logits, int ld, const int32_t* tgt, void* G,
                                  int ldg, float* lse, float* rowloss, float* loss, int N, int vocab, int* flag) {
  if (!logits || !tgt || !G || !lse || !rowloss || !loss || !flag || N < 1 || ld < vocab || ldg < vocab) return OURO_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = launch_ce_rows(s, dtype, logits, ld, tgt, G, ldg, lse, rowloss, N, vocab, flag);
  if (e == hipSuccess) e = launch_sum_rows(s, rowloss, N, loss);
  return rc_of(e);
}

extern "C" int ouro_op_update(void* stream, float* w, float* m, float* v, void* shadow, const float* g0, float s0,
                              const float* g1, float s1, size_t n, int adam, float lr, float beta1, float beta2,
                              float eps, int64_t t) {
  if (!w || (adam && (!m || !v)) || t < 0) return OURO_E_ARG;
  UpdateDesc u;
  memset(&u, 0, sizeof u);
  u.w = w; u.m = m; u.v = v; u.shadow = (bf16_t*)shadow; u.g0 = g0; u.g1 = g1; u.gscale0 = s0; u.gscale1 = s1;
  u.n = n; u.adam = adam; u.lr = lr; u.beta1 = beta1; u.beta2 = beta2; u.eps = eps;
  u.bc1 = (float)(1.0 - std::pow((double)beta1, (double)(t + 1)));
  u.bc2 = (float)(1.0 - std::pow((double)beta2, (double)(t + 1)));
  return rc_of(launch_update((hipStream_t)stream, u));
}

extern "C" int ouro_op_from_f32(void* stream, int dtype, void* dst, const float* src, size_t n) {
  if (!dst || !src) return OURO_E_ARG;
  return rc_of(launch_convert((hipStream_t)stream, dtype, dst, src, n));
}
extern "C" int ouro_op_to_f32(void* stream, int dtype, float* dst, const void* src, size_t n) {
  if (!dst || !src) return OURO_E_ARG;
  return rc_of(launch_to_f32((hipStream_t)stream, dtype, dst, src, n));
}
