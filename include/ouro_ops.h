/* ouro_ops.h -- single-kernel entry points of libouro, for per-kernel parity tests and
 * micro-benchmarks.  Every pointer is a device address unless named host_*; work is
 * enqueued on `stream` (a hipStream_t, NULL = null stream) and the call returns at once.
 * dtype: 0 = fp32 elements, 1 = bf16 elements ("T" below).  Returns OURO_OK or a negative
 * OURO_E_* code (see ouro.h); buffers are owned by the caller.
 */
#ifndef OURO_OPS_H
#define OURO_OPS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = alpha * op(A) op(B) with fp32 accumulation, then
 *   + bias[n] (fp32, may be NULL); epilogue 1: Z = v (type T), v = GELU(v);
 *   epilogue 2: v *= GELU'(Z) ; + residual[m,n] (type T, may be NULL); stored as T, or
 *   as fp32 when out_fp32; accumulate != 0 adds atomically into fp32 C instead
 *   (no bias / residual / epilogue then).
 * transA == 0: A is [M,K] row-major with leading dimension lda; 1: A is [K,M].
 * transB == 0: B is [K,N]; 1: B is [N,K].  force_generic: 0 = automatic kernel choice, 1 = the
 * plain tiled kernel, 10..14 = one MFMA tile configuration (10 register-staged 128x128,
 * 11 direct-to-LDS 128x128, 12 direct-to-LDS 128x64, 13 register-prefetch 128x128 with a
 * four-stage ring, 14 direct-to-LDS 256x256; 11..14 fall back to 10 unless K % 64 == 0),
 * for tests and tuning.
 * These are the layer contractions of Eq. 2 / Eq. 6 (forward, input- and weight-gradient). */
int ouro_op_gemm(void* stream, int dtype, int transA, int transB, int M, int N, int K, float alpha,
                 const void* A, int lda, const void* B, int ldb, void* C, int ldc, int out_fp32,
                 int accumulate, const float* bias, const void* residual, int ldr, int epilogue,
                 void* Z, int ldz, int force_generic);
/* A grid of by x bz products of one shape in one call (plain epilogue): product (y, z) reads
 * A + y*sAy + z*sAz and B + y*sBy + z*sBz and writes C + y*sCy + z*sCz (strides in elements).
 * With C2 != NULL a second grid of the same shape, strides and leading dimensions runs in the
 * same launch with A2, B2, C2, alpha2.  bf16 products with K % 64 == 0 and 16-byte aligned
 * strides run as one launch of the MFMA kernel, anything else as one launch per product.
 * accumulate: 0 C = alpha A B; 1 fp32 C += alpha A B with the contraction split over workgroups
 * (atomic adds); 2 fp32 C += alpha A B in the epilogue of a single pass (one grid only).
 * The relative-position attention backward forms dK, dV (Eq. 6 inside the attention block) this
 * way, and adds the input gradient of the key / value projection over the current rows of every
 * batch element (the memory rows of [memory ; segment] are constants) with accumulate = 2. */
int ouro_op_gemm_batched(void* stream, int dtype, int transA, int transB, int M, int N, int K, float alpha,
                         const void* A, int lda, const void* B, int ldb, void* C, int ldc, int out_fp32,
                         int accumulate, int by, int bz, long long sAy, long long sAz, long long sBy,
                         long long sBz, long long sCy, long long sCz, const void* A2, const void* B2,
                         void* C2, float alpha2, int force_generic);
/* n <= 6 accumulating products C_i (fp32 [M_i, N_i]) += alpha * A_i^T B_i with A_i [K_i, M_i] and
 * B_i [K_i, N_i] (the weight-gradient contractions of a layer, Eq. 6-7: contraction over all
 * tokens onto small outputs).  Products that admit it (bf16, K_i a multiple of 64 and >= 512) share
 * one launch in which every workgroup takes a long K range; the rest run one by one. */
int ouro_op_gemm_group(void* stream, int dtype, int n, const int* M, const int* N, const int* K,
                       const void* const* A, const int* lda, const void* const* B, const int* ldb,
                       float* const* C, const int* ldc, float alpha);
/* 1 if ouro_op_gemm would run the MFMA kernel for these arguments (host only). */
int ouro_op_gemm_uses_mfma(int dtype, int transA, int transB, int M, int N, int K, const void* A,
                           int lda, const void* B, int ldb);

/* Causal attention over [memory ; segment].  q, o, d_o, dq: rows b*T+i; k, v, dk, dv: rows
 * b*S+j with S = Mv+T; head h in columns [h*dh, (h+1)*dh) of a row (ld* in elements).
 * Query i sits at position Mv+i and sees keys j <= Mv+i.  lse: fp32 [B,H,T].
 * rel != 0: score = ((q+u_h).k_j + (q+vb_h).r_h[Mv+i-j]) * scale, with u, vb [H,dh] (T) and
 * r [S, H*dh] (T) indexed by distance; else score = q.k_j * scale. */
int ouro_op_attention_fwd(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv,
                          float scale, const void* q, int ldq, const void* k, int ldk,
                          const void* v, int ldv, void* o, int ldo, float* lse, int rel,
                          const void* u, const void* vb, const void* r, int ldr, int force_generic);
/* Backward of the above.  du, dvb (fp32 [H,dh]) and dr (fp32 [S, H*dh]) are overwritten when
 * rel != 0 (may be NULL otherwise).  scratch: fp32, ouro_op_attention_bwd_scratch() floats,
 * 16-byte aligned: enough for either form (with rel != 0, bf16 and dh == 64 the pass leaves the
 * probabilities and score gradients there, about B*H*S*T floats, and forms dk, dv and dr from
 * them). */
int ouro_op_attention_bwd(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv,
                          float scale, const void* q, int ldq, const void* k, int ldk,
                          const void* v, int ldv, const void* o, int ldo, const float* lse,
                          const void* d_o, int lddo, void* dq, int lddq, void* dk, int lddk,
                          void* dv, int lddv, int rel, const void* u, const void* vb, const void* r,
                          int ldr, float* du, float* dvb, float* dr, float* scratch, int force_generic);
size_t ouro_op_attention_bwd_scratch(int B, int H, int T, int S, int dh);
/* ouro_op_attention_bwd for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same arguments without
 * `scratch`; the workspace is a device array inside the library, 4 Mi floats (16 MiB) on every
 * GPU the library runs on, held until the process ends.  Sizes that need more than 4194304
 * floats (rel != 0: ouro_op_attention_bwd_scratch(); rel == 0: 2*B*S*H*dh + 2*B*H*T) are refused
 * with OURO_E_ARG (ouro_last_error says how much was needed).  The call allocates and frees nothing; it clears
 * the part of the workspace it uses with a fill kernel on `stream`, then enqueues the same
 * kernels as ouro_op_attention_bwd.  All calls on one GPU share that GPU's workspace: calls
 * that may overlap on one GPU (different streams, different threads) race; keep them on one
 * stream or order them with events. */
int ouro_op_attention_bwd_noalloc(void* stream, int dtype, int B, int H, int T, int S, int dh, int Mv,
                                  float scale, const void* q, int ldq, const void* k, int ldk,
                                  const void* v, int ldv, const void* o, int ldo, const float* lse,
                                  const void* d_o, int lddo, void* dq, int lddq, void* dk, int lddk,
                                  void* dv, int lddv, int rel, const void* u, const void* vb, const void* r,
                                  int ldr, float* du, float* dvb, float* dr, int force_generic);

/* Repeatable dropout (Section 5.2): dst[r,c] = src[r,c] * f(r*drop_ld + c), f(i) = 1/(1-p) if the high
 * 32 bits of output i + stream_id*2^40 + 1 of the SplitMix64 sequence started at `seed` are >=
 * floor(p*2^32), else 0.  rows x cols elements of type T, row stride ld on both sides; 0 <= p < 1. */
int ouro_op_dropout(void* stream, int dtype, const void* src, void* dst, int rows, int cols, int ld,
                    float p, uint64_t seed, uint32_t stream_id, int drop_ld);
/* C = dropout(op(A) op(B) + bias) + residual with the mask above at element index m*drop_ld + n
 * (the fused form the layers use for the attention projection and the feed-forward output).
 * C, residual type T; bias fp32 or NULL; residual may be NULL. */
int ouro_op_gemm_dropout(void* stream, int dtype, int transA, int transB, int M, int N, int K,
                         const void* A, int lda, const void* B, int ldb, void* C, int ldc, const float* bias,
                         const void* residual, int ldr, float p, uint64_t seed, uint32_t stream_id, int drop_ld,
                         int force_generic);

/* C = op(A) op(B) + bias + R, the form of the two contractions of a block that close a residual
 * connection, with the residual taken from fp32: R[m,n] = res32[m,n] when mean is NULL, else the
 * LayerNorm of res32 recomputed in place, (res32[m,n] - mean[m]) * rstd[m] * g[n] + b[n] (a block's
 * input is the LayerNorm of the sum before it; its stored, rounded copy is only the contraction
 * operand).  res32 fp32 [M, ldr32]; mean, rstd fp32 [M]; g, b fp32 [N]; C type T or fp32 (out_fp32). */
int ouro_op_gemm_ln_residual(void* stream, int dtype, int transA, int transB, int M, int N, int K,
                             const void* A, int lda, const void* B, int ldb, void* C, int ldc, int out_fp32,
                             const float* bias, const float* res32, int ldr32, const float* mean,
                             const float* rstd, const float* g, const float* b, int force_generic);

/* y = (x-mean)*rstd*g + b over rows of d (biased variance, eps 1e-5); g, b, mean, rstd fp32.
 * The two LayerNorm calls also take dtype 2: rows read (x, and dy in the backward call) are fp32,
 * rows written (y, dx) bf16 -- the form the bf16 model runs, whose sums entering a LayerNorm and
 * whose gradients of the normalised rows stay in fp32.
 * dn in (0, d): the statistics run over the first dn columns only and the other d-dn columns are
 * zero padding (x, g, b zero there; y then is zero there too).  dn = 0 means dn = d. */
int ouro_op_layernorm_fwd(void* stream, int dtype, const void* x, const float* g, const float* b,
                          void* y, float* mean, float* rstd, int rows, int d, int dn);
/* dx (T) and dg, db (fp32 [d], overwritten).  dn as above; dx is zero in the padding columns. */
int ouro_op_layernorm_bwd(void* stream, int dtype, const void* dy, const void* x, const float* g,
                          const float* mean, const float* rstd, void* dx, float* dg, float* db,
                          int rows, int d, int dn);
/* out[c] = sum_r x[r,c]  (fp32 [cols], overwritten). */
int ouro_op_colsum(void* stream, int dtype, const void* x, int ldx, float* out, int rows, int cols);
/* h[n,:] = scale*V[tok[n],:] (+ pe[n%T,:], fp32, may be NULL).  *flag (device int) gets bit 0 set
 * for ids outside [0,vocab), whose rows become zero (Eq. 1). */
int ouro_op_embed_fwd(void* stream, int dtype, const int32_t* tok, const void* V, const float* pe,
                      void* h, int N, int T, int d, int vocab, float scale, int* flag);
/* dVi (fp32 [vocab,d], overwritten) = scatter-add of scale*dh rows (Eq. 7, left). */
int ouro_op_embed_bwd(void* stream, int dtype, const int32_t* tok, const void* dh, float* dVi,
                      int N, int d, int vocab, float scale);
/* Rows of logits [N, ld] (type T): lse[n]; rowloss[n] = lse - logit[tgt]; G (T, [N, ldg]) =
 * (softmax - onehot)/N, which may be the logits buffer itself (in place); *loss =
 * mean(rowloss) (Eq. 4).  flag bit 1: target out of range. */
int ouro_op_softmax_ce(void* stream, int dtype, const void* logits, int ld, const int32_t* tgt,
                       void* G, int ldg, float* lse, float* rowloss, float* loss, int N, int vocab,
                       int* flag);
/* Algorithm 1 (adam == 0) or Algorithm 2 on n fp32 elements with g = s0*g0 + s1*g1 (NULL = 0);
 * t is the global iteration (bias correction 1-beta^(t+1)); shadow (bf16 copy of w) may be NULL. */
int ouro_op_update(void* stream, float* w, float* m, float* v, void* shadow, const float* g0,
                   float s0, const float* g1, float s1, size_t n, int adam, float lr, float beta1,
                   float beta2, float eps, int64_t t);
/* dst (type T) = src (fp32), n elements; and back. */
int ouro_op_from_f32(void* stream, int dtype, void* dst, const float* src, size_t n);
int ouro_op_to_f32(void* stream, int dtype, float* dst, const void* src, size_t n);

#ifdef __cplusplus
}
#endif
#endif
