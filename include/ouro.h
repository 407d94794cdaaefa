/* ouro.h -- C boundary of the MI355X (gfx950) Ouroboros training-step library.
 *
 * One training iteration of a Transformer language model whose L layers are split
 * into K contiguous modules G(1..K) (paper Section 3.1).  Every iteration runs the
 * forward pass (Eq. 1-4) and backpropagation (Eq. 6-7) of the current mini-batch at the
 * current weights, parks each module's weight gradient in a per-module ring, and
 * updates module k with the gradient computed K-k iterations earlier (Eq. 8), and the
 * tied embedding/softmax matrix V with half the fresh output-projection gradient
 * plus half the input-embedding gradient from K-1 iterations earlier (Eq. 9), using
 * SGD (Algorithm 1) or Adam (Algorithm 2, appendix).
 *
 * Conventions
 *   - Every function returns OURO_OK (0) or a negative OURO_E_* code; nothing throws
 *     or aborts.  ouro_last_error() returns a description of the last failure of the
 *     calling thread.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *   - The caller owns the device arena and the HIP stream.  The library carves the
 *     arena and allocates no device memory itself.  ouro_create_model also creates
 *     internal non-blocking streams and events of default priority (two streams per
 *     model, plus two per module above the first under schedule = 1) for work that may
 *     run beside the caller's stream.  Ordering contract: every call first orders its
 *     work after whatever the caller's stream holds at entry; ouro_step, ouro_eval_step
 *     and the last ouro_delayed_update of an iteration join all internal streams back
 *     into the caller's stream before they return, and so does every module-level call
 *     for what a later call or a read through this interface depends on.  Work the
 *     caller enqueues on the caller's stream after such a call therefore sees its
 *     results; between the module-level calls of one iteration the arena is in use by
 *     internal streams and must only be touched through this interface.  The caller's
 *     own other streams are not ordered against the arena.
 *     Calls return after enqueueing unless stated otherwise.
 *   - A model object is not thread-safe; use one thread per model.
 *   - Only gfx950 code is built; there is no host fallback: without a usable GPU,
 *     ouro_create_model fails with OURO_E_HIP.
 */
#ifndef OURO_H
#define OURO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  OURO_OK = 0,
  OURO_E_CONFIG = -1,   /* invalid configuration field or combination           */
  OURO_E_ARG = -2,      /* null pointer, wrong length, index out of range        */
  OURO_E_ARENA = -3,    /* arena too small or misaligned (256 B)                 */
  OURO_E_SEQUENCE = -4, /* call order violates the per-iteration contract        */
  OURO_E_TOKEN = -5,    /* a token or target id was outside [0, vocab)           */
  OURO_E_STALE = -6,    /* a ring slot's tag did not match the iteration wanted  */
  OURO_E_HIP = -7       /* a HIP runtime call or kernel launch failed            */
};

typedef struct ouro_model ouro_model; /* opaque host object */

/* Model and method configuration.  Layer internals (not defined by the paper):
 * post-LayerNorm blocks y = LN(h + Attn(h)), h' = LN(y + FFN(y)); attention
 * projections without bias; FFN = GELU(y W_1 + b_1) W_2 + b_2 with the erf-form
 * GELU x*Phi(x), erf evaluated to 1.5e-7 absolute (a rational approximation) in both dtypes; scores scaled by 1/sqrt(d_head), causal; LayerNorm eps 1e-5; LM head
 * logits = h_L V^T without bias; loss = mean over batch*seq_len targets of the
 * natural-log cross entropy (Eq. 4). */
typedef struct {
  int32_t n_layer, d_model, n_head, d_head, d_ff, vocab; /* n_head*d_head == d_model, d_model even */
  int32_t seq_len;   /* T: tokens per stream per iteration                                  */
  int32_t mem_len;   /* M: Transformer-XL segment memory length (0 = none; needs rel_pos=1)  */
  int32_t batch;     /* B: independent token streams                                         */
  int32_t n_module;  /* K >= 1, K <= n_layer                                                 */
  const int32_t* layers_per_module; /* host, K entries summing to n_layer; NULL = contiguous
                                       split, remainder to the interior modules first        */
  int32_t rel_pos;   /* 0: fixed sinusoid positions added to the embedding;
                        1: Transformer-XL relative attention (per-layer W_r, u, v)           */
  int32_t dtype;     /* 0: fp32 weights and activations;
                        1: bf16 weights/activations, fp32 accumulation, statistics,
                           gradients slots, master weights and moments                      */
  int32_t optimizer; /* 0: SGD (Algorithm 1); 1: Adam (Algorithm 2)                          */
  float beta1, beta2, eps; /* Adam constants (Algorithm 2: 0.9, 0.999, 1e-8)                 */
  int32_t embed_warm_mode; /* Eq. 9 while t-K+1 < 0.  0: g_V = 0 (literal);
                              1: only the input-embedding term is dropped                   */
  float emb_scale;   /* factor on the embedding lookup (1.0)                                */
  int32_t schedule;  /* 0: Eq. 8 to the letter: the gradient of mini-batch t-K+k at the full
                           weights of iteration t-K+k, kept in a ring of gradients;
                        1: the memory-saving schedule of Section 3.1 ("Memory Consumption"):
                           each module keeps its inputs instead, recomputes its activations
                           of mini-batch t-K+k with the weights it holds at iteration t and
                           back-propagates the error gradient its upper neighbour produced
                           at iteration t-1; segment memories are stored with the inputs     */
  float dropout;     /* p in [0, 1): inverted dropout on the embedding sum and on the outputs of
                        the attention projection and of the feed-forward block, before the
                        residual additions (0 = none).  Section 5.2, "Repeatable Dropout": the
                        mask is a pure function of (seed + iteration of the mini-batch, place,
                        element), so a recomputation reproduces it                          */
  uint64_t seed;     /* dropout seed of iteration 0; iteration t uses seed + t               */
} ouro_config;

/* Parameter groups: group 0 is V [vocab, d_model]; group k = 1..K is module k.
 * A module blob is its layers in order, each layer (row-major fp32):
 *   W_qkv[d,3d], W_o[d,d], (rel_pos only: W_r[d,d], u[H,d_head], v[H,d_head]),
 *   ln1_g[d], ln1_b[d], W_1[d,F], b_1[F], W_2[F,d], b_2[d], ln2_g[d], ln2_b[d].
 * Linear maps are y = x W with W stored [in, out].
 * Gradient stores use the same ids plus OURO_GRAD_VO(K) = K+1:
 *   id 0 = ring of dV_i (depth K), id k = ring of module k (depth K-k+1),
 *   id K+1 = dV_o of the current iteration (depth 1). */
#define OURO_GROUP_V 0

const char* ouro_last_error(void);

/* Bytes of device arena needed for cfg (256-byte aligned base).  Host only. */
int ouro_query_arena_bytes(const ouro_config* cfg, size_t* bytes);

/* Validates cfg, lays out the arena (dev pointer, at least `bytes` from the query),
 * zeroes optimizer state, gradient rings and memories, and returns a model in *out.
 * hip_stream is a hipStream_t (NULL = the null stream).  Parameters are undefined
 * until ouro_set_params has been called for every group. */
int ouro_create_model(const ouro_config* cfg, void* dev_arena, size_t bytes, void* hip_stream,
                      ouro_model** out);
/* Synchronises the stream and frees the host object; never frees the arena. */
int ouro_destroy_model(ouro_model* m);

int ouro_param_count(const ouro_model* m, int group, int64_t* n);
/* Copies n fp32 values (n must equal the group's count) into the master weights and,
 * in bf16 mode, refreshes the bf16 copy.  src is host memory unless src_is_device.
 * Blocking for host sources. */
int ouro_set_params(ouro_model* m, int group, const float* src, int64_t n, int src_is_device);
/* Copies the fp32 master weights out; synchronises the stream for host destinations. */
int ouro_get_params(ouro_model* m, int group, float* dst, int64_t n, int dst_is_device);

/* --- the iteration (Algorithm 1 / 2, inner loop), iteration counter t starts at 0 ---
 * Contract inside iteration t (else OURO_E_SEQUENCE):
 *   module_forward k = 1..K ascending; module_backward k = K..1 descending after
 *   forward K; delayed_update once for each group 0..K, any order, after backward 1.
 *   The last of the K+1 updates closes the iteration: segment memories roll and t
 *   becomes t+1.  Under this order no update of iteration t reads anything another
 *   update of iteration t writes, so the result equals the "for k in parallel" loop.
 *
 * ouro_module_forward: k==1 reads dev_tokens (int32 [batch, seq_len]) and looks up the
 *   embedding with V^t (Eq. 1); runs the layers of G(k) (Eq. 2); k==K reads dev_targets
 *   (int32 [batch, seq_len]) and evaluates the loss through V^t (Eq. 3-4).  The buffers
 *   stay owned by the caller and must remain valid until the stream has passed
 *   module_backward(1) of the same iteration.  Unused pointers may be NULL.
 * ouro_module_backward: Eq. 6-7 for the layers of G(k) at w^t; k==K also produces
 *   dV_o(t); k==1 also produces dV_i(t).  Writes ring slot t mod depth, tagged t.
 * ouro_delayed_update: group k in 1..K applies Eq. 8: gradient slot of iteration
 *   t-(K-k), or a zero gradient while that is negative; group 0 applies Eq. 9.
 *   lr is gamma_t of the current iteration.
 * ouro_step: all of the above for one mini-batch.  If host_loss is not NULL the
 *   stream is synchronised and the loss (and OURO_E_TOKEN, if any id was out of
 *   range; such ids are skipped, never dereferenced) is returned.
 *
 * schedule = 1 keeps the same calls and order.  module_forward(k), k < K, also stores the
 *   module's input (token ids for k = 1) in a ring of depth K-k+1, tagged t.
 *   module_backward(k), k < K, does nothing while t-K+k < 0; otherwise it recomputes the
 *   module's activations from the stored input of iteration t-K+k (OURO_E_STALE if the slot's
 *   tag differs) with the current weights, takes the error gradient module k+1 left at
 *   iteration t-1 and writes the gradient store of module k (depth 1, tagged t) and the error
 *   gradient for module k-1 (k = 1: dV_i of mini-batch t-K+1).  The token buffer of
 *   iteration t may be released once module_forward(1) has run on the stream.
 *   delayed_update applies what this iteration computed (zero while t-K+k < 0; Eq. 9 for V). */
int ouro_module_forward(ouro_model* m, int k, const int32_t* dev_tokens, const int32_t* dev_targets);
int ouro_module_backward(ouro_model* m, int k);
int ouro_delayed_update(ouro_model* m, int group, float lr);
int ouro_step(ouro_model* m, const int32_t* dev_tokens, const int32_t* dev_targets, float lr,
              float* host_loss);
/* --- evaluation and checkpoints ---
 * ouro_eval_step: a forward-only iteration with the current weights: the loss of the mini-batch
 *   (Eq. 4; bits per character = loss / ln 2, perplexity = exp(loss)), no dropout, no gradient,
 *   no update, nothing stored for a later backward pass.  Segment memories roll and the
 *   iteration counter advances as after a training iteration, so a stream of consecutive
 *   segments is evaluated with carried-over memory; evaluate on a model of its own (it may have
 *   a longer mem_len than the training model; copy the weights with ouro_get_params /
 *   ouro_set_params on device pointers), not between the training iterations of one model.
 *   Only at an iteration boundary (OURO_E_SEQUENCE otherwise).
 * ouro_state_bytes / ouro_save_state / ouro_load_state: the whole training state at an
 *   iteration boundary as one host buffer: iteration counter, master weights and their bf16
 *   copies, Adam moments, every gradient and input ring with its tags (the pending stale
 *   gradients), error-gradient mailboxes, segment memories.  A model created with the same
 *   configuration continues from a loaded state exactly where the saved one stood.  bytes must
 *   equal ouro_state_bytes; a buffer of another configuration is refused (OURO_E_CONFIG).
 *   Both calls synchronise the model's streams. */
int ouro_eval_step(ouro_model* m, const int32_t* dev_tokens, const int32_t* dev_targets, float* host_loss);
int ouro_state_bytes(const ouro_model* m, size_t* bytes);
int ouro_save_state(ouro_model* m, void* host_dst, size_t bytes);
int ouro_load_state(ouro_model* m, const void* host_src, size_t bytes);

/* Loss of the most recent forward of module K; synchronises the stream. */
int ouro_get_loss(ouro_model* m, float* host_loss);
int64_t ouro_current_step(const ouro_model* m);

/* --- staleness contract: pure host integer function, usable without a GPU ---
 * For K modules, group id (0 = dV_i ring, 1..K = module rings, K+1 = dV_o) and
 * iteration t: write != 0 gives the slot written at t (*tau = t); write == 0 gives the
 * slot read by the update of iteration t and the iteration *tau whose gradient it holds
 * (Eq. 8: t-K+k; Eq. 9: t-K+1 for dV_i, t for dV_o), or *slot = -1, *tau = -1 when the
 * rule prescribes a zero gradient. */
int ouro_slot_index(int K, int id, int64_t t, int write, int64_t* slot, int64_t* tau);
int ouro_ring_depth(int K, int id, int64_t* depth);

/* --- step size (Section 5.2: gradual warm-up, then a cosine schedule); pure host function ---
 * *lr = gamma_t for iteration t >= 0: base*(t+1)/warmup while t < warmup; then
 * floor + (base-floor)*(1+cos(pi*(t-warmup)/(total-warmup)))/2 until t = total; floor from
 * there on.  Requires 0 <= warmup < total (warmup = 0: no warm-up) and 0 <= floor <= base;
 * OURO_E_ARG otherwise.  The caller passes the result to ouro_step / ouro_delayed_update, which
 * take the step size per call (a stale gradient is applied with the current gamma_t). */
int ouro_lr_schedule(double base, int64_t warmup, int64_t total, double floor, int64_t t, double* lr);

/* --- test / debug surface --- */
int ouro_debug_slot_tag(ouro_model* m, int id, int64_t slot, int64_t* tag); /* -1 = never written */
int ouro_debug_last_read(ouro_model* m, int id, int64_t* slot, int64_t* tau);
/* schedule = 1: tag (iteration, -1 = never written) of slot `slot` of module k's input ring, and
 * the slot and mini-batch the last module_backward(k) recomputed from (-1, -1: it computed nothing). */
int ouro_debug_input_tag(ouro_model* m, int k, int64_t slot, int64_t* tag);
int ouro_debug_last_input_read(ouro_model* m, int k, int64_t* slot, int64_t* tau);
/* Stands in for forward+backward of the current iteration: writes the fp32 host vector g
 * (the store's element count) as store `id`'s gradient of iteration t.  After all K+2
 * stores are injected the iteration is in the "backward done" state. */
int ouro_debug_inject_grad(ouro_model* m, int id, const float* host_g, int64_t n);
/* Copies the gradient that store `id` holds for iteration tau to host memory
 * (OURO_E_STALE if it has been overwritten); synchronises the stream. */
int ouro_get_grad_slot(ouro_model* m, int id, int64_t tau, float* host_dst, int64_t n);
/* Segment memory of a layer as fp32 [batch, valid_len, d_model]; *valid_len is returned.
 * host_dst may be NULL to query the length only. */
int ouro_get_mems(ouro_model* m, int layer, float* host_dst, int64_t* valid_len);
/* Input activation of a layer (0-based), or with layer == n_layer the final hidden
 * state, of the latest forward, as fp32 [batch*seq_len, d_model]. */
int ouro_debug_get_hidden(ouro_model* m, int layer, float* host_dst, int64_t n);
/* Optional per-launch HIP event timing on the model's stream (slows the step while on).
 * OURO_TIMING_CONTRACTION: the MFMA contraction kernel, work = 2*M*N*K flops per launch;
 * OURO_TIMING_UPDATE: the delayed-update kernel (zero-gradient warm-up launches excluded), work =
 *         algorithmic bytes (gradient reads 4 B each, w 8 B, Adam moments 16 B, bf16 copy 2 B);
 * OURO_TIMING_ATTENTION: attention forward and backward launches, work = algorithmic flops
 *         (visible query-key pairs x 4 d_head forward, 6 d_head with the relative-position term;
 *         a backward launch counts twice its forward);
 * OURO_TIMING_LAYERNORM: LayerNorm forward and input-gradient launches, work = bytes (rows read
 *         and written in the activation type, 8 B of statistics per row);
 * OURO_TIMING_CE_ROWS: the row pass of the softmax cross entropy, work = bytes (logits read once,
 *         the logit gradient written once).
 * timing_read synchronises the stream, returns the totals since the last read of that
 * kind and resets them. */
enum { OURO_TIMING_CONTRACTION = 0, OURO_TIMING_UPDATE = 1, OURO_TIMING_ATTENTION = 2, OURO_TIMING_LAYERNORM = 3,
       OURO_TIMING_CE_ROWS = 4, OURO_TIMING_KINDS = 5 };
int ouro_debug_timing_enable(ouro_model* m, int on);
/* Stream overlap switch. on = 1 (default): weight-gradient contractions run on a second
 * stream beside the error-gradient chain and ouro_step enqueues each module's update behind
 * its backward pass on a third. on = 0: every kernel runs on the model's stream in program
 * order, so a HIP-event bracket or a profiler's kernel duration measures that kernel alone.
 * The results are the same in both modes up to the order of atomic float additions. Call it
 * between iterations; it drains the extra streams. */
int ouro_debug_set_overlap(ouro_model* m, int on);
int ouro_debug_timing_read(ouro_model* m, int kind, double* ms, int64_t* launches, double* work);
/* Cost of one timing bracket by itself: enqueues `reps` (at most 4096) empty brackets (two
 * event records with nothing between them) back to back on the model's stream and returns their
 * mean elapsed time in milliseconds. A bracket around a kernel reads that kernel's duration plus
 * this event-marker cost, so callers subtract it to compare with a profiler's kernel durations. */
int ouro_debug_timing_overhead(ouro_model* m, int reps, double* ms_mean);

#ifdef __cplusplus
}
#endif
#endif /* OURO_H */
