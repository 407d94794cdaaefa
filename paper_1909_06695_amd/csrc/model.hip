// Host side of the C boundary: configuration checks, arena layout, the per-iteration
// call contract, the staleness rings (Eq. 8-9) and the sequence of kernel launches that
// make up module_forward / module_backward / delayed_update.
#include "common.h"
#include "../../include/ouro.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace ouro;

static thread_local std::string g_err;
static int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
#define HIPCHK(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return fail(OURO_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

extern "C" const char* ouro_last_error(void) { return g_err.c_str(); }
namespace ouro {
int set_error(int code, const char* msg) { g_err = msg ? msg : ""; return code; }
}

// ------------------------------------------------------------------ staleness integers
// Eq. 8: module k at iteration t consumes the gradient of iteration t-K+k.  A ring of
// K-k+1 slots is enough: slot (t mod depth) is written at t and read K-k iterations
// later, just before it would be overwritten.  Eq. 9: dV_i of iteration t-K+1 (ring of K
// slots) and dV_o of iteration t (one slot).
extern "C" int ouro_ring_depth(int K, int id, int64_t* depth) {
  if (!depth || K < 1 || id < 0 || id > K + 1) return fail(OURO_E_ARG, "ring_depth: bad K=%d id=%d", K, id);
  if (id == 0) *depth = K;
  else if (id == K + 1) *depth = 1;
  else *depth = K - id + 1;
  return OURO_OK;
}

extern "C" int ouro_slot_index(int K, int id, int64_t t, int write, int64_t* slot, int64_t* tau) {
  int64_t depth;
  if (!slot || !tau || t < 0) return fail(OURO_E_ARG, "slot_index: bad argument");
  int rc = ouro_ring_depth(K, id, &depth);
  if (rc) return rc;
  int64_t want = t;
  if (!write) {
    if (id == 0) want = t - K + 1;
    else if (id <= K) want = t - K + id;
  }
  if (want < 0) { *slot = -1; *tau = -1; return OURO_OK; }
  *slot = want % depth;
  *tau = want;
  return OURO_OK;
}

extern "C" int ouro_lr_schedule(double base, int64_t warmup, int64_t total, double floor, int64_t t, double* lr) {
  if (!lr) return fail(OURO_E_ARG, "lr_schedule: lr is null");
  if (!(warmup >= 0 && warmup < total && t >= 0 && floor >= 0 && floor <= base))
    return fail(OURO_E_ARG, "lr_schedule: need 0 <= warmup < total, t >= 0, 0 <= floor <= base");
  if (t < warmup) *lr = base * (double)(t + 1) / (double)warmup;
  else if (t >= total) *lr = floor;
  else *lr = floor + (base - floor) * 0.5 * (1.0 + std::cos(M_PI * (double)(t - warmup) / (double)(total - warmup)));
  return OURO_OK;
}

// ------------------------------------------------------------------------------ layout
struct LayerOff {   // element offsets inside a module blob
  size_t W_qkv, W_o, W_r, u, v, ln1_g, ln1_b, W_1, b_1, W_2, b_2, ln2_g, ln2_b, end;
};
// Offsets of one layer's tensors, in the documented order, for a model width d, a joint width
// hd of all heads (n_head * d_head) and an inner width F.
static LayerOff layer_offsets(bool rel, size_t d, size_t hd, size_t F, size_t base) {
  LayerOff o;
  size_t p = base;
  o.W_qkv = p; p += d * 3 * hd;
  o.W_o = p; p += hd * d;
  o.W_r = o.u = o.v = 0;
  if (rel) {
    o.W_r = p; p += d * hd;
    o.u = p; p += hd;
    o.v = p; p += hd;
  }
  o.ln1_g = p; p += d;
  o.ln1_b = p; p += d;
  o.W_1 = p; p += d * F;
  o.b_1 = p; p += F;
  o.W_2 = p; p += F * d;
  o.b_2 = p; p += d;
  o.ln2_g = p; p += d;
  o.ln2_b = p; p += d;
  o.end = p;
  return o;
}

// One tensor of a parameter group: where it sits in the caller's blob (rows x cols, dense) and in
// the stored one (leading dimension pcols).  A "head" axis runs over n_head slices of d_head
// elements, stored d_head_stored apart.
struct TensorMap {
  size_t loff, poff;
  int rows, cols, pcols;
  bool row_heads, col_heads;
};

struct LayerBuf {   // saved activations of one layer (element type T unless noted)
  char* x;          // input [N, d]
  char* cat;        // [B, Mv+T, d] memory ; input (relative mode with memory)
  char* qkv;        // plain: [N, 3d]; relative: q [N, d] then kv [B*S, 2d]
  char* a;          // attention output before W_o [N, d]
  char* s1;         // x + a W_o  [N, d], fp32 in every mode (see lnk)
  char* y;          // LN1 output [N, d]
  char* z;          // FFN pre-activation [N, F]
  char* uact;       // GELU(z) [N, F]
  char* s2;         // y + FFN [N, d], fp32
  char* r;          // W_r-projected distance table [S, d]
  char* mem;        // segment memory [B, Mv, d] (stored-input schedule: the ring slot in use)
  char* memring;    // stored-input schedule: the memories of iterations t-(K-k) .. t+1, slot = iteration mod memdepth
  size_t memstride;
  int memdepth;
  float *lse, *mean1, *rstd1, *mean2, *rstd2;
};

struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off += (bytes + 255) & ~(size_t)255;
    return o;
  }
};

// What one module's backward pass works with: its streams, the events between them and its
// scratch buffers.  The model's own members of these names are the set in use; under the
// stored-input schedule every module has a set of its own (ouro_model::ctxs), because the K
// backward passes of an iteration are independent and ouro_step runs them side by side.
struct BwdCtx {
  hipStream_t stream;          // the error-gradient chain (set 0: the caller's stream, which also carries the forward pass)
  // Weight-gradient GEMMs and bias column sums only feed the gradient ring, so they run on
  // a second stream beside the error-gradient chain (both default priority); events order
  // them against the producers of their operands and against the reuse of those buffers.
  hipStream_t side;
  hipEvent_t ev_ready[4];      // ds2 / dz / ds1 / dqkv of the current layer written (main)
  hipEvent_t ev_side_done[2];  // side work that reads buffer set p finished
  bool side_busy[2];
  hipEvent_t ev_join;
  hipEvent_t ev_done;          // sets 1..: this module's backward pass and update are enqueued up to here
  // backward scratch
  char *dhb[3], *dy[2], *da, *dcat, *dr_t[2];   // layer l reads dhb[l % 3], writes dhb[(l + 2) % 3]; dhb and dy are fp32
  // gradients that the weight-gradient GEMMs read on the side stream: two sets, by layer parity
  char *ds2[2], *dz[2], *ds1[2], *dqkv[2];
  char *ds2m[2], *ds1m[2];         // ds2 / ds1 times the dropout masks (the same buffers without dropout)
  float *attn_scratch, *dr_f32[2];
  int attn_scratch_Mv;           // relative mode: memory length of the passes since the workspace was last cleared (-1: none)
  char* hscratch;                 // output of a recomputed module's last layer (never read)
};

struct ouro_model : BwdCtx {
  std::vector<BwdCtx> ctxs;      // [K] under the stored-input schedule (entry of the set in use is stale), else empty
  int cur_ctx;
  hipEvent_t ev_fwd;             // forward pass of the iteration enqueued (the other sets wait for it)
  ouro_config cfg;
  std::vector<int> lpm;          // layers per module
  std::vector<int> first_layer;  // first layer of module k (index k-1), plus end
  std::vector<int> layer_mod;    // module (1..K) of each layer
  std::vector<LayerOff> loff;    // per layer, offsets inside its module's stored blob
  // Stored widths.  bf16 mode with d_head <= 64 stores every tensor with d_head rounded up to
  // 64, d_model and d_ff rounded up to multiples of 64, the padding zero: the contractions and
  // the attention then run on the MFMA kernels for any such shape.  Zero padding is preserved
  // by every step (a zero weight with a zero gradient stays zero under SGD and Adam), so the
  // results in the unpadded positions are those of the unpadded model.
  bool padded;
  int pd, pdh, phd, pF;           // stored d_model, d_head, n_head * d_head, d_ff
  std::vector<std::vector<TensorMap>> tmap;   // per group 0..K
  std::vector<int64_t> pcount;    // stored elements per group
  char* arena;
  size_t bytes;
  int esz;                        // bytes per activation element
  int N, S;                       // tokens per step, max keys per stream (T + M)
  // parameter groups 0..K
  std::vector<int64_t> count;
  std::vector<float*> master, adam_m, adam_v;
  std::vector<bf16_t*> shadow;
  // bf16 mode: every weight matrix also transposed ([out, in]), at the same offsets, refreshed after
  // each update: y = x W then contracts two operands that are both contiguous along the
  // contraction index, the fastest form of the contraction kernels (the input-gradient
  // contractions already have it with W itself).  V^T (leading dimension = padded vocabulary)
  // serves dh_L = G V.
  std::vector<bf16_t*> shadowT;
  std::vector<std::vector<TransposeEntry>> ttab;
  std::vector<TransposeEntry*> ttab_dev;
  std::vector<int> ttiles;
  // gradient stores 0..K+1
  std::vector<int64_t> gcount, gstride, depth;   // elements per gradient (caller's), slot stride (stored, 256-byte multiple)
  std::vector<float*> ring;
  std::vector<std::vector<int64_t>> tags;
  std::vector<int64_t> last_slot, last_tau;
  // activations
  std::vector<LayerBuf> L;
  char* hL;                       // final hidden state [N, d]
  float* pe;                      // [T, d] fp32 (absolute mode)
  char* rtab;                     // [S, d] distance sinusoids, type T (relative mode)
  char* G;                        // [N, ldv] type T: logits, then overwritten by d loss / d logits
  int ldv;                        // vocab rounded up to 64: leading dimension of G and, in bf16 mode, the
                                  // extent the two contractions over / onto the vocabulary run with (padding is zero)
  float *lse_ce, *rowloss, *loss;
  int* flag;
  uint64_t cur_seed;               // dropout seed of the mini-batch being worked on
  bool eval_mode;                  // inside ouro_eval_step: no dropout, no stored inputs
  size_t persist_end;              // arena[0, persist_end): weights, moments, gradient and input rings, mailboxes
  float* dbg_f32;
  size_t dbg_floats;
  // Gradients of a layer's vectors (LayerNorm scales and shifts, the two FFN biases) are sums
  // over all rows that many blocks add to: they are collected in 8 copies (one per XCD, see
  // launch_layernorm_bwd), vec_stride floats apart, layer l's vectors at vec_off[l] in the
  // order ln2_g, ln2_b, b_2, ln1_g, ln1_b, b_1; at the end of a module's backward pass one
  // launch adds the sum of the copies to the gradient slot (segs: the pieces, per module) and
  // leaves the copies zero.
  float* vec_copies;
  size_t vec_stride;
  std::vector<size_t> vec_off;
  std::vector<std::vector<SumSegment>> segs;
  std::vector<SumSegment*> segs_dev;
  // Stored-input schedule (cfg.schedule == 1): module k < K keeps the input of its last
  // K-k+1 forward passes (token ids for k = 1, the hidden state at the boundary otherwise),
  // tagged with the iteration; the error gradient of module k's output travels from module
  // k+1 to module k through a double-buffered mailbox (written at t, read at t+1).
  std::vector<char*> inring;
  std::vector<size_t> instride;
  std::vector<int64_t> indepth, in_last_slot, in_last_tau;
  std::vector<std::vector<int64_t>> intags;
  std::vector<char*> mail[2];
  std::vector<int64_t> mailtag[2];
  // iteration state
  int64_t t;
  int fwd_next, bwd_next;         // next module expected by forward (1..K+1) / backward (K..0)
  uint64_t upd_mask, inject_mask;
  int mem_valid;                  // valid rows in every layer memory
  const int32_t* tok;
  const int32_t* tgt;
  bool use_side;               // run gradient-only work beside the error-gradient chain (BwdCtx::side)
  // A third stream carries (inside ouro_step) the update of a module as soon as its backward
  // pass is done, beside the backward of the modules below.
  hipStream_t aux;
  hipEvent_t ev_bwd_done, ev_upd_done;
  bool upd_pending;            // updates enqueued on aux that main has not waited for yet
  // optional per-launch HIP event timing, by kind of kernel (see ouro_debug_timing_enable)
  int timing;
  std::vector<hipEvent_t> ev[OURO_TIMING_KINDS];
  size_t ev_used[OURO_TIMING_KINDS];
  double timed_work[OURO_TIMING_KINDS];
  int64_t timed_launches[OURO_TIMING_KINDS];

  const char* wT(int layer, size_t off) const {   // weight as activation-typed operand
    int k = layer_mod[layer];
    return cfg.dtype == 1 ? (const char*)(shadow[k] + off) : (const char*)(master[k] + off);
  }
  const float* wF(int layer, size_t off) const { return master[layer_mod[layer]] + off; }
  const char* vT() const { return cfg.dtype == 1 ? (const char*)shadow[0] : (const char*)master[0]; }
  const char* wTt(int layer, size_t off) const { return (const char*)(shadowT[layer_mod[layer]] + off); }   // bf16 mode only
  float* slot_ptr(int id, int64_t slot) const { return ring[id] + (size_t)slot * gstride[id]; }
};

static int default_split(int L, int K, std::vector<int>& out) {
  int base = L / K, rem = L % K;
  out.assign(K, base);
  std::vector<int> order;
  for (int i = 1; i < K - 1; ++i) order.push_back(i);
  order.push_back(0);
  if (K > 1) order.push_back(K - 1);
  for (int i = 0; i < rem; ++i) out[order[i % order.size()]] += 1;
  return 0;
}

static int validate(const ouro_config* c, std::vector<int>& lpm) {
  if (!c) return fail(OURO_E_ARG, "config is null");
  if (c->n_layer < 1 || c->d_model < 2 || c->n_head < 1 || c->d_head < 1 || c->d_ff < 1 || c->vocab < 2 ||
      c->seq_len < 1 || c->batch < 1 || c->mem_len < 0)
    return fail(OURO_E_CONFIG, "sizes must be positive");
  if ((int64_t)c->n_head * c->d_head != c->d_model) return fail(OURO_E_CONFIG, "n_head*d_head != d_model");
  if (c->d_model % 2) return fail(OURO_E_CONFIG, "d_model must be even");
  if (c->d_head > 256) return fail(OURO_E_CONFIG, "d_head > 256 unsupported");
  if (c->n_module < 1 || c->n_module > c->n_layer || c->n_module > 62)
    return fail(OURO_E_CONFIG, "n_module must be in [1, min(n_layer, 62)]");
  if (c->mem_len > 0 && !c->rel_pos) return fail(OURO_E_CONFIG, "mem_len > 0 needs rel_pos = 1");
  if (c->rel_pos != 0 && c->rel_pos != 1) return fail(OURO_E_CONFIG, "rel_pos must be 0 or 1");
  if (c->dtype != 0 && c->dtype != 1) return fail(OURO_E_CONFIG, "dtype must be 0 or 1");
  if (c->optimizer != 0 && c->optimizer != 1) return fail(OURO_E_CONFIG, "optimizer must be 0 or 1");
  if (c->embed_warm_mode != 0 && c->embed_warm_mode != 1) return fail(OURO_E_CONFIG, "embed_warm_mode must be 0 or 1");
  if (c->schedule != 0 && c->schedule != 1) return fail(OURO_E_CONFIG, "schedule must be 0 or 1");
  if (!(c->dropout >= 0.f && c->dropout < 1.f)) return fail(OURO_E_CONFIG, "dropout must be in [0, 1)");
  if (c->optimizer == 1 && !(c->beta1 >= 0 && c->beta1 < 1 && c->beta2 >= 0 && c->beta2 < 1 && c->eps > 0))
    return fail(OURO_E_CONFIG, "Adam constants out of range");
  if ((int64_t)c->batch * c->seq_len > (1 << 24)) return fail(OURO_E_CONFIG, "batch*seq_len too large");
  if ((int64_t)(c->seq_len + c->mem_len) > 6000) return fail(OURO_E_CONFIG, "seq_len+mem_len > 6000 unsupported");
  if (c->layers_per_module) {
    int sum = 0;
    lpm.assign(c->layers_per_module, c->layers_per_module + c->n_module);
    for (int v : lpm) {
      if (v < 1) return fail(OURO_E_CONFIG, "every module needs at least one layer");
      sum += v;
    }
    if (sum != c->n_layer) return fail(OURO_E_CONFIG, "layers_per_module does not sum to n_layer");
  } else {
    default_split(c->n_layer, c->n_module, lpm);
  }
  return OURO_OK;
}

// Fills every pointer of m relative to base (base may be null: sizing only).
static size_t lay_out(ouro_model& m, char* base) {
  const ouro_config& c = m.cfg;
  const int K = c.n_module, L = c.n_layer;
  const size_t V = c.vocab, T = c.seq_len, M = c.mem_len, B = c.batch;
  const size_t N = B * T, S = T + M, es = m.esz;
  const size_t vpad = (V + 63) / 64 * 64;
  const size_t dl = c.d_model, Fl = c.d_ff, dhl = c.d_head, H = c.n_head;   // the caller's widths
  auto up64 = [](size_t x) { return (x + 63) / 64 * 64; };
  m.padded = c.dtype == 1 && dhl <= 64 && (dhl != 64 || dl % 64 || Fl % 64);
  m.pd = (int)(m.padded ? up64(dl) : dl);
  m.pdh = (int)(m.padded ? 64 : dhl);
  m.phd = (int)(H * m.pdh);
  m.pF = (int)(m.padded ? up64(Fl) : Fl);
  const size_t d = m.pd, F = m.pF, hd = m.phd;                              // stored widths from here on
  Bump bp;
  auto P = [&](size_t bytes) { return base + bp.take(bytes); };
  m.count.assign(K + 1, 0); m.pcount.assign(K + 1, 0);
  m.count[0] = (int64_t)(V * dl); m.pcount[0] = (int64_t)(V * d);
  m.tmap.assign(K + 1, {});
  m.tmap[0].push_back({0, 0, (int)V, (int)dl, (int)d, false, false});
  m.first_layer.assign(K + 1, 0);
  m.layer_mod.assign(L, 0);
  m.loff.resize(L);
  int l = 0;
  for (int k = 1; k <= K; ++k) {
    m.first_layer[k - 1] = l;
    size_t off = 0, lo_off = 0;
    for (int i = 0; i < m.lpm[k - 1]; ++i, ++l) {
      m.layer_mod[l] = k;
      const LayerOff po = layer_offsets(c.rel_pos != 0, d, hd, F, off);
      const LayerOff lo = layer_offsets(c.rel_pos != 0, dl, dl, Fl, lo_off);
      m.loff[l] = po;
      std::vector<TensorMap>& tm = m.tmap[k];
      tm.push_back({lo.W_qkv, po.W_qkv, (int)dl, (int)(3 * dl), (int)(3 * hd), false, true});
      tm.push_back({lo.W_o, po.W_o, (int)dl, (int)dl, (int)d, true, false});
      if (c.rel_pos) {
        tm.push_back({lo.W_r, po.W_r, (int)dl, (int)dl, (int)hd, false, true});
        tm.push_back({lo.u, po.u, 1, (int)dl, (int)hd, false, true});
        tm.push_back({lo.v, po.v, 1, (int)dl, (int)hd, false, true});
      }
      tm.push_back({lo.ln1_g, po.ln1_g, 1, (int)dl, (int)d, false, false});
      tm.push_back({lo.ln1_b, po.ln1_b, 1, (int)dl, (int)d, false, false});
      tm.push_back({lo.W_1, po.W_1, (int)dl, (int)Fl, (int)F, false, false});
      tm.push_back({lo.b_1, po.b_1, 1, (int)Fl, (int)F, false, false});
      tm.push_back({lo.W_2, po.W_2, (int)Fl, (int)dl, (int)d, false, false});
      tm.push_back({lo.b_2, po.b_2, 1, (int)dl, (int)d, false, false});
      tm.push_back({lo.ln2_g, po.ln2_g, 1, (int)dl, (int)d, false, false});
      tm.push_back({lo.ln2_b, po.ln2_b, 1, (int)dl, (int)d, false, false});
      off = po.end;
      lo_off = lo.end;
    }
    m.count[k] = (int64_t)lo_off;
    m.pcount[k] = (int64_t)off;
  }
  m.first_layer[K] = L;
  m.master.assign(K + 1, nullptr); m.shadow.assign(K + 1, nullptr);
  m.adam_m.assign(K + 1, nullptr); m.adam_v.assign(K + 1, nullptr);
  for (int k = 0; k <= K; ++k) {
    m.master[k] = (float*)P(m.pcount[k] * 4);
    // V's bf16 copy carries zero rows up to the padded vocabulary (never written after the arena clear)
    if (c.dtype == 1) m.shadow[k] = (bf16_t*)P((k == 0 ? vpad * d : (size_t)m.pcount[k]) * 2);
    if (c.optimizer == 1) {
      m.adam_m[k] = (float*)P(m.pcount[k] * 4);
      m.adam_v[k] = (float*)P(m.pcount[k] * 4);
    }
  }
  m.shadowT.assign(K + 1, nullptr); m.ttab.assign(K + 1, {}); m.ttab_dev.assign(K + 1, nullptr); m.ttiles.assign(K + 1, 0);
  if (c.dtype == 1) {
    auto add = [&](int k, size_t off, size_t rows, size_t cols, size_t ld_out) {
      TransposeEntry t{(unsigned long long)off, (int)rows, (int)cols, (int)ld_out, m.ttiles[k]};
      m.ttab[k].push_back(t);
      m.ttiles[k] += (int)(((rows + 63) / 64) * ((cols + 63) / 64));
    };
    add(0, 0, V, d, vpad);
    for (int li = 0; li < L; ++li) {
      const int k = m.layer_mod[li];
      const LayerOff& o = m.loff[li];
      add(k, o.W_qkv, d, 3 * hd, d);
      add(k, o.W_o, hd, d, hd);
      if (c.rel_pos) add(k, o.W_r, d, hd, d);
      add(k, o.W_1, d, F, d);
      add(k, o.W_2, F, d, F);
    }
    for (int k = 0; k <= K; ++k) {
      m.shadowT[k] = (bf16_t*)P((k == 0 ? vpad * d : (size_t)m.pcount[k]) * 2);
      m.ttab_dev[k] = (TransposeEntry*)P(m.ttab[k].size() * sizeof(TransposeEntry));
    }
  }
  m.gcount.assign(K + 2, 0); m.gstride.assign(K + 2, 0); m.depth.assign(K + 2, 0); m.ring.assign(K + 2, nullptr);
  for (int id = 0; id <= K + 1; ++id) {
    const int grp = (id == 0 || id == K + 1) ? 0 : id;
    m.gcount[id] = m.count[grp];
    m.gstride[id] = (m.pcount[grp] + 63) / 64 * 64;
    if (id == K + 1 && (int64_t)(vpad * d) > m.gstride[id]) m.gstride[id] = (int64_t)(vpad * d);   // dV_o rows of the padding
    ouro_ring_depth(K, id, &m.depth[id]);
    if (c.schedule == 1) m.depth[id] = 1;     // a gradient is applied in the iteration that computes it
    m.ring[id] = (float*)P((size_t)m.depth[id] * m.gstride[id] * 4);
  }
  m.inring.assign(K + 1, nullptr); m.instride.assign(K + 1, 0); m.indepth.assign(K + 1, 0);
  for (int p2 = 0; p2 < 2; ++p2) m.mail[p2].assign(K + 1, nullptr);
  if (c.schedule == 1) {
    for (int k = 1; k < K; ++k) {
      m.indepth[k] = K - k + 1;
      m.instride[k] = ((k == 1 ? N * 4 : N * d * es) + 255) & ~(size_t)255;
      m.inring[k] = P(m.instride[k] * (size_t)m.indepth[k]);
      for (int p2 = 0; p2 < 2; ++p2) m.mail[p2][k] = P(N * d * 4);
    }
  }
  m.persist_end = bp.off;
  m.L.resize(L);
  const size_t qkv_elems = c.rel_pos ? (N * hd + B * S * 2 * hd) : (N * 3 * hd);
  for (int i = 0; i < L; ++i) {
    LayerBuf& b = m.L[i];
    b.x = P(N * d * es);
    b.cat = (M > 0) ? P(B * S * d * es) : nullptr;
    b.qkv = P(qkv_elems * es);
    b.a = P(N * hd * es);
    b.s1 = P(N * d * 4);
    b.y = P(N * d * es);
    b.z = P(N * F * es);
    b.uact = P(N * F * es);
    b.s2 = P(N * d * 4);
    b.r = c.rel_pos ? P(S * hd * es) : nullptr;
    b.memring = nullptr; b.memstride = 0; b.memdepth = 0;
    if (M > 0 && c.schedule == 1) {
      // a module's memories are part of its stored input: one slot per iteration still to be
      // recomputed, plus the one the running forward pass fills for the next iteration
      b.memdepth = K - m.layer_mod[i] + 2;
      b.memstride = (B * M * d * es + 255) & ~(size_t)255;
      b.memring = P(b.memstride * (size_t)b.memdepth);
      b.mem = b.memring;
    } else {
      b.mem = (M > 0) ? P(B * M * d * es) : nullptr;
    }
    b.lse = (float*)P(B * c.n_head * T * 4);
    b.mean1 = (float*)P(N * 4); b.rstd1 = (float*)P(N * 4);
    b.mean2 = (float*)P(N * 4); b.rstd2 = (float*)P(N * 4);
  }
  m.hL = P(N * d * es);
  m.pe = c.rel_pos ? nullptr : (float*)P(T * d * 4);
  m.rtab = c.rel_pos ? P(S * d * es) : nullptr;
  m.ldv = (int)vpad;
  m.G = P(N * (size_t)m.ldv * es);
  m.lse_ce = (float*)P(N * 4);
  m.rowloss = (float*)P(N * 4);
  m.loss = (float*)P(256);
  m.flag = (int*)P(256);
  // backward scratch: one set, or one per module under the stored-input schedule
  auto scratch = [&](BwdCtx& x) {
    for (int i = 0; i < 3; ++i) x.dhb[i] = P(N * d * 4);
    x.dy[0] = P(N * d * 4); x.dy[1] = P(N * d * 4); x.da = P(N * hd * es);
    for (int p2 = 0; p2 < 2; ++p2) {
      x.ds2[p2] = P(N * d * es); x.dz[p2] = P(N * F * es);
      x.ds1[p2] = P(N * d * es); x.dqkv[p2] = P(qkv_elems * es);
      x.ds2m[p2] = c.dropout > 0 ? P(N * d * es) : x.ds2[p2];
      x.ds1m[p2] = c.dropout > 0 ? P(N * d * es) : x.ds1[p2];
    }
    x.dcat = (c.rel_pos && c.dtype != 1) ? P(B * S * d * es) : nullptr;   // fp32 mode: d[mem ; x] before its current rows are added to dx
    for (int p2 = 0; p2 < 2; ++p2) {
      x.dr_t[p2] = c.rel_pos ? P(S * hd * es) : nullptr;
      x.dr_f32[p2] = c.rel_pos ? (float*)P(S * hd * 4) : nullptr;
    }
    x.attn_scratch = (float*)P((c.rel_pos ? attn_bwd_scratch_floats_any(c.batch, c.n_head, c.seq_len, (int)S, m.pdh)
                                          : attn_bwd_scratch_floats(c.batch, c.n_head, c.seq_len, (int)S, m.pdh)) * 4);
    x.attn_scratch_Mv = -1;
    x.hscratch = c.schedule == 1 ? P(N * d * es) : nullptr;
  };
  scratch(m);
  if (m.ctxs.empty() && c.schedule == 1 && K > 1) {
    BwdCtx z;
    memset(&z, 0, sizeof z);
    m.ctxs.assign(K, z);
  }
  for (size_t i = 1; i < m.ctxs.size(); ++i) scratch(m.ctxs[i]);
  m.dbg_floats = N * d > B * M * d ? N * d : B * M * d;
  if (m.dbg_floats < S * d) m.dbg_floats = S * d;
  m.dbg_f32 = (float*)P(m.dbg_floats * 4);
  m.vec_off.assign(L, 0);
  m.segs.assign(K + 1, {});
  m.segs_dev.assign(K + 1, nullptr);
  size_t vtot = 0;
  for (int li = 0; li < L; ++li) {
    m.vec_off[li] = vtot;
    const LayerOff& o = m.loff[li];
    const size_t dst[6] = {o.ln2_g, o.ln2_b, o.b_2, o.ln1_g, o.ln1_b, o.b_1};
    for (int i = 0; i < 6; ++i) {
      const size_t len = i == 5 ? F : d;
      for (size_t c0 = 0; c0 < len; c0 += 256)
        m.segs[m.layer_mod[li]].push_back({(unsigned)(vtot + c0), (unsigned)(dst[i] + c0), (unsigned)std::min<size_t>(256, len - c0)});
      vtot += len;
    }
  }
  m.vec_stride = (vtot + 63) / 64 * 64;
  m.vec_copies = (float*)P(8 * m.vec_stride * 4);
  for (int k = 1; k <= K; ++k) m.segs_dev[k] = (SumSegment*)P(m.segs[k].size() * sizeof(SumSegment));
  return bp.off;
}

extern "C" int ouro_query_arena_bytes(const ouro_config* cfg, size_t* bytes) {
  if (!bytes) return fail(OURO_E_ARG, "bytes is null");
  ouro_model m;
  int rc = validate(cfg, m.lpm);
  if (rc) return rc;
  m.cfg = *cfg;
  m.esz = cfg->dtype == 1 ? 2 : 4;
  *bytes = lay_out(m, nullptr);
  return OURO_OK;
}

// rows x d sinusoids in rows of ld floats (columns d..ld-1 zero)
static void host_sinusoid(std::vector<float>& out, int rows, int d, int ld) {
  out.assign((size_t)rows * ld, 0.f);
  for (int p = 0; p < rows; ++p)
    for (int i = 0; i < d / 2; ++i) {
      double w = std::pow(10000.0, -2.0 * i / d);
      out[(size_t)p * ld + i] = (float)std::sin(p * w);
      out[(size_t)p * ld + d / 2 + i] = (float)std::cos(p * w);
    }
}

// Copies a parameter group between the caller's dense blob and the stored layout (host memory
// both; the stored blob is zero-filled by the caller before to_stored).
static void remap_group(const ouro_model* m, int group, float* stored, float* blob, bool to_stored);

extern "C" int ouro_create_model(const ouro_config* cfg, void* dev_arena, size_t bytes, void* hip_stream,
                                 ouro_model** out) {
  if (!out) return fail(OURO_E_ARG, "out is null");
  *out = nullptr;
  ouro_model* m = new ouro_model();
  int rc = validate(cfg, m->lpm);
  if (rc) { delete m; return rc; }
  m->cfg = *cfg;
  m->cfg.layers_per_module = nullptr;
  m->esz = cfg->dtype == 1 ? 2 : 4;
  m->N = cfg->batch * cfg->seq_len;
  m->S = cfg->seq_len + cfg->mem_len;
  if (!dev_arena || (reinterpret_cast<uintptr_t>(dev_arena) & 255)) { delete m; return fail(OURO_E_ARENA, "arena null or not 256-byte aligned"); }
  size_t need = lay_out(*m, (char*)dev_arena);
  if (bytes < need) { delete m; return fail(OURO_E_ARENA, "arena has %zu bytes, %zu needed", bytes, need); }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { delete m; return fail(OURO_E_HIP, "no HIP device available"); }
  m->arena = (char*)dev_arena;
  m->bytes = need;
  m->stream = (hipStream_t)hip_stream;
  const int K = cfg->n_module;
  m->tags.resize(K + 2);
  for (int id = 0; id <= K + 1; ++id) m->tags[id].assign((size_t)m->depth[id], -1);
  m->last_slot.assign(K + 2, -1); m->last_tau.assign(K + 2, -1);
  m->intags.resize(K + 1);
  for (int k = 0; k <= K; ++k) m->intags[k].assign((size_t)m->indepth[k], -1);
  m->in_last_slot.assign(K + 1, -1); m->in_last_tau.assign(K + 1, -1);
  for (int p2 = 0; p2 < 2; ++p2) m->mailtag[p2].assign(K + 1, -1);
  m->t = 0; m->fwd_next = 1; m->bwd_next = K; m->upd_mask = 0; m->inject_mask = 0; m->mem_valid = 0;
  m->tok = m->tgt = nullptr;
  m->timing = 0;
  m->eval_mode = false; m->cur_seed = cfg->seed;
  for (int i = 0; i < OURO_TIMING_KINDS; ++i) { m->ev_used[i] = 0; m->timed_work[i] = 0; m->timed_launches[i] = 0; }
  m->side = nullptr; m->use_side = false; m->ev_join = nullptr;
  m->aux = nullptr; m->ev_bwd_done = m->ev_upd_done = nullptr; m->upd_pending = false;
  for (int i = 0; i < 4; ++i) m->ev_ready[i] = nullptr;
  for (int i = 0; i < 2; ++i) { m->ev_side_done[i] = nullptr; m->side_busy[i] = false; }
  {
    hipError_t es_ = hipStreamCreateWithFlags(&m->side, hipStreamNonBlocking);
    for (int i = 0; i < 4 && es_ == hipSuccess; ++i) es_ = hipEventCreateWithFlags(&m->ev_ready[i], hipEventDisableTiming);
    for (int i = 0; i < 2 && es_ == hipSuccess; ++i) es_ = hipEventCreateWithFlags(&m->ev_side_done[i], hipEventDisableTiming);
    if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming);
    if (es_ == hipSuccess) es_ = hipStreamCreateWithFlags(&m->aux, hipStreamNonBlocking);
    for (hipEvent_t* pe : {&m->ev_bwd_done, &m->ev_upd_done})
      if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(pe, hipEventDisableTiming);
    m->ev_done = nullptr; m->ev_fwd = nullptr; m->cur_ctx = 0;
    if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&m->ev_fwd, hipEventDisableTiming);
    for (size_t i = 1; i < m->ctxs.size() && es_ == hipSuccess; ++i) {
      BwdCtx& x = m->ctxs[i];
      es_ = hipStreamCreateWithFlags(&x.stream, hipStreamNonBlocking);
      if (es_ == hipSuccess) es_ = hipStreamCreateWithFlags(&x.side, hipStreamNonBlocking);
      for (int j = 0; j < 4 && es_ == hipSuccess; ++j) es_ = hipEventCreateWithFlags(&x.ev_ready[j], hipEventDisableTiming);
      for (int j = 0; j < 2 && es_ == hipSuccess; ++j) es_ = hipEventCreateWithFlags(&x.ev_side_done[j], hipEventDisableTiming);
      if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&x.ev_join, hipEventDisableTiming);
      if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&x.ev_done, hipEventDisableTiming);
    }
    if (es_ != hipSuccess) { ouro_destroy_model(m); return fail(OURO_E_HIP, "streams / events: %s", hipGetErrorString(es_)); }
    m->use_side = true;
  }
  // zero optimizer state, rings, everything else too (one fill over the arena)
  hipError_t e = launch_fill_zero(m->stream, m->arena, need);
  if (e != hipSuccess) { ouro_destroy_model(m); return fail(OURO_E_HIP, "arena clear: %s", hipGetErrorString(e)); }
  for (int k = 0; k <= K && e == hipSuccess; ++k)
    if (m->ttab_dev[k])
      e = hipMemcpyAsync(m->ttab_dev[k], m->ttab[k].data(), m->ttab[k].size() * sizeof(TransposeEntry), hipMemcpyHostToDevice, m->stream);
  for (int k = 1; k <= K && e == hipSuccess; ++k)
    if (!m->segs[k].empty())
      e = hipMemcpyAsync(m->segs_dev[k], m->segs[k].data(), m->segs[k].size() * sizeof(SumSegment), hipMemcpyHostToDevice, m->stream);
  if (e != hipSuccess) { ouro_destroy_model(m); return fail(OURO_E_HIP, "table upload: %s", hipGetErrorString(e)); }
  std::vector<float> tab;
  if (!cfg->rel_pos) {
    host_sinusoid(tab, cfg->seq_len, cfg->d_model, m->pd);
    e = hipMemcpyAsync(m->pe, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, m->stream);
  } else {
    host_sinusoid(tab, m->S, cfg->d_model, m->pd);
    e = hipMemcpyAsync(m->dbg_f32, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, m->stream);
    if (e == hipSuccess) e = launch_convert(m->stream, cfg->dtype, m->rtab, m->dbg_f32, tab.size());
  }
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  if (e != hipSuccess) { ouro_destroy_model(m); return fail(OURO_E_HIP, "table upload: %s", hipGetErrorString(e)); }
  *out = m;
  return OURO_OK;
}

// Makes backward set i the one in use (host bookkeeping only).
static void activate(ouro_model* m, int i) {
  if (i == m->cur_ctx || m->ctxs.empty()) return;
  m->ctxs[m->cur_ctx] = *static_cast<BwdCtx*>(m);
  *static_cast<BwdCtx*>(m) = m->ctxs[i];
  m->cur_ctx = i;
}

extern "C" int ouro_destroy_model(ouro_model* m) {
  if (!m) return OURO_OK;
  activate(m, 0);
  for (size_t i = 1; i < m->ctxs.size(); ++i) {
    BwdCtx& x = m->ctxs[i];
    if (x.stream) { (void)hipStreamSynchronize(x.stream); (void)hipStreamDestroy(x.stream); }
    if (x.side) { (void)hipStreamSynchronize(x.side); (void)hipStreamDestroy(x.side); }
    for (hipEvent_t e : {x.ev_ready[0], x.ev_ready[1], x.ev_ready[2], x.ev_ready[3], x.ev_side_done[0], x.ev_side_done[1], x.ev_join, x.ev_done})
      if (e) (void)hipEventDestroy(e);
  }
  if (m->ev_fwd) (void)hipEventDestroy(m->ev_fwd);
  (void)hipStreamSynchronize(m->stream);
  if (m->side) { (void)hipStreamSynchronize(m->side); (void)hipStreamDestroy(m->side); }
  for (int i = 0; i < 4; ++i) if (m->ev_ready[i]) (void)hipEventDestroy(m->ev_ready[i]);
  for (int i = 0; i < 2; ++i) if (m->ev_side_done[i]) (void)hipEventDestroy(m->ev_side_done[i]);
  if (m->ev_join) (void)hipEventDestroy(m->ev_join);
  if (m->aux) { (void)hipStreamSynchronize(m->aux); (void)hipStreamDestroy(m->aux); }
  for (hipEvent_t e : {m->ev_bwd_done, m->ev_upd_done}) if (e) (void)hipEventDestroy(e);
  for (int i = 0; i < OURO_TIMING_KINDS; ++i)
    for (hipEvent_t e : m->ev[i]) (void)hipEventDestroy(e);
  delete m;
  return OURO_OK;
}

extern "C" int ouro_param_count(const ouro_model* m, int group, int64_t* n) {
  if (!m || !n || group < 0 || group > m->cfg.n_module) return fail(OURO_E_ARG, "param_count: bad argument");
  *n = m->count[group];
  return OURO_OK;
}

// bf16 mode: the transposed copies of a group's weight matrices follow its bf16 copy
static int refresh_transposed(ouro_model* m, int group, hipStream_t st) {
  if (m->cfg.dtype != 1) return OURO_OK;
  HIPCHK(launch_transpose_table(st, m->shadow[group], m->shadowT[group], m->ttab_dev[group], (int)m->ttab[group].size(), m->ttiles[group]));
  return OURO_OK;
}

extern "C" int ouro_set_params(ouro_model* m, int group, const float* src, int64_t n, int src_is_device) {
  if (!m || !src || group < 0 || group > m->cfg.n_module) return fail(OURO_E_ARG, "set_params: bad argument");
  if (n != m->count[group]) return fail(OURO_E_ARG, "set_params: group %d has %lld elements, got %lld", group, (long long)m->count[group], (long long)n);
  if (m->padded) {
    std::vector<float> blob, stored((size_t)m->pcount[group], 0.f);
    const float* hsrc = src;
    if (src_is_device) {
      blob.resize((size_t)n);
      HIPCHK(hipMemcpyAsync(blob.data(), src, (size_t)n * 4, hipMemcpyDeviceToHost, m->stream));
      HIPCHK(hipStreamSynchronize(m->stream));
      hsrc = blob.data();
    }
    remap_group(m, group, stored.data(), const_cast<float*>(hsrc), true);
    HIPCHK(hipMemcpyAsync(m->master[group], stored.data(), stored.size() * 4, hipMemcpyHostToDevice, m->stream));
    HIPCHK(launch_convert(m->stream, 1, m->shadow[group], m->master[group], stored.size()));
    if (int rc = refresh_transposed(m, group, m->stream)) return rc;
    HIPCHK(hipStreamSynchronize(m->stream));
    return OURO_OK;
  }
  HIPCHK(hipMemcpyAsync(m->master[group], src, (size_t)n * 4, src_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, m->stream));
  if (m->cfg.dtype == 1) HIPCHK(launch_convert(m->stream, 1, m->shadow[group], m->master[group], (size_t)n));
  if (int rc = refresh_transposed(m, group, m->stream)) return rc;
  if (!src_is_device) HIPCHK(hipStreamSynchronize(m->stream));
  return OURO_OK;
}

extern "C" int ouro_get_params(ouro_model* m, int group, float* dst, int64_t n, int dst_is_device) {
  if (!m || !dst || group < 0 || group > m->cfg.n_module) return fail(OURO_E_ARG, "get_params: bad argument");
  if (n != m->count[group]) return fail(OURO_E_ARG, "get_params: wrong element count");
  if (m->padded) {
    std::vector<float> stored((size_t)m->pcount[group]), blob;
    HIPCHK(hipMemcpyAsync(stored.data(), m->master[group], stored.size() * 4, hipMemcpyDeviceToHost, m->stream));
    HIPCHK(hipStreamSynchronize(m->stream));
    if (!dst_is_device) { remap_group(m, group, stored.data(), dst, false); return OURO_OK; }
    blob.resize((size_t)n);
    remap_group(m, group, stored.data(), blob.data(), false);
    HIPCHK(hipMemcpyAsync(dst, blob.data(), (size_t)n * 4, hipMemcpyHostToDevice, m->stream));
    HIPCHK(hipStreamSynchronize(m->stream));
    return OURO_OK;
  }
  HIPCHK(hipMemcpyAsync(dst, m->master[group], (size_t)n * 4, dst_is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, m->stream));
  if (!dst_is_device) HIPCHK(hipStreamSynchronize(m->stream));
  return OURO_OK;
}

extern "C" int64_t ouro_current_step(const ouro_model* m) { return m ? m->t : -1; }

static void remap_group(const ouro_model* m, int group, float* stored, float* blob, bool to_stored) {
  const int dh = m->cfg.d_head, pdh = m->pdh;
  for (const TensorMap& t : m->tmap[group]) {
    for (int r = 0; r < t.rows; ++r) {
      const size_t pr = t.row_heads ? (size_t)(r / dh) * pdh + r % dh : (size_t)r;
      float* srow = stored + t.poff + pr * t.pcols;
      float* brow = blob + t.loff + (size_t)r * t.cols;
      if (!t.col_heads) {
        if (to_stored) memcpy(srow, brow, (size_t)t.cols * 4);
        else memcpy(brow, srow, (size_t)t.cols * 4);
      } else {
        for (int c0 = 0; c0 < t.cols; c0 += dh) {
          float* sp = srow + (size_t)(c0 / dh) * pdh;
          if (to_stored) memcpy(sp, brow + c0, (size_t)dh * 4);
          else memcpy(brow + c0, sp, (size_t)dh * 4);
        }
      }
    }
  }
}

// --------------------------------------------------------------------- launch helpers
static int timing_begin(ouro_model* m, int kind, hipStream_t st) {
  while (m->ev[kind].size() < m->ev_used[kind] + 2) {
    hipEvent_t e;
    HIPCHK(hipEventCreate(&e));
    m->ev[kind].push_back(e);
  }
  HIPCHK(hipEventRecord(m->ev[kind][m->ev_used[kind]], st));
  return OURO_OK;
}
static int timing_end(ouro_model* m, int kind, double work, hipStream_t st) {
  HIPCHK(hipEventRecord(m->ev[kind][m->ev_used[kind] + 1], st));
  m->ev_used[kind] += 2;
  m->timed_work[kind] += work;
  m->timed_launches[kind] += 1;
  return OURO_OK;
}

// Runs `launch` (a callable returning hipError_t) on st, inside a timing bracket of `kind` when timing is on.
template <typename F>
static int timed_launch(ouro_model* m, int kind, double work, hipStream_t st, F&& launch) {
  const bool timed = m->timing != 0;
  if (timed) { int rc = timing_begin(m, kind, st); if (rc) return rc; }
  HIPCHK(launch());
  if (timed) return timing_end(m, kind, work, st);
  return OURO_OK;
}
// Algorithmic flops of one attention forward launch: visible (query, key) pairs x 4 d_head (scores
// and P V), 6 d_head with the relative-position term; the backward pass counts twice that.
static double attn_fwd_flops(const ouro_model* m, int Mv) {
  const ouro_config& c = m->cfg;
  const double pairs = (double)c.seq_len * Mv + 0.5 * (double)c.seq_len * (c.seq_len + 1);
  return pairs * c.batch * c.n_head * c.d_head * (c.rel_pos ? 6.0 : 4.0);
}

static int run_gemm_on(ouro_model* m, GemmDesc g, hipStream_t st) {
  const bool timed = m->timing && gemm_uses_mfma(m->cfg.dtype, g);
  if (timed) { int rc = timing_begin(m, OURO_TIMING_CONTRACTION, st); if (rc) return rc; }
  HIPCHK(launch_gemm(st, m->cfg.dtype, g, 0));
  if (timed) return timing_end(m, OURO_TIMING_CONTRACTION, 2.0 * g.M * g.N * g.K * std::max(1, g.by) * std::max(1, g.bz), st);
  return OURO_OK;
}
static int run_gemm(ouro_model* m, GemmDesc g) { return run_gemm_on(m, g, m->stream); }
// The weight-gradient contractions of a layer in one launch where they admit it (launch_gemm_group).
static int run_gemm_group_on(ouro_model* m, const GemmDesc* g, int n, hipStream_t st) {
  if (n == 0) return OURO_OK;
  bool timed = m->timing;
  double flops = 0;
  for (int i = 0; i < n; ++i) { timed = timed && gemm_uses_mfma(m->cfg.dtype, g[i]); flops += 2.0 * g[i].M * g[i].N * g[i].K; }
  if (timed) { int rc = timing_begin(m, OURO_TIMING_CONTRACTION, st); if (rc) return rc; }
  HIPCHK(launch_gemm_group(st, m->cfg.dtype, g, n));
  if (timed) return timing_end(m, OURO_TIMING_CONTRACTION, flops, st);
  return OURO_OK;
}

static GemmDesc gd(const void* A, int lda, int tA, const void* B, int ldb, int tB, void* C, int ldc, int M, int N, int K) {
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.transA = tA; g.transB = tB; g.alpha = 1.f;
  return g;
}
#define RUN(expr) do { int rc_ = (expr); if (rc_) return rc_; } while (0)

// ------------------------------------------------------------------------------ forward
// Dropout descriptor of a place (0: embedding sum; 2l+1 / 2l+2: attention-projection / feed-forward
// output of layer l) under the seed of the mini-batch being worked on; rows are d_model long.
static DropDesc drop_at(const ouro_model* m, uint32_t place) {
  return make_drop(m->eval_mode ? 0.f : m->cfg.dropout, m->cur_seed, place, m->cfg.d_model);
}

// Valid rows of every segment memory at the forward pass of iteration t.
static int mem_valid_at(const ouro_model* m, int64_t t) {
  const int64_t rows = t * (int64_t)m->cfg.seq_len;
  return (int)std::min<int64_t>(m->cfg.mem_len, rows);
}
// Stored-input schedule: layer l uses the memory of iteration t from here on.
static void select_memory(ouro_model* m, int l, int64_t t) {
  LayerBuf& b = m->L[l];
  if (b.memring) b.mem = b.memring + (size_t)(t % b.memdepth) * b.memstride;
}

// out_override: where the layer's output goes instead of the next layer's input buffer.
// x_is_ln_of_prev: the layer's input b.x is the stored (rounded) output of layer l-1's second LayerNorm
// in this same pass, so the residual addition takes it unrounded from that layer's fp32 sum.
static int layer_forward(ouro_model* m, int l, char* out_override = nullptr, bool x_is_ln_of_prev = false) {
  const ouro_config& c = m->cfg;
  const int d = m->pd, F = m->pF, hd = m->phd, dn = c.d_model;   // stored widths; dn = normalised width
  const int N = m->N, T = c.seq_len, B = c.batch, es = m->esz;
  const LayerOff& o = m->loff[l];
  LayerBuf& b = m->L[l];
  const bool bt = c.dtype == 1;               // weights are at hand transposed: both operands contraction-contiguous
  char* out = out_override ? out_override : (l + 1 < c.n_layer) ? m->L[l + 1].x : m->hL;
  const int Mv = m->mem_valid, S = Mv + T;
  AttnDesc a;
  memset(&a, 0, sizeof a);
  a.B = B; a.H = c.n_head; a.T = T; a.S = S; a.dh = m->pdh; a.Mv = Mv;
  a.scale = 1.f / std::sqrt((float)c.d_head);
  a.o = b.a; a.ldo = hd; a.lse = b.lse;
  if (!c.rel_pos) {
    if (bt) RUN(run_gemm(m, gd(b.x, d, 0, m->wTt(l, o.W_qkv), d, 1, b.qkv, 3 * hd, N, 3 * hd, d)));
    else RUN(run_gemm(m, gd(b.x, d, 0, m->wT(l, o.W_qkv), 3 * hd, 0, b.qkv, 3 * hd, N, 3 * hd, d)));
    a.q = b.qkv; a.ldq = 3 * hd;
    a.k = b.qkv + (size_t)hd * es; a.ldk = 3 * hd;
    a.v = b.qkv + (size_t)2 * hd * es; a.ldv = 3 * hd;
  } else {
    const char* cat = b.x;
    if (Mv > 0) {
      HIPCHK(launch_copy_rows(m->stream, c.dtype, b.cat, (size_t)S * d, 0, b.mem, (size_t)Mv * d, 0, B, Mv, d));
      HIPCHK(launch_copy_rows(m->stream, c.dtype, b.cat, (size_t)S * d, (size_t)Mv * d, b.x, (size_t)T * d, 0, B, T, d));
      cat = b.cat;
    }
    char* q = b.qkv;
    char* kv = b.qkv + (size_t)N * hd * es;
    if (bt) {
      // rows 0..hd-1 of W_qkv^T are the query projection, the rest the key / value projections
      RUN(run_gemm(m, gd(b.x, d, 0, m->wTt(l, o.W_qkv), d, 1, q, hd, N, hd, d)));
      RUN(run_gemm(m, gd(cat, d, 0, m->wTt(l, o.W_qkv) + (size_t)hd * d * es, d, 1, kv, 2 * hd, B * S, 2 * hd, d)));
      RUN(run_gemm(m, gd(m->rtab, d, 0, m->wTt(l, o.W_r), d, 1, b.r, hd, S, hd, d)));
    } else {
      RUN(run_gemm(m, gd(b.x, d, 0, m->wT(l, o.W_qkv), 3 * hd, 0, q, hd, N, hd, d)));
      RUN(run_gemm(m, gd(cat, d, 0, m->wT(l, o.W_qkv) + (size_t)hd * es, 3 * hd, 0, kv, 2 * hd, B * S, 2 * hd, d)));
      RUN(run_gemm(m, gd(m->rtab, d, 0, m->wT(l, o.W_r), hd, 0, b.r, hd, S, hd, d)));
    }
    a.q = q; a.ldq = hd;
    a.k = kv; a.ldk = 2 * hd;
    a.v = kv + (size_t)hd * es; a.ldv = 2 * hd;
    a.rel = 1; a.u = m->wT(l, o.u); a.vb = m->wT(l, o.v); a.r = b.r; a.ldr = hd;
  }
  RUN(timed_launch(m, OURO_TIMING_ATTENTION, attn_fwd_flops(m, Mv), m->stream, [&] { return launch_attn_fwd(m->stream, c.dtype, a, 0); }));
  {
    GemmDesc g = bt ? gd(b.a, hd, 0, m->wTt(l, o.W_o), hd, 1, b.s1, d, N, d, hd) : gd(b.a, hd, 0, m->wT(l, o.W_o), d, 0, b.s1, d, N, d, hd);
    if (x_is_ln_of_prev && l > 0) {
      const LayerBuf& pb = m->L[l - 1];
      const LayerOff& po = m->loff[l - 1];
      g.res32 = (const float*)pb.s2; g.ldr32 = d; g.ln_mean = pb.mean2; g.ln_rstd = pb.rstd2;
      g.ln_g = m->wF(l - 1, po.ln2_g); g.ln_b = m->wF(l - 1, po.ln2_b);
    } else {
      g.residual = b.x; g.ldr = d;
    }
    g.drop = drop_at(m, 2 * l + 1); g.out_fp32 = 1;
    RUN(run_gemm(m, g));
  }
  // The sums that enter a LayerNorm stay in fp32 (in bf16 mode too): every layer's rounding error travels
  // along this path, and bf16 sums alone put the gradients of a 24-layer model at the 2e-2 bar.
  const int lnk = c.dtype == 1 ? 2 : 0;
  const double ln_fwd_bytes = (double)N * dn * (4 + es) + 8.0 * N;      // fp32 row read, row written, two statistics per row
  RUN(timed_launch(m, OURO_TIMING_LAYERNORM, ln_fwd_bytes, m->stream, [&] {
    return launch_layernorm_fwd(m->stream, lnk, b.s1, m->wF(l, o.ln1_g), m->wF(l, o.ln1_b), b.y, b.mean1, b.rstd1, N, d, dn); }));
  {
    GemmDesc g = bt ? gd(b.y, d, 0, m->wTt(l, o.W_1), d, 1, b.uact, F, N, F, d) : gd(b.y, d, 0, m->wT(l, o.W_1), F, 0, b.uact, F, N, F, d);
    g.bias = m->wF(l, o.b_1); g.epilogue = EPI_GELU; g.Z = b.z; g.ldz = F;
    RUN(run_gemm(m, g));
  }
  {
    GemmDesc g = bt ? gd(b.uact, F, 0, m->wTt(l, o.W_2), F, 1, b.s2, d, N, d, F) : gd(b.uact, F, 0, m->wT(l, o.W_2), d, 0, b.s2, d, N, d, F);
    g.bias = m->wF(l, o.b_2);
    g.res32 = (const float*)b.s1; g.ldr32 = d; g.ln_mean = b.mean1; g.ln_rstd = b.rstd1;      // y, unrounded
    g.ln_g = m->wF(l, o.ln1_g); g.ln_b = m->wF(l, o.ln1_b);
    g.drop = drop_at(m, 2 * l + 2); g.out_fp32 = 1;
    RUN(run_gemm(m, g));
  }
  RUN(timed_launch(m, OURO_TIMING_LAYERNORM, ln_fwd_bytes, m->stream, [&] {
    return launch_layernorm_fwd(m->stream, lnk, b.s2, m->wF(l, o.ln2_g), m->wF(l, o.ln2_b), out, b.mean2, b.rstd2, N, d, dn); }));
  return OURO_OK;
}

extern "C" int ouro_module_forward(ouro_model* m, int k, const int32_t* dev_tokens, const int32_t* dev_targets) {
  if (!m) return fail(OURO_E_ARG, "model is null");
  const ouro_config& c = m->cfg;
  const int K = c.n_module;
  if (k < 1 || k > K) return fail(OURO_E_ARG, "module_forward: k=%d outside 1..%d", k, K);
  if (m->inject_mask) return fail(OURO_E_SEQUENCE, "module_forward after inject_grad in the same iteration");
  if (k != m->fwd_next) return fail(OURO_E_SEQUENCE, "module_forward(%d) but module %d is next", k, m->fwd_next);
  if (k == 1) {
    if (!dev_tokens) return fail(OURO_E_ARG, "module_forward(1) needs tokens");
    m->tok = dev_tokens;
    m->cur_seed = c.seed + (uint64_t)m->t;
    HIPCHK(launch_fill_zero(m->stream, m->flag, 256));
    const DropDesc dd = drop_at(m, 0);
    HIPCHK(launch_embed_fwd(m->stream, c.dtype, m->tok, m->vT(), m->pe, m->L[0].x, m->N, c.seq_len, m->pd, c.vocab, c.emb_scale, m->flag, &dd));
  }
  if (k == K && !dev_targets) return fail(OURO_E_ARG, "module_forward(K) needs targets");
  if (c.schedule == 1 && k < K && !m->eval_mode) {
    // the module's input of this iteration, for the backward pass K-k iterations from now
    const int64_t slot = m->t % m->indepth[k];
    char* dst = m->inring[k] + (size_t)slot * m->instride[k];
    if (k == 1) HIPCHK(hipMemcpyAsync(dst, m->tok, (size_t)m->N * 4, hipMemcpyDeviceToDevice, m->stream));
    else HIPCHK(hipMemcpyAsync(dst, m->L[m->first_layer[k - 1]].x, (size_t)m->N * m->pd * m->esz, hipMemcpyDeviceToDevice, m->stream));
    m->intags[k][slot] = m->t;
  }
  for (int l = m->first_layer[k - 1]; l < m->first_layer[k]; ++l) {
    RUN(layer_forward(m, l, nullptr, l > 0));       // layer l-1 ran earlier in this forward pass
    LayerBuf& b = m->L[l];
    if (b.memring) {
      // the memory of iteration t+1 = last M rows of [memory ; layer input], taken now: the
      // backward passes of this iteration recompute over these buffers
      const int T = c.seq_len, dd = m->pd, Mv = m->mem_valid, S = Mv + T, Mn = std::min(c.mem_len, S);
      const char* cat = Mv > 0 ? b.cat : b.x;
      char* nxt = b.memring + (size_t)((m->t + 1) % b.memdepth) * b.memstride;
      HIPCHK(launch_copy_rows(m->stream, c.dtype, nxt, (size_t)Mn * dd, 0, cat, (size_t)S * dd, (size_t)(S - Mn) * dd, c.batch, Mn, dd));
    }
  }
  if (k == K) {
    m->tgt = dev_targets;
    const int d = m->pd, V = c.vocab, N = m->N;
    GemmDesc g = gd(m->hL, d, 0, m->vT(), d, 1, m->G, m->ldv, N, V, d);   // logits = h_L V^T (Eq. 3)
    RUN(run_gemm(m, g));
    // logits read once, d loss / d logits written once, per row the log-sum-exp and the loss
    RUN(timed_launch(m, OURO_TIMING_CE_ROWS, 2.0 * N * (double)V * m->esz + 12.0 * N, m->stream, [&] {
      return launch_ce_rows(m->stream, c.dtype, m->G, m->ldv, m->tgt, m->G, m->ldv, m->lse_ce, m->rowloss, N, V, m->flag); }));
    HIPCHK(launch_sum_rows(m->stream, m->rowloss, N, m->loss));
  }
  m->fwd_next = k + 1;
  if (k == K) m->bwd_next = K;
  return OURO_OK;
}

// ----------------------------------------------------------------------------- backward
template <typename T>
__global__ void add_rows_kernel(float* dst, size_t dst_bstride, const T* src, size_t src_bstride, size_t src_off, size_t n) {
  const int b = blockIdx.y;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    size_t di = b * dst_bstride + i;
    dst[di] += to_f32(src[b * src_bstride + src_off + i]);
  }
}

static int layer_backward(ouro_model* m, int l, char* dh, char* dx, float* gslot) {
  const ouro_config& c = m->cfg;
  const int d = m->pd, F = m->pF, hd = m->phd, dn = c.d_model;   // stored widths; dn = normalised width
  const int N = m->N, T = c.seq_len, B = c.batch, es = m->esz;
  const LayerOff& o = m->loff[l];
  LayerBuf& b = m->L[l];
  const int Mv = m->mem_valid, S = Mv + T;
  hipStream_t st = m->stream;
  const int ps = l & 1;                               // buffer set of this layer
  const bool side = m->use_side;
  hipStream_t sw = side ? m->side : st;               // stream of the weight-gradient work
  char* ds2 = m->ds2[ps]; char* dz = m->dz[ps]; char* ds1 = m->ds1[ps]; char* dqkv = m->dqkv[ps];
  // what flows into the two dropped branches: the LayerNorm input gradients times the masks
  char* ds2m = m->ds2m[ps]; char* ds1m = m->ds1m[ps];
  const bool dropping = c.dropout > 0;
  char* dy = m->dy[ps];
  // the side stream may still be reading this buffer set (layer l+2 of this module)
  if (side && m->side_busy[ps]) { HIPCHK(hipStreamWaitEvent(st, m->ev_side_done[ps], 0)); m->side_busy[ps] = false; }
  auto ready = [&](int i) -> int {                    // operand i written on main; side may start
    if (!side) return OURO_OK;
    HIPCHK(hipEventRecord(m->ev_ready[i], st));
    HIPCHK(hipStreamWaitEvent(sw, m->ev_ready[i], 0));
    return OURO_OK;
  };
  // the gradients of this layer's vectors gather in the per-XCD copies; module_backward adds them to gslot
  float* vc = m->vec_copies + m->vec_off[l];
  // The layer's weight-gradient contractions (small outputs, contraction over all tokens) are
  // collected and go out together once the last operand exists: each alone cannot give its
  // workgroups a long K range and fill the chip in whole rounds.
  GemmDesc wg[GEMM_GROUP_MAX];
  int nwg = 0;
  // LN2
  // the scale / shift gradients come from the same kernel (one pass over dh and s2)
  // dh, dy (gradients of the normalised rows) and the saved sums s1, s2 are fp32 in every mode
  const int lnk = c.dtype == 1 ? 2 : 0;
  const double ln_bwd_bytes = (double)N * dn * (8 + es) + 8.0 * N;      // fp32 gradient and input rows read, one row written, statistics
  RUN(timed_launch(m, OURO_TIMING_LAYERNORM, ln_bwd_bytes, st, [&] {
    return launch_layernorm_bwd(st, lnk, dh, b.s2, m->wF(l, o.ln2_g), b.mean2, b.rstd2, ds2,
                                vc, vc + d, N, d, dn, true, m->vec_stride); }));
  if (dropping) HIPCHK(launch_dropout_apply(st, c.dtype, ds2, ds2m, N, d, d, drop_at(m, 2 * l + 2)));
  RUN(ready(0));
  // FFN2
  {
    GemmDesc g = gd(b.uact, F, 1, ds2m, d, 0, gslot + o.W_2, d, F, d, N);
    g.out_fp32 = 1; g.accumulate = 1;
    wg[nwg++] = g;
  }
  HIPCHK(launch_colsum(sw, c.dtype, ds2m, d, vc + 2 * d, N, d, m->vec_stride));
  {
    GemmDesc g = gd(ds2m, d, 0, m->wT(l, o.W_2), d, 1, dz, F, N, F, d);
    g.epilogue = EPI_GELUGRAD; g.Z = b.z; g.ldz = F;
    RUN(run_gemm(m, g));
  }
  RUN(ready(1));
  // FFN1
  {
    GemmDesc g = gd(b.y, d, 1, dz, F, 0, gslot + o.W_1, F, d, F, N);
    g.out_fp32 = 1; g.accumulate = 1;
    wg[nwg++] = g;
  }
  HIPCHK(launch_colsum(sw, c.dtype, dz, F, vc + 5 * d, N, F, m->vec_stride));
  {
    GemmDesc g = gd(dz, F, 0, m->wT(l, o.W_1), F, 1, dy, d, N, d, F);
    g.residual = ds2; g.ldr = d; g.out_fp32 = 1;
    RUN(run_gemm(m, g));
  }
  // LN1
  RUN(timed_launch(m, OURO_TIMING_LAYERNORM, ln_bwd_bytes, st, [&] {
    return launch_layernorm_bwd(st, lnk, dy, b.s1, m->wF(l, o.ln1_g), b.mean1, b.rstd1, ds1,
                                vc + 3 * d, vc + 4 * d, N, d, dn, true, m->vec_stride); }));
  if (dropping) HIPCHK(launch_dropout_apply(st, c.dtype, ds1, ds1m, N, d, d, drop_at(m, 2 * l + 1)));
  RUN(ready(2));
  // output projection
  {
    GemmDesc g = gd(b.a, hd, 1, ds1m, d, 0, gslot + o.W_o, d, hd, d, N);
    g.out_fp32 = 1; g.accumulate = 1;
    wg[nwg++] = g;
  }
  RUN(run_gemm(m, gd(ds1m, d, 0, m->wT(l, o.W_o), d, 1, m->da, hd, N, hd, d)));
  // attention
  AttnDesc a;
  memset(&a, 0, sizeof a);
  a.B = B; a.H = c.n_head; a.T = T; a.S = S; a.dh = m->pdh; a.Mv = Mv;
  a.scale = 1.f / std::sqrt((float)c.d_head);
  a.o = b.a; a.ldo = hd; a.lse = b.lse; a.d_o = m->da; a.lddo = hd; a.scratch = m->attn_scratch;
  if (!c.rel_pos) {
    a.q = b.qkv; a.ldq = 3 * hd;
    a.k = b.qkv + (size_t)hd * es; a.ldk = 3 * hd;
    a.v = b.qkv + (size_t)2 * hd * es; a.ldv = 3 * hd;
    a.dq = dqkv; a.lddq = 3 * hd;
    a.dk = dqkv + (size_t)hd * es; a.lddk = 3 * hd;
    a.dv = dqkv + (size_t)2 * hd * es; a.lddv = 3 * hd;
    RUN(timed_launch(m, OURO_TIMING_ATTENTION, 2.0 * attn_fwd_flops(m, Mv), st, [&] { return launch_attn_bwd(st, c.dtype, a, 0); }));
    RUN(ready(3));
    {
      GemmDesc g = gd(b.x, d, 1, dqkv, 3 * hd, 0, gslot + o.W_qkv, 3 * hd, d, 3 * hd, N);
      g.out_fp32 = 1; g.accumulate = 1;
      wg[nwg++] = g;
    }
    RUN(run_gemm_group_on(m, wg, nwg, sw));
    {
      GemmDesc g = gd(dqkv, 3 * hd, 0, m->wT(l, o.W_qkv), 3 * hd, 1, dx, d, N, d, 3 * hd);
      g.residual = ds1; g.ldr = d; g.out_fp32 = 1;
      RUN(run_gemm(m, g));
    }
  } else {
    const char* cat = Mv > 0 ? b.cat : b.x;
    char* q = b.qkv;
    char* kv = b.qkv + (size_t)N * hd * es;
    char* dq = dqkv;
    char* dkv = dqkv + (size_t)N * hd * es;
    a.q = q; a.ldq = hd; a.k = kv; a.ldk = 2 * hd; a.v = kv + (size_t)hd * es; a.ldv = 2 * hd;
    a.rel = 1; a.u = m->wT(l, o.u); a.vb = m->wT(l, o.v); a.r = b.r; a.ldr = hd;
    a.dq = dq; a.lddq = hd; a.dk = dkv; a.lddk = 2 * hd; a.dv = dkv + (size_t)hd * es; a.lddv = 2 * hd;
    float* drf = m->dr_f32[ps];
    a.du = gslot + o.u; a.dvb = gslot + o.v; a.dr = drf;
    // The fused path leaves matrices in the workspace whose unwritten cells must be zero; they are
    // the same cells while the memory length stays the same, so it is cleared when that changes.
    if (m->attn_scratch_Mv != Mv) {
      HIPCHK(launch_fill_zero(st, m->attn_scratch, attn_bwd_scratch_floats_any(B, c.n_head, T, m->S, m->pdh) * 4));
      m->attn_scratch_Mv = Mv;
    }
    a.scratch_clean = 1;
    HIPCHK(launch_fill_zero(st, drf, (size_t)S * hd * 4));
    RUN(timed_launch(m, OURO_TIMING_ATTENTION, 2.0 * attn_fwd_flops(m, Mv), st, [&] { return launch_attn_bwd(st, c.dtype, a, 0); }));
    const void* drp = drf;
    if (c.dtype == 1) { HIPCHK(launch_convert(st, 1, m->dr_t[ps], drf, (size_t)S * hd)); drp = m->dr_t[ps]; }
    RUN(ready(3));
    // weight gradients: dW_r = R^T dr, dW_q = x^T dq, dW_kv = [mem ; x]^T dkv
    {
      GemmDesc g = gd(m->rtab, d, 1, drp, hd, 0, gslot + o.W_r, hd, d, hd, S);
      g.out_fp32 = 1; g.accumulate = 1;
      wg[nwg++] = g;
    }
    {
      GemmDesc g = gd(b.x, d, 1, dq, hd, 0, gslot + o.W_qkv, 3 * hd, d, hd, N);
      g.out_fp32 = 1; g.accumulate = 1;
      wg[nwg++] = g;
    }
    {
      GemmDesc g = gd(cat, d, 1, dkv, 2 * hd, 0, gslot + o.W_qkv + hd, 3 * hd, d, 2 * hd, B * S);
      g.out_fp32 = 1; g.accumulate = 1;
      wg[nwg++] = g;
    }
    RUN(run_gemm_group_on(m, wg, nwg, sw));
    {
      GemmDesc g = gd(dq, hd, 0, m->wT(l, o.W_qkv), 3 * hd, 1, dx, d, N, d, hd);
      g.residual = ds1; g.ldr = d; g.out_fp32 = 1;
      RUN(run_gemm(m, g));
    }
    // the memory rows are constants: only the current rows of d[mem ; x] reach dx
    if (c.dtype == 1) {
      // one product per batch element over its T current rows of dkv, added to dx in place
      GemmDesc g = gd(dkv + (size_t)Mv * 2 * hd * es, 2 * hd, 0, m->wT(l, o.W_qkv) + (size_t)hd * es, 3 * hd, 1, dx, d, T, d, 2 * hd);
      g.by = B; g.sAy = (long long)S * 2 * hd; g.sCy = (long long)T * d;
      g.out_fp32 = 1; g.res32 = (const float*)dx; g.ldr32 = d;
      RUN(run_gemm(m, g));
    } else {
      RUN(run_gemm(m, gd(dkv, 2 * hd, 0, m->wT(l, o.W_qkv) + (size_t)hd * es, 3 * hd, 1, m->dcat, d, B * S, d, 2 * hd)));
      size_t n = (size_t)T * d;
      dim3 grid((unsigned)std::min<size_t>((n + 255) / 256, 1024), B), block(256);
      hipLaunchKernelGGL(add_rows_kernel<float>, grid, block, 0, st, (float*)dx, n, (const float*)m->dcat, (size_t)S * d, (size_t)Mv * d, n);
      HIPCHK(hipGetLastError());
    }
  }
  if (side) { HIPCHK(hipEventRecord(m->ev_side_done[ps], sw)); m->side_busy[ps] = true; }
  return OURO_OK;
}

// defer_join: leave the side stream's share of this module's gradient unjoined (ev_join is
// recorded on the side stream; the caller orders the gradient's reader behind it).
static int module_backward_impl(ouro_model* m, int k, bool defer_join) {
  const ouro_config& c = m->cfg;
  const int K = c.n_module, d = m->pd, V = c.vocab, N = m->N;
  if (k < 1 || k > K) return fail(OURO_E_ARG, "module_backward: k=%d outside 1..%d", k, K);
  if (m->inject_mask) return fail(OURO_E_SEQUENCE, "module_backward after inject_grad in the same iteration");
  if (m->fwd_next != K + 1) return fail(OURO_E_SEQUENCE, "module_backward before forward of module %d", m->fwd_next);
  if (k != m->bwd_next) return fail(OURO_E_SEQUENCE, "module_backward(%d) but module %d is next", k, m->bwd_next);
  const bool stored = c.schedule == 1;          // stored-input schedule: this pass is for mini-batch t-K+k
  int64_t slot, tau;
  if (stored) { slot = 0; tau = m->t - K + k; }
  else ouro_slot_index(K, k, m->t, 1, &slot, &tau);
  if (stored && tau < 0) {
    // no error gradient has reached this module yet: it computes nothing (zero gradient)
    m->in_last_slot[k] = -1; m->in_last_tau[k] = -1;
    if (m->use_side) HIPCHK(hipEventRecord(m->ev_join, m->side));
    m->bwd_next = k - 1;
    return OURO_OK;
  }
  const int first = m->first_layer[k - 1], last = m->first_layer[k] - 1;
  const int32_t* tok = m->tok;
  char* dh_top = m->dhb[last % 3];
  if (stored && k < K) {
    // recompute the module's activations from its stored input of iteration tau with the
    // weights it holds now; the last layer's output is not needed
    const int64_t is = tau % m->indepth[k];
    if (m->intags[k][is] != tau) return fail(OURO_E_STALE, "module %d input slot %lld holds iteration %lld, wanted %lld", k, (long long)is, (long long)m->intags[k][is], (long long)tau);
    m->in_last_slot[k] = is; m->in_last_tau[k] = tau;
    const char* src = m->inring[k] + (size_t)is * m->instride[k];
    m->cur_seed = c.seed + (uint64_t)tau;           // the stored seed: the masks of the original pass
    if (k == 1) {
      tok = (const int32_t*)src;
      const DropDesc dd = drop_at(m, 0);
      HIPCHK(launch_embed_fwd(m->stream, c.dtype, tok, m->vT(), m->pe, m->L[0].x, N, c.seq_len, d, V, c.emb_scale, m->flag, &dd));
    } else {
      HIPCHK(hipMemcpyAsync(m->L[first].x, src, (size_t)N * d * m->esz, hipMemcpyDeviceToDevice, m->stream));
    }
    m->mem_valid = mem_valid_at(m, tau);            // this module works on iteration tau's memories
    for (int l = first; l <= last; ++l) {
      select_memory(m, l, tau);
      RUN(layer_forward(m, l, l == last ? m->hscratch : nullptr, l > first));   // the first layer's input is the stored one
    }
    // error gradient of this module's output, left by module k+1 one iteration ago
    const int pr = (int)((m->t + 1) & 1);
    if (m->mailtag[pr][k] != tau) return fail(OURO_E_STALE, "module %d error gradient is of mini-batch %lld, wanted %lld", k, (long long)m->mailtag[pr][k], (long long)tau);
    dh_top = m->mail[pr][k];
  }
  float* gslot = m->slot_ptr(k, slot);
  HIPCHK(launch_fill_zero(m->stream, gslot, (size_t)m->gstride[k] * 4));
  if (k == K) {
    // Eq. 7 (right): dV_o = G^T h_L ; error gradient dh_L = G V
    float* dvo = m->slot_ptr(K + 1, 0);
    // bf16 mode: both contractions run over the padded vocabulary (G's padding columns and
    // V's padding rows are zero), which keeps them on the MFMA kernels for any vocabulary size
    const int Vx = c.dtype == 1 ? m->ldv : V;
    GemmDesc g = gd(m->G, m->ldv, 1, m->hL, d, 0, dvo, d, Vx, d, N);
    g.out_fp32 = 1;
    if (m->use_side) {        // independent of the error-gradient chain: beside dh_L = G V
      HIPCHK(hipEventRecord(m->ev_ready[0], m->stream));
      HIPCHK(hipStreamWaitEvent(m->side, m->ev_ready[0], 0));
      RUN(run_gemm_on(m, g, m->side));
    } else {
      RUN(run_gemm(m, g));
    }
    m->tags[K + 1][0] = m->t;
    GemmDesc gh = c.dtype == 1 ? gd(m->G, m->ldv, 0, (const char*)m->shadowT[0], m->ldv, 1, dh_top, d, N, d, Vx)
                               : gd(m->G, m->ldv, 0, m->vT(), d, 0, dh_top, d, N, d, Vx);
    gh.out_fp32 = 1;                                  // the error gradient between layers is fp32
    if (c.dtype == 1 && gemm_uses_mfma(c.dtype, gh) && V >= 8192) {
      // The contraction runs over the whole vocabulary onto a narrow output: split it over
      // the grid (two workgroups per CU instead of one), adding into the zeroed fp32 result.
      HIPCHK(launch_fill_zero(m->stream, dh_top, (size_t)N * d * 4));
      gh.accumulate = 1;
      RUN(run_gemm(m, gh));
    } else {
      RUN(run_gemm(m, gh));
    }
  }
  // layer l reads its output gradient from dhb[l % 3] and writes its input gradient to dhb[(l + 2) % 3]:
  // three buffers, so that side-stream readers of layer l's input are two layers away from its next writer.
  // Stored-input schedule: the top layer of a module below K reads the mailbox instead, and the
  // bottom layer of a module above 1 writes the mailbox of the module below.
  for (int l = last; l >= first; --l) {
    char* dh = l == last ? dh_top : m->dhb[l % 3];
    char* dx = m->dhb[(l + 2) % 3];
    if (stored && k > 1 && l == first) {
      const int pw = (int)(m->t & 1);
      dx = m->mail[pw][k - 1];
      m->mailtag[pw][k - 1] = tau;
    }
    RUN(layer_backward(m, l, dh, dx, gslot));
  }
  if (stored) m->mem_valid = mem_valid_at(m, m->t);
  // the layers' vector gradients: sum of the copies into the slot.  On the stream of the
  // weight-gradient work, which has waited for every LayerNorm kernel of the module.
  HIPCHK(launch_sum_segments(m->use_side ? m->side : m->stream, m->segs_dev[k], (int)m->segs[k].size(), m->vec_copies, m->vec_stride, gslot));
  if (m->use_side) {          // the module's gradient is complete once the side work has joined
    HIPCHK(hipEventRecord(m->ev_join, m->side));
    if (!defer_join) {
      HIPCHK(hipStreamWaitEvent(m->stream, m->ev_join, 0));
      m->side_busy[0] = m->side_busy[1] = false;
    }
  }
  m->tags[k][slot] = m->t;
  if (k == 1) {
    // Eq. 7 (left): dV_i rows = scattered error gradient of the embedding output
    int64_t s0 = 0, t0;
    if (!stored) ouro_slot_index(K, 0, m->t, 1, &s0, &t0);
    float* dvi = m->slot_ptr(0, s0);
    HIPCHK(launch_fill_zero(m->stream, dvi, (size_t)m->gstride[0] * 4));
    const DropDesc dd = drop_at(m, 0);
    HIPCHK(launch_embed_bwd(m->stream, 0, tok, m->dhb[2], dvi, N, d, V, c.emb_scale, &dd));   // dh is fp32
    m->tags[0][s0] = m->t;
  }
  m->cur_seed = c.seed + (uint64_t)m->t;
  m->bwd_next = k - 1;
  return OURO_OK;
}

extern "C" int ouro_module_backward(ouro_model* m, int k) {
  if (!m) return fail(OURO_E_ARG, "model is null");
  return module_backward_impl(m, k, false);
}

// ------------------------------------------------------------------------------- update
static int close_iteration(ouro_model* m) {
  const ouro_config& c = m->cfg;
  if (c.mem_len > 0 && c.schedule == 1) {
    // the forward pass already filled the slots of iteration t+1
    for (int l = 0; l < c.n_layer; ++l) select_memory(m, l, m->t + 1);
    m->mem_valid = mem_valid_at(m, m->t + 1);
  } else if (c.mem_len > 0) {
    // memory for t+1 = last M rows of [memory ; layer input] (constants, no gradient)
    const int T = c.seq_len, d = m->pd, Mv = m->mem_valid, S = Mv + T;
    const int Mn = std::min(c.mem_len, S);
    for (int l = 0; l < c.n_layer; ++l) {
      LayerBuf& b = m->L[l];
      const char* cat = Mv > 0 ? b.cat : b.x;
      HIPCHK(launch_copy_rows(m->stream, c.dtype, b.mem, (size_t)Mn * d, 0, cat, (size_t)S * d, (size_t)(S - Mn) * d, c.batch, Mn, d));
    }
    m->mem_valid = Mn;
  }
  m->t += 1;
  m->fwd_next = 1; m->bwd_next = c.n_module; m->upd_mask = 0; m->inject_mask = 0;
  return OURO_OK;
}

// One optimizer step of a parameter group with the gradient Eq. 8 / Eq. 9 select, on stream st.
static int update_group(ouro_model* m, int group, float lr, hipStream_t st) {
  const ouro_config& c = m->cfg;
  const int K = c.n_module;
  UpdateDesc u;
  memset(&u, 0, sizeof u);
  u.w = m->master[group]; u.m = m->adam_m[group]; u.v = m->adam_v[group]; u.shadow = m->shadow[group];
  u.n = (size_t)m->pcount[group]; u.adam = c.optimizer; u.lr = lr;
  u.beta1 = c.beta1; u.beta2 = c.beta2; u.eps = c.eps;
  u.bc1 = (float)(1.0 - std::pow((double)c.beta1, (double)(m->t + 1)));   // global t+1 (Algorithm 2)
  u.bc2 = (float)(1.0 - std::pow((double)c.beta2, (double)(m->t + 1)));
  int64_t slot, tau;
  const bool stored = c.schedule == 1;
  if (group >= 1 && stored) {
    // the gradient of mini-batch t-K+k was computed in this iteration (or nothing was)
    tau = m->t - K + group;
    m->last_slot[group] = tau >= 0 ? 0 : -1; m->last_tau[group] = tau >= 0 ? tau : -1;
    if (tau >= 0) {
      if (m->tags[group][0] != m->t) return fail(OURO_E_STALE, "module %d gradient is of iteration %lld, wanted %lld", group, (long long)m->tags[group][0], (long long)m->t);
      u.g0 = m->slot_ptr(group, 0); u.gscale0 = 1.f;
    }
  } else if (group >= 1) {
    ouro_slot_index(K, group, m->t, 0, &slot, &tau);                        // Eq. 8
    m->last_slot[group] = slot; m->last_tau[group] = tau;
    if (tau >= 0) {
      if (m->tags[group][slot] != tau) return fail(OURO_E_STALE, "module %d slot %lld holds iteration %lld, wanted %lld", group, (long long)slot, (long long)m->tags[group][slot], (long long)tau);
      u.g0 = m->slot_ptr(group, slot); u.gscale0 = 1.f;
    }
  } else {
    int64_t si, ti;                                                         // Eq. 9
    ouro_slot_index(K, 0, m->t, 0, &si, &ti);
    int64_t want = ti;                        // tag the dV_i slot must carry
    if (stored) { si = ti >= 0 ? 0 : -1; want = m->t; }
    m->last_slot[0] = si; m->last_tau[0] = ti;
    m->last_slot[K + 1] = -1; m->last_tau[K + 1] = -1;
    if (ti >= 0 || c.embed_warm_mode == 1) {
      if (m->tags[K + 1][0] != m->t) return fail(OURO_E_STALE, "dV_o slot holds iteration %lld, wanted %lld", (long long)m->tags[K + 1][0], (long long)m->t);
      u.g0 = m->slot_ptr(K + 1, 0); u.gscale0 = 0.5f;
      m->last_slot[K + 1] = 0; m->last_tau[K + 1] = m->t;
    }
    if (ti >= 0) {
      if (m->tags[0][si] != want) return fail(OURO_E_STALE, "dV_i slot %lld holds iteration %lld, wanted %lld", (long long)si, (long long)m->tags[0][si], (long long)want);
      u.g1 = m->slot_ptr(0, si); u.gscale1 = 0.5f;
    }
  }
  const bool timed = m->timing && u.g0;
  if (timed) RUN(timing_begin(m, OURO_TIMING_UPDATE, st));
  HIPCHK(launch_update(st, u));
  if (timed) {
    // algorithmic bytes per element: gradient(s) 4 each, w read+write 8, Adam m,v read+write 16, bf16 copy 2
    double per = 4.0 * ((u.g0 ? 1 : 0) + (u.g1 ? 1 : 0)) + 8.0 + (u.adam ? 16.0 : 0.0) + (u.shadow ? 2.0 : 0.0);
    RUN(timing_end(m, OURO_TIMING_UPDATE, per * (double)u.n, st));
  }
  RUN(refresh_transposed(m, group, st));
  m->upd_mask |= 1ull << group;
  if (m->upd_mask == (1ull << (K + 1)) - 1) {
    if (m->upd_pending) {       // the next iteration reads every weight: main waits for aux
      HIPCHK(hipEventRecord(m->ev_upd_done, m->aux));
      HIPCHK(hipStreamWaitEvent(m->stream, m->ev_upd_done, 0));
      m->upd_pending = false;
    }
    return close_iteration(m);
  }
  return OURO_OK;
}

extern "C" int ouro_delayed_update(ouro_model* m, int group, float lr) {
  if (!m) return fail(OURO_E_ARG, "model is null");
  const int K = m->cfg.n_module;
  if (group < 0 || group > K) return fail(OURO_E_ARG, "delayed_update: group=%d outside 0..%d", group, K);
  if (m->fwd_next != K + 1 || m->bwd_next != 0) return fail(OURO_E_SEQUENCE, "delayed_update before backward of module 1");
  if (m->upd_mask & (1ull << group)) return fail(OURO_E_SEQUENCE, "delayed_update(%d) twice in one iteration", group);
  return update_group(m, group, lr, m->stream);
}

static int read_loss(ouro_model* m, float* host_loss) {
  struct { float loss; int flag; } h;
  HIPCHK(hipMemcpyAsync(&h.loss, m->loss, 4, hipMemcpyDeviceToHost, m->stream));
  HIPCHK(hipMemcpyAsync(&h.flag, m->flag, 4, hipMemcpyDeviceToHost, m->stream));
  HIPCHK(hipStreamSynchronize(m->stream));
  *host_loss = h.loss;
  if (h.flag) return fail(OURO_E_TOKEN, "token or target id outside [0, vocab) (flag %d)", h.flag);
  return OURO_OK;
}

extern "C" int ouro_get_loss(ouro_model* m, float* host_loss) {
  if (!m || !host_loss) return fail(OURO_E_ARG, "get_loss: bad argument");
  return read_loss(m, host_loss);
}

extern "C" int ouro_step(ouro_model* m, const int32_t* dev_tokens, const int32_t* dev_targets, float lr,
                         float* host_loss) {
  if (!m || !dev_tokens || !dev_targets) return fail(OURO_E_ARG, "step: null argument");
  const int K = m->cfg.n_module;
  for (int k = 1; k <= K; ++k) RUN(ouro_module_forward(m, k, dev_tokens, dev_targets));
  // Module k's weights are last read by its own backward pass, and the gradient Eq. 8 hands
  // it is either an older ring slot or (k = K) the one that pass just completed; V is last
  // read by module K's backward, and for K > 1 Eq. 9 pairs the fresh dV_o with an older dV_i.
  // So each update is enqueued on the third stream right behind that backward pass and
  // overlaps the backward passes of the modules below; the results are those of the serial
  // order, since the groups are disjoint. Per-launch timing keeps the serial order.
  if (m->cfg.schedule == 1 && K > 1 && m->use_side && !m->timing) {
    // Stored-input schedule: the K backward passes of an iteration are independent (each works
    // on its own mini-batch from its own stored input and mailbox), so each runs on the streams
    // and scratch buffers of its own set, followed there by its module's update; module 1 stays
    // on the caller's stream.  V waits for both of its halves (modules 1 and K).
    HIPCHK(hipEventRecord(m->ev_fwd, m->stream));
    hipEvent_t fwd = m->ev_fwd;
    int rc = OURO_OK;
    for (int k = K; k >= 1 && rc == OURO_OK; --k) {
      activate(m, k - 1);
      if (k > 1) {
        hipError_t e = hipStreamWaitEvent(m->stream, fwd, 0);
        if (e != hipSuccess) { rc = fail(OURO_E_HIP, "%s", hipGetErrorString(e)); break; }
      }
      rc = module_backward_impl(m, k, false);
      if (rc == OURO_OK && k > 1) {
        rc = update_group(m, k, lr, m->stream);
        if (rc == OURO_OK && hipEventRecord(m->ev_done, m->stream) != hipSuccess) rc = fail(OURO_E_HIP, "event record failed");
      }
    }
    activate(m, 0);
    if (rc) return rc;
    for (size_t i = 1; i < m->ctxs.size(); ++i) HIPCHK(hipStreamWaitEvent(m->stream, m->ctxs[i].ev_done, 0));
    RUN(update_group(m, 1, lr, m->stream));
    RUN(update_group(m, 0, lr, m->stream));
    if (host_loss) return read_loss(m, host_loss);
    return OURO_OK;
  }
  const bool early = m->use_side && !m->timing;
  for (int k = K; k >= 1; --k) {
    RUN(module_backward_impl(m, k, early && k > 1));
    if (early && k > 1) {
      // the update waits for both halves of the gradient; the main stream goes straight on
      HIPCHK(hipEventRecord(m->ev_bwd_done, m->stream));
      HIPCHK(hipStreamWaitEvent(m->aux, m->ev_bwd_done, 0));
      HIPCHK(hipStreamWaitEvent(m->aux, m->ev_join, 0));
      m->upd_pending = true;
      RUN(update_group(m, k, lr, m->aux));
      // (stored-input schedule: module 1's recomputation still reads V, so V waits)
      if (k == K && m->cfg.schedule == 0) RUN(update_group(m, 0, lr, m->aux));
    }
  }
  const uint64_t done = m->upd_mask;    // the last update closes the iteration and clears the mask
  for (int k = 0; k <= K; ++k)
    if (!(done & (1ull << k))) RUN(update_group(m, k, lr, m->stream));
  if (host_loss) return read_loss(m, host_loss);
  return OURO_OK;
}

// ------------------------------------------------------------------- evaluation, state
extern "C" int ouro_eval_step(ouro_model* m, const int32_t* dev_tokens, const int32_t* dev_targets, float* host_loss) {
  if (!m || !dev_tokens || !dev_targets) return fail(OURO_E_ARG, "eval_step: null argument");
  if (m->fwd_next != 1 || m->inject_mask) return fail(OURO_E_SEQUENCE, "eval_step inside a training iteration");
  const int K = m->cfg.n_module;
  m->eval_mode = true;
  int rc = OURO_OK;
  for (int k = 1; k <= K && rc == OURO_OK; ++k) rc = ouro_module_forward(m, k, dev_tokens, dev_targets);
  m->eval_mode = false;
  if (rc) { m->fwd_next = 1; return rc; }
  rc = close_iteration(m);          // segment memories roll; the counter moves on
  if (rc) return rc;
  if (host_loss) return read_loss(m, host_loss);
  return OURO_OK;
}

namespace {
struct StateHeader {
  uint64_t magic;
  uint32_t version, header_bytes;
  ouro_config cfg;                  // layers_per_module pointer zeroed
  int32_t lpm[64];
  int64_t t;
  int32_t mem_valid, n_tags;
  uint64_t persist_bytes, mem_bytes;
};
const uint64_t STATE_MAGIC = 0x4f55524f53544154ull;   // "OUROSTAT"

void fill_header(const ouro_model* m, StateHeader& h) {
  memset(&h, 0, sizeof h);
  h.magic = STATE_MAGIC; h.version = 1; h.header_bytes = (uint32_t)sizeof(StateHeader);
  h.cfg = m->cfg; h.cfg.layers_per_module = nullptr;
  for (size_t i = 0; i < m->lpm.size(); ++i) h.lpm[i] = m->lpm[i];
  h.t = m->t; h.mem_valid = m->mem_valid;
  size_t nt = 0;
  for (const auto& v : m->tags) nt += v.size();
  for (const auto& v : m->intags) nt += v.size();
  nt += m->mailtag[0].size() + m->mailtag[1].size();
  h.n_tags = (int32_t)nt;
  h.persist_bytes = m->persist_end;
  size_t mb = 0;
  for (const LayerBuf& b : m->L) {
    if (b.memring) mb += b.memstride * (size_t)b.memdepth;
    else if (b.mem) mb += (size_t)m->cfg.batch * m->cfg.mem_len * m->pd * m->esz;
  }
  h.mem_bytes = mb;
}
bool same_config(const ouro_config& a, const ouro_config& b) {
  return a.n_layer == b.n_layer && a.d_model == b.d_model && a.n_head == b.n_head && a.d_head == b.d_head &&
         a.d_ff == b.d_ff && a.vocab == b.vocab && a.seq_len == b.seq_len && a.mem_len == b.mem_len &&
         a.batch == b.batch && a.n_module == b.n_module && a.rel_pos == b.rel_pos && a.dtype == b.dtype &&
         a.optimizer == b.optimizer && a.beta1 == b.beta1 && a.beta2 == b.beta2 && a.eps == b.eps &&
         a.embed_warm_mode == b.embed_warm_mode && a.emb_scale == b.emb_scale && a.schedule == b.schedule &&
         a.dropout == b.dropout && a.seed == b.seed;
}
size_t state_bytes(const StateHeader& h) { return sizeof(StateHeader) + (size_t)h.n_tags * 8 + h.persist_bytes + h.mem_bytes; }
}  // namespace

extern "C" int ouro_state_bytes(const ouro_model* m, size_t* bytes) {
  if (!m || !bytes) return fail(OURO_E_ARG, "state_bytes: null argument");
  StateHeader h;
  fill_header(m, h);
  *bytes = state_bytes(h);
  return OURO_OK;
}

extern "C" int ouro_save_state(ouro_model* m, void* host_dst, size_t bytes) {
  if (!m || !host_dst) return fail(OURO_E_ARG, "save_state: null argument");
  if (m->fwd_next != 1 || m->inject_mask) return fail(OURO_E_SEQUENCE, "save_state inside an iteration");
  StateHeader h;
  fill_header(m, h);
  if (bytes != state_bytes(h)) return fail(OURO_E_ARG, "save_state: buffer has %zu bytes, state has %zu", bytes, state_bytes(h));
  char* p = (char*)host_dst;
  memcpy(p, &h, sizeof h); p += sizeof h;
  int64_t* tg = (int64_t*)p;
  for (const auto& v : m->tags) for (int64_t x : v) *tg++ = x;
  for (const auto& v : m->intags) for (int64_t x : v) *tg++ = x;
  for (int q = 0; q < 2; ++q) for (int64_t x : m->mailtag[q]) *tg++ = x;
  p = (char*)tg;
  HIPCHK(hipStreamSynchronize(m->side));
  HIPCHK(hipStreamSynchronize(m->aux));
  HIPCHK(hipMemcpyAsync(p, m->arena, m->persist_end, hipMemcpyDeviceToHost, m->stream)); p += m->persist_end;
  for (const LayerBuf& b : m->L) {
    const size_t n = b.memring ? b.memstride * (size_t)b.memdepth : b.mem ? (size_t)m->cfg.batch * m->cfg.mem_len * m->pd * m->esz : 0;
    if (!n) continue;
    HIPCHK(hipMemcpyAsync(p, b.memring ? b.memring : b.mem, n, hipMemcpyDeviceToHost, m->stream)); p += n;
  }
  HIPCHK(hipStreamSynchronize(m->stream));
  return OURO_OK;
}

extern "C" int ouro_load_state(ouro_model* m, const void* host_src, size_t bytes) {
  if (!m || !host_src) return fail(OURO_E_ARG, "load_state: null argument");
  if (m->fwd_next != 1 || m->inject_mask) return fail(OURO_E_SEQUENCE, "load_state inside an iteration");
  if (bytes < sizeof(StateHeader)) return fail(OURO_E_ARG, "load_state: buffer too short");
  StateHeader h, mine;
  memcpy(&h, host_src, sizeof h);
  fill_header(m, mine);
  if (h.magic != STATE_MAGIC || h.version != 1 || h.header_bytes != sizeof(StateHeader)) return fail(OURO_E_ARG, "load_state: not a state of this library version");
  if (!same_config(h.cfg, mine.cfg) || memcmp(h.lpm, mine.lpm, sizeof h.lpm) || h.n_tags != mine.n_tags ||
      h.persist_bytes != mine.persist_bytes || h.mem_bytes != mine.mem_bytes)
    return fail(OURO_E_CONFIG, "load_state: the state was saved by a model with another configuration");
  if (bytes != state_bytes(h)) return fail(OURO_E_ARG, "load_state: buffer has %zu bytes, state has %zu", bytes, state_bytes(h));
  const char* p = (const char*)host_src + sizeof h;
  const int64_t* tg = (const int64_t*)p;
  for (auto& v : m->tags) for (int64_t& x : v) x = *tg++;
  for (auto& v : m->intags) for (int64_t& x : v) x = *tg++;
  for (int q = 0; q < 2; ++q) for (int64_t& x : m->mailtag[q]) x = *tg++;
  p = (const char*)tg;
  HIPCHK(hipStreamSynchronize(m->side));
  HIPCHK(hipStreamSynchronize(m->aux));
  HIPCHK(hipMemcpyAsync(m->arena, p, m->persist_end, hipMemcpyHostToDevice, m->stream)); p += m->persist_end;
  for (LayerBuf& b : m->L) {
    const size_t n = b.memring ? b.memstride * (size_t)b.memdepth : b.mem ? (size_t)m->cfg.batch * m->cfg.mem_len * m->pd * m->esz : 0;
    if (!n) continue;
    HIPCHK(hipMemcpyAsync(b.memring ? b.memring : b.mem, p, n, hipMemcpyHostToDevice, m->stream)); p += n;
  }
  HIPCHK(hipStreamSynchronize(m->stream));
  m->t = h.t; m->mem_valid = h.mem_valid;
  m->cur_seed = m->cfg.seed + (uint64_t)m->t;
  for (int l = 0; l < m->cfg.n_layer; ++l) select_memory(m, l, m->t);
  m->upd_mask = 0; m->upd_pending = false;
  m->side_busy[0] = m->side_busy[1] = false;
  std::fill(m->last_slot.begin(), m->last_slot.end(), -1); std::fill(m->last_tau.begin(), m->last_tau.end(), -1);
  return OURO_OK;
}

// -------------------------------------------------------------------------- debug hooks
extern "C" int ouro_debug_slot_tag(ouro_model* m, int id, int64_t slot, int64_t* tag) {
  if (!m || !tag || id < 0 || id > m->cfg.n_module + 1 || slot < 0 || slot >= m->depth[id]) return fail(OURO_E_ARG, "slot_tag: bad argument");
  *tag = m->tags[id][slot];
  return OURO_OK;
}

extern "C" int ouro_debug_last_read(ouro_model* m, int id, int64_t* slot, int64_t* tau) {
  if (!m || !slot || !tau || id < 0 || id > m->cfg.n_module + 1) return fail(OURO_E_ARG, "last_read: bad argument");
  *slot = m->last_slot[id];
  *tau = m->last_tau[id];
  return OURO_OK;
}

extern "C" int ouro_debug_input_tag(ouro_model* m, int k, int64_t slot, int64_t* tag) {
  if (!m || !tag || k < 1 || k > m->cfg.n_module || slot < 0 || slot >= m->indepth[k]) return fail(OURO_E_ARG, "input_tag: bad argument");
  *tag = m->intags[k][slot];
  return OURO_OK;
}

extern "C" int ouro_debug_last_input_read(ouro_model* m, int k, int64_t* slot, int64_t* tau) {
  if (!m || !slot || !tau || k < 1 || k > m->cfg.n_module) return fail(OURO_E_ARG, "last_input_read: bad argument");
  *slot = m->in_last_slot[k];
  *tau = m->in_last_tau[k];
  return OURO_OK;
}

extern "C" int ouro_debug_inject_grad(ouro_model* m, int id, const float* host_g, int64_t n) {
  if (!m || !host_g) return fail(OURO_E_ARG, "inject_grad: null argument");
  const int K = m->cfg.n_module;
  if (id < 0 || id > K + 1) return fail(OURO_E_ARG, "inject_grad: id=%d outside 0..%d", id, K + 1);
  if (n != m->gcount[id]) return fail(OURO_E_ARG, "inject_grad: store %d has %lld elements", id, (long long)m->gcount[id]);
  if (m->fwd_next != 1 && !m->inject_mask) return fail(OURO_E_SEQUENCE, "inject_grad after module_forward in the same iteration");
  if (m->inject_mask & (1ull << id)) return fail(OURO_E_SEQUENCE, "inject_grad(%d) twice in one iteration", id);
  int64_t slot, tau;
  ouro_slot_index(K, id, m->t, 1, &slot, &tau);
  if (m->cfg.schedule == 1) slot = 0;
  if (m->padded) {
    const int grp = (id == 0 || id == K + 1) ? 0 : id;
    std::vector<float> stored((size_t)m->pcount[grp], 0.f);
    remap_group(m, grp, stored.data(), const_cast<float*>(host_g), true);
    HIPCHK(hipMemcpyAsync(m->slot_ptr(id, slot), stored.data(), stored.size() * 4, hipMemcpyHostToDevice, m->stream));
  } else {
    HIPCHK(hipMemcpyAsync(m->slot_ptr(id, slot), host_g, (size_t)n * 4, hipMemcpyHostToDevice, m->stream));
  }
  HIPCHK(hipStreamSynchronize(m->stream));
  m->tags[id][slot] = m->t;
  m->inject_mask |= 1ull << id;
  if (m->inject_mask == (1ull << (K + 2)) - 1) { m->fwd_next = K + 1; m->bwd_next = 0; }
  return OURO_OK;
}

extern "C" int ouro_get_grad_slot(ouro_model* m, int id, int64_t tau, float* host_dst, int64_t n) {
  if (!m || !host_dst || id < 0 || id > m->cfg.n_module + 1 || tau < 0) return fail(OURO_E_ARG, "get_grad_slot: bad argument");
  if (n != m->gcount[id]) return fail(OURO_E_ARG, "get_grad_slot: wrong element count");
  int64_t slot = tau % m->depth[id];
  if (m->tags[id][slot] != tau) return fail(OURO_E_STALE, "store %d no longer holds iteration %lld", id, (long long)tau);
  if (m->padded) {
    const int grp = (id == 0 || id == m->cfg.n_module + 1) ? 0 : id;
    std::vector<float> stored((size_t)m->pcount[grp]);
    HIPCHK(hipMemcpyAsync(stored.data(), m->slot_ptr(id, slot), stored.size() * 4, hipMemcpyDeviceToHost, m->stream));
    HIPCHK(hipStreamSynchronize(m->stream));
    remap_group(m, grp, stored.data(), host_dst, false);
    return OURO_OK;
  }
  HIPCHK(hipMemcpyAsync(host_dst, m->slot_ptr(id, slot), (size_t)n * 4, hipMemcpyDeviceToHost, m->stream));
  HIPCHK(hipStreamSynchronize(m->stream));
  return OURO_OK;
}

// rows of the stored width in dbg_f32 -> dense rows of d_model floats in host memory
static int rows_to_host(ouro_model* m, float* host_dst, size_t rows) {
  const size_t dl = m->cfg.d_model;
  HIPCHK(hipMemcpy2DAsync(host_dst, dl * 4, m->dbg_f32, (size_t)m->pd * 4, dl * 4, rows, hipMemcpyDeviceToHost, m->stream));
  HIPCHK(hipStreamSynchronize(m->stream));
  return OURO_OK;
}

extern "C" int ouro_get_mems(ouro_model* m, int layer, float* host_dst, int64_t* valid_len) {
  if (!m || !valid_len || layer < 0 || layer >= m->cfg.n_layer) return fail(OURO_E_ARG, "get_mems: bad argument");
  *valid_len = m->mem_valid;
  if (!host_dst || m->mem_valid == 0) return OURO_OK;
  const size_t rows = (size_t)m->cfg.batch * m->mem_valid;
  HIPCHK(launch_to_f32(m->stream, m->cfg.dtype, m->dbg_f32, m->L[layer].mem, rows * m->pd));
  return rows_to_host(m, host_dst, rows);
}

extern "C" int ouro_debug_get_hidden(ouro_model* m, int layer, float* host_dst, int64_t n) {
  if (!m || !host_dst || layer < 0 || layer > m->cfg.n_layer) return fail(OURO_E_ARG, "get_hidden: bad argument");
  size_t cnt = (size_t)m->N * m->cfg.d_model;
  if ((size_t)n != cnt) return fail(OURO_E_ARG, "get_hidden: wrong element count");
  const char* src = layer < m->cfg.n_layer ? m->L[layer].x : m->hL;
  HIPCHK(launch_to_f32(m->stream, m->cfg.dtype, m->dbg_f32, src, (size_t)m->N * m->pd));
  return rows_to_host(m, host_dst, (size_t)m->N);
}

extern "C" int ouro_debug_timing_enable(ouro_model* m, int on) {
  if (!m) return fail(OURO_E_ARG, "model is null");
  m->timing = on ? 1 : 0;
  return OURO_OK;
}

extern "C" int ouro_debug_timing_overhead(ouro_model* m, int reps, double* ms_mean) {
  if (!m || !ms_mean || reps < 1 || reps > 4096) return fail(OURO_E_ARG, "timing_overhead: bad argument");
  // empty brackets (two event records, nothing between), enqueued back to back as in a
  // timed step and read after one wait
  const int warm = 8;
  std::vector<hipEvent_t> ev(2 * (size_t)(reps + warm), nullptr);
  hipError_t e = hipSuccess;
  for (size_t i = 0; i < ev.size() && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
  for (int i = 0; i < reps + warm && e == hipSuccess; ++i) {
    e = hipEventRecord(ev[2 * i], m->stream);
    if (e == hipSuccess) e = hipEventRecord(ev[2 * i + 1], m->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  double total = 0;
  for (int i = warm; i < reps + warm && e == hipSuccess; ++i) {
    float t = 0;
    e = hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1]);
    total += t;
  }
  for (hipEvent_t x : ev) if (x) (void)hipEventDestroy(x);
  if (e != hipSuccess) return fail(OURO_E_HIP, "timing_overhead: %s", hipGetErrorString(e));
  *ms_mean = total / reps;
  return OURO_OK;
}

extern "C" int ouro_debug_set_overlap(ouro_model* m, int on) {
  if (!m) return fail(OURO_E_ARG, "model is null");
  if (m->fwd_next != 1) return fail(OURO_E_SEQUENCE, "set_overlap inside an iteration");
  HIPCHK(hipStreamSynchronize(m->stream));
  HIPCHK(hipStreamSynchronize(m->side));
  HIPCHK(hipStreamSynchronize(m->aux));
  for (size_t i = 1; i < m->ctxs.size(); ++i) {
    HIPCHK(hipStreamSynchronize(m->ctxs[i].stream));
    HIPCHK(hipStreamSynchronize(m->ctxs[i].side));
    m->ctxs[i].side_busy[0] = m->ctxs[i].side_busy[1] = false;
  }
  m->side_busy[0] = m->side_busy[1] = false;
  m->use_side = on != 0;
  return OURO_OK;
}

extern "C" int ouro_debug_timing_read(ouro_model* m, int kind, double* ms, int64_t* launches, double* work) {
  if (!m || kind < 0 || kind >= OURO_TIMING_KINDS) return fail(OURO_E_ARG, "timing_read: bad argument");
  HIPCHK(hipStreamSynchronize(m->stream));
  double total = 0;
  for (size_t i = 0; i + 1 < m->ev_used[kind]; i += 2) {
    float t = 0;
    HIPCHK(hipEventElapsedTime(&t, m->ev[kind][i], m->ev[kind][i + 1]));
    total += t;
  }
  if (ms) *ms = total;
  if (launches) *launches = m->timed_launches[kind];
  if (work) *work = m->timed_work[kind];
  m->ev_used[kind] = 0; m->timed_work[kind] = 0; m->timed_launches[kind] = 0;
  return OURO_OK;
}
