"""CPU fp64 oracle for the Ouroboros training step.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module; the product path (the HIP library and its binding) never does.  It shares no
code with the HIP path: plain numpy in fp64, no blocking, no fusion, no ring buffers.

What it computes, with the passage of the paper each part follows:

  * The network is a chain of L layers with a tied input-embedding / output-projection
    matrix V = V_i = V_o (Section 2, Eq. 1-3) trained on the LM loss (Eq. 4).
  * Backpropagation is the chain rule of Eq. 6; V_i and V_o are differentiated as two
    separate leaves that hold equal values (Eq. 7).
  * The layers are split into K contiguous modules G(1..K) (Section 3.1).  At iteration
    t module k uses the gradient of mini-batch t-K+k evaluated at the full weight
    vector of iteration t-K+k, or zero while t-K+k < 0 (Eq. 8).
  * The tied matrix uses g_V = 1/2 dV_o(t) + 1/2 dV_i(t-K+1), zero while t-K+1 < 0
    (Eq. 9; `embed_warm_mode=1` is the term-wise reading where only the V_i term is
    dropped during those steps).
  * The step size follows a linear warm-up and then a cosine decay (`learning_rate`,
    Section 5.2).
  * SGD (Algorithm 1) or Adam (Algorithm 2, appendix): every group steps at every t,
    also with a zero gradient; bias correction uses the global t+1; epsilon is added
    outside the square root after bias correction.

The paper does not define the Transformer layer itself; the oracle fixes the reading
(post-LN blocks, bias-free attention projections, exact-erf GELU, fixed sinusoid
positions, Transformer-XL relative attention with per-layer u, v, W_r and a constant
segment memory).  Those readings are pinned by finite differences, closed forms and an
independent autograd model in tests/, not by the paper: "parity unpinned" against the
paper for the layer internals and for whole-trajectory loss values (the paper prints
none).

`RecomputeOracle` is the memory-saving schedule of Section 3.1 ("Memory Consumption") and
Section 5.2 ("Repeatable Dropout"): every module stores only its input of each iteration,
re-runs its forward pass on the input of mini-batch t-K+k with the weights it holds now, and
back-propagates the error gradient the module above produced one iteration earlier.

The oracle keeps the gradient of every past step in an unbounded list indexed by the
step number (no modulo arithmetic), and `brute_check` re-derives any used gradient from
a stored copy of that step's full weights and batch.
"""
from __future__ import annotations

import copy
import math

import numpy as np
from scipy.special import erf

LN_EPS = 1e-5


# ----------------------------------------------------------------------------- config
class Config:
    def __init__(self, n_layer, d_model, n_head, d_head, d_ff, vocab, seq_len, batch,
                 n_module=1, mem_len=0, rel_pos=0, layers_per_module=None, optimizer=0,
                 beta1=0.9, beta2=0.999, eps=1e-8, embed_warm_mode=0, emb_scale=1.0,
                 dropout=0.0, seed=0, **_):
        assert n_head * d_head == d_model
        assert d_model % 2 == 0
        assert mem_len == 0 or rel_pos
        self.n_layer, self.d_model, self.n_head, self.d_head = n_layer, d_model, n_head, d_head
        self.d_ff, self.vocab, self.seq_len, self.batch = d_ff, vocab, seq_len, batch
        self.n_module, self.mem_len, self.rel_pos = n_module, mem_len, rel_pos
        self.optimizer, self.beta1, self.beta2, self.eps = optimizer, beta1, beta2, eps
        self.embed_warm_mode, self.emb_scale = embed_warm_mode, emb_scale
        assert 0.0 <= dropout < 1.0
        self.dropout, self.seed = float(dropout), int(seed)
        if layers_per_module is None:
            layers_per_module = split_layers(n_layer, n_module)
        assert len(layers_per_module) == n_module and sum(layers_per_module) == n_layer
        self.layers_per_module = list(layers_per_module)


def split_layers(n_layer, n_module):
    """Contiguous groups G(k) (Section 3.1); if K does not divide L the interior
    modules take the extra layers first."""
    base, rem = divmod(n_layer, n_module)
    sizes = [base] * n_module
    order = list(range(1, n_module - 1)) + [0, n_module - 1]
    for i in range(rem):
        sizes[order[i % n_module]] += 1
    return sizes


PARAM_ORDER_PLAIN = ["W_qkv", "W_o", "ln1_g", "ln1_b", "W_1", "b_1", "W_2", "b_2", "ln2_g", "ln2_b"]
PARAM_ORDER_XL = ["W_qkv", "W_o", "W_r", "u", "v", "ln1_g", "ln1_b", "W_1", "b_1", "W_2", "b_2",
                  "ln2_g", "ln2_b"]


def param_shapes(cfg):
    d, f, h, dh = cfg.d_model, cfg.d_ff, cfg.n_head, cfg.d_head
    s = {"W_qkv": (d, 3 * d), "W_o": (d, d), "W_r": (d, d), "u": (h, dh), "v": (h, dh),
         "ln1_g": (d,), "ln1_b": (d,), "W_1": (d, f), "b_1": (f,), "W_2": (f, d), "b_2": (d,),
         "ln2_g": (d,), "ln2_b": (d,)}
    order = PARAM_ORDER_XL if cfg.rel_pos else PARAM_ORDER_PLAIN
    return [(n, s[n]) for n in order]


def unpack_layers(cfg, blob, n_layers):
    """Module blob (flat, documented order) -> list of per-layer dicts of fp64 arrays."""
    blob = np.asarray(blob, dtype=np.float64)
    out, off = [], 0
    for _ in range(n_layers):
        p = {}
        for name, shape in param_shapes(cfg):
            n = int(np.prod(shape))
            p[name] = blob[off:off + n].reshape(shape).copy()
            off += n
        out.append(p)
    assert off == blob.size
    return out


def pack_layers(cfg, layers):
    parts = []
    for p in layers:
        for name, _ in param_shapes(cfg):
            parts.append(np.asarray(p[name], dtype=np.float64).ravel())
    return np.concatenate(parts) if parts else np.zeros(0)


# ----------------------------------------------------------------------- elementary ops
def sinusoid(positions, d):
    """[len(positions), d] table: first half sin(p*w_m), second half cos(p*w_m),
    w_m = 10000^(-2m/d), m < d/2."""
    pos = np.asarray(positions, dtype=np.float64)[:, None]
    m = np.arange(d // 2, dtype=np.float64)[None, :]
    ang = pos * (10000.0 ** (-2.0 * m / d))
    return np.concatenate([np.sin(ang), np.cos(ang)], axis=1)


def layernorm_fwd(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)          # biased variance
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, g, cache):
    xhat, rstd = cache
    dg = (dy * xhat).reshape(-1, xhat.shape[-1]).sum(axis=0)
    db = dy.reshape(-1, xhat.shape[-1]).sum(axis=0)
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True)
                 - xhat * (dxh * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def gelu_grad(x):
    return 0.5 * (1.0 + erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def split_heads(x, h, dh):
    """[B, S, h*dh] -> [B, h, S, dh]"""
    b, s, _ = x.shape
    return x.reshape(b, s, h, dh).transpose(0, 2, 1, 3)


def merge_heads(x):
    b, h, s, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(b, s, h * dh)


# --------------------------------------------------------------------------- attention
def attention_core_fwd(q, k, v, Mv, scale, u=None, vb=None, r=None):
    """Causal attention on projected heads.  q [B,H,T,dh]; k, v [B,H,S,dh], S = Mv+T.
    Query i sits at absolute position Mv+i and sees keys j <= Mv+i.  With u, vb [H,dh] and
    r [H,S,dh] (row = relative distance) the score is the Transformer-XL form
    (q_i+u).k_j + (q_i+vb).r[Mv+i-j], indexed directly by distance (no shift trick)."""
    T, S = q.shape[2], k.shape[2]
    delta = Mv + np.arange(T)[:, None] - np.arange(S)[None, :]     # p_i - p_j
    visible = delta >= 0
    c = dict(q=q, k=k, v=v, Mv=Mv, visible=visible, delta=delta, scale=scale, rel=r is not None)
    if r is not None:
        qu = q + u[None, :, None, :]
        qv = q + vb[None, :, None, :]
        AC = qu @ k.transpose(0, 1, 3, 2)                          # [B,H,T,S]
        QR = np.einsum("bhic,hpc->bhip", qv, r)                    # [B,H,T,S] indexed by distance
        dcl = np.where(visible, delta, 0)
        BD = np.take_along_axis(QR, np.broadcast_to(dcl, QR.shape), axis=3)
        s = (AC + BD) * scale
        c.update(r=r, qu=qu, qv=qv)
    else:
        s = (q @ k.transpose(0, 1, 3, 2)) * scale
    s = np.where(visible, s, -np.inf)
    mx = s.max(axis=-1, keepdims=True)
    e = np.exp(s - mx)
    den = e.sum(axis=-1, keepdims=True)
    P = e / den
    c.update(P=P, lse=(mx + np.log(den))[..., 0])
    return P @ v, c


def attention_core_bwd(do, c):
    """Gradients of attention_core_fwd's output w.r.t. q, k, v (and u, vb, r)."""
    q, k, v, P, scale = c["q"], c["k"], c["v"], c["P"], c["scale"]
    dv = P.transpose(0, 1, 3, 2) @ do
    dP = do @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dS = np.where(c["visible"], dS, 0.0) * scale
    if not c["rel"]:
        return dS @ k, dS.transpose(0, 1, 3, 2) @ q, dv, None, None, None
    r, qu, qv = c["r"], c["qu"], c["qv"]
    dqu = dS @ k
    dk = dS.transpose(0, 1, 3, 2) @ qu
    # dS[b,h,i,j] belongs to relative distance delta(i,j); for a fixed i the map
    # j -> delta is one-to-one over the visible keys, so plain assignment is exact
    dQR = np.zeros_like(dS)
    ii, jj = np.nonzero(c["visible"])
    dQR[:, :, ii, c["delta"][ii, jj]] = dS[:, :, ii, jj]
    dqv = np.einsum("bhip,hpc->bhic", dQR, r)
    dr = np.einsum("bhip,bhic->hpc", dQR, qv)                      # [H,S,dh]
    return dqu + dqv, dk, dv, dqu.sum(axis=(0, 2)), dqv.sum(axis=(0, 2)), dr


def attention_fwd(cfg, p, x, mem):
    """Self-attention of one layer.  x [B,T,d] current segment, mem [B,Mv,d] or None
    (a constant: previous inputs of this layer); keys and values span [mem ; x]."""
    B, T, d = x.shape
    H, dh = cfg.n_head, cfg.d_head
    Mv = 0 if mem is None else mem.shape[1]
    cat = x if Mv == 0 else np.concatenate([mem, x], axis=1)
    S = Mv + T
    Wq, Wk, Wv = p["W_qkv"][:, :d], p["W_qkv"][:, d:2 * d], p["W_qkv"][:, 2 * d:]
    q = split_heads(x @ Wq, H, dh)            # [B,H,T,dh]
    k = split_heads(cat @ Wk, H, dh)          # [B,H,S,dh]
    v = split_heads(cat @ Wv, H, dh)
    scale = 1.0 / math.sqrt(dh)
    if cfg.rel_pos:
        R = sinusoid(np.arange(S), d)                               # R_delta, delta = 0..S-1
        r = (R @ p["W_r"]).reshape(S, H, dh).transpose(1, 0, 2)     # [H,S,dh]
        oh, cc = attention_core_fwd(q, k, v, Mv, scale, p["u"], p["v"], r)
        cc["R"] = R
    else:
        oh, cc = attention_core_fwd(q, k, v, Mv, scale)
    a = merge_heads(oh)                                             # [B,T,d]
    cc.update(x=x, cat=cat, a=a)
    return a @ p["W_o"], cc


def attention_bwd(cfg, p, do, c):
    d = cfg.d_model
    H, dh = cfg.n_head, cfg.d_head
    x, cat, a, Mv = c["x"], c["cat"], c["a"], c["Mv"]
    g = {}
    g["W_o"] = a.reshape(-1, d).T @ do.reshape(-1, d)
    da = split_heads(do @ p["W_o"].T, H, dh)                        # [B,H,T,dh]
    dq, dk, dv, du, dvb, dr = attention_core_bwd(da, c)
    if cfg.rel_pos:
        g["u"], g["v"] = du, dvb
        g["W_r"] = c["R"].T @ dr.transpose(1, 0, 2).reshape(-1, d)
    dq, dk, dv = merge_heads(dq), merge_heads(dk), merge_heads(dv)
    x2, cat2 = x.reshape(-1, d), cat.reshape(-1, d)
    g["W_qkv"] = np.concatenate([x2.T @ dq.reshape(-1, d), cat2.T @ dk.reshape(-1, d),
                                 cat2.T @ dv.reshape(-1, d)], axis=1)
    Wq, Wk, Wv = p["W_qkv"][:, :d], p["W_qkv"][:, d:2 * d], p["W_qkv"][:, 2 * d:]
    dx = dq @ Wq.T + (dk[:, Mv:] @ Wk.T) + (dv[:, Mv:] @ Wv.T)      # memory is a constant
    return dx, g


# ----------------------------------------------------------------------------- dropout
MASK64 = (1 << 64) - 1


def random_u32(seed, stream, idx):
    """Counter-based generator shared (as an algorithm, not as code) with the HIP path:
    the high 32 bits of output number idx + stream*2^40 + 1 of the SplitMix64 sequence
    (Steele, Lea, Flood 2014) started at `seed`, i.e. the 64-bit finaliser applied to
    seed + gamma*(idx + stream*2^40 + 1).  idx: uint64 array; returns uint32."""
    idx = np.asarray(idx, dtype=np.uint64)
    with np.errstate(over="ignore"):
        ctr = idx + np.uint64((int(stream) << 40) + 1)
        z = np.uint64(int(seed) & MASK64) + np.uint64(0x9E3779B97F4A7C15) * ctr
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return (z >> np.uint64(32)).astype(np.uint32)


def dropout_mask(cfg, seed, stream, shape):
    """Inverted dropout (Srivastava et al. 2014, cited in Section 5.2): element i (row-major
    index) is kept iff its 32 random bits are >= floor(p * 2^32); kept elements are scaled
    by 1/(1-p).  The mask is a pure function of (seed, stream, i): "repeatable"."""
    n = int(np.prod(shape))
    bits = random_u32(seed, stream, np.arange(n, dtype=np.uint64))
    thresh = np.uint32(int(cfg.dropout * 4294967296.0))
    return ((bits >= thresh).astype(np.float64) / (1.0 - cfg.dropout)).reshape(shape)


def embed_stream():
    return 0


def layer_stream(l, site):
    """site 1: output of the attention projection; site 2: output of the feed-forward block."""
    return 2 * l + site


# ------------------------------------------------------------------------------- layer
def layer_fwd(cfg, p, x, mem, drop=None):
    """drop = (seed, layer index) switches dropout on at the two sublayer outputs, before the
    residual additions (the paper names dropout, Section 5.2, not its places: a reading)."""
    o, ca = attention_fwd(cfg, p, x, mem)
    m1 = m2 = None
    if drop is not None and cfg.dropout > 0:
        m1 = dropout_mask(cfg, drop[0], layer_stream(drop[1], 1), o.shape)
        o = o * m1
    y, c1 = layernorm_fwd(x + o, p["ln1_g"], p["ln1_b"])
    z = y @ p["W_1"] + p["b_1"]
    u = gelu(z)
    f = u @ p["W_2"] + p["b_2"]
    if m1 is not None:
        m2 = dropout_mask(cfg, drop[0], layer_stream(drop[1], 2), f.shape)
        f = f * m2
    h, c2 = layernorm_fwd(y + f, p["ln2_g"], p["ln2_b"])
    return h, dict(att=ca, ln1=c1, y=y, z=z, u=u, ln2=c2, m1=m1, m2=m2)


def layer_bwd(cfg, p, dh, c):
    d, F = cfg.d_model, cfg.d_ff
    g = {}
    ds2_res, g["ln2_g"], g["ln2_b"] = layernorm_bwd(dh, p["ln2_g"], c["ln2"])
    ds2 = ds2_res if c.get("m2") is None else ds2_res * c["m2"]      # into the feed-forward branch
    g["W_2"] = c["u"].reshape(-1, F).T @ ds2.reshape(-1, d)
    g["b_2"] = ds2.reshape(-1, d).sum(axis=0)
    dz = (ds2 @ p["W_2"].T) * gelu_grad(c["z"])
    g["W_1"] = c["y"].reshape(-1, d).T @ dz.reshape(-1, F)
    g["b_1"] = dz.reshape(-1, F).sum(axis=0)
    dy = ds2_res + dz @ p["W_1"].T
    ds1, g["ln1_g"], g["ln1_b"] = layernorm_bwd(dy, p["ln1_g"], c["ln1"])
    do = ds1 if c.get("m1") is None else ds1 * c["m1"]                # into the attention branch
    dx_att, ga = attention_bwd(cfg, p, do, c["att"])
    g.update(ga)
    return ds1 + dx_att, g


# ------------------------------------------------------------------------------- model
def cross_entropy_fwd(logits, targets):
    """Eq. 4 with f = mean over all targets of (logsumexp(logits) - logit[target])."""
    mx = logits.max(axis=-1, keepdims=True)
    lse = mx[..., 0] + np.log(np.exp(logits - mx).sum(axis=-1))
    tgt_logit = np.take_along_axis(logits, targets[..., None].astype(np.int64), axis=-1)[..., 0]
    return float((lse - tgt_logit).mean()), lse


def cross_entropy_bwd(logits, lse, targets):
    """d loss / d logits = (softmax - onehot) / (number of targets)."""
    G = np.exp(logits - lse[..., None])
    idx = targets[..., None].astype(np.int64)
    np.put_along_axis(G, idx, np.take_along_axis(G, idx, axis=-1) - 1.0, axis=-1)
    return G / targets.size


def embed_fwd(cfg, Vi, tokens, seed=None):
    """Eq. 1 (+ fixed positions, + dropout on the sum when a seed is given)."""
    h = cfg.emb_scale * Vi[tokens]                            # Eq. 1: V_i enters layer 1
    if not cfg.rel_pos:
        h = h + sinusoid(np.arange(tokens.shape[1]), cfg.d_model)[None]
    m0 = None
    if seed is not None and cfg.dropout > 0:
        m0 = dropout_mask(cfg, seed, embed_stream(), h.shape)
        h = h * m0
    return h, m0


def model_forward(cfg, layers, Vi, Vo, tokens, targets, mems=None, seed=None):
    """Eq. 1-4.  Returns loss (mean over all B*T targets, natural log) and a cache.
    seed: dropout seed of this pass (None or cfg.dropout = 0: no dropout)."""
    h, m0 = embed_fwd(cfg, Vi, tokens, seed)
    inputs, caches = [], []
    for l, p in enumerate(layers):
        inputs.append(h)
        h, c = layer_fwd(cfg, p, h, None if mems is None else mems[l], None if seed is None else (seed, l))
        caches.append(c)
    logits = h @ Vo.T                                         # Eq. 3: V_o leaves layer L
    loss, lse = cross_entropy_fwd(logits, targets)
    return loss, dict(inputs=inputs, caches=caches, hL=h, logits=logits, lse=lse, m0=m0)


def model_backward(cfg, layers, Vi, Vo, tokens, targets, fw):
    """Eq. 6-7: full gradient {dw_l for all l, dV_i, dV_o}."""
    B, T = tokens.shape
    N = B * T
    d = cfg.d_model
    G = cross_entropy_bwd(fw["logits"], fw["lse"], targets)
    dVo = G.reshape(N, -1).T @ fw["hL"].reshape(N, d)
    dh = G @ Vo
    grads = [None] * len(layers)
    for l in reversed(range(len(layers))):
        dh, grads[l] = layer_bwd(cfg, layers[l], dh, fw["caches"][l])
    if fw.get("m0") is not None:
        dh = dh * fw["m0"]
    dVi = np.zeros_like(Vi)
    np.add.at(dVi, tokens.reshape(-1), cfg.emb_scale * dh.reshape(N, d))
    return grads, dVi, dVo


def full_gradient(cfg, layers, V, tokens, targets, mems=None, seed=None):
    loss, fw = model_forward(cfg, layers, V, V, tokens, targets, mems, seed)
    grads, dVi, dVo = model_backward(cfg, layers, V, V, tokens, targets, fw)
    return loss, grads, dVi, dVo, fw["inputs"]


# -------------------------------------------------------------------------- step size
def learning_rate(t, base, warmup, total, floor=0.0):
    """Step size gamma_t of iteration t = 0, 1, ... (Section 5.2, "Warm-up Training" and
    the cosine schedule named beside the optimiser settings).

    Reading (the paper gives the two phases and the warm-up length, not the formula):
    a gradual linear warm-up that reaches `base` at the last warm-up iteration,
    gamma_t = base * (t+1) / warmup for t < warmup, then one half cosine period from
    `base` down to `floor` at iteration `total` (the cited restart schedule with a
    single period), constant `floor` afterwards."""
    if t < warmup:
        return base * (t + 1) / warmup
    if t >= total:
        return floor
    return floor + (base - floor) * 0.5 * (1.0 + math.cos(math.pi * (t - warmup) / (total - warmup)))


# ------------------------------------------------------------------- training iteration
class Oracle:
    """Algorithm 1 / Algorithm 2 with the delayed gradients of Eq. 8-9."""

    def __init__(self, cfg: Config, blobs, keep_history=True):
        """blobs: [V flat, module 1 flat, ..., module K flat] (documented blob order)."""
        self.cfg = cfg
        self.V = np.asarray(blobs[0], dtype=np.float64).reshape(cfg.vocab, cfg.d_model).copy()
        self.layers = []
        for k in range(cfg.n_module):
            self.layers += unpack_layers(cfg, blobs[k + 1], cfg.layers_per_module[k])
        self.bounds = np.concatenate([[0], np.cumsum(cfg.layers_per_module)])  # G(k) = [b[k-1], b[k])
        self.t = 0
        self.mems = None
        self.grad_hist = []      # step -> (per-layer grads, dV_i, dV_o); never a ring
        self.state_hist = []     # step -> (layers, V, mems, tokens, targets)
        self.keep_history = keep_history
        self.used = []           # step -> {k: tau} actually used, for the index pins
        if cfg.optimizer == 1:
            self.m = [{n: np.zeros_like(a) for n, a in p.items()} for p in self.layers]
            self.v = [{n: np.zeros_like(a) for n, a in p.items()} for p in self.layers]
            self.mV, self.vV = np.zeros_like(self.V), np.zeros_like(self.V)

    def seed_of(self, t):
        """Dropout seed of mini-batch t (stored with the module inputs, Section 5.2
        "Repeatable Dropout"): the configured seed plus t; None when dropout is off."""
        return (self.cfg.seed + t) & MASK64 if self.cfg.dropout > 0 else None

    def module_layers(self, k):
        """Layer indices of G(k), k = 1..K."""
        return range(int(self.bounds[k - 1]), int(self.bounds[k]))

    def module_blob(self, k):
        return self.V.ravel().copy() if k == 0 else pack_layers(self.cfg, [self.layers[l] for l in self.module_layers(k)])

    def grad_blob(self, k, tau):
        """Flat gradient of module k (1..K) computed at step tau."""
        return pack_layers(self.cfg, [self.grad_hist[tau][0][l] for l in self.module_layers(k)])

    def _apply(self, w, g, m, v, lr):
        c = self.cfg
        if c.optimizer == 0:
            w -= lr * g                                      # Algorithm 1
            return
        m *= c.beta1; m += (1 - c.beta1) * g                 # Algorithm 2
        v *= c.beta2; v += (1 - c.beta2) * g * g
        mh = m / (1 - c.beta1 ** (self.t + 1))
        vh = v / (1 - c.beta2 ** (self.t + 1))
        w -= lr * mh / (np.sqrt(vh) + c.eps)

    def step(self, tokens, targets, lr):
        c, t, K = self.cfg, self.t, self.cfg.n_module
        tokens = np.asarray(tokens); targets = np.asarray(targets)
        if self.keep_history:
            self.state_hist.append((copy.deepcopy(self.layers), self.V.copy(),
                                    copy.deepcopy(self.mems), tokens.copy(), targets.copy()))
        loss, grads, dVi, dVo, inputs = full_gradient(c, self.layers, self.V, tokens, targets, self.mems,
                                                      self.seed_of(t))
        self.grad_hist.append((grads, dVi, dVo))
        used = {}
        for k in range(1, K + 1):                            # Eq. 8
            tau = t - K + k
            used[k] = tau if tau >= 0 else -1
            for l in self.module_layers(k):
                for name in self.layers[l]:
                    g = self.grad_hist[tau][0][l][name] if tau >= 0 else np.zeros_like(self.layers[l][name])
                    mm = self.m[l][name] if c.optimizer == 1 else None
                    vv = self.v[l][name] if c.optimizer == 1 else None
                    self._apply(self.layers[l][name], g, mm, vv, lr)
        tau_i = t - K + 1                                    # Eq. 9
        if tau_i >= 0:
            gV = 0.5 * self.grad_hist[t][2] + 0.5 * self.grad_hist[tau_i][1]
            used[0] = (t, tau_i)
        elif c.embed_warm_mode == 1:
            gV = 0.5 * self.grad_hist[t][2]
            used[0] = (t, -1)
        else:
            gV = np.zeros_like(self.V)
            used[0] = (-1, -1)
        self._apply(self.V, gV, getattr(self, "mV", None), getattr(self, "vV", None), lr)
        self.used.append(used)
        if c.mem_len > 0:                                    # segment memory for step t+1
            new = []
            for l in range(c.n_layer):
                cat = inputs[l] if self.mems is None else np.concatenate([self.mems[l], inputs[l]], axis=1)
                new.append(cat[:, -c.mem_len:].copy())
            self.mems = new
        self.t += 1
        return loss

    def eval_step(self, tokens, targets):
        """Forward-only pass with the current weights (Eq. 1-4, no dropout): the loss in nats
        per token, from which the paper's tables report bits per character (loss / ln 2) or
        perplexity (exp(loss)).  Segment memories roll and the counter advances, so that
        consecutive segments are evaluated with carried-over memory."""
        c = self.cfg
        loss, fw = model_forward(c, self.layers, self.V, self.V, np.asarray(tokens), np.asarray(targets), self.mems, None)
        if c.mem_len > 0:
            new = []
            for l in range(c.n_layer):
                cat = fw["inputs"][l] if self.mems is None else np.concatenate([self.mems[l], fw["inputs"][l]], axis=1)
                new.append(cat[:, -c.mem_len:].copy())
            self.mems = new
        self.t += 1
        return loss

    def brute_check(self, t):
        """Re-derive, from the stored full state of step tau, every gradient that the
        update of iteration t consumed, and compare with what was used (Eq. 8-9)."""
        K = self.cfg.n_module
        worst = 0.0
        for k in range(1, K + 1):
            tau = t - K + k
            assert self.used[t][k] == (tau if tau >= 0 else -1)
            if tau < 0:
                continue
            layers, V, mems, tok, tgt = self.state_hist[tau]
            _, grads, _, _, _ = full_gradient(self.cfg, layers, V, tok, tgt, mems, self.seed_of(tau))
            for l in self.module_layers(k):
                for name in grads[l]:
                    worst = max(worst, float(np.abs(grads[l][name] - self.grad_hist[tau][0][l][name]).max()))
        return worst


# ------------------------------------------------- stored-input / recompute schedule
def module_fwd(cfg, k, layers_k, V, inp, mems_k, seed=None, first_layer=0):
    """Forward pass of module k on its stored input: token ids for k = 1 (the embedding
    lookup of Eq. 1 belongs to module 1), the hidden state at the module boundary
    otherwise.  seed: the stored dropout seed of that mini-batch; first_layer: index of
    the module's first layer in the network (it keys the dropout streams).  Returns the
    module's output, the per-layer caches and the embedding mask (k = 1, else None)."""
    m0 = None
    if k == 1:
        h, m0 = embed_fwd(cfg, V, inp, seed)
    else:
        h = inp
    caches = []
    for i, p in enumerate(layers_k):
        h, c = layer_fwd(cfg, p, h, None if mems_k is None else mems_k[i],
                         None if seed is None else (seed, first_layer + i))
        caches.append(c)
    return h, caches, m0


def module_bwd(cfg, layers_k, caches, dh):
    """Eq. 6 inside one module: error gradient of the module's output -> per-layer weight
    gradients and the error gradient of the module's input."""
    grads = [None] * len(layers_k)
    for i in reversed(range(len(layers_k))):
        dh, grads[i] = layer_bwd(cfg, layers_k[i], dh, caches[i])
    return dh, grads


class RecomputeOracle(Oracle):
    """The schedule the paper runs on its GPUs (Section 3.1, "Memory Consumption"): module k
    stores its input of every iteration instead of a gradient.  At iteration t it

      * runs the forward pass of mini-batch t on the current weights (all modules in
        sequence; the loss reported is that of mini-batch t),
      * and, "in parallel" over k, takes mini-batch tau = t-K+k: it recomputes its
        activations from the stored input of iteration tau with the weights it holds at
        iteration t, and back-propagates the error gradient of its output that module
        k+1 produced at iteration t-1 (module K differentiates the loss of mini-batch t
        itself).  The error gradient of its own input goes to module k-1, which uses
        it at iteration t+1; module 1 turns it into dV_i of mini-batch t-K+1.
      * Then every group takes its step with the gradient just computed (zero while
        tau < 0); V mixes dV_o(t) and that dV_i as in Eq. 9.

    Reading: the paper says that inputs are stored and activations recomputed, not with
    which weights; this class recomputes with the module's current weights (what a
    device that keeps one copy of its weights does).  With frozen weights the gradients
    coincide with Eq. 8's; with moving weights they differ from it at first order in the
    step size.  Segment memories are part of a module's stored input.

    grad_hist[t] holds what iteration t computed: module k's entry is the gradient of
    mini-batch t-K+k (zeros while that is negative), dV_i that of mini-batch t-K+1."""

    def __init__(self, cfg, blobs, keep_history=True, repeatable=True):
        """repeatable=False is the ablation of Section 6.3 (recompute under the dropout seed
        of the running iteration instead of the stored one); tests use it as a planted error."""
        super().__init__(cfg, blobs, keep_history)
        self.repeatable = repeatable
        self.inputs = {}         # (k, t) -> (input of module k at iteration t, its layers' memories)
        self.mail = {}           # k -> (tau, error gradient of module k's output for mini-batch tau)
        self.batch_of = []       # t -> {k: tau}

    def step(self, tokens, targets, lr):
        c, t, K = self.cfg, self.t, self.cfg.n_module
        tokens = np.asarray(tokens); targets = np.asarray(targets)
        # forward pass of mini-batch t, storing every module's input (and the dropout seed)
        h = tokens
        layer_inputs = []
        seed_t = self.seed_of(t)
        for k in range(1, K + 1):
            ls = list(self.module_layers(k))
            mems_k = None if self.mems is None else [self.mems[l] for l in ls]
            self.inputs[(k, t)] = (h.copy(), copy.deepcopy(mems_k), seed_t)
            if k == 1:
                x, m0_t = embed_fwd(c, self.V, tokens, seed_t)
            else:
                x = h
            caches = []
            for i, l in enumerate(ls):
                layer_inputs.append(x)
                x, cc = layer_fwd(c, self.layers[l], x, None if mems_k is None else mems_k[i],
                                  None if seed_t is None else (seed_t, l))
                caches.append(cc)
            h = x
        hL, top_caches = h, caches
        logits = hL @ self.V.T
        loss, lse = cross_entropy_fwd(logits, targets)
        # backward passes, one per module, all from the state iteration t-1 left behind
        N, d = tokens.size, c.d_model
        grads = [{n: np.zeros_like(a) for n, a in p.items()} for p in self.layers]
        dVi, dVo = np.zeros_like(self.V), np.zeros_like(self.V)
        new_mail, batch_of = {}, {}
        for k in range(1, K + 1):
            tau = t - K + k
            batch_of[k] = tau if tau >= 0 else -1
            if tau < 0:
                continue
            ls = list(self.module_layers(k))
            layers_k = [self.layers[l] for l in ls]
            if k == K:                                        # tau = t: the pass just made
                G = cross_entropy_bwd(logits, lse, targets)
                dVo = G.reshape(N, -1).T @ hL.reshape(N, d)
                dh = G @ self.V
                caches_k = top_caches
                m0 = m0_t if K == 1 else None
            else:
                inp, mems_k, seed_tau = self.inputs[(k, tau)]
                if not self.repeatable:
                    seed_tau = seed_t
                _, caches_k, m0 = module_fwd(c, k, layers_k, self.V, inp, mems_k, seed_tau, ls[0])
                mtau, dh = self.mail[k]
                assert mtau == tau
            dx, gk = module_bwd(c, layers_k, caches_k, dh)
            for i, l in enumerate(ls):
                grads[l] = gk[i]
            if k > 1:
                new_mail[k - 1] = (tau, dx)
            else:
                tok_tau = self.inputs[(1, tau)][0]
                if m0 is not None:
                    dx = dx * m0
                np.add.at(dVi, tok_tau.reshape(-1), c.emb_scale * dx.reshape(N, d))
        self.mail = new_mail
        self.grad_hist.append((grads, dVi, dVo))
        self.batch_of.append(batch_of)
        used = {}
        for k in range(1, K + 1):
            used[k] = t if batch_of[k] >= 0 else -1
            for l in self.module_layers(k):
                for name in self.layers[l]:
                    mm = self.m[l][name] if c.optimizer == 1 else None
                    vv = self.v[l][name] if c.optimizer == 1 else None
                    self._apply(self.layers[l][name], grads[l][name], mm, vv, lr)
        if batch_of[1] >= 0:                                  # Eq. 9
            gV = 0.5 * dVo + 0.5 * dVi
            used[0] = (t, t)
        elif c.embed_warm_mode == 1:
            gV = 0.5 * dVo
            used[0] = (t, -1)
        else:
            gV = np.zeros_like(self.V)
            used[0] = (-1, -1)
        self._apply(self.V, gV, getattr(self, "mV", None), getattr(self, "vV", None), lr)
        self.used.append(used)
        if c.mem_len > 0:
            new = []
            for l in range(c.n_layer):
                cat = layer_inputs[l] if self.mems is None else np.concatenate([self.mems[l], layer_inputs[l]], axis=1)
                new.append(cat[:, -c.mem_len:].copy())
            self.mems = new
        self.t += 1
        return loss
