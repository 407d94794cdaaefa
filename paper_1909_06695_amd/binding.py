"""Thin ctypes binding of libouro.so: argument marshalling only.

Every step of the training iteration runs inside the HIP library; PyTorch is used here
for device memory (the arena, token buffers) and the stream handle.  There is no CPU
fallback: loading fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("OURO_LIB_PATH", os.path.join(_HERE, "libouro.so"))

OK, E_CONFIG, E_ARG, E_ARENA, E_SEQUENCE, E_TOKEN, E_STALE, E_HIP = 0, -1, -2, -3, -4, -5, -6, -7


class OuroError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libouro error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("n_layer", C.c_int32), ("d_model", C.c_int32), ("n_head", C.c_int32),
                ("d_head", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("seq_len", C.c_int32), ("mem_len", C.c_int32), ("batch", C.c_int32),
                ("n_module", C.c_int32), ("layers_per_module", C.POINTER(C.c_int32)),
                ("rel_pos", C.c_int32), ("dtype", C.c_int32), ("optimizer", C.c_int32),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("embed_warm_mode", C.c_int32), ("emb_scale", C.c_float), ("schedule", C.c_int32),
                ("dropout", C.c_float), ("seed", C.c_uint64)]


_lib = None


def lib():
    """Loads libouro.so (built by `python -m paper_1909_06695_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise OuroError(E_HIP, f"{LIB_PATH} is missing: build it with `python -m paper_1909_06695_amd.build`; "
                               "there is no CPU fallback")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t
    P = C.POINTER
    sig = {
        "ouro_last_error": (C.c_char_p, []),
        "ouro_query_arena_bytes": (i32, [P(Config), P(sz)]),
        "ouro_create_model": (i32, [P(Config), vp, sz, vp, P(vp)]),
        "ouro_destroy_model": (i32, [vp]),
        "ouro_param_count": (i32, [vp, i32, P(i64)]),
        "ouro_set_params": (i32, [vp, i32, vp, i64, i32]),
        "ouro_get_params": (i32, [vp, i32, vp, i64, i32]),
        "ouro_module_forward": (i32, [vp, i32, vp, vp]),
        "ouro_module_backward": (i32, [vp, i32]),
        "ouro_delayed_update": (i32, [vp, i32, f32]),
        "ouro_step": (i32, [vp, vp, vp, f32, P(f32)]),
        "ouro_get_loss": (i32, [vp, P(f32)]),
        "ouro_eval_step": (i32, [vp, vp, vp, P(f32)]),
        "ouro_state_bytes": (i32, [vp, P(sz)]),
        "ouro_save_state": (i32, [vp, vp, sz]),
        "ouro_load_state": (i32, [vp, vp, sz]),
        "ouro_current_step": (i64, [vp]),
        "ouro_slot_index": (i32, [i32, i32, i64, i32, P(i64), P(i64)]),
        "ouro_ring_depth": (i32, [i32, i32, P(i64)]),
        "ouro_lr_schedule": (i32, [C.c_double, i64, i64, C.c_double, i64, P(C.c_double)]),
        "ouro_debug_slot_tag": (i32, [vp, i32, i64, P(i64)]),
        "ouro_debug_last_read": (i32, [vp, i32, P(i64), P(i64)]),
        "ouro_debug_input_tag": (i32, [vp, i32, i64, P(i64)]),
        "ouro_debug_last_input_read": (i32, [vp, i32, P(i64), P(i64)]),
        "ouro_debug_inject_grad": (i32, [vp, i32, vp, i64]),
        "ouro_get_grad_slot": (i32, [vp, i32, i64, vp, i64]),
        "ouro_get_mems": (i32, [vp, i32, vp, P(i64)]),
        "ouro_debug_get_hidden": (i32, [vp, i32, vp, i64]),
        "ouro_debug_timing_enable": (i32, [vp, i32]),
        "ouro_debug_set_overlap": (i32, [vp, i32]),
        "ouro_debug_timing_overhead": (i32, [vp, i32, P(C.c_double)]),
        "ouro_debug_timing_read": (i32, [vp, i32, P(C.c_double), P(i64), P(C.c_double)]),
        # single-kernel entry points
        "ouro_op_gemm": (i32, [vp, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, i32, i32, vp, vp,
                               i32, i32, vp, i32, i32]),
        "ouro_op_gemm_batched": (i32, [vp, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, i32, i32, i32, i32,
                                       C.c_longlong, C.c_longlong, C.c_longlong, C.c_longlong, C.c_longlong, C.c_longlong,
                                       vp, vp, vp, f32, i32]),
        "ouro_op_gemm_group": (i32, [vp, i32, i32, P(i32), P(i32), P(i32), P(vp), P(i32), P(vp), P(i32), P(vp), P(i32), f32]),
        "ouro_op_gemm_uses_mfma": (i32, [i32, i32, i32, i32, i32, i32, vp, i32, vp, i32]),
        "ouro_op_attention_fwd": (i32, [vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, vp,
                                        i32, vp, i32, vp, vp, vp, i32, i32]),
        "ouro_op_attention_bwd": (i32, [vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, vp,
                                        i32, vp, vp, i32, vp, i32, vp, i32, vp, i32, i32, vp, vp, vp, i32, vp, vp,
                                        vp, vp, i32]),
        "ouro_op_attention_bwd_scratch": (sz, [i32, i32, i32, i32, i32]),
        "ouro_op_attention_bwd_noalloc": (i32, [vp, i32, i32, i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, vp,
                                                i32, vp, vp, i32, vp, i32, vp, i32, vp, i32, i32, vp, vp, vp, i32, vp, vp,
                                                vp, i32]),
        "ouro_op_dropout": (i32, [vp, i32, vp, vp, i32, i32, i32, f32, C.c_uint64, C.c_uint32, i32]),
        "ouro_op_gemm_dropout": (i32, [vp, i32, i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, vp, vp, i32, f32,
                                       C.c_uint64, C.c_uint32, i32, i32]),
        "ouro_op_gemm_ln_residual": (i32, [vp, i32, i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, i32, vp, vp, i32, vp,
                                           vp, vp, vp, i32]),
        "ouro_op_layernorm_fwd": (i32, [vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32]),
        "ouro_op_layernorm_bwd": (i32, [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32]),
        "ouro_op_colsum": (i32, [vp, i32, vp, i32, vp, i32, i32]),
        "ouro_op_embed_fwd": (i32, [vp, i32, vp, vp, vp, vp, i32, i32, i32, i32, f32, vp]),
        "ouro_op_embed_bwd": (i32, [vp, i32, vp, vp, vp, i32, i32, i32, f32]),
        "ouro_op_softmax_ce": (i32, [vp, i32, vp, i32, vp, vp, i32, vp, vp, vp, i32, i32, vp]),
        "ouro_op_update": (i32, [vp, vp, vp, vp, vp, vp, f32, vp, f32, sz, i32, f32, f32, f32, f32, i64]),
        "ouro_op_from_f32": (i32, [vp, i32, vp, vp, sz]),
        "ouro_op_to_f32": (i32, [vp, i32, vp, vp, sz]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    L._sig = sig
    _lib = L
    return L


EXPORTS = None  # filled lazily by exported_symbols()


def exported_symbols():
    return sorted(lib()._sig.keys())


def check(rc):
    if rc != 0:
        raise OuroError(rc, lib().ouro_last_error().decode())


def make_config(n_layer, d_model, n_head, d_head, d_ff, vocab, seq_len, batch, n_module=1, mem_len=0,
                rel_pos=0, dtype=0, optimizer=0, layers_per_module=None, beta1=0.9, beta2=0.999,
                eps=1e-8, embed_warm_mode=0, emb_scale=1.0, schedule=0, dropout=0.0, seed=0, **_):
    cfg = Config()
    cfg.n_layer, cfg.d_model, cfg.n_head, cfg.d_head = n_layer, d_model, n_head, d_head
    cfg.d_ff, cfg.vocab, cfg.seq_len, cfg.mem_len, cfg.batch = d_ff, vocab, seq_len, mem_len, batch
    cfg.n_module, cfg.rel_pos, cfg.dtype, cfg.optimizer = n_module, rel_pos, dtype, optimizer
    cfg.beta1, cfg.beta2, cfg.eps = beta1, beta2, eps
    cfg.embed_warm_mode, cfg.emb_scale, cfg.schedule = embed_warm_mode, emb_scale, schedule
    cfg.dropout, cfg.seed = dropout, seed
    if layers_per_module is not None:
        arr = (C.c_int32 * len(layers_per_module))(*layers_per_module)
        cfg._keep = arr
        cfg.layers_per_module = C.cast(arr, C.POINTER(C.c_int32))
    return cfg


def slot_index(K, store, t, write):
    s, tau = C.c_int64(), C.c_int64()
    check(lib().ouro_slot_index(K, store, t, int(write), C.byref(s), C.byref(tau)))
    return s.value, tau.value


def lr_schedule(base, warmup, total, t, floor=0.0):
    """Step size of iteration t: linear warm-up, then cosine decay to `floor` at `total`."""
    v = C.c_double()
    check(lib().ouro_lr_schedule(float(base), int(warmup), int(total), float(floor), int(t), C.byref(v)))
    return v.value


def ring_depth(K, store):
    d = C.c_int64()
    check(lib().ouro_ring_depth(K, store, C.byref(d)))
    return d.value


def query_arena_bytes(cfg: Config) -> int:
    n = C.c_size_t()
    check(lib().ouro_query_arena_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Model:
    """create_model / module_forward / module_backward / delayed_update / step."""

    def __init__(self, device="cuda:0", stream=None, **cfg_kw):
        import torch
        self.torch = torch
        self.cfg_kw = dict(cfg_kw)
        self.cfg = make_config(**cfg_kw)
        self.L = lib()
        nbytes = query_arena_bytes(self.cfg)
        self.device = torch.device(device)
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)   # caller-owned arena
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        check(self.L.ouro_create_model(C.byref(self.cfg), C.c_void_p(self.arena.data_ptr()), nbytes,
                                       C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self.h = h
        self.K = self.cfg.n_module

    def close(self):
        if getattr(self, "h", None):
            self.L.ouro_destroy_model(self.h)
            self.h = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- parameters
    def param_count(self, group):
        n = C.c_int64()
        check(self.L.ouro_param_count(self.h, group, C.byref(n)))
        return n.value

    def set_params(self, group, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32).ravel()
        check(self.L.ouro_set_params(self.h, group, a.ctypes.data_as(C.c_void_p), a.size, 0))

    def get_params(self, group):
        out = np.empty(self.param_count(group), dtype=np.float32)
        check(self.L.ouro_get_params(self.h, group, out.ctypes.data_as(C.c_void_p), out.size, 0))
        return out

    # ---- the iteration
    def module_forward(self, k, tokens=None, targets=None):
        check(self.L.ouro_module_forward(self.h, k, _ptr(tokens), _ptr(targets)))

    def module_backward(self, k):
        check(self.L.ouro_module_backward(self.h, k))

    def delayed_update(self, group, lr):
        check(self.L.ouro_delayed_update(self.h, group, lr))

    def step(self, tokens, targets, lr, want_loss=True):
        loss = C.c_float()
        check(self.L.ouro_step(self.h, _ptr(tokens), _ptr(targets), lr, C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def eval_step(self, tokens, targets, want_loss=True):
        """Forward-only iteration: loss of the mini-batch in nats per token (bits per character =
        loss / ln 2, perplexity = exp(loss)); memories roll."""
        loss = C.c_float()
        check(self.L.ouro_eval_step(self.h, _ptr(tokens), _ptr(targets), C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def copy_params_from(self, other):
        """Device-to-device copy of every parameter group of `other` (same layer shapes)."""
        import torch
        for g in range(self.K + 1):
            n = other.param_count(g)
            buf = torch.empty(n, dtype=torch.float32, device="cuda")
            check(other.L.ouro_get_params(other.h, g, C.c_void_p(buf.data_ptr()), n, 1))
            check(self.L.ouro_set_params(self.h, g, C.c_void_p(buf.data_ptr()), n, 1))
            torch.cuda.synchronize()

    def save_state(self):
        """The whole training state at an iteration boundary as a numpy byte array."""
        n = C.c_size_t()
        check(self.L.ouro_state_bytes(self.h, C.byref(n)))
        buf = np.empty(n.value, dtype=np.uint8)
        check(self.L.ouro_save_state(self.h, buf.ctypes.data_as(C.c_void_p), n.value))
        return buf

    def load_state(self, buf):
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        check(self.L.ouro_load_state(self.h, buf.ctypes.data_as(C.c_void_p), buf.size))

    def get_loss(self):
        loss = C.c_float()
        check(self.L.ouro_get_loss(self.h, C.byref(loss)))
        return loss.value

    def current_step(self):
        return self.L.ouro_current_step(self.h)

    # ---- debug surface
    def slot_tag(self, store, slot):
        t = C.c_int64()
        check(self.L.ouro_debug_slot_tag(self.h, store, slot, C.byref(t)))
        return t.value

    def last_read(self, store):
        s, tau = C.c_int64(), C.c_int64()
        check(self.L.ouro_debug_last_read(self.h, store, C.byref(s), C.byref(tau)))
        return s.value, tau.value

    def input_tag(self, k, slot):
        t = C.c_int64()
        check(self.L.ouro_debug_input_tag(self.h, k, slot, C.byref(t)))
        return t.value

    def last_input_read(self, k):
        s, tau = C.c_int64(), C.c_int64()
        check(self.L.ouro_debug_last_input_read(self.h, k, C.byref(s), C.byref(tau)))
        return s.value, tau.value

    def grad_count(self, store):
        return self.param_count(0 if store in (0, self.K + 1) else store)

    def inject_grad(self, store, g):
        a = np.ascontiguousarray(g, dtype=np.float32).ravel()
        check(self.L.ouro_debug_inject_grad(self.h, store, a.ctypes.data_as(C.c_void_p), a.size))

    def get_grad_slot(self, store, tau):
        out = np.empty(self.grad_count(store), dtype=np.float32)
        check(self.L.ouro_get_grad_slot(self.h, store, tau, out.ctypes.data_as(C.c_void_p), out.size))
        return out

    def get_mems(self, layer):
        n = C.c_int64()
        check(self.L.ouro_get_mems(self.h, layer, None, C.byref(n)))
        if n.value == 0:
            return np.zeros((self.cfg.batch, 0, self.cfg.d_model), np.float32)
        out = np.empty((self.cfg.batch, n.value, self.cfg.d_model), dtype=np.float32)
        check(self.L.ouro_get_mems(self.h, layer, out.ctypes.data_as(C.c_void_p), C.byref(n)))
        return out

    def get_hidden(self, layer):
        out = np.empty((self.cfg.batch * self.cfg.seq_len, self.cfg.d_model), dtype=np.float32)
        check(self.L.ouro_debug_get_hidden(self.h, layer, out.ctypes.data_as(C.c_void_p), out.size))
        return out

    def timing_enable(self, on):
        check(self.L.ouro_debug_timing_enable(self.h, int(on)))

    def timing_overhead(self, reps=200):
        """Mean elapsed milliseconds of an empty timing bracket (two event records)."""
        ms = C.c_double()
        check(self.L.ouro_debug_timing_overhead(self.h, int(reps), C.byref(ms)))
        return ms.value

    def set_overlap(self, on):
        check(self.L.ouro_debug_set_overlap(self.h, int(on)))

    def timing_read(self, kind):
        """(ms, launches, work) since the last read: kind 0 = MFMA contraction kernel (flops), 1 = update
        kernel (bytes), 2 = attention (flops), 3 = LayerNorm (bytes), 4 = cross-entropy row pass (bytes)."""
        ms, n, w = C.c_double(), C.c_int64(), C.c_double()
        check(self.L.ouro_debug_timing_read(self.h, kind, C.byref(ms), C.byref(n), C.byref(w)))
        return ms.value, n.value, w.value


def create_model(**kw):
    return Model(**kw)
