"""Pins of the oracle's layer arithmetic against things other than itself:
closed forms, invariants, brute-force loops, finite differences and an independent
autograd model made of torch library routines."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import ouro_oracle as O
import synth_inputs as S
from tests import torch_ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_closed_forms():
    out = {}
    for line in open(os.path.join(GOLD, "closed_forms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def tiny_cfg(rel_pos=0, mem_len=0, **kw):
    base = dict(n_layer=2, d_model=8, n_head=2, d_head=4, d_ff=12, vocab=11, seq_len=5, batch=2,
                n_module=1, mem_len=mem_len, rel_pos=rel_pos)
    base.update(kw)
    return O.Config(**base)


def rand_layers(cfg, rng, std=0.3):
    layers = []
    for _ in range(cfg.n_layer):
        p = {}
        for n, shp in O.param_shapes(cfg):
            p[n] = rng.standard_normal(shp) * std
            if n.endswith("_g"):
                p[n] += 1.0
        layers.append(p)
    return layers


# ------------------------------------------------------------------ closed forms
def test_gelu_closed_forms():
    cf = read_closed_forms()
    for x in (-3.0, -1.0, -0.5, 0.0, 0.5, 1.0, 3.0):
        assert abs(O.gelu(np.array(x)) - cf[f"gelu({x})"]) < 1e-15
    assert O.gelu(np.array(0.0)) == 0.0
    assert O.gelu_grad(np.array(0.0)) == 0.5
    x = np.linspace(-4, 4, 41)
    fd = (O.gelu(x + 1e-6) - O.gelu(x - 1e-6)) / 2e-6
    assert np.abs(fd - O.gelu_grad(x)).max() < 1e-8


def test_layernorm_constant_row_and_library():
    g = np.array([1.5, -2.0, 0.5, 3.0]); b = np.array([0.1, 0.2, -0.3, 0.4])
    y, _ = O.layernorm_fwd(np.full((3, 4), 7.25), g, b)
    assert np.allclose(y, b, atol=1e-12)                      # LN of a constant row = beta
    rng = np.random.default_rng(0)
    x = rng.standard_normal((6, 4))
    y, c = O.layernorm_fwd(x, g, b)
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(g, requires_grad=True); bt = torch.tensor(b, requires_grad=True)
    yt = torch.nn.functional.layer_norm(xt, (4,), gt, bt, 1e-5)
    assert np.abs(y - yt.detach().numpy()).max() < 1e-13
    dy = rng.standard_normal((6, 4))
    yt.backward(torch.tensor(dy))
    dx, dg, db = O.layernorm_bwd(dy, g, c)
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-12
    assert np.abs(dg - gt.grad.numpy()).max() < 1e-12
    assert np.abs(db - bt.grad.numpy()).max() < 1e-12


def test_sinusoid_form():
    t = O.sinusoid(np.arange(4), 6)
    assert t.shape == (4, 6)
    assert np.allclose(t[0], [0, 0, 0, 1, 1, 1])
    for p in range(4):
        for m in range(3):
            w = 10000.0 ** (-2.0 * m / 6)
            assert abs(t[p, m] - math.sin(p * w)) < 1e-15
            assert abs(t[p, 3 + m] - math.cos(p * w)) < 1e-15


def test_zero_logit_loss_is_ln_vocab():
    cf = read_closed_forms()
    cfg = O.Config(n_layer=1, d_model=8, n_head=2, d_head=4, d_ff=8, vocab=256, seq_len=4, batch=2)
    rng = np.random.default_rng(1)
    layers = rand_layers(cfg, rng)
    V = np.zeros((256, 8))
    tok = rng.integers(0, 256, (2, 4)); tgt = rng.integers(0, 256, (2, 4))
    loss, fw = O.model_forward(cfg, layers, V, V, tok, tgt)
    assert abs(loss - cf["ln256"]) < 1e-14
    # dlogits = (1/V - onehot)/N: rows sum to zero, and dV_o rows: sum over vocab of dV_o = 0
    grads, dVi, dVo = O.model_backward(cfg, layers, V, V, tok, tgt, fw)
    assert np.abs(dVo.sum(axis=0)).max() < 1e-14
    N = 8
    hL = fw["hL"].reshape(N, 8)
    exp = np.tile(hL.sum(0) / 256 / N, (256, 1))
    np.subtract.at(exp, tgt.reshape(-1), hL / N)
    assert np.abs(dVo - exp).max() < 1e-14


# ------------------------------------------------------------------ attention pins
def test_attention_rows_sum_to_one_and_special_cases():
    cfg = tiny_cfg()
    rng = np.random.default_rng(2)
    p = rand_layers(cfg, rng)[0]
    x = rng.standard_normal((2, 5, 8))
    o, c = O.attention_fwd(cfg, p, x, None)
    assert np.abs(c["P"].sum(-1) - 1).max() < 1e-14
    assert np.all(c["P"][:, :, np.triu_indices(5, 1)[0], np.triu_indices(5, 1)[1]] == 0)
    # first query sees only key 0: output = v_0 (per head), before W_o
    v0 = (x[:, 0] @ p["W_qkv"][:, 16:])
    assert np.abs(c["a"][:, 0] - v0).max() < 1e-13
    # equal scores (W_q = 0) -> output = running mean of the visible values
    p2 = dict(p); p2["W_qkv"] = p["W_qkv"].copy(); p2["W_qkv"][:, :8] = 0
    o2, c2 = O.attention_fwd(cfg, p2, x, None)
    vals = x @ p2["W_qkv"][:, 16:]
    run = np.cumsum(vals, axis=1) / np.arange(1, 6)[None, :, None]
    assert np.abs(c2["a"] - run).max() < 1e-13


def test_xl_reduces_to_plain_attention():
    cfgx = tiny_cfg(rel_pos=1)
    cfgp = tiny_cfg(rel_pos=0)
    rng = np.random.default_rng(3)
    p = rand_layers(cfgx, rng)[0]
    p["u"][:] = 0; p["v"][:] = 0; p["W_r"][:] = 0
    x = rng.standard_normal((2, 5, 8))
    ox, _ = O.attention_fwd(cfgx, p, x, None)
    op, _ = O.attention_fwd(cfgp, p, x, None)
    assert np.abs(ox - op).max() < 1e-14


def test_xl_relative_indexing_brute_force():
    """T=3, M=2: scores recomputed with pure-Python loops straight from
    score(i,j) = (q_i+u).k_j + (q_i+v).(W_r R_{p_i-p_j}) over [mem ; cur]."""
    cfg = O.Config(n_layer=1, d_model=4, n_head=2, d_head=2, d_ff=4, vocab=5, seq_len=3, batch=1,
                   mem_len=2, rel_pos=1)
    rng = np.random.default_rng(4)
    p = rand_layers(cfg, rng, std=0.7)[0]
    x = rng.standard_normal((1, 3, 4)); mem = rng.standard_normal((1, 2, 4))
    _, c = O.attention_fwd(cfg, p, x, mem)
    cat = np.concatenate([mem, x], axis=1)[0]
    T, Sx, d, H, dh = 3, 5, 4, 2, 2
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        for i in range(T):
            q = x[0, i] @ p["W_qkv"][:, :d][:, sl]
            sc = []
            for j in range(Sx):
                pi, pj = 2 + i, j
                if pj > pi:
                    sc.append(-math.inf); continue
                kj = cat[j] @ p["W_qkv"][:, d:2 * d][:, sl]
                dist = pi - pj
                R = np.array([math.sin(dist * 10000.0 ** (-2.0 * m / d)) for m in range(d // 2)]
                             + [math.cos(dist * 10000.0 ** (-2.0 * m / d)) for m in range(d // 2)])
                rr = (R @ p["W_r"])[sl]
                sc.append((float((q + p["u"][h]) @ kj) + float((q + p["v"][h]) @ rr)) / math.sqrt(dh))
            mx = max(sc)
            e = [math.exp(s - mx) for s in sc]
            P = np.array(e) / sum(e)
            assert np.abs(P - c["P"][0, h, i]).max() < 1e-14


# ------------------------------------------------------------------ gradients
def _fd_check(cfg, mems, seed, n_probe=6):
    rng = np.random.default_rng(seed)
    layers = rand_layers(cfg, rng)
    Vi = rng.standard_normal((cfg.vocab, cfg.d_model)) * 0.5
    Vo = rng.standard_normal((cfg.vocab, cfg.d_model)) * 0.5      # separate leaves, unequal on purpose
    tok = rng.integers(0, cfg.vocab, (cfg.batch, cfg.seq_len))
    tgt = rng.integers(0, cfg.vocab, (cfg.batch, cfg.seq_len))
    loss, fw = O.model_forward(cfg, layers, Vi, Vo, tok, tgt, mems)
    grads, dVi, dVo = O.model_backward(cfg, layers, Vi, Vo, tok, tgt, fw)
    eps = 1e-5

    def probe(arr, garr, what):
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=min(n_probe, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp, _ = O.model_forward(cfg, layers, Vi, Vo, tok, tgt, mems)
            flat[idx] = old - eps
            lm, _ = O.model_forward(cfg, layers, Vi, Vo, tok, tgt, mems)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            an = garr.reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 2e-9, (what, idx, fd, an)

    for l, p in enumerate(layers):
        for n in p:
            probe(p[n], grads[l][n], (l, n))
    # V_i: probe rows that occur in the batch, V_o: any
    for t in np.unique(tok)[:3]:
        probe(Vi[t], dVi[t], ("Vi", t))
    probe(Vo, dVo, "Vo")
    unused = np.setdiff1d(np.arange(cfg.vocab), tok.reshape(-1))
    assert np.all(dVi[unused] == 0)


def test_finite_differences_plain():
    _fd_check(tiny_cfg(), None, 10)


def test_finite_differences_xl_no_mem():
    _fd_check(tiny_cfg(rel_pos=1, mem_len=3), None, 11)


def test_finite_differences_xl_with_mem():
    cfg = tiny_cfg(rel_pos=1, mem_len=3)
    rng = np.random.default_rng(12)
    mems = [rng.standard_normal((2, 3, 8)) for _ in range(cfg.n_layer)]
    _fd_check(cfg, mems, 13)


@pytest.mark.parametrize("rel_pos,mem", [(0, 0), (1, 0), (1, 4)])
def test_against_autograd_model(rel_pos, mem):
    """Loss and every gradient against an independent model of torch library routines."""
    cfg = O.Config(n_layer=3, d_model=12, n_head=3, d_head=4, d_ff=20, vocab=17, seq_len=7, batch=3,
                   mem_len=mem, rel_pos=rel_pos, emb_scale=1.7)
    rng = np.random.default_rng(20 + rel_pos + mem)
    layers = rand_layers(cfg, rng)
    Vi = rng.standard_normal((17, 12)) * 0.5
    Vo = rng.standard_normal((17, 12)) * 0.5
    tok = rng.integers(0, 17, (3, 7)); tgt = rng.integers(0, 17, (3, 7))
    mems = [rng.standard_normal((3, mem, 12)) for _ in range(3)] if mem else None
    loss, fw = O.model_forward(cfg, layers, Vi, Vo, tok, tgt, mems)
    grads, dVi, dVo = O.model_backward(cfg, layers, Vi, Vo, tok, tgt, fw)
    tl = [{n: torch.tensor(a, requires_grad=True) for n, a in p.items()} for p in layers]
    tVi = torch.tensor(Vi, requires_grad=True); tVo = torch.tensor(Vo, requires_grad=True)
    tm = None if mems is None else [torch.tensor(m) for m in mems]
    tloss, tin = torch_ref.forward(cfg, tl, tVi, tVo, torch.tensor(tok), torch.tensor(tgt), tm)
    tloss.backward()
    assert abs(loss - tloss.item()) < 1e-12
    for l in range(3):
        assert np.abs(fw["inputs"][l] - tin[l].detach().numpy()).max() < 1e-12
        for n in layers[l]:
            assert np.abs(grads[l][n] - tl[l][n].grad.numpy()).max() < 1e-11, (l, n)
    assert np.abs(dVi - tVi.grad.numpy()).max() < 1e-11
    assert np.abs(dVo - tVo.grad.numpy()).max() < 1e-11


def test_blob_roundtrip_and_layout():
    for rel in (0, 1):
        cfg = tiny_cfg(rel_pos=rel)
        names = [n for n, _ in O.param_shapes(cfg)]
        assert names == [n for n, _, _ in S.layer_param_layout(8, 2, 4, 12, rel)]
        n = sum(int(np.prod(s)) for _, s in O.param_shapes(cfg))
        assert n == S.layer_param_count(8, 2, 4, 12, rel)
        blob = np.arange(2 * n, dtype=np.float64)
        layers = O.unpack_layers(cfg, blob, 2)
        assert layers[0]["W_qkv"][0, 1] == 1.0 and layers[0]["W_o"][0, 0] == 8 * 24
        assert np.array_equal(O.pack_layers(cfg, layers), blob)


def test_split_layers():
    assert O.split_layers(18, 4) == [4, 5, 5, 4]
    assert O.split_layers(12, 4) == [3, 3, 3, 3]
    assert O.split_layers(2, 2) == [1, 1]
    assert O.split_layers(5, 1) == [5]
    assert S.default_layers_per_module(18, 4) == [4, 5, 5, 4]
