"""Pins of the oracle's training iteration (Eq. 8, Eq. 9, Algorithm 1, Algorithm 2)."""
import os

import numpy as np
import pytest
import torch

from oracle import ouro_oracle as O
import synth_inputs as S
from tests import torch_ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_cfg(K, L=None, **kw):
    base = dict(n_layer=L or K, d_model=8, n_head=2, d_head=4, d_ff=12, vocab=13, seq_len=5, batch=2,
                n_module=K, mem_len=0, rel_pos=0, dtype=0, optimizer=0)
    base.update(kw)
    return base


def make(K, seed=0, steps=8, **kw):
    c = small_cfg(K, **kw)
    cfg = O.Config(**c)
    blobs = S.init_params(c, seed=seed, std=0.3, perturb=0.1)
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], steps, 1.1, seed + 1,
                               contiguous=bool(c["mem_len"]))
    return c, cfg, blobs, tok, tgt


def test_eq8_eq9_index_table_K4():
    rows = [l.split() for l in open(os.path.join(GOLD, "eq8_index_table_K4.txt")) if not l.startswith("#")]
    c, cfg, blobs, tok, tgt = make(4, steps=7)
    orc = O.Oracle(cfg, blobs)
    for t in range(7):
        orc.step(tok[t], tgt[t], 0.05)
    conv = lambda s: -1 if s == "-" else int(s)
    for r in rows:
        t = int(r[0])
        for k in range(1, 5):
            assert orc.used[t][k] == conv(r[k])
        assert orc.used[t][0] == (conv(r[5]), conv(r[6]))


@pytest.mark.parametrize("K", [1, 2, 3, 4])
@pytest.mark.parametrize("opt", [0, 1])
def test_brute_force_replay(K, opt):
    """Every gradient consumed at iteration t equals the gradient recomputed from the
    stored full state of iteration t-K+k; the weights follow by re-applying the
    update rule outside the oracle."""
    c, cfg, blobs, tok, tgt = make(K, seed=K, steps=K + 3, optimizer=opt)
    orc = O.Oracle(cfg, blobs)
    lr = 0.05 if opt == 0 else 0.01
    # independent replay of Alg. 1 / Alg. 2 on flat module blobs
    w = [np.asarray(b, np.float64).copy() for b in blobs]
    m = [np.zeros_like(x) for x in w]; v = [np.zeros_like(x) for x in w]
    for t in range(K + 3):
        before = [orc.module_blob(k) for k in range(K + 1)]
        for k in range(K + 1):
            assert np.array_equal(before[k], w[k])
        orc.step(tok[t], tgt[t], lr)
        assert orc.brute_check(t) == 0.0
        for k in range(K + 1):
            if k == 0:
                ti = t - K + 1
                if ti >= 0:
                    layers, V, mems, tk, tg = orc.state_hist[t]
                    _, _, _, dVo, _ = O.full_gradient(cfg, layers, V, tk, tg, mems)
                    layers, V, mems, tk, tg = orc.state_hist[ti]
                    _, _, dVi, _, _ = O.full_gradient(cfg, layers, V, tk, tg, mems)
                    g = (0.5 * dVo + 0.5 * dVi).ravel()
                else:
                    g = np.zeros_like(w[0])
            else:
                tau = t - K + k
                if tau >= 0:
                    layers, V, mems, tk, tg = orc.state_hist[tau]
                    _, grads, _, _, _ = O.full_gradient(cfg, layers, V, tk, tg, mems)
                    g = O.pack_layers(cfg, [grads[l] for l in orc.module_layers(k)])
                else:
                    g = np.zeros_like(w[k])
            if opt == 0:
                w[k] = w[k] - lr * g
            else:
                m[k] = 0.9 * m[k] + (1 - 0.9) * g
                v[k] = 0.999 * v[k] + (1 - 0.999) * g * g
                w[k] = w[k] - lr * (m[k] / (1 - 0.9 ** (t + 1))) / (np.sqrt(v[k] / (1 - 0.999 ** (t + 1))) + 1e-8)
            assert np.abs(orc.module_blob(k) - w[k]).max() <= 1e-15 * max(1.0, np.abs(w[k]).max()), (t, k)
            w[k] = orc.module_blob(k)


def test_modules_frozen_until_first_gradient():
    K = 4
    c, cfg, blobs, tok, tgt = make(K, steps=6)
    for opt in (0, 1):
        cfg.optimizer = opt
        orc = O.Oracle(cfg, blobs)
        init = [orc.module_blob(k) for k in range(K + 1)]
        for t in range(6):
            orc.step(tok[t], tgt[t], 0.05)
            for k in range(1, K + 1):
                same = np.array_equal(orc.module_blob(k), init[k])
                assert same == (t < K - k), (opt, t, k)       # first real update at t = K-k
            assert np.array_equal(orc.module_blob(0), init[0]) == (t < K - 1)


def test_embed_warm_mode_termwise():
    K = 3
    c, cfg, blobs, tok, tgt = make(K, steps=2, embed_warm_mode=1)
    orc = O.Oracle(cfg, blobs)
    V0 = orc.module_blob(0)
    orc.step(tok[0], tgt[0], 0.1)
    _, _, _, dVo = orc.grad_hist[0][0], None, None, orc.grad_hist[0][2]
    assert np.abs(orc.module_blob(0) - (V0 - 0.1 * 0.5 * dVo.ravel())).max() < 1e-16
    assert orc.used[0][0] == (0, -1)


def test_tagged_gradient_plumbing(monkeypatch):
    """Replace backprop by integer-tagged gradients g(t, group) so the final weights have
    a closed form: w_k^T = -lr * sum over t with tau>=0 of (1000*tau + k)."""
    K, T = 4, 9
    c, cfg, blobs, tok, tgt = make(K, steps=T)
    calls = {"t": 0}

    def fake(cfg_, layers, V, tokens, targets, mems=None, seed=None):
        t = calls["t"]; calls["t"] += 1
        bounds = np.concatenate([[0], np.cumsum(cfg_.layers_per_module)])
        grads = []
        for l, p in enumerate(layers):
            k = int(np.searchsorted(bounds, l, side="right"))
            grads.append({n: np.full_like(a, 1000.0 * t + k) for n, a in p.items()})
        return 0.0, grads, np.full_like(V, 1000.0 * t + 0.25), np.full_like(V, 1000.0 * t + 0.75), [None] * len(layers)

    monkeypatch.setattr(O, "full_gradient", fake)
    zero = [np.zeros_like(b) for b in blobs]
    orc = O.Oracle(cfg, zero)
    lr = 2.0 ** -10
    for t in range(T):
        orc.step(tok[t], tgt[t], lr)
    for k in range(1, K + 1):
        expect = -lr * sum(1000.0 * (t - K + k) + k for t in range(T) if t - K + k >= 0)
        assert np.all(orc.module_blob(k) == expect)
    expect = -lr * sum(0.5 * (1000.0 * t + 0.75) + 0.5 * (1000.0 * (t - K + 1) + 0.25)
                       for t in range(T) if t - K + 1 >= 0)
    assert np.all(orc.module_blob(0) == expect)


def test_sgd_linearity_and_tied_invariant():
    K = 3
    c, cfg, blobs, tok, tgt = make(K, steps=6)
    orc = O.Oracle(cfg, blobs)
    w0 = [orc.module_blob(k) for k in range(K + 1)]
    lrs = [0.1, 0.05, 0.02, 0.07, 0.03, 0.01]
    for t in range(6):
        orc.step(tok[t], tgt[t], lrs[t])                      # the step uses gamma_t, not gamma_tau
    for k in range(1, K + 1):
        acc = sum(lrs[t] * orc.grad_blob(k, t - K + k) for t in range(6) if t - K + k >= 0)
        assert np.abs(orc.module_blob(k) - (w0[k] - acc)).max() < 1e-14


@pytest.mark.parametrize("opt", [0, 1])
def test_K1_is_ordinary_backprop(opt):
    """K=1: layer weights follow plain SGD/Adam on the autograd gradient; the tied matrix
    receives the mean (half the sum) of its two gradients."""
    c, cfg, blobs, tok, tgt = make(1, L=2, steps=3, optimizer=opt)
    orc = O.Oracle(cfg, blobs)
    tl = [{n: torch.tensor(a.copy(), requires_grad=True) for n, a in p.items()} for p in orc.layers]
    tV = torch.tensor(orc.V.copy(), requires_grad=True)
    params = [x for p in tl for x in p.values()] + [tV]
    lr = 0.05 if opt == 0 else 0.01
    optim = torch.optim.SGD(params, lr=lr) if opt == 0 else torch.optim.Adam(params, lr=lr, betas=(0.9, 0.999), eps=1e-8)
    for t in range(3):
        lo = orc.step(tok[t], tgt[t], lr)
        Vi = tV.detach().clone().requires_grad_(True)
        Vo = tV.detach().clone().requires_grad_(True)
        optim.zero_grad()
        loss, _ = torch_ref.forward(cfg, tl, Vi, Vo, torch.tensor(tok[t]), torch.tensor(tgt[t]))
        loss.backward()
        tV.grad = 0.5 * (Vi.grad + Vo.grad)
        optim.step()
        assert abs(lo - loss.item()) < 1e-12
        for l in range(2):
            for n in tl[l]:
                assert np.abs(orc.layers[l][n] - tl[l][n].detach().numpy()).max() < 1e-10, (t, l, n)
        assert np.abs(orc.V - tV.detach().numpy()).max() < 1e-10


def test_adam_closed_forms():
    cfg = O.Config(**small_cfg(1, optimizer=1))
    orc = O.Oracle(cfg, S.init_params(small_cfg(1), seed=0))
    w = np.array([1.0, -2.0, 3.0]); g = np.array([0.5, -4.0, 1e-3])
    m = np.zeros(3); v = np.zeros(3)
    orc._apply(w, g, m, v, 0.1)                                # t = 0: dw = -lr * g / (|g| + eps)
    assert np.abs(w - (np.array([1.0, -2.0, 3.0]) - 0.1 * g / (np.abs(g) + 1e-8))).max() < 1e-15
    w2 = np.array([1.0, -2.0]); m2 = np.zeros(2); v2 = np.zeros(2)
    orc._apply(w2, np.zeros(2), m2, v2, 0.1)                   # zero gradient, zero moments: no change
    assert np.array_equal(w2, [1.0, -2.0]) and not m2.any() and not v2.any()


def test_xl_memory_carry():
    c = small_cfg(2, L=2, rel_pos=1, mem_len=7)
    cfg = O.Config(**c)
    blobs = S.init_params(c, seed=3, std=0.3)
    tok, tgt = S.token_batches(13, 2, 5, 3, 1.1, 4, contiguous=True)
    assert np.array_equal(tok[1][:, 0], tgt[0][:, -1])          # streams are contiguous
    orc = O.Oracle(cfg, blobs)
    orc.step(tok[0], tgt[0], 0.05)
    assert orc.mems[0].shape == (2, 5, 8)                       # valid length min(M, T) after one step
    first_inputs = orc.mems[0].copy()
    orc.step(tok[1], tgt[1], 0.05)
    assert orc.mems[0].shape == (2, 7, 8)                       # last 7 rows of [old ; new]
    assert np.array_equal(orc.mems[0][:, :2], first_inputs[:, 3:])
    assert orc.brute_check(1) == 0.0


def test_learning_rate_schedule_closed_forms():
    """Warm-up then cosine (Section 5.2), pinned by what the two phases fix: the warm-up is an
    arithmetic progression that ends exactly at the base rate; the cosine phase starts there,
    passes the midpoint of [floor, base] half-way, is point-symmetric about it, decreases
    monotonically and ends at the floor, where it stays."""
    base, W, T, floor = 2.5e-4, 5000, 200000, 1e-6
    lr = lambda t: O.learning_rate(t, base, W, T, floor)
    assert lr(0) == base / W and lr(W - 1) == base
    d = [lr(t + 1) - lr(t) for t in range(0, W - 1, 97)]
    assert np.allclose(d, base / W, rtol=1e-9)
    assert lr(W) == base
    mid = W + (T - W) // 2
    assert abs(lr(mid) - 0.5 * (base + floor)) < 1e-15
    for x in (1, 17, 4000, 90000):
        assert abs(lr(W + x) + lr(T - x) - (base + floor)) < 1e-15
    ts = np.arange(W, T + 1, 331)
    v = np.array([lr(int(t)) for t in ts])
    assert np.all(np.diff(v) < 0)
    assert lr(T) == floor and lr(T + 12345) == floor
    # quarter points of a cosine: (1 + cos(pi/4)) / 2 and (1 + cos(3 pi/4)) / 2
    q = (T - W) // 4
    assert abs(lr(W + q) - (floor + (base - floor) * (2 + np.sqrt(2)) / 4)) < 1e-15
    assert abs(lr(W + 3 * q) - (floor + (base - floor) * (2 - np.sqrt(2)) / 4)) < 1e-15
    # no warm-up
    assert O.learning_rate(0, 1.0, 0, 10) == 1.0 and abs(O.learning_rate(5, 1.0, 0, 10) - 0.5) < 1e-15


# ------------------------------------------------ stored-input / recompute schedule
@pytest.mark.parametrize("K,kw", [(2, {}), (3, {}), (4, {}), (3, dict(rel_pos=1, mem_len=7, L=5))])
def test_recompute_with_frozen_weights_is_eq8(K, kw):
    """With step size 0 the weights never move, so recomputing from the stored input with the
    current weights must give exactly Eq. 8's gradient: the k-th slice of the full gradient of
    mini-batch t-K+k.  This pins the index plumbing of the schedule (which stored input, which
    error gradient, which iteration) to the already pinned full gradient."""
    c, cfg, blobs, tok, tgt = make(K, seed=10 + K, steps=K + 3, **kw)
    a, b = O.Oracle(cfg, blobs), O.RecomputeOracle(cfg, blobs)
    for t in range(K + 3):
        la, lb = a.step(tok[t], tgt[t], 0.0), b.step(tok[t], tgt[t], 0.0)
        assert la == lb
        for k in range(1, K + 1):
            tau = t - K + k
            assert b.batch_of[t][k] == (tau if tau >= 0 else -1)
            assert b.used[t][k] == (t if tau >= 0 else -1)
            for l in b.module_layers(k):
                for n in b.layers[l]:
                    ref = a.grad_hist[tau][0][l][n] if tau >= 0 else np.zeros_like(b.layers[l][n])
                    assert np.abs(b.grad_hist[t][0][l][n] - ref).max() < 1e-12, (t, k, l, n)
        ti = t - K + 1
        assert np.abs(b.grad_hist[t][1] - (a.grad_hist[ti][1] if ti >= 0 else 0.0)).max() < 1e-12
        assert np.abs(b.grad_hist[t][2] - a.grad_hist[t][2]).max() < 1e-12


@pytest.mark.parametrize("opt", [0, 1])
def test_recompute_K1_is_the_plain_schedule(opt):
    c, cfg, blobs, tok, tgt = make(1, L=2, steps=4, optimizer=opt)
    a, b = O.Oracle(cfg, blobs), O.RecomputeOracle(cfg, blobs)
    for t in range(4):
        assert a.step(tok[t], tgt[t], 0.03) == b.step(tok[t], tgt[t], 0.03)
        for k in range(2):
            assert np.array_equal(a.module_blob(k), b.module_blob(k))


@pytest.mark.parametrize("opt,kw", [(0, {}), (1, {}), (0, dict(rel_pos=1, mem_len=6))])
def test_recompute_schedule_against_autograd_pipeline(opt, kw):
    """The whole schedule rebuilt from torch autograd, module by module: every iteration each
    module re-runs its layers on its stored (detached) input of mini-batch t-K+k with the
    weights it holds now and calls backward with the error gradient its upper neighbour left the
    iteration before; the tied matrix mixes the two halves as in Eq. 9.  Weights, error
    gradients and losses must follow the oracle's over more iterations than the pipeline is deep,
    with weights that move (so a recompute with stale weights, or a wrong mailbox delay, shows)."""
    K, L, steps = 3, 4, 7
    c, cfg, blobs, tok, tgt = make(K, L=L, seed=5, steps=steps, optimizer=opt, **kw)
    orc = O.RecomputeOracle(cfg, blobs)
    lr = 0.05 if opt == 0 else 0.01
    tl = [{n: torch.tensor(a.copy(), requires_grad=True) for n, a in p.items()} for p in orc.layers]
    tV = torch.tensor(orc.V.copy(), requires_grad=True)
    params = [x for p in tl for x in p.values()] + [tV]
    optim = torch.optim.SGD(params, lr=lr) if opt == 0 else torch.optim.Adam(params, lr=lr, betas=(0.9, 0.999), eps=1e-8)
    bounds = np.concatenate([[0], np.cumsum(cfg.layers_per_module)])
    stored, mail, mems = {}, {}, None
    for t in range(steps):
        lo = orc.step(tok[t], tgt[t], lr)
        optim.zero_grad()
        for x in params:
            x.grad = torch.zeros_like(x)
        ttok, ttgt = torch.tensor(tok[t]), torch.tensor(tgt[t])
        with torch.no_grad():                                  # forward of mini-batch t: store inputs
            h, layer_in = ttok, []
            for k in range(1, K + 1):
                mk = None if mems is None else [mems[l] for l in range(bounds[k - 1], bounds[k])]
                stored[(k, t)] = (h, mk)
                x = torch_ref.embed(cfg, tV, h) if k == 1 else h
                for i, l in enumerate(range(bounds[k - 1], bounds[k])):
                    layer_in.append(x)
                    x = torch_ref.layer_forward(cfg, tl[l], x, None if mk is None else mk[i])
                h = x
            loss_t = torch.nn.functional.cross_entropy(h.reshape(-1, cfg.d_model) @ tV.t(), ttgt.reshape(-1).long()).item()
        assert abs(lo - loss_t) < 1e-12
        new_mail = {}
        gVi = torch.zeros_like(tV); gVo = torch.zeros_like(tV)
        for k in range(1, K + 1):
            tau = t - K + k
            if tau < 0:
                continue
            inp, mk = stored[(k, tau)]
            Vi = tV.detach().clone().requires_grad_(True)
            Vo = tV.detach().clone().requires_grad_(True)
            if k == 1:
                x0 = None
                x = torch_ref.embed(cfg, Vi, inp)
            else:
                x0 = inp.detach().clone().requires_grad_(True)
                x = x0
            for i, l in enumerate(range(bounds[k - 1], bounds[k])):
                x = torch_ref.layer_forward(cfg, tl[l], x, None if mk is None else mk[i])
            if k == K:
                lossk = torch.nn.functional.cross_entropy(x.reshape(-1, cfg.d_model) @ Vo.t(), ttgt.reshape(-1).long())
                lossk.backward()
                gVo = Vo.grad
            else:
                x.backward(mail[k])
            if k == 1:
                gVi = Vi.grad
            else:
                new_mail[k - 1] = x0.grad
        mail = new_mail
        if t - K + 1 >= 0:
            tV.grad = 0.5 * gVo + 0.5 * gVi
        else:
            tV.grad = torch.zeros_like(tV)
        optim.step()
        if cfg.mem_len:
            mems = [(layer_in[l] if mems is None else torch.cat([mems[l], layer_in[l]], dim=1))[:, -cfg.mem_len:] for l in range(L)]
        for k in list(orc.mail):
            assert np.abs(orc.mail[k][1] - mail[k].numpy()).max() < 1e-10, (t, k)
        for l in range(L):
            for n in tl[l]:
                assert np.abs(orc.layers[l][n] - tl[l][n].detach().numpy()).max() < 1e-9, (t, l, n)
        assert np.abs(orc.V - tV.detach().numpy()).max() < 1e-9


def test_recompute_differs_from_eq8_once_weights_move():
    """The two schedules are different iterations: same losses and gradients until the first
    delayed gradient meets weights that have moved, different from there on (so the frozen-weight
    pin above does not hide an oracle that simply replays Eq. 8)."""
    K = 3
    c, cfg, blobs, tok, tgt = make(K, seed=2, steps=6)
    a, b = O.Oracle(cfg, blobs), O.RecomputeOracle(cfg, blobs)
    diff = []
    for t in range(6):
        a.step(tok[t], tgt[t], 0.1); b.step(tok[t], tgt[t], 0.1)
        diff.append(max(np.abs(a.module_blob(k) - b.module_blob(k)).max() for k in range(K + 1)))
    assert diff[0] == 0.0                      # only module K (tau = t) has a gradient: identical
    assert diff[-1] > 1e-4


# ---------------------------------------------------------------- repeatable dropout
def splitmix64_python(seed, n):
    """The SplitMix64 sequence written with Python integers (state += gamma; finalise)."""
    M = (1 << 64) - 1
    out, s = [], seed & M
    for _ in range(n):
        s = (s + 0x9E3779B97F4A7C15) & M
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        out.append(z ^ (z >> 31))
    return out


def test_random_bits_are_the_splitmix_sequence_and_look_uniform():
    """The vectorised generator against the sequential definition in big-integer arithmetic
    (stream 0: output i is element i+1 of the sequence; stream s starts 2^40*s further on), then
    what dropout needs of it: the keep rate within binomial bounds for several p, balanced bits,
    and no visible correlation between neighbours, streams or consecutive seeds."""
    seq = splitmix64_python(12345, 40)
    got = O.random_u32(12345, 0, np.arange(40))
    assert [int(x) for x in got] == [z >> 32 for z in seq]
    g = 0x9E3779B97F4A7C15
    jump = splitmix64_python((12345 + g * (3 << 40)) & ((1 << 64) - 1), 5)
    assert [int(x) for x in O.random_u32(12345, 3, np.arange(5))] == [z >> 32 for z in jump]
    n = 1 << 20
    idx = np.arange(n, dtype=np.uint64)
    a = O.random_u32(7, 5, idx)
    for p in (0.1, 0.5, 0.9):
        keep = (a >= np.uint32(int(p * 2 ** 32))).mean()
        assert abs(keep - (1 - p)) < 5 * np.sqrt(p * (1 - p) / n)
    for bit in range(32):
        assert abs(((a >> np.uint32(bit)) & 1).mean() - 0.5) < 5 * 0.5 / np.sqrt(n)
    u = a.astype(np.float64) / 2 ** 32 - 0.5
    for other in (np.roll(u, 1), O.random_u32(7, 6, idx) / 2 ** 32 - 0.5, O.random_u32(8, 5, idx) / 2 ** 32 - 0.5):
        assert abs(np.mean(u * other)) < 5 / (12 * np.sqrt(n))


def test_dropout_mask_semantics():
    cfg = O.Config(**small_cfg(1, dropout=0.25, seed=9))
    m = O.dropout_mask(cfg, 9, 3, (4, 5, 6))
    assert set(np.unique(m)) == {0.0, 1 / 0.75}
    assert np.array_equal(m, O.dropout_mask(cfg, 9, 3, (4, 5, 6)))          # repeatable
    assert not np.array_equal(m, O.dropout_mask(cfg, 10, 3, (4, 5, 6)))
    assert not np.array_equal(m, O.dropout_mask(cfg, 9, 4, (4, 5, 6)))
    assert np.array_equal(m.ravel()[:30], O.dropout_mask(cfg, 9, 3, (30,)))   # row-major element index
    big = O.dropout_mask(cfg, 1, 0, (1 << 18,))
    assert abs(big.mean() - 1.0) < 0.01                                     # inverted scaling keeps the mean
    cfg0 = O.Config(**small_cfg(1, dropout=0.0))
    assert np.all(O.dropout_mask(cfg0, 1, 0, (100,)) == 1.0)


@pytest.mark.parametrize("kw", [{}, dict(rel_pos=1, mem_len=4)])
def test_dropout_gradients_by_finite_differences_and_autograd(kw):
    """With the masks fixed by the seed the network is a smooth function again: the oracle's
    gradient under dropout against central differences along random directions, and against the
    autograd model that receives the same masks as constants."""
    c = small_cfg(1, L=2, dropout=0.3, seed=4, **kw)
    cfg = O.Config(**c)
    blobs = S.init_params(c, seed=1, std=0.3, perturb=0.1)
    tok, tgt = S.token_batches(13, 2, 5, 1, 1.1, 2, False)
    orc = O.Oracle(cfg, blobs)
    rng = np.random.default_rng(0)
    mems = [rng.standard_normal((2, 4, 8)) for _ in range(2)] if kw else None
    seed = 77
    loss, grads, dVi, dVo, _ = O.full_gradient(cfg, orc.layers, orc.V, tok[0], tgt[0], mems, seed)
    loss0, *_ = O.full_gradient(cfg, orc.layers, orc.V, tok[0], tgt[0], mems, None)
    assert abs(loss - loss0) > 1e-3                                         # dropout is on
    for _ in range(4):
        dirs = [{n: rng.standard_normal(a.shape) for n, a in p.items()} for p in orc.layers]
        dV = rng.standard_normal(orc.V.shape)
        eps = 1e-6
        def at(sgn):
            ls = [{n: a + sgn * eps * dirs[l][n] for n, a in p.items()} for l, p in enumerate(orc.layers)]
            V = orc.V + sgn * eps * dV
            return O.model_forward(cfg, ls, V, V, tok[0], tgt[0], mems, seed)[0]
        fd = (at(+1) - at(-1)) / (2 * eps)
        an = sum(float((grads[l][n] * dirs[l][n]).sum()) for l in range(2) for n in grads[l]) + float(((dVi + dVo) * dV).sum())
        assert abs(fd - an) < 1e-6 * max(1.0, abs(an))
    # autograd with the same masks
    tl = [{n: torch.tensor(a.copy(), requires_grad=True) for n, a in p.items()} for p in orc.layers]
    Vi = torch.tensor(orc.V.copy(), requires_grad=True); Vo = torch.tensor(orc.V.copy(), requires_grad=True)
    masks = {"emb": torch.tensor(O.dropout_mask(cfg, seed, O.embed_stream(), (2, 5, 8)))}
    for l in range(2):
        for site in (1, 2):
            masks[(l, site)] = torch.tensor(O.dropout_mask(cfg, seed, O.layer_stream(l, site), (2, 5, 8)))
    tm = None if mems is None else [torch.tensor(x) for x in mems]
    tloss, _ = torch_ref.forward(cfg, tl, Vi, Vo, torch.tensor(tok[0]), torch.tensor(tgt[0]), tm, masks)
    tloss.backward()
    assert abs(tloss.item() - loss) < 1e-12
    assert np.abs(Vi.grad.numpy() - dVi).max() < 1e-10 and np.abs(Vo.grad.numpy() - dVo).max() < 1e-10
    for l in range(2):
        for n in grads[l]:
            assert np.abs(tl[l][n].grad.numpy() - grads[l][n]).max() < 1e-10, (l, n)


def test_repeatable_dropout_in_the_recompute_schedule():
    """Section 5.2, "Repeatable Dropout": with the seed stored beside the module input, the
    recomputation sees the masks of the original pass, so at frozen weights the schedule still
    yields Eq. 8's gradient (now of the dropout network of mini-batch t-K+k).  Recomputing under
    the running iteration's seed instead (the ablation) breaks exactly that."""
    K = 3
    c, cfg, blobs, tok, tgt = make(K, seed=21, steps=K + 3, dropout=0.2)
    cfg.seed = 1000
    a, b = O.Oracle(cfg, blobs), O.RecomputeOracle(cfg, blobs)
    bad = O.RecomputeOracle(cfg, blobs, repeatable=False)
    worst_bad = 0.0
    for t in range(K + 3):
        la, lb = a.step(tok[t], tgt[t], 0.0), b.step(tok[t], tgt[t], 0.0)
        bad.step(tok[t], tgt[t], 0.0)
        assert la == lb
        assert a.brute_check(t) == 0.0
        for k in range(1, K + 1):
            tau = t - K + k
            if tau < 0:
                continue
            for l in b.module_layers(k):
                for n in b.layers[l]:
                    ref = a.grad_hist[tau][0][l][n]
                    assert np.abs(b.grad_hist[t][0][l][n] - ref).max() < 1e-12, (t, k, l, n)
                    if k < K:
                        worst_bad = max(worst_bad, float(np.abs(bad.grad_hist[t][0][l][n] - ref).max()))
        ti = t - K + 1
        if ti >= 0:
            assert np.abs(b.grad_hist[t][1] - a.grad_hist[ti][1]).max() < 1e-12
    assert worst_bad > 1e-3


def test_eval_step_is_the_forward_pass():
    """Evaluation = the forward half of a training iteration at frozen weights: same loss, same
    memory roll as a training step with step size 0 and no dropout; with dropout configured it
    still reports the loss of the network without masks; weights never move."""
    c, cfg, blobs, tok, tgt = make(2, L=2, steps=4, rel_pos=1, mem_len=7)
    a, b = O.Oracle(cfg, blobs), O.Oracle(cfg, blobs)
    cd = dict(c, dropout=0.3, seed=5)
    d = O.Oracle(O.Config(**cd), blobs)
    w0 = [a.module_blob(k) for k in range(3)]
    for t in range(4):
        la, lb, ld = a.step(tok[t], tgt[t], 0.0), b.eval_step(tok[t], tgt[t]), d.eval_step(tok[t], tgt[t])
        assert la == lb == ld
        for l in range(2):
            assert np.array_equal(a.mems[l], b.mems[l]) and np.array_equal(a.mems[l], d.mems[l])
        assert b.t == t + 1
    for k in range(3):
        assert np.array_equal(b.module_blob(k), w0[k])
    # uniform predictions: loss = ln(vocab) exactly, i.e. log2(vocab) bits per character
    z = [np.zeros_like(x) for x in blobs]
    assert abs(O.Oracle(cfg, z).eval_step(tok[0], tgt[0]) - np.log(13)) < 1e-12
