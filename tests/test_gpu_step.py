"""End-to-end parity of the HIP training iteration against the CPU oracle, through the
C boundary: losses, every gradient store, updated weights, segment memories, and the
bit-exact staleness bookkeeping (Eq. 8-9)."""
import json
import os

import numpy as np
import pytest

from oracle import ouro_oracle as O
import synth_inputs as S

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def P():
    import paper_1909_06695_amd as pkg
    return pkg


def rel_err(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


# Element-wise bound beside every norm ratio: |a - b| <= f * tol * (|b| + EW_ATOL * scale), f the factor
# the norm ratio is held to (1, or 5 for a single small parameter tensor).  The norm ratio alone
# lets a fraction tol^2 of a tensor be entirely wrong (three rows of an [8192, 512] activation at
# the bf16 bar); under this bound one wrong element (an error of the size of its scale) fails it
# 1 / (f * tol * EW_ATOL) times over.  `scale` is the size elements have at that place: the
# tensor's RMS for a vector; for a matrix the larger of the element's row RMS and column RMS,
# because gradient matrices are sums of outer products whose rows and columns carry very
# different sizes (a row of dV_i is the sum over the occurrences of one token: 14 % of a Zipf
# stream for the first id, none at all for most).  EW_ATOL = 6: rounding
# errors are close to normal, a tensor that just meets the norm bound f * tol has a per-element
# standard deviation of f * tol * scale, and the largest of 5e7 normal draws sits near 6 standard
# deviations.
EW_ATOL = 6.0
# The element-wise bound never runs tighter than EW_FLOOR x tol: the errors' tails are heavier than
# normal (a few elements in 4e6 reach 2.7 x tol x (|b| + 6 scale) after four Adam iterations, when the
# two sides' weights have also drifted apart); a wrong element still fails 1 / (4 x 0.02 x 6) = 2 times over.
EW_FLOOR = 4.0
RECORD_ONLY = bool(os.environ.get("OURO_PARITY_RECORD"))   # calibration runs: collect WORST without failing
WORST = {}          # what -> (largest norm ratio / tol, largest element-wise excess), for the calibration record


def elem_scale(ref, shape=None, whole=False):
    """Element-wise size of a reference tensor (flat array out): see EW_ATOL.  `whole`: never below
    the whole tensor's RMS (see cancels_by_rows)."""
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    if shape is None or len(shape) != 2 or rms == 0.0:
        return np.full(ref.size, rms)
    r2 = ref.reshape(shape)
    sc = np.maximum(np.sqrt(np.mean(r2 * r2, axis=1))[:, None], np.sqrt(np.mean(r2 * r2, axis=0))[None, :]).ravel()
    return np.maximum(sc, rms) if whole else sc


def cancels_by_rows(name):
    """The gradient of W_r has rows that vanish by cancellation, not because their summands are small:
    the low-frequency cosine features of the distance encoding (Section 5.2's Transformer-XL attention)
    are close to 1 at every distance, so their rows of the gradient are close to sum_ij dS_ij (q_i + v),
    and the softmax gradient dS sums to zero over the keys of every query.  The oracle's fp64 sum
    reaches 1e-3 of the tensor's RMS there; rounded summands cannot, so the scale of such a tensor's
    elements is never taken below the tensor's own RMS."""
    return name == "W_r"


def record(key, nr_over_tol, excess):
    if RECORD_ONLY:
        key = os.environ.get("PYTEST_CURRENT_TEST", "").split("::")[-1].split(" ")[0] + " :: " + key
    w = WORST.get(key, (0.0, 0.0))
    WORST[key] = (max(w[0], nr_over_tol), max(w[1], excess))


def assert_close(got, ref, tol, what, norm_factor=1.0, shape=None, whole=False):
    got = np.asarray(got, np.float64).ravel(); ref = np.asarray(ref, np.float64).ravel()
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), (what, "non-finite values")
    diff = np.abs(got - ref)
    nr = float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-30))
    ew = UV_ELEMENT_FACTOR if norm_factor == UV_FACTOR else max(norm_factor, EW_FLOOR)
    bound = ew * tol * (np.abs(ref) + EW_ATOL * elem_scale(ref, shape, whole))
    over = diff > bound
    ratio = diff / np.maximum(bound, 1e-300)
    excess = float(np.max(ratio))
    record(what[0] if isinstance(what, tuple) else what, nr / tol, min(excess, 1e9))
    if RECORD_ONLY and isinstance(what, tuple) and what[0] in ("dVi", "dVo"):
        record(f"{what[0]} t={what[-1]}", nr / tol, min(excess, 1e9))
    if RECORD_ONLY:
        return
    assert nr < norm_factor * tol, (what, "norm ratio", nr)
    if over.any():
        i = int(np.argmax(ratio))
        raise AssertionError((what, "element", i, got[i], ref[i], "bound", bound[i], "excess", excess, "bad elements", int(over.sum())))


# Error budget of a weight after an optimiser step with a gradient that carries the rounding noise
# the gradient bound allows (per element up to tol * (|g| + EW_ATOL * scale)).  SGD: lr times that.
# Adam: the step lr * m^ / (sqrt(v^) + eps) does not depend on the size of g but on ratios, so the
# error of one step is lr * (noise / sqrt(v^)) * 2 (numerator and denominator move), capped by the
# largest change a step can make at all, ADAM_CAP * lr (a sign flip of a step of lr *
# (1-beta1)/sqrt(1-beta2) = 3.2 lr at most, in practice of about lr); where sqrt(v^) is far below
# the noise the step is ill-conditioned and only that cap holds.  Every element is checked against
# the sum of its per-iteration budgets.
ADAM_CAP = 4.0


@pytest.fixture(autouse=True, scope="module")
def _dump_worst():
    """With OURO_PARITY_RECORD=<file> the largest ratios seen per kind of tensor are written there."""
    yield
    if RECORD_ONLY:
        with open(os.environ["OURO_PARITY_RECORD"], "w") as f:
            json.dump({k: list(v) for k, v in sorted(WORST.items())}, f, indent=1)


UV_FACTOR = 10.0
# Single elements of du, dv: the noise of one element is set by the size of the summands of its sum,
# not by the sum (1.4 times the RMS of the oracle's tensor seen on one of 1024 elements, at d = 1024
# after four Adam iterations, the norm ratio of the same tensor being inside 10 tol), so the
# element-wise bound of these two vectors runs at twice their norm factor.
UV_ELEMENT_FACTOR = 2.0 * UV_FACTOR


def tensor_factor(name, shape):
    """Multiple of tol a single parameter tensor's gradient is held to (a whole module's gradient: 1).
    Small tensors (biases, LayerNorm scales and shifts) are averages over little data; the gradient
    of W_r is a sum over distances of oscillating terms; the gradients of the two bias vectors u, v
    of the relative scores are sums over every (query, key) pair of a head of signed terms, so the
    rounding noise of the summands, which adds up like a random walk, stands against a sum that
    largely cancels (observed: 3.5 to 6 tol at d = 1024, segment and memory 384, after Adam steps)."""
    if name in ("u", "v"):
        return UV_FACTOR
    return 5.0 if int(np.prod(shape)) < 65536 or name == "W_r" else 1.5


def param_shapes_of_groups(cfg, orc):
    """Per parameter group a list of (offset, count, shape, tolerance factor) of its tensors in blob order."""
    K = cfg.n_module
    out = [[(0, cfg.vocab * cfg.d_model, (cfg.vocab, cfg.d_model), 1.0, False)]]
    for k in range(1, K + 1):
        off, lst = 0, []
        for _ in orc.module_layers(k):
            for name, shape in O.param_shapes(cfg):
                n = int(np.prod(shape))
                lst.append((off, n, shape, tensor_factor(name, shape), cancels_by_rows(name)))
                off += n
        out.append(lst)
    return out


def run_both(c, steps, lr, seed=0, std=0.02, perturb=0.0, check_grads=True, tol=1e-4, module_api=False, rep=1):
    """Runs `steps` iterations on both sides; returns nothing, asserts parity.

    rep > 1: the HIP model runs with batch * rep streams, each of the oracle's streams
    replicated rep times.  Streams do not interact and the loss is a mean over all targets, so
    the loss, every gradient and every weight equal those of the oracle's batch exactly (up to
    summation order): the full-size launch configuration is checked element by element at
    the oracle cost of the small batch."""
    pkg = P()
    blobs = S.init_params(c, seed=seed, std=std, perturb=perturb)
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], steps, c.get("zipf_s", 1.1), seed + 1,
                               contiguous=bool(c.get("mem_len", 0)))
    cfg = O.Config(**c)
    stored = c.get("schedule", 0) == 1                    # stored-input / recompute schedule
    orc = (O.RecomputeOracle if stored else O.Oracle)(cfg, blobs, keep_history=False)
    m = pkg.create_model(**dict(c, batch=c["batch"] * rep))
    K = c["n_module"]
    for g in range(K + 1):
        assert m.param_count(g) == blobs[g].size
        m.set_params(g, blobs[g])
    dtok = torch.from_numpy(np.tile(tok, (1, rep, 1))).cuda(); dtgt = torch.from_numpy(np.tile(tgt, (1, rep, 1))).cuda()
    budget = [np.zeros(b.size) for b in blobs]            # per-element error budget of the weights, see ADAM_CAP
    w0 = [b.astype(np.float64) for b in blobs]
    moved = [False] * (K + 1)
    shapes = param_shapes_of_groups(cfg, orc)
    for t in range(steps):
        lo = orc.step(tok[t], tgt[t], lr)
        for g in range(K + 1):
            u = orc.used[t][g]
            if g >= 1 and u >= 0:
                gg = orc.grad_blob(g, u)
            elif g == 0 and u[0] >= 0:
                gg = 0.5 * orc.grad_hist[u[0]][2].ravel()
                if u[1] >= 0:
                    gg = gg + 0.5 * orc.grad_hist[u[1]][1].ravel()
            else:
                continue
            moved[g] = True
            noise = np.concatenate([(UV_ELEMENT_FACTOR if f == UV_FACTOR else max(f, EW_FLOOR)) * tol * (np.abs(gg[o:o + n]) + EW_ATOL * elem_scale(gg[o:o + n], sh, wh)) for o, n, sh, f, wh in shapes[g]])
            if c["optimizer"] == 0:
                budget[g] += lr * noise
            else:
                v = orc.vV.ravel() if g == 0 else O.pack_layers(cfg, [orc.v[l] for l in orc.module_layers(g)])
                vhat = v / (1.0 - c.get("beta2", 0.999) ** orc.t)             # orc.t: iterations done, = t + 1
                budget[g] += lr * np.minimum(ADAM_CAP, 2.0 * noise / np.maximum(np.sqrt(vhat), 1e-300))
        if module_api:
            for k in range(1, K + 1):
                m.module_forward(k, dtok[t], dtgt[t])
            lg = m.get_loss()
            for k in range(K, 0, -1):
                m.module_backward(k)
            order = list(range(K + 1))
            np.random.default_rng(t).shuffle(order)          # updates commute within an iteration
            for g in order:
                m.delayed_update(g, lr)
        else:
            lg = m.step(dtok[t], dtgt[t], lr)
        assert abs(lg - lo) / abs(lo) < tol, (t, lg, lo)
        assert m.current_step() == t + 1
        if check_grads:
            grads, dVi, dVo = orc.grad_hist[t]
            assert_close(m.get_grad_slot(K + 1, t), dVo, tol, ("dVo", t), shape=dVo.shape)
            if not stored or t - K + 1 >= 0:
                assert_close(m.get_grad_slot(0, t), dVi, tol, ("dVi", t), shape=dVi.shape)
            for k in range(1, K + 1):
                if stored:
                    # the pass of iteration t is for mini-batch t-K+k, recomputed from input slot (t-K+k) mod (K-k+1)
                    tau = t - K + k
                    if k < K:
                        assert m.last_input_read(k) == ((tau % (K - k + 1), tau) if tau >= 0 else (-1, -1))
                        assert m.input_tag(k, t % (K - k + 1)) == t
                    assert m.last_read(k) == ((0, tau) if tau >= 0 else (-1, -1))
                    if tau < 0:
                        continue
                got = m.get_grad_slot(k, t)
                nrm = rel_err(got, orc.grad_blob(k, t))
                record(f"module grad k={k} t={t}" if RECORD_ONLY else "module grad", nrm / tol, 0.0)
                assert RECORD_ONLY or nrm < tol, ("module grad", k, t, nrm)
                # per-parameter check so that small tensors (biases, u, v) are not drowned
                off = 0
                for l in orc.module_layers(k):
                    for name, shape in O.param_shapes(cfg):
                        n = int(np.prod(shape))
                        assert_close(got[off:off + n], grads[l][name], tol, ("grad " + name, l, t), norm_factor=tensor_factor(name, shape), shape=shape, whole=cancels_by_rows(name))
                        off += n
        for g in range(K + 1):
            got, ref = m.get_params(g).astype(np.float64), orc.module_blob(g)
            if not moved[g]:
                assert np.array_equal(got, w0[g]), ("group moved before its first gradient", g, t)
                continue
            assert np.all(np.isfinite(got)), ("weights", g, t)
            diff = np.abs(got - ref)
            allow = budget[g] + 1e-6 * np.abs(ref)               # + fp32 rounding of the master weights
            excess = float(np.max(diff / np.maximum(allow, 1e-300)))
            # the movement itself in the norm: against the size of the weights a lost update hides under tol
            nr = rel_err(got - w0[g], ref - w0[g])
            record("weights", nr / tol, excess)
            if RECORD_ONLY and excess > 1.0:
                i = int(np.argmax(diff / np.maximum(allow, 1e-300)))
                WORST[os.environ.get("PYTEST_CURRENT_TEST", "").split("::")[-1].split(" ")[0] + f" :: weights detail g{g} t{t}"] = (
                    float(i), float(got[i]), float(ref[i]), float(w0[g][i]), float(budget[g][i]), float((diff > allow).sum()), float(diff.size))
            if not RECORD_ONLY:
                assert excess <= 1.0, ("weights", g, t, "element", int(np.argmax(diff / np.maximum(allow, 1e-300))), excess)
                assert c["optimizer"] == 1 or nr < MOVE_FACTOR * tol, ("weight movement", g, t, nr)
        if c.get("mem_len", 0):
            for l in range(c["n_layer"]):
                mem = m.get_mems(l)
                assert mem.shape[0] == orc.mems[l].shape[0] * rep and mem.shape[1:] == orc.mems[l].shape[1:]
                assert_close(mem, np.tile(orc.mems[l], (rep, 1, 1)), tol, ("memory", l, t))
    m.close()


# SGD only: bound on the relative error of the whole group's movement w_t - w_0 (norm ratio, in units
# of tol).  The movement is a sum of gradients, so the gradients' own bound applies with slack for
# the bf16 working copy that later iterations see.  (Under Adam every element moves by about lr per
# iteration whatever |g| is, so the few elements whose gradient is below the rounding noise weigh
# as much in that norm as all others; there the per-element budget above is the check.)
MOVE_FACTOR = 3.0


def test_config1_fp32_sgd_three_steps():
    c = dict(S.CONFIGS["cfg1"])
    run_both(c, steps=3, lr=c["lr"], seed=c["seed"])


def test_config1_perturbed_params_module_api():
    """Same shape with non-trivial biases / gains, Adam, more steps than K, driven through
    module_forward / module_backward / delayed_update with shuffled update order."""
    c = dict(S.CONFIGS["cfg1"], optimizer=1)
    run_both(c, steps=5, lr=1e-3, seed=3, std=0.08, perturb=0.1, module_api=True)


def test_ragged_shapes_K3_fp32():
    c = dict(n_layer=4, d_model=40, n_head=5, d_head=8, d_ff=72, vocab=131, seq_len=19, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=0, optimizer=0)
    run_both(c, steps=5, lr=0.05, seed=5, std=0.1, perturb=0.1)


def test_K1_fp32_adam():
    c = dict(n_layer=2, d_model=32, n_head=2, d_head=16, d_ff=64, vocab=97, seq_len=16, mem_len=0, batch=2,
             n_module=1, rel_pos=0, dtype=0, optimizer=1)
    run_both(c, steps=3, lr=1e-3, seed=6, std=0.1, perturb=0.1)


def test_xl_fp32_memory_carry():
    """Relative attention with a segment memory that is empty, then partial, then rolling."""
    c = dict(n_layer=3, d_model=32, n_head=2, d_head=16, d_ff=48, vocab=61, seq_len=6, mem_len=10, batch=2,
             n_module=3, rel_pos=1, dtype=0, optimizer=0)
    run_both(c, steps=5, lr=0.05, seed=7, std=0.15, perturb=0.1)


def test_xl_fp32_odd_dims_adam():
    c = dict(n_layer=2, d_model=82, n_head=2, d_head=41, d_ff=100, vocab=73, seq_len=9, mem_len=9, batch=2,
             n_module=2, rel_pos=1, dtype=0, optimizer=1, embed_warm_mode=1)
    run_both(c, steps=4, lr=1e-3, seed=8, std=0.1, perturb=0.1)


@pytest.mark.parametrize("K,opt,api", [(2, 0, False), (3, 0, True), (4, 1, False), (1, 1, False)])
def test_stored_input_schedule_fp32(K, opt, api):
    """The memory-saving schedule (stored module inputs, recomputation with the current weights,
    error gradients handed down one iteration late) against its oracle in fp32: losses, every
    gradient with the mini-batch and ring slot it was recomputed from, and the weights, over more
    iterations than the pipeline is deep."""
    c = dict(n_layer=max(K, 4), d_model=40, n_head=5, d_head=8, d_ff=72, vocab=131, seq_len=19, mem_len=0, batch=3,
             n_module=K, rel_pos=0, dtype=0, optimizer=opt, schedule=1)
    run_both(c, steps=K + 4, lr=0.05 if opt == 0 else 1e-3, seed=50 + K, std=0.1, perturb=0.1, module_api=api)


def test_stored_input_schedule_xl_blocks_fp32():
    c = dict(n_layer=3, d_model=32, n_head=2, d_head=16, d_ff=48, vocab=61, seq_len=12, mem_len=0, batch=2,
             n_module=3, rel_pos=1, dtype=0, optimizer=0, schedule=1, embed_warm_mode=1)
    run_both(c, steps=6, lr=0.05, seed=57, std=0.15, perturb=0.1)


def test_stored_input_schedule_with_segment_memory():
    """Transformer-XL memories under the stored-input schedule: a module recomputes mini-batch
    t-K+k against the memories its layers held at that iteration, while the forward pass rolls
    them on.  fp32 (general kernels), then bf16 at head size 64 (fused kernels)."""
    c = dict(n_layer=4, d_model=32, n_head=2, d_head=16, d_ff=48, vocab=61, seq_len=6, mem_len=10, batch=2,
             n_module=3, rel_pos=1, dtype=0, optimizer=0, schedule=1)
    run_both(c, steps=7, lr=0.05, seed=71, std=0.15, perturb=0.1)
    c = dict(n_layer=3, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=512, seq_len=80, mem_len=112, batch=2,
             n_module=3, rel_pos=1, dtype=1, optimizer=0, embed_warm_mode=1, schedule=1)
    run_both(c, steps=6, lr=0.05, seed=73, std=0.05, perturb=0.05, tol=2e-2)


def test_stored_input_schedule_bf16():
    """bf16 mode, K = 4, shapes that span several MFMA tiles; then K = 3 with Adam through the
    zero-padded storage."""
    c = dict(n_layer=4, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=1001, seq_len=96, mem_len=0, batch=3,
             n_module=4, rel_pos=0, dtype=1, optimizer=0, schedule=1)
    run_both(c, steps=7, lr=0.05, seed=61, std=0.05, perturb=0.05, tol=2e-2)
    c = dict(n_layer=3, d_model=82, n_head=2, d_head=41, d_ff=100, vocab=203, seq_len=70, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=1, optimizer=1, schedule=1)
    run_both(c, steps=5, lr=1e-3, seed=63, std=0.05, perturb=0.05, tol=2e-2)


@pytest.mark.parametrize("schedule", [0, 1])
def test_dropout_fp32(schedule):
    """Repeatable dropout (embedding sum, attention-projection and feed-forward outputs) in both
    schedules against the oracle, fp32: the masks are bit-identical on both sides, so the usual
    tolerance holds.  Under schedule 1 the recomputation of mini-batch t-K+k must regenerate that
    mini-batch's masks from the stored seed (a recomputation under the running seed fails this)."""
    c = dict(n_layer=4, d_model=40, n_head=5, d_head=8, d_ff=72, vocab=131, seq_len=19, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=0, optimizer=0, schedule=schedule, dropout=0.1875, seed=2 ** 40 + 17)
    run_both(c, steps=6, lr=0.05, seed=81, std=0.1, perturb=0.1)


def test_dropout_xl_memory_adam_fp32():
    c = dict(n_layer=3, d_model=32, n_head=2, d_head=16, d_ff=48, vocab=61, seq_len=6, mem_len=10, batch=2,
             n_module=3, rel_pos=1, dtype=0, optimizer=1, schedule=1, dropout=0.125, seed=5)
    run_both(c, steps=6, lr=1e-3, seed=83, std=0.15, perturb=0.1)


@pytest.mark.parametrize("schedule", [0, 1])
def test_dropout_bf16(schedule):
    """bf16: fused masks in the MFMA epilogues (16-byte store path) and through zero-padded storage."""
    c = dict(n_layer=3, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=512, seq_len=96, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=1, optimizer=0, schedule=schedule, dropout=0.15625, seed=99)
    run_both(c, steps=5, lr=0.05, seed=85, std=0.05, perturb=0.05, tol=2e-2)
    c = dict(n_layer=2, d_model=82, n_head=2, d_head=41, d_ff=100, vocab=203, seq_len=70, mem_len=0, batch=3,
             n_module=2, rel_pos=0, dtype=1, optimizer=0, schedule=schedule, dropout=0.15625, seed=7)
    run_both(c, steps=4, lr=0.05, seed=87, std=0.05, perturb=0.05, tol=2e-2)


@pytest.mark.parametrize("dtype,tol", [(0, 1e-4), (1, 2e-2)])
@pytest.mark.parametrize("kw", [dict(seq_len=1, batch=5), dict(seq_len=2, batch=1, n_layer=1, n_module=1),
                                dict(seq_len=3, batch=2, rel_pos=1, mem_len=7, embed_warm_mode=1),
                                dict(seq_len=5, batch=1, n_layer=4, n_module=4, schedule=1, rel_pos=1, mem_len=1),
                                dict(seq_len=4, batch=2, vocab=2, d_ff=1)])
def test_degenerate_shapes(dtype, tol, kw):
    """Single-token segments (each query sees only itself), one layer in one module, a memory
    longer than the segment or of one row, as many modules as layers, a two-word vocabulary and a
    one-unit feed-forward layer: both modes, every gradient and the weights against the oracle."""
    c = dict(n_layer=2, d_model=16, n_head=2, d_head=8, d_ff=24, vocab=37, seq_len=4, mem_len=0, batch=2,
             n_module=2, rel_pos=0, dtype=dtype, optimizer=0)
    c.update(kw)
    if dtype == 1 and c["d_ff"] == 1:
        pytest.skip("8 tokens through one bf16 hidden unit: rounding noise is averaged over nothing, the 2e-2 bar does not apply")
    run_both(c, steps=c["n_module"] + 3, lr=0.05, seed=91, std=0.2, perturb=0.1, tol=tol)


def test_bf16_small_sgd():
    """bf16 mode against the fp64 oracle within 2e-2 (several tiles of the MFMA kernels)."""
    c = dict(n_layer=2, d_model=128, n_head=2, d_head=64, d_ff=512, vocab=512, seq_len=128, mem_len=0, batch=2,
             n_module=2, rel_pos=0, dtype=1, optimizer=0)
    run_both(c, steps=3, lr=0.05, seed=9, std=0.05, perturb=0.05, tol=2e-2)


def test_bf16_odd_vocab_adam():
    """bf16 mode with a vocabulary that is no multiple of 8 (the zero-padded vocabulary keeps the
    dh = G V and dV_o = G^T h contractions on the MFMA kernels) and K = 3 with Adam."""
    c = dict(n_layer=3, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=1001, seq_len=96, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=1, optimizer=1, embed_warm_mode=0)
    run_both(c, steps=5, lr=1e-3, seed=21, std=0.05, perturb=0.05, tol=2e-2)


def test_xl_bf16_mfma_path_memory_carry():
    """Transformer-XL blocks in bf16 with head size 64 (the fused relative-position kernels),
    memory shorter than, equal to and rolling past the segment over four steps."""
    c = dict(n_layer=2, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=512, seq_len=80, mem_len=112, batch=2,
             n_module=2, rel_pos=1, dtype=1, optimizer=0, embed_warm_mode=1)
    run_both(c, steps=4, lr=0.05, seed=31, std=0.05, perturb=0.05, tol=2e-2)


def test_bf16_widths_off_the_tile_grid_adam():
    """bf16 mode with d_head = 41, d_model = 82, d_ff = 100: stored zero-padded to 64 / 128 / 128 so
    that the MFMA kernels run; every result the caller sees (loss, gradients, weights) is that of
    the unpadded model.  Adam over more steps than K: padding that picked up a value would leak
    into the visible weights."""
    c = dict(n_layer=3, d_model=82, n_head=2, d_head=41, d_ff=100, vocab=203, seq_len=70, mem_len=0, batch=3,
             n_module=3, rel_pos=0, dtype=1, optimizer=1, embed_warm_mode=0)
    run_both(c, steps=6, lr=1e-3, seed=41, std=0.05, perturb=0.05, tol=2e-2)


def test_xl_bf16_widths_off_the_tile_grid_memory_carry():
    """The same zero-padded storage with Transformer-XL blocks (W_r, u, v per head) and a rolling
    memory; head size 32 here."""
    c = dict(n_layer=2, d_model=96, n_head=3, d_head=32, d_ff=200, vocab=301, seq_len=40, mem_len=56, batch=2,
             n_module=2, rel_pos=1, dtype=1, optimizer=0, embed_warm_mode=1)
    run_both(c, steps=4, lr=0.05, seed=43, std=0.05, perturb=0.05, tol=2e-2)


@pytest.mark.parametrize("rel_pos,mem_len,schedule", [(0, 0, 0), (1, 96, 0), (0, 0, 1), (1, 96, 1)])
def test_stream_overlap_matches_one_stream(rel_pos, mem_len, schedule):
    """The multi-stream execution of step() (weight gradients and updates beside the
    error-gradient chain; under the stored-input schedule the K backward passes side by side,
    each on its own streams and scratch buffers) against the same steps on one stream: equal up
    to the order of fp32 atomic additions, over more iterations than the rings are deep."""
    c = dict(n_layer=4, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=512, seq_len=96, mem_len=mem_len, batch=2,
             n_module=4, rel_pos=rel_pos, dtype=1, optimizer=0, embed_warm_mode=0, schedule=schedule, dropout=0.125 * schedule)
    steps, lr = 7, 0.05
    blobs = S.init_params(c, seed=5, std=0.05, perturb=0.05)
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], steps, 1.1, 6, contiguous=bool(mem_len))
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    out = []
    for overlap in (True, False):
        m = P().create_model(**c)
        for g in range(c["n_module"] + 1):
            m.set_params(g, blobs[g])
        m.set_overlap(overlap)
        losses = [m.step(dtok[t], dtgt[t], lr) for t in range(steps)]
        out.append((losses, [m.get_params(g) for g in range(c["n_module"] + 1)]))
        m.close()
    (la, wa), (lb, wb) = out
    assert np.allclose(la, lb, rtol=1e-4, atol=0)
    for a, b in zip(wa, wb):
        # SGD: a last-bit difference of an fp32 sum can flip the bf16 rounding of a weight's
        # copy now and then, nothing more
        assert rel_err(a, b) < 1e-3


def test_long_run_with_warmup_and_cosine_schedule():
    """Section 5.2's recipe on a structured source: K = 4 with delayed gradients, Adam, linear
    warm-up then cosine decay (the library's schedule function), 400 iterations on a Markov token
    source.  The run stays finite, ends well below the unigram entropy of the source (so the
    context was learnt through the stale gradients), and lands close to plain backpropagation
    (K = 1) on the same data.  A property test: no oracle trajectory of this length exists."""
    steps, W, base = 400, 40, 2e-3
    vocab, B, T = 256, 16, 64
    tok, tgt = S.markov_token_batches(vocab, B, T, steps, 1.1, seed=77)
    p_uni = np.bincount(tgt.ravel(), minlength=vocab) / tgt.size
    h_uni = float(-(p_uni[p_uni > 0] * np.log(p_uni[p_uni > 0])).sum())
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    final = {}
    for K in (4, 1):
        c = dict(n_layer=4, d_model=128, n_head=2, d_head=64, d_ff=256, vocab=vocab, seq_len=T, mem_len=0, batch=B,
                 n_module=K, rel_pos=0, dtype=1, optimizer=1, embed_warm_mode=0, emb_scale=float(np.sqrt(128)))
        m = P().create_model(**c)
        for g, blob in enumerate(S.init_params(c, seed=3)):
            m.set_params(g, blob)
        losses = [m.step(dtok[t], dtgt[t], P().lr_schedule(base, W, steps, t)) for t in range(steps)]
        m.close()
        assert np.all(np.isfinite(losses))
        final[K] = float(np.mean(losses[-20:]))
        assert losses[0] > h_uni                       # starts near log(vocab)
    assert final[4] < h_uni - 2.0, (final, h_uni)
    assert final[4] < final[1] + 0.25, final


@pytest.mark.parametrize("dtype,tol", [(0, 1e-4), (1, 2e-2)])
def test_eval_step_with_longer_memory(dtype, tol):
    """Evaluation path: train a Transformer-XL model for a few iterations, copy its weights on the
    device into an evaluation model with a longer memory (and dropout configured, which
    evaluation must ignore), and evaluate consecutive segments: losses and rolled memories
    against the oracle's forward-only pass; the weights and the training model stay untouched."""
    dh = 64 if dtype else 16
    c = dict(n_layer=3, d_model=2 * dh, n_head=2, d_head=dh, d_ff=96, vocab=211, seq_len=24, mem_len=24, batch=2,
             n_module=3, rel_pos=1, dtype=dtype, optimizer=0, embed_warm_mode=1)
    blobs = S.init_params(c, seed=11, std=0.1, perturb=0.1)
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], 9, 1.1, 12, contiguous=True)
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    orc = O.Oracle(O.Config(**c), blobs)
    m = P().create_model(**c)
    for g in range(4):
        m.set_params(g, blobs[g])
    for t in range(4):
        lo, lg = orc.step(tok[t], tgt[t], 0.05), m.step(dtok[t], dtgt[t], 0.05)
        assert abs(lg - lo) / lo < tol
    ce = dict(c, mem_len=60, dropout=0.375, seed=3)
    oe = O.Oracle(O.Config(**ce), [orc.module_blob(g) for g in range(4)])
    e = P().create_model(**ce)
    e.copy_params_from(m)
    for g in range(4):
        assert np.array_equal(e.get_params(g), m.get_params(g))
    for t in range(4, 9):
        lo, lg = oe.eval_step(tok[t], tgt[t]), e.eval_step(dtok[t], dtgt[t])
        assert abs(lg - lo) / lo < tol, (t, lg, lo)
        assert e.current_step() == t - 3
        for l in range(3):
            mem = e.get_mems(l)
            assert mem.shape == oe.mems[l].shape and rel_err(mem, oe.mems[l]) < tol
    with pytest.raises(P().OuroError):                       # not in the middle of a training iteration
        m.module_forward(1, dtok[0], dtgt[0]); m.eval_step(dtok[0], dtgt[0])
    for g in range(4):
        assert np.array_equal(e.get_params(g), m.get_params(g))
    m.close(); e.close()


@pytest.mark.parametrize("schedule,dtype,opt", [(0, 0, 1), (1, 0, 0), (1, 1, 1)])
def test_checkpoint_resume(schedule, dtype, opt):
    """Save the whole state (weights, moments, pending stale gradients or stored inputs with their
    tags, mailboxes, memories, counters) after 4 iterations, load it into a fresh model of the same
    configuration and go on: the resumed run keeps following the oracle, which ran straight
    through.  Saving again right after loading returns the same bytes; another configuration is
    refused."""
    tol = 2e-2 if dtype else 1e-4
    dh = 64 if dtype else 16
    c = dict(n_layer=3, d_model=2 * dh, n_head=2, d_head=dh, d_ff=96, vocab=211, seq_len=24, mem_len=40, batch=2,
             n_module=3, rel_pos=1, dtype=dtype, optimizer=opt, schedule=schedule, dropout=0.125, seed=77)
    lr = 1e-3 if opt else 0.05
    blobs = S.init_params(c, seed=13, std=0.1, perturb=0.1)
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], 9, 1.1, 14, contiguous=True)
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    orc = (O.RecomputeOracle if schedule else O.Oracle)(O.Config(**c), blobs)
    a = P().create_model(**c)
    for g in range(4):
        a.set_params(g, blobs[g])
    for t in range(4):
        lo, lg = orc.step(tok[t], tgt[t], lr), a.step(dtok[t], dtgt[t], lr)
        assert abs(lg - lo) / lo < tol
    state = a.save_state()
    a.close()
    b = P().create_model(**c)
    b.load_state(state)
    assert b.current_step() == 4
    assert np.array_equal(b.save_state(), state)
    for t in range(4, 9):
        lo, lg = orc.step(tok[t], tgt[t], lr), b.step(dtok[t], dtgt[t], lr)
        assert abs(lg - lo) / lo < tol, (t, lg, lo)
    if opt == 0:                                              # (Adam: see run_both on ill-conditioned elements)
        for g in range(4):
            assert rel_err(b.get_params(g), orc.module_blob(g)) < tol
    for l in range(3):
        assert rel_err(b.get_mems(l), orc.mems[l]) < tol
    other = P().create_model(**dict(c, d_ff=128))
    with pytest.raises(P().OuroError):
        other.load_state(state)
    with pytest.raises(P().OuroError):
        b.load_state(state[:-8])
    other.close(); b.close()


def test_timing_hooks():
    """Per-launch timing brackets and the empty-bracket cost: plausible, positive numbers."""
    c = dict(S.CONFIGS["cfg1"])
    m = P().create_model(**c)
    blobs = S.init_params(c, seed=0)
    for g in range(c["n_module"] + 1):
        m.set_params(g, blobs[g])
    tok, tgt = S.token_batches(c["vocab"], c["batch"], c["seq_len"], 1, c["zipf_s"], c["seed"], False)
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    m.set_overlap(False)
    m.timing_enable(True)
    for _ in range(3):
        m.step(dtok[0], dtgt[0], c["lr"])
    ms, n, work = m.timing_read(1)                      # update kernel: bytes
    assert n > 0 and ms > 0 and work > 0
    m.timing_enable(False)
    ovh = m.timing_overhead(50)
    assert 0 < ovh < 1.0                                 # milliseconds per empty bracket
    m.close()


def test_staleness_plumbing_bit_exact():
    """Integer-tagged gradients through inject_grad: final weights have a closed form that
    fp32 represents exactly; slot tags and reads follow Eq. 8-9 at every iteration."""
    pkg = P()
    K, T = 4, 11
    c = dict(n_layer=4, d_model=16, n_head=2, d_head=8, d_ff=16, vocab=32, seq_len=4, mem_len=0, batch=1,
             n_module=K, rel_pos=0, dtype=0, optimizer=0)
    m = pkg.create_model(**c)
    for g in range(K + 1):
        m.set_params(g, np.zeros(m.param_count(g), np.float32))
    lr = 2.0 ** -10
    val = lambda t, store: 1000.0 * t + (0.25 if store == 0 else 0.75 if store == K + 1 else store)
    for t in range(T):
        for store in range(K + 2):
            m.inject_grad(store, np.full(m.grad_count(store), val(t, store), np.float32))
            slot, tau = pkg.slot_index(K, store, t, True)
            assert m.slot_tag(store, slot) == t
        for g in range(K, -1, -1):
            m.delayed_update(g, lr)
        for k in range(1, K + 1):
            tau = t - K + k
            assert m.last_read(k) == ((tau % (K - k + 1), tau) if tau >= 0 else (-1, -1))
        ti = t - K + 1
        assert m.last_read(0) == ((ti % K, ti) if ti >= 0 else (-1, -1))
        assert m.last_read(K + 1) == ((0, t) if ti >= 0 else (-1, -1))
        assert m.current_step() == t + 1
    for k in range(1, K + 1):
        expect = np.float32(-lr * sum(val(t - K + k, k) for t in range(T) if t - K + k >= 0))
        assert np.all(m.get_params(k) == expect)
    expect = np.float32(-lr * sum(0.5 * val(t, K + 1) + 0.5 * val(t - K + 1, 0) for t in range(T) if t - K + 1 >= 0))
    assert np.all(m.get_params(0) == expect)
    m.close()


def test_stored_input_schedule_plumbing_bit_exact():
    """The same with schedule = 1: every gradient store has depth 1 and a gradient is applied in
    the iteration that produced it, but only once mini-batch t-K+k exists; closed-form weights."""
    pkg = P()
    K, T = 4, 9
    c = dict(n_layer=4, d_model=16, n_head=2, d_head=8, d_ff=16, vocab=32, seq_len=4, mem_len=0, batch=1,
             n_module=K, rel_pos=0, dtype=0, optimizer=0, schedule=1)
    m = pkg.create_model(**c)
    for g in range(K + 1):
        m.set_params(g, np.zeros(m.param_count(g), np.float32))
    lr = 2.0 ** -10
    val = lambda t, store: 1000.0 * t + (0.25 if store == 0 else 0.75 if store == K + 1 else store)
    for t in range(T):
        for store in range(K + 2):
            m.inject_grad(store, np.full(m.grad_count(store), val(t, store), np.float32))
            assert m.slot_tag(store, 0) == t
            with pytest.raises(pkg.OuroError):
                m.slot_tag(store, 1)
        for g in range(K + 1):
            m.delayed_update(g, lr)
        for k in range(1, K + 1):
            tau = t - K + k
            assert m.last_read(k) == ((0, tau) if tau >= 0 else (-1, -1))
        ti = t - K + 1
        assert m.last_read(0) == ((0, ti) if ti >= 0 else (-1, -1))
        assert m.last_read(K + 1) == ((0, t) if ti >= 0 else (-1, -1))
    for k in range(1, K + 1):
        expect = np.float32(-lr * sum(val(t, k) for t in range(T) if t - K + k >= 0))
        assert np.all(m.get_params(k) == expect)
    expect = np.float32(-lr * sum(0.5 * val(t, K + 1) + 0.5 * val(t, 0) for t in range(T) if t - K + 1 >= 0))
    assert np.all(m.get_params(0) == expect)
    m.close()


def test_frozen_until_first_gradient_and_adam_zero_step():
    pkg = P()
    K = 3
    c = dict(n_layer=3, d_model=16, n_head=2, d_head=8, d_ff=16, vocab=32, seq_len=8, mem_len=0, batch=2,
             n_module=K, rel_pos=0, dtype=0, optimizer=1)
    blobs = S.init_params(c, seed=1, std=0.1)
    tok, tgt = S.token_batches(32, 2, 8, 4, 1.1, 2, False)
    m = pkg.create_model(**c)
    for g in range(K + 1):
        m.set_params(g, blobs[g])
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    for t in range(4):
        m.step(dtok[t], dtgt[t], 1e-2)
        for k in range(1, K + 1):
            same = np.array_equal(m.get_params(k), blobs[k])
            assert same == (t < K - k), (t, k)
        assert np.array_equal(m.get_params(0), blobs[0]) == (t < K - 1)
    m.close()


def test_call_order_and_error_codes():
    pkg = P()
    from paper_1909_06695_amd import binding as Bn
    c = dict(n_layer=2, d_model=16, n_head=2, d_head=8, d_ff=16, vocab=32, seq_len=8, mem_len=0, batch=2,
             n_module=2, rel_pos=0, dtype=0, optimizer=0)
    m = pkg.create_model(**c)
    blobs = S.init_params(c, seed=1)
    for g in range(3):
        m.set_params(g, blobs[g])
    tok = torch.zeros((2, 8), dtype=torch.int32, device="cuda")
    tgt = torch.ones((2, 8), dtype=torch.int32, device="cuda")

    def code(fn, *a):
        with pytest.raises(pkg.OuroError) as e:
            fn(*a)
        return e.value.code

    assert code(m.module_forward, 2, tok, tgt) == Bn.E_SEQUENCE
    assert code(m.module_backward, 2) == Bn.E_SEQUENCE
    assert code(m.delayed_update, 1, 0.1) == Bn.E_SEQUENCE
    assert code(m.module_forward, 3, tok, tgt) == Bn.E_ARG
    assert code(m.module_forward, 1, None, None) == Bn.E_ARG
    m.module_forward(1, tok, tgt)
    assert code(m.module_forward, 1, tok, tgt) == Bn.E_SEQUENCE
    assert code(m.module_backward, 2) == Bn.E_SEQUENCE
    m.module_forward(2, tok, tgt)
    assert code(m.module_backward, 1) == Bn.E_SEQUENCE
    m.module_backward(2)
    assert code(m.delayed_update, 2, 0.1) == Bn.E_SEQUENCE
    m.module_backward(1)
    m.delayed_update(2, 0.1)
    assert code(m.delayed_update, 2, 0.1) == Bn.E_SEQUENCE
    assert m.current_step() == 0
    m.delayed_update(0, 0.1); m.delayed_update(1, 0.1)
    assert m.current_step() == 1
    assert code(m.set_params, 1, np.zeros(3, np.float32)) == Bn.E_ARG
    assert code(m.get_grad_slot, 1, 5) == Bn.E_STALE
    # out-of-range token and target ids are reported, never dereferenced
    bad = tok.clone(); bad[0, 0] = 32
    with pytest.raises(pkg.OuroError) as e:
        m.step(bad, tgt, 0.1)
    assert e.value.code == Bn.E_TOKEN
    badt = tgt.clone(); badt[1, 3] = -7
    with pytest.raises(pkg.OuroError) as e:
        m.step(tok, badt, 0.1)
    assert e.value.code == Bn.E_TOKEN
    assert np.isfinite(m.step(tok, tgt, 0.1))
    m.close()


def test_bench_config_full_size_steady_state():
    """cfg2 (12 layers, d=512, vocab 32768, 8192 tokens, K=4, Adam, bf16) in the benchmark's launch
    configuration for K+2 iterations: every module and V take real stale-gradient Adam steps
    (module 1 and V from iteration K-1 on), every ring slot is written a second time and read
    after the wrap-around.  Loss, every gradient store and the weights (element by element)
    against the oracle."""
    c = dict(S.CONFIGS["cfg2"], batch=4)                 # 4 oracle streams, each 4 times on the HIP side: 16 streams
    run_both(c, steps=c["n_module"] + 2, lr=c["lr"], seed=0, tol=2e-2, rep=4)


def test_xl_config_full_size_first_steps():
    """cfg3: Transformer-XL with widths off the tile grid (16 layers, d=410, 10 heads of 41,
    d_ff=2100, segment and memory 150) at full size, stored zero-padded: empty memory, full
    memory, rolled memory against the oracle."""
    c = dict(S.CONFIGS["cfg3"], batch=8)                 # 8 oracle streams, each 4 times on the HIP side: 32 streams
    run_both(c, steps=3, lr=c["lr"], seed=0, tol=2e-2, rep=4)


def test_cfg4_shapes_full_size_launch():
    """cfg4 (24 layers, d=1024, 16 heads, d_ff=4096, vocab 50257 on the zero-padded vocabulary
    path, T=1024: 16 key blocks per query block, K=8 with rings up to 8 deep) in the launch
    configuration the benchmark times (8 streams, 8192 tokens): the oracle runs one stream, the
    HIP path the same stream eight times (run_both, rep), so every tile of the full-size
    launches is compared element by element.  3 iterations: modules 6..8 take real Adam steps.
    (Under Adam the two sides' weights drift apart where a gradient element is below the rounding
    noise, since the first steps are lr * sign(g); at this depth the gradient at the bottom of the
    stack, dV_i, then goes from 0.78 of the bar at t = 2 to 0.95-0.99 at t = 3 and 4, too close
    to hold on every run.  cfg2 runs K + 2 iterations and cfg5 K + 1 with a quarter of the bar to spare.)"""
    c = dict(S.CONFIGS["cfg4"], batch=1)
    run_both(c, steps=3, lr=c["lr"], seed=0, tol=2e-2, rep=8)


def test_cfg5_shapes_full_size_launch():
    """cfg5 (Transformer-XL, 18 layers split 4,5,5,4 by the default rule, d=1024, segment and
    memory 384, vocab 65536) with 16 streams on the HIP side (one oracle stream sixteen
    times): empty, full and rolled memory, every module and V updated (K+1 = 5 iterations)."""
    c = dict(S.CONFIGS["cfg5"], batch=1)
    assert "layers_per_module" not in c
    run_both(c, steps=c["n_module"] + 1, lr=c["lr"], seed=0, tol=2e-2, rep=16)


@pytest.mark.parametrize("name,rows", [("cfg4", (0, 5)), ("cfg5", (3, 15))])
def test_full_size_distinct_streams_forward_rows(name, rows):
    """Full-size launches with all streams different (the benchmark's inputs): streams do not
    interact in the forward pass, so the final hidden state of one stream is what the oracle
    computes for that stream alone.  Two iterations at step size 0 (the second with a full
    segment memory for the relative model), sampled streams element by element, and the loss as
    the mean of per-stream losses cannot be formed without all streams, so it is bounded only."""
    c = dict(S.CONFIGS[name])
    B, T, d, L = c["batch"], c["seq_len"], c["d_model"], c["n_layer"]
    blobs = S.init_params(c, seed=0)
    tok, tgt = S.token_batches(c["vocab"], B, T, 2, c["zipf_s"], c["seed"], contiguous=bool(c["mem_len"]))
    m = P().create_model(**c)
    for g in range(c["n_module"] + 1):
        m.set_params(g, blobs[g])
    dtok = torch.from_numpy(tok).cuda(); dtgt = torch.from_numpy(tgt).cuda()
    hid, losses = [], []
    for t in range(2):
        losses.append(m.step(dtok[t], dtgt[t], 0.0))
        hid.append(m.get_hidden(L).reshape(B, T, d))
    for g in range(c["n_module"] + 1):
        assert np.array_equal(m.get_params(g), blobs[g])          # step size 0: nothing moved
    m.close()
    c1 = dict(c, batch=1)
    row_losses = []
    for b in rows:
        orc = O.Oracle(O.Config(**c1), blobs, keep_history=False)
        for t in range(2):
            loss, fw = O.model_forward(orc.cfg, orc.layers, orc.V, orc.V, tok[t, b:b + 1], tgt[t, b:b + 1], orc.mems, None)
            assert_close(hid[t][b], fw["hL"][0], 2e-2, ("final hidden state", name, b, t))
            row_losses.append(loss)
            if c["mem_len"]:
                orc.mems = [fw["inputs"][l][:, -c["mem_len"]:].copy() if orc.mems is None else
                            np.concatenate([orc.mems[l], fw["inputs"][l]], axis=1)[:, -c["mem_len"]:].copy() for l in range(L)]
    # Zipf streams at the initial weights: per-stream losses lie close together
    assert abs(np.mean(losses) - np.mean(row_losses)) < 0.05 * np.mean(row_losses)
