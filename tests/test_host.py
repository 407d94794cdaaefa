"""Host-only checks of the HIP library: it loads, exports every symbol the headers
declare, and its pure-integer staleness functions follow Eq. 8-9 (brute force)."""
import ctypes
import os
import re

import pytest

import paper_1909_06695_amd as P
from paper_1909_06695_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in ("ouro.h", "ouro_ops.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ouro_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = P.lib()
    decl = declared_symbols()
    assert len(decl) >= 30
    for name in decl:
        assert hasattr(L, name), name
    assert decl == set(P.exported_symbols())        # the binding covers the whole boundary


def test_ring_depths():
    for K in range(1, 9):
        assert P.ring_depth(K, 0) == K
        assert P.ring_depth(K, K + 1) == 1
        for k in range(1, K + 1):
            assert P.ring_depth(K, k) == K - k + 1
    with pytest.raises(P.OuroError):
        P.ring_depth(3, 5)


@pytest.mark.parametrize("K", [1, 2, 3, 4, 8])
def test_slot_index_against_brute_force(K):
    """Simulate the rings literally: a slot read at iteration t must still hold the
    gradient of iteration t-K+k (Eq. 8) / t-K+1 (Eq. 9), i.e. no later write has landed on
    it, and a zero gradient is prescribed exactly while that index is negative."""
    stores = {i: [None] * P.ring_depth(K, i) for i in range(K + 2)}
    for t in range(3 * K + 5):
        for i in range(K + 2):                       # backward of iteration t writes
            slot, tau = P.slot_index(K, i, t, True)
            assert tau == t and 0 <= slot < len(stores[i])
            stores[i][slot] = t
        for i in range(K + 2):                       # updates of iteration t read
            slot, tau = P.slot_index(K, i, t, False)
            want = t if i == K + 1 else (t - K + 1 if i == 0 else t - K + i)
            if want < 0:
                assert (slot, tau) == (-1, -1)
            else:
                assert tau == want and stores[i][slot] == want, (K, i, t)


def test_config_validation_is_host_side():
    good = dict(n_layer=2, d_model=64, n_head=2, d_head=32, d_ff=256, vocab=256, seq_len=32, batch=4, n_module=2)
    assert P.query_arena_bytes(P.make_config(**good)) > 0
    bad = [dict(n_head=3), dict(d_model=63, n_head=1, d_head=63), dict(n_module=3), dict(n_module=0),
           dict(mem_len=4), dict(dtype=2), dict(optimizer=5), dict(layers_per_module=[2, 1]),
           dict(layers_per_module=[2, 0]), dict(vocab=1), dict(rel_pos=2), dict(schedule=2), dict(schedule=-1),
           dict(dropout=1.0), dict(dropout=-0.1), dict(dropout=float("nan"))]
    for b in bad:
        kw = dict(good); kw.update(b)
        with pytest.raises(P.OuroError) as e:
            P.query_arena_bytes(P.make_config(**kw))
        assert e.value.code == binding.E_CONFIG, b
    # bf16 + Adam needs more arena than fp32 + SGD of the same shape? (shadow + moments vs half-size activations)
    a = P.query_arena_bytes(P.make_config(**good))
    b = P.query_arena_bytes(P.make_config(**dict(good, optimizer=1)))
    assert b > a
    # the stored-input schedule keeps module inputs instead of rings of gradients: for a deep
    # pipeline of wide layers that is the smaller arena (the point of the memory paragraph)
    big = dict(n_layer=8, d_model=256, n_head=4, d_head=64, d_ff=1024, vocab=512, seq_len=64, batch=2, n_module=8, dtype=1, optimizer=1)
    assert P.query_arena_bytes(P.make_config(**dict(big, schedule=1))) < P.query_arena_bytes(P.make_config(**big))


def test_create_model_rejects_bad_arena_without_touching_it():
    cfg = P.make_config(n_layer=1, d_model=8, n_head=2, d_head=4, d_ff=8, vocab=8, seq_len=4, batch=1)
    h = ctypes.c_void_p()
    rc = P.lib().ouro_create_model(ctypes.byref(cfg), None, 0, None, ctypes.byref(h))
    assert rc == binding.E_ARENA and not h.value
    rc = P.lib().ouro_create_model(ctypes.byref(cfg), ctypes.c_void_p(256), 16, None, ctypes.byref(h))
    assert rc == binding.E_ARENA and not h.value


def test_lr_schedule_matches_the_oracle():
    """The library's host-side step-size function against the oracle's, over both phases and
    the boundaries (both fp64: agreement to rounding); bad arguments are refused."""
    from oracle import ouro_oracle as O
    for base, W, T, floor in [(2.5e-4, 5000, 200000, 0.0), (1e-3, 0, 1000, 1e-5), (0.1, 50, 51, 0.0), (3e-4, 500, 40000, 3e-6)]:
        for t in sorted({0, 1, W - 1 if W else 0, W, W + 1, (W + T) // 2, T - 1, T, T + 7, 12345 % (T + 1)}):
            got, ref = P.lr_schedule(base, W, T, t, floor), O.learning_rate(t, base, W, T, floor)
            assert abs(got - ref) <= 1e-15 + 1e-13 * abs(ref), (base, W, T, floor, t)
    for bad in [(1.0, 10, 10, 0, 0.0), (1.0, -1, 10, 0, 0.0), (1.0, 2, 10, -1, 0.0), (1.0, 2, 10, 0, 2.0), (1.0, 2, 10, 0, -0.1)]:
        with pytest.raises(P.OuroError):
            P.lr_schedule(bad[0], bad[1], bad[2], bad[3], bad[4])
