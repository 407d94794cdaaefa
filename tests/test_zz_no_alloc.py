"""The attention backward entry point that allocates nothing (workspace inside the library)
against the entry point that takes the caller's workspace: same inputs, same outputs, on two
calls in a row, the second with a smaller input (the shared workspace keeps the first call's
contents), and a size beyond the built-in workspace is refused."""
import ctypes as C
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def L():
    import paper_1909_06695_amd as P
    return P.lib()


def p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _case(dtype, B, H, T, Mv, dh, rel, seed):
    """Returns (outputs of the workspace entry point, outputs of the no-allocation one)."""
    lib = L()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(seed)
    S, d = Mv + T, H * dh
    tdt = torch.bfloat16 if dtype else torch.float32
    mk = lambda shape, s=1.0: torch.from_numpy((rng.standard_normal(shape) * s).astype(np.float32)).cuda().to(tdt).contiguous()
    q, kv, do, u, vb, r = mk((B * T, d)), mk((B * S, 2 * d)), mk((B * T, d)), mk((H, dh), 0.5), mk((H, dh), 0.5), mk((S, d))
    o = torch.zeros((B * T, d), dtype=tdt, device="cuda")
    lse = torch.zeros((B, H, T), dtype=torch.float32, device="cuda")
    scale = 1.0 / math.sqrt(dh)
    kp = C.c_void_p(kv.data_ptr()); vp = C.c_void_p(kv.data_ptr() + d * kv.element_size())
    assert lib.ouro_op_attention_fwd(st, dtype, B, H, T, S, dh, Mv, scale, p(q), d, kp, 2 * d, vp, 2 * d, p(o), d, p(lse),
                                     rel, p(u), p(vb), p(r), d, 0) == 0
    outs = []
    for noalloc in (False, True):
        gq = torch.full((B * T, d), 3.0, dtype=tdt, device="cuda")
        gkv = torch.full((B * S, 2 * d), 3.0, dtype=tdt, device="cuda")
        gu = torch.full((H, dh), 3.0, dtype=torch.float32, device="cuda")
        gvb = torch.full((H, dh), 3.0, dtype=torch.float32, device="cuda")
        gr = torch.full((S, d), 3.0, dtype=torch.float32, device="cuda")
        gk = C.c_void_p(gkv.data_ptr()); gv = C.c_void_p(gkv.data_ptr() + d * gkv.element_size())
        head = (st, dtype, B, H, T, S, dh, Mv, scale, p(q), d, kp, 2 * d, vp, 2 * d, p(o), d, p(lse), p(do), d, p(gq), d,
                gk, 2 * d, gv, 2 * d, rel, p(u), p(vb), p(r), d, p(gu), p(gvb), p(gr))
        if noalloc:
            rc = lib.ouro_op_attention_bwd_noalloc(*head, 0)
        else:
            scr = torch.full((max(lib.ouro_op_attention_bwd_scratch(B, H, T, S, dh), 1),), 7.0, dtype=torch.float32, device="cuda")
            rc = lib.ouro_op_attention_bwd(*head, p(scr), 0)
        assert rc == 0, lib.ouro_last_error()
        torch.cuda.synchronize()
        res = [gq.float().cpu().numpy(), gkv.float().cpu().numpy()]
        if rel:
            res += [gu.cpu().numpy(), gvb.cpu().numpy(), gr.cpu().numpy()]
        outs.append(res)
    return outs


def _same(a, b, exact):
    for x, y in zip(a, b):
        assert np.all(np.isfinite(x)) and np.all(np.isfinite(y))
        if exact:
            assert np.array_equal(x, y)
        else:                       # kernels that add with fp32 atomics: equal up to the order of the additions
            x = x.astype(np.float64); y = y.astype(np.float64)
            assert np.linalg.norm(x - y) <= 1e-4 * max(np.linalg.norm(y), 1e-30)
            assert np.max(np.abs(x - y)) <= 1e-3 * (np.abs(y).max() + 1e-30)


@pytest.mark.parametrize("dtype,dh,rel,big,small", [
    (1, 64, 0, (2, 3, 200, 0), (1, 2, 70, 0)),        # fused MFMA kernels (no atomics: bit-equal)
    (1, 64, 1, (2, 2, 150, 150), (1, 2, 96, 40)),     # relative-position MFMA kernels (atomic adds into dr)
    (0, 16, 1, (2, 2, 24, 17), (1, 1, 5, 0)),         # general kernels, fp32
])
def test_no_alloc_entry_matches_workspace_entry(dtype, dh, rel, big, small):
    for (B, H, T, Mv), seed in ((big, 1), (small, 2)):          # two calls in a row, the second smaller
        ref, got = _case(dtype, B, H, T, Mv, dh, rel, seed)
        _same(got, ref, exact=(rel == 0))


def test_no_alloc_entry_refuses_sizes_beyond_its_workspace():
    lib = L()
    B, H, T, dh = 64, 16, 4096, 64
    assert lib.ouro_op_attention_bwd_scratch(B, H, T, T, dh) > 4 << 20
    one = torch.zeros(8, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.ouro_op_attention_bwd_noalloc(st, 1, B, H, T, T, dh, 0, 0.125, p(one), 64, p(one), 64, p(one), 64, p(one), 64,
                                           p(one), p(one), 64, p(one), 64, p(one), 64, p(one), 64, 0, None, None, None, 0,
                                           None, None, None, 0)
    assert rc == -2                                             # OURO_E_ARG, before anything is enqueued
    assert b"workspace" in lib.ouro_last_error()
    torch.cuda.synchronize()
