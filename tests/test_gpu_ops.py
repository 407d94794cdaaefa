"""Per-kernel parity: each HIP kernel, called through the C boundary, against the CPU
oracle's function for the same operation on the same seeded inputs."""
import ctypes as C
import math

import numpy as np
import pytest

from oracle import ouro_oracle as O

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def L():
    import paper_1909_06695_amd as P
    return P.lib()


def stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def dev(a, dtype):
    """numpy -> device tensor of the op's element type (dtype 0 fp32, 1 bf16)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == 1 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def rel_err(a, b):
    # the floor keeps exactly-zero references (a single visible key has zero score gradient)
    # from turning rounding noise into an infinite ratio
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-2 * math.sqrt(b.size)))


def ok(rc):
    assert rc == 0, L().ouro_last_error()


TOL = {0: 2e-5, 1: 1e-2}


# ------------------------------------------------------------------------------- GEMM
# force: 0 automatic, 1 plain kernel, 10..14 one MFMA tile configuration each
@pytest.mark.parametrize("dtype,force", [(0, 0), (1, 1), (1, 0), (1, 10), (1, 11), (1, 12), (1, 13), (1, 14)])
@pytest.mark.parametrize("tA,tB", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(200, 136, 328), (128, 256, 64), (72, 40, 1000), (384, 520, 96), (136, 264, 512),
                                   (392, 136, 192), (520, 392, 1024)])
def test_gemm_forms(dtype, force, tA, tB, M, N, K):
    rng = np.random.default_rng(M + 7 * N + 13 * K + tA * 2 + tB)
    A = rng.standard_normal((K, M) if tA else (M, K)).astype(np.float32)
    B = rng.standard_normal((N, K) if tB else (K, N)).astype(np.float32)
    dA, dB = dev(A, dtype), dev(B, dtype)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    ok(L().ouro_op_gemm(stream(), dtype, tA, tB, M, N, K, 1.0, p(dA), dA.shape[1], p(dB), dB.shape[1], p(out), N,
                        1, 0, None, None, 0, 0, None, 0, force))
    torch.cuda.synchronize()
    a64, b64 = host(dA), host(dB)
    ref = (a64.T if tA else a64) @ (b64.T if tB else b64)
    assert rel_err(host(out), ref) < 2e-6
    if dtype == 1 and force != 1:
        assert L().ouro_op_gemm_uses_mfma(dtype, tA, tB, M, N, K, p(dA), dA.shape[1], p(dB), dB.shape[1]) == 1


def test_gemm_row_tail():
    """A product on 256x256 tiles whose tile rows end a little past a full round of workgroups:
    the rows of the last partial round come from a second, split-K launch.  Rows on both sides
    of the seam and the last rows against fp64."""
    M, N, K = 16384 + 520, 1024, 4096
    rng = np.random.default_rng(77)
    dA = dev(rng.standard_normal((K, M)).astype(np.float32), 1)
    dB = dev(rng.standard_normal((K, N)).astype(np.float32), 1)
    out = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
    ok(L().ouro_op_gemm(stream(), 1, 1, 0, M, N, K, 1.0, p(dA), M, p(dB), N, p(out), N, 1, 0, None, None, 0, 0, None, 0, 0))
    torch.cuda.synchronize()
    rows = np.r_[0:4, 8190:8194, 16376:16392, 16640:16644, M - 9:M]
    a64, b64 = host(dA), host(dB)
    ref = a64[:, rows].T @ b64
    assert rel_err(host(out)[rows], ref) < 2e-6


@pytest.mark.parametrize("dtype,tA,tB,M,N,K,by,bz,second,acc", [
    (1, 0, 0, 200, 64, 128, 3, 2, True, 0),      # one launch of the MFMA kernel over the grid, two grids, ragged M
    (1, 0, 1, 136, 72, 192, 2, 1, False, 0),
    (1, 1, 0, 128, 64, 2048, 3, 1, False, 1),    # split K with atomic adds inside a grid of products
    (1, 0, 0, 20, 64, 64, 2, 2, True, 0),        # fewer rows than an MFMA tile: one launch per product
    (1, 0, 0, 72, 40, 40, 2, 3, False, 0),       # K off the tile grid: one launch per product
    (1, 0, 1, 200, 136, 256, 3, 2, False, 2),    # added to C in the epilogue, one launch
    (1, 0, 1, 72, 40, 40, 2, 1, False, 2),       # ... one launch per product
    (0, 0, 1, 33, 17, 29, 2, 2, False, 2),       # ... fp32
    (0, 0, 1, 33, 17, 29, 2, 2, True, 0)])       # fp32
def test_gemm_batched(dtype, tA, tB, M, N, K, by, bz, second, acc):
    """Grids of equal products (operands laid out back to back, batch y fastest), optionally two
    grids in one call, against the fp64 product of the rounded operands."""
    rng = np.random.default_rng(1000 * M + 10 * K + by + bz)
    nb = by * bz
    shA, shB = ((K, M) if tA else (M, K)), ((N, K) if tB else (K, N))
    grids = 2 if second else 1
    A = rng.standard_normal((grids, nb) + shA).astype(np.float32)
    B = rng.standard_normal((grids, nb) + shB).astype(np.float32)
    dA, dB = dev(A, dtype), dev(B, dtype)
    init = rng.standard_normal((grids, nb, M, N)).astype(np.float32) if acc else np.zeros((grids, nb, M, N), np.float32)
    out = torch.from_numpy(init.copy()).cuda()
    nA, nB, nC = shA[0] * shA[1], shB[0] * shB[1], M * N
    at = lambda t, g: C.c_void_p(t.data_ptr() + g * nb * (t.numel() // (grids * nb)) * t.element_size())
    ok(L().ouro_op_gemm_batched(stream(), dtype, tA, tB, M, N, K, 0.5, at(dA, 0), shA[1], at(dB, 0), shB[1], at(out, 0), N,
                                1, acc, by, bz, nA, by * nA, nB, by * nB, nC, by * nC,
                                at(dA, 1) if second else None, at(dB, 1) if second else None, at(out, 1) if second else None, -2.0, 0))
    torch.cuda.synchronize()
    a64, b64, got = host(dA), host(dB), host(out)
    for g in range(grids):
        alpha = -2.0 if g else 0.5
        for i in range(nb):
            a, b = a64[g, i], b64[g, i]
            ref = init[g, i] + alpha * ((a.T if tA else a) @ (b.T if tB else b))
            assert rel_err(got[g, i], ref) < 2e-6, (g, i)


@pytest.mark.parametrize("dtype,shapes", [
    (1, [(256, 128, 2048), (128, 384, 2048), (136, 72, 1024), (128, 128, 512)]),     # all in one launch, ragged tiles
    (1, [(256, 128, 1024), (72, 40, 1000), (128, 256, 4096), (64, 64, 320)]),        # two of them go by themselves
    (1, [(128, 128, 1024)]),
    (0, [(33, 17, 29), (40, 24, 64)])])                                              # fp32: one by one
def test_gemm_group(dtype, shapes):
    """Several accumulating products C_i += alpha A_i^T B_i in one call against fp64."""
    rng = np.random.default_rng(sum(m + n + k for m, n, k in shapes))
    n = len(shapes)
    dA = [dev(rng.standard_normal((k, m)).astype(np.float32), dtype) for m, nn, k in shapes]
    dB = [dev(rng.standard_normal((k, nn)).astype(np.float32), dtype) for m, nn, k in shapes]
    init = [rng.standard_normal((m, nn)).astype(np.float32) for m, nn, k in shapes]
    out = [torch.from_numpy(x.copy()).cuda() for x in init]
    ia = lambda v: (C.c_int * n)(*v)
    pa = lambda ts: (C.c_void_p * n)(*[t.data_ptr() for t in ts])
    ok(L().ouro_op_gemm_group(stream(), dtype, n, ia([s[0] for s in shapes]), ia([s[1] for s in shapes]), ia([s[2] for s in shapes]),
                              pa(dA), ia([s[0] for s in shapes]), pa(dB), ia([s[1] for s in shapes]), pa(out), ia([s[1] for s in shapes]), 0.25))
    torch.cuda.synchronize()
    for i in range(n):
        ref = init[i] + 0.25 * (host(dA[i]).T @ host(dB[i]))
        assert rel_err(host(out[i]), ref) < 2e-6, i


@pytest.mark.parametrize("dtype,force", [(0, 0), (1, 0), (1, 10), (1, 11), (1, 12), (1, 13), (1, 14)])
def test_gemm_epilogues_and_strides(dtype, force):
    rng = np.random.default_rng(5)
    M, N, K = 264, 200, 136
    lda, ldb, ldc = K + 8, N + 16, N + 24
    A = rng.standard_normal((M, lda)).astype(np.float32)
    B = (rng.standard_normal((K, ldb)) * 0.2).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    R = rng.standard_normal((M, N)).astype(np.float32)
    dA, dB, dR = dev(A, dtype), dev(B, dtype), dev(R, dtype)
    dbias = torch.from_numpy(bias).cuda()
    tdt = torch.bfloat16 if dtype else torch.float32
    out = torch.zeros((M, ldc), dtype=tdt, device="cuda")
    Z = torch.zeros((M, N), dtype=tdt, device="cuda")
    a64, b64 = host(dA)[:, :K], host(dB)[:, :N]
    pre = a64 @ b64 + bias
    # bias + GELU (writes Z) + residual
    ok(L().ouro_op_gemm(stream(), dtype, 0, 0, M, N, K, 1.0, p(dA), lda, p(dB), ldb, p(out), ldc, 0, 0, p(dbias), p(dR), N,
                        1, p(Z), N, force))
    torch.cuda.synchronize()
    assert rel_err(host(Z), pre) < TOL[dtype]
    assert rel_err(host(out)[:, :N], O.gelu(pre) + host(dR)) < TOL[dtype]
    assert np.all(host(out)[:, N:] == 0)
    # multiply by GELU'(Z)
    out2 = torch.zeros((M, N), dtype=tdt, device="cuda")
    ok(L().ouro_op_gemm(stream(), dtype, 0, 0, M, N, K, 1.0, p(dA), lda, p(dB), ldb, p(out2), N, 0, 0, None, None, 0,
                        2, p(Z), N, force))
    torch.cuda.synchronize()
    assert rel_err(host(out2), (a64 @ b64) * O.gelu_grad(host(Z))) < TOL[dtype]
    # accumulate (split-K path for bf16): C += A^T-form product
    M2, N2, K2 = 136, 264, 4096
    A2 = rng.standard_normal((K2, M2)).astype(np.float32)
    B2 = rng.standard_normal((K2, N2)).astype(np.float32)
    dA2, dB2 = dev(A2, dtype), dev(B2, dtype)
    acc = torch.ones((M2, N2), dtype=torch.float32, device="cuda")
    ok(L().ouro_op_gemm(stream(), dtype, 1, 0, M2, N2, K2, 1.0, p(dA2), M2, p(dB2), N2, p(acc), N2, 1, 1, None, None, 0,
                        0, None, 0, force))
    torch.cuda.synchronize()
    assert rel_err(host(acc), 1.0 + host(dA2).T @ host(dB2)) < 3e-6


# -------------------------------------------------------------------------- attention
def _attn_case(dtype, B, H, T, Mv, dh, rel, seed, force=1):
    rng = np.random.default_rng(seed)
    S = Mv + T
    d = H * dh
    q = rng.standard_normal((B * T, d)).astype(np.float32)
    kv = rng.standard_normal((B * S, 2 * d)).astype(np.float32)
    do = rng.standard_normal((B * T, d)).astype(np.float32)
    u = (rng.standard_normal((H, dh)) * 0.5).astype(np.float32)
    vb = (rng.standard_normal((H, dh)) * 0.5).astype(np.float32)
    r = rng.standard_normal((S, d)).astype(np.float32)
    dq_, dkv, ddo, du_, dvb_, dr_ = (dev(x, dtype) for x in (q, kv, do, u, vb, r))
    tdt = torch.bfloat16 if dtype else torch.float32
    o = torch.zeros((B * T, d), dtype=tdt, device="cuda")
    lse = torch.zeros((B, H, T), dtype=torch.float32, device="cuda")
    scale = 1.0 / math.sqrt(dh)
    kptr = C.c_void_p(dkv.data_ptr())
    vptr = C.c_void_p(dkv.data_ptr() + d * dkv.element_size())
    ok(L().ouro_op_attention_fwd(stream(), dtype, B, H, T, S, dh, Mv, scale, p(dq_), d, kptr, 2 * d, vptr, 2 * d, p(o), d,
                                 p(lse), rel, p(du_), p(dvb_), p(dr_), d, force))
    # oracle on the same (rounded) inputs
    q64 = host(dq_).reshape(B, T, H, dh).transpose(0, 2, 1, 3)
    k64 = host(dkv)[:, :d].reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    v64 = host(dkv)[:, d:].reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    r64 = host(dr_).reshape(S, H, dh).transpose(1, 0, 2)
    if rel:
        oo, cache = O.attention_core_fwd(q64, k64, v64, Mv, scale, host(du_), host(dvb_), r64)
    else:
        oo, cache = O.attention_core_fwd(q64, k64, v64, Mv, scale)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_err(host(o), oo.transpose(0, 2, 1, 3).reshape(B * T, d)) < tol
    assert np.abs(host(lse) - cache["lse"]).max() < (1e-4 if dtype == 0 else 2e-2)
    # backward
    n_scr = L().ouro_op_attention_bwd_scratch(B, H, T, S, dh)
    scr = torch.zeros(max(n_scr, 1), dtype=torch.float32, device="cuda")
    gq = torch.zeros((B * T, d), dtype=tdt, device="cuda")
    gkv = torch.zeros((B * S, 2 * d), dtype=tdt, device="cuda")
    gu = torch.zeros((H, dh), dtype=torch.float32, device="cuda")
    gvb = torch.zeros((H, dh), dtype=torch.float32, device="cuda")
    gr = torch.zeros((S, d), dtype=torch.float32, device="cuda")
    gk = C.c_void_p(gkv.data_ptr())
    gv = C.c_void_p(gkv.data_ptr() + d * gkv.element_size())
    ok(L().ouro_op_attention_bwd(stream(), dtype, B, H, T, S, dh, Mv, scale, p(dq_), d, kptr, 2 * d, vptr, 2 * d, p(o), d,
                                 p(lse), p(ddo), d, p(gq), d, gk, 2 * d, gv, 2 * d, rel, p(du_), p(dvb_), p(dr_), d,
                                 p(gu), p(gvb), p(gr), p(scr), force))
    torch.cuda.synchronize()
    do64 = host(ddo).reshape(B, T, H, dh).transpose(0, 2, 1, 3)
    rq, rk, rv, ru, rvb, rr = O.attention_core_bwd(do64, cache)
    mh = lambda x, n: x.transpose(0, 2, 1, 3).reshape(B * n, d)
    btol = tol * 2
    assert rel_err(host(gq), mh(rq, T)) < btol
    assert rel_err(host(gkv)[:, :d], mh(rk, S)) < btol
    assert rel_err(host(gkv)[:, d:], mh(rv, S)) < btol
    if rel:
        assert rel_err(host(gu), ru) < btol
        assert rel_err(host(gvb), rvb) < btol
        assert rel_err(host(gr), rr.transpose(1, 0, 2).reshape(S, d)) < btol


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("B,H,T,Mv,dh,rel", [(2, 2, 32, 0, 32, 0), (1, 3, 70, 0, 41, 0), (2, 2, 24, 17, 16, 1),
                                               (1, 2, 67, 130, 41, 1), (1, 1, 1, 0, 8, 0), (2, 1, 5, 0, 8, 1)])
def test_attention_general_kernel(dtype, B, H, T, Mv, dh, rel):
    _attn_case(dtype, B, H, T, Mv, dh, rel, seed=B + H + T + Mv + dh)


@pytest.mark.parametrize("B,H,T,Mv", [(2, 2, 128, 0), (1, 3, 200, 0), (2, 1, 96, 40), (1, 2, 512, 0), (1, 1, 33, 0),
                                      (1, 2, 300, 77), (32, 16, 256, 0), (16, 16, 384, 0), (16, 16, 300, 90)])
def test_attention_mfma_kernel(B, H, T, Mv):
    """Fused matrix-core kernels (bf16, head size 64): several query/key blocks, ragged
    tails, and a key prefix (Mv) that every query sees.  The last three cases have enough
    (batch, head) pairs for the backward kernels to take two blocks per workgroup (an even
    count, an odd one whose middle block goes alone, and unequal query / key block counts)."""
    _attn_case(1, B, H, T, Mv, 64, 0, seed=100 + T + Mv, force=0)


@pytest.mark.parametrize("B,H,T,Mv", [(2, 2, 128, 0), (1, 3, 200, 0), (2, 1, 96, 40), (1, 2, 384, 384), (1, 1, 33, 0),
                                      (1, 2, 300, 77), (2, 2, 150, 150), (3, 2, 20, 5), (2, 3, 64, 200)])
def test_attention_xl_mfma_kernel(B, H, T, Mv):
    """Fused matrix-core kernels with the relative-position term (bf16, head size 64): with and
    without memory, several query/key blocks, ragged tails, fewer keys than a contraction tile
    (dK, dV and dr are contractions of what the dQ kernel leaves), memory longer than the segment."""
    _attn_case(1, B, H, T, Mv, 64, 1, seed=200 + T + Mv, force=0)


@pytest.mark.parametrize("dtype,force", [(0, 0), (1, 1), (1, 0), (1, 10), (1, 11), (1, 12), (1, 13), (1, 14)])
@pytest.mark.parametrize("M,N,K,ln", [(200, 136, 328, 1), (384, 520, 192, 1), (130, 88, 128, 0), (260, 256, 64, 1)])
def test_gemm_with_fp32_layernorm_residual(dtype, force, M, N, K, ln):
    """C = A B + bias + R with R the LayerNorm of an fp32 matrix recomputed in the epilogue (ln = 1) or
    that fp32 matrix itself (ln = 0); fp32 result; every contraction kernel, ragged tiles."""
    rng = np.random.default_rng(M + N + K + force + ln)
    A = rng.standard_normal((M, K)).astype(np.float32); B = rng.standard_normal((K, N)).astype(np.float32) / math.sqrt(K)
    bias = rng.standard_normal(N).astype(np.float32)
    S_ = (rng.standard_normal((M, N)) * 2 + 0.3).astype(np.float32)
    g = (1 + 0.3 * rng.standard_normal(N)).astype(np.float32); b = (0.2 * rng.standard_normal(N)).astype(np.float32)
    dA, dB = dev(A, dtype), dev(B, dtype)
    dS, dbias, dg, db = (torch.from_numpy(x).cuda() for x in (S_, bias, g, b))
    R, cache = O.layernorm_fwd(S_.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    mean = torch.from_numpy(S_.astype(np.float64).mean(axis=1).astype(np.float32)).cuda()      # row statistics are inputs here
    rstd = torch.from_numpy(cache[1][:, 0].astype(np.float32)).cuda()
    Cc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    ok(L().ouro_op_gemm_ln_residual(stream(), dtype, 0, 0, M, N, K, p(dA), K, p(dB), N, p(Cc), N, 1, p(dbias), p(dS), N,
                                    p(mean) if ln else None, p(rstd) if ln else None, p(dg) if ln else None,
                                    p(db) if ln else None, force))
    torch.cuda.synchronize()
    ref = host(dA) @ host(dB) + bias + (R if ln else S_.astype(np.float64))
    assert rel_err(host(Cc), ref) < TOL[dtype]
    assert np.abs(host(Cc) - ref).max() < (1e-4 if dtype == 0 else 0.1) * np.abs(ref).max()


# ------------------------------------------------------------------ row-wise kernels
@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("rows,d", [(37, 64), (130, 512), (9, 410), (5, 1024), (3, 4100), (517, 1024), (66, 2048)])
def test_layernorm(dtype, rows, d):
    """dtype 2: fp32 rows read, bf16 rows written (the bf16 model's form)."""
    rng = np.random.default_rng(rows + d)
    x = (rng.standard_normal((rows, d)) * 2 + 0.5).astype(np.float32)
    dy = rng.standard_normal((rows, d)).astype(np.float32)
    g = (1 + 0.3 * rng.standard_normal(d)).astype(np.float32)
    b = (0.2 * rng.standard_normal(d)).astype(np.float32)
    dx_, ddy = dev(x, 1 if dtype == 1 else 0), dev(dy, 1 if dtype == 1 else 0)
    dg_, db_ = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    tdt = torch.bfloat16 if dtype else torch.float32
    y = torch.zeros((rows, d), dtype=tdt, device="cuda")
    mean = torch.zeros(rows, device="cuda"); rstd = torch.zeros(rows, device="cuda")
    ok(L().ouro_op_layernorm_fwd(stream(), dtype, p(dx_), p(dg_), p(db_), p(y), p(mean), p(rstd), rows, d, 0))
    yr, cache = O.layernorm_fwd(host(dx_), g.astype(np.float64), b.astype(np.float64))
    torch.cuda.synchronize()
    assert rel_err(host(y), yr) < TOL[min(dtype, 1)]
    assert rel_err(host(rstd), cache[1][:, 0]) < 1e-5
    gx = torch.zeros((rows, d), dtype=tdt, device="cuda")
    gg = torch.full((d,), 7.0, device="cuda"); gb = torch.full((d,), 7.0, device="cuda")
    ok(L().ouro_op_layernorm_bwd(stream(), dtype, p(ddy), p(dx_), p(dg_), p(mean), p(rstd), p(gx), p(gg), p(gb), rows, d, 0))
    torch.cuda.synchronize()
    rx, rg, rb = O.layernorm_bwd(host(ddy), g.astype(np.float64), cache)
    assert rel_err(host(gx), rx) < TOL[min(dtype, 1)]
    assert rel_err(host(gg), rg) < 1e-4
    assert rel_err(host(gb), rb) < 1e-4


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("rows,dn,d", [(37, 410, 448), (9, 41, 64), (130, 100, 101)])
def test_layernorm_zero_padded_rows(dtype, rows, dn, d):
    """Rows of d columns whose last d-dn are zero padding: statistics over dn columns only, the
    padding stays zero in y and dx, and the first dn columns equal LayerNorm of the unpadded rows."""
    rng = np.random.default_rng(rows + d)
    x = np.zeros((rows, d), np.float32); dy = np.zeros((rows, d), np.float32)
    g = np.zeros(d, np.float32); b = np.zeros(d, np.float32)
    x[:, :dn] = rng.standard_normal((rows, dn)) * 2 + 0.5
    dy[:, :dn] = rng.standard_normal((rows, dn))
    g[:dn] = 1 + 0.3 * rng.standard_normal(dn); b[:dn] = 0.2 * rng.standard_normal(dn)
    dx_, ddy = dev(x, dtype), dev(dy, dtype)
    dg_, db_ = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
    tdt = torch.bfloat16 if dtype else torch.float32
    y = torch.full((rows, d), 3.0, dtype=tdt, device="cuda")
    mean = torch.zeros(rows, device="cuda"); rstd = torch.zeros(rows, device="cuda")
    ok(L().ouro_op_layernorm_fwd(stream(), dtype, p(dx_), p(dg_), p(db_), p(y), p(mean), p(rstd), rows, d, dn))
    yr, cache = O.layernorm_fwd(host(dx_)[:, :dn], g[:dn].astype(np.float64), b[:dn].astype(np.float64))
    torch.cuda.synchronize()
    assert rel_err(host(y)[:, :dn], yr) < TOL[dtype]
    assert not host(y)[:, dn:].any()
    assert rel_err(host(rstd), cache[1][:, 0]) < 1e-5
    gx = torch.full((rows, d), 3.0, dtype=tdt, device="cuda")
    gg = torch.full((d,), 7.0, device="cuda"); gb = torch.full((d,), 7.0, device="cuda")
    ok(L().ouro_op_layernorm_bwd(stream(), dtype, p(ddy), p(dx_), p(dg_), p(mean), p(rstd), p(gx), p(gg), p(gb), rows, d, dn))
    torch.cuda.synchronize()
    rx, rg, rb = O.layernorm_bwd(host(ddy)[:, :dn], g[:dn].astype(np.float64), cache)
    assert rel_err(host(gx)[:, :dn], rx) < TOL[dtype]
    assert not host(gx)[:, dn:].any()
    assert rel_err(host(gg)[:dn], rg) < 1e-4 and not host(gg)[dn:].any()
    assert rel_err(host(gb)[:dn], rb) < 1e-4 and not host(gb)[dn:].any()


# ---------------------------------------------------------------------------- dropout
@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("rows,cols,ld,drop_ld", [(37, 64, 64, 64), (130, 410, 448, 410), (3, 5, 9, 7)])
def test_dropout_mask_bit_exact(dtype, rows, cols, ld, drop_ld):
    """The kernel's generator against the oracle's: every element kept or dropped alike (integer
    work: bit-exact), kept elements scaled by 1/(1-p); element index = row * drop_ld + column."""
    pr, seed, sid = 0.3125, 0xDEADBEEF12345678, 11   # rates are dyadic: the same number in fp32 (boundary) and fp64 (oracle)
    cfg = O.Config(n_layer=1, d_model=2, n_head=1, d_head=2, d_ff=1, vocab=2, seq_len=1, batch=1, dropout=pr)
    src = np.zeros((rows, ld), np.float32)
    src[:, :cols] = 1.0 + np.arange(rows * cols, dtype=np.float32).reshape(rows, cols) % 7
    d_src = dev(src, dtype)
    dst = torch.zeros_like(d_src)
    ok(L().ouro_op_dropout(stream(), dtype, p(d_src), p(dst), rows, cols, ld, pr, seed, sid, drop_ld))
    torch.cuda.synchronize()
    mask = O.dropout_mask(cfg, seed, sid, (rows, drop_ld))[:, :cols]
    got = host(dst)[:, :cols]
    assert np.array_equal(got != 0, mask != 0)
    assert rel_err(got, host(d_src)[:, :cols] * mask) < TOL[dtype]
    assert 0.58 < (mask != 0).mean() < 0.8 or mask.size < 100


@pytest.mark.parametrize("dtype,force", [(0, 0), (1, 1), (1, 0), (1, 10), (1, 11), (1, 12), (1, 13), (1, 14)])
@pytest.mark.parametrize("M,N,K", [(200, 136, 328), (384, 520, 192), (130, 82, 128)])
def test_gemm_with_fused_dropout(dtype, force, M, N, K):
    """C = dropout(A B + bias) + residual in every contraction kernel's epilogue (16-byte and
    scalar store paths, ragged tiles): the mask is the oracle's at element m*N + n."""
    rng = np.random.default_rng(M + N + K + force)
    A = rng.standard_normal((M, K)).astype(np.float32); B = rng.standard_normal((K, N)).astype(np.float32) / math.sqrt(K)
    bias = rng.standard_normal(N).astype(np.float32); R = rng.standard_normal((M, N)).astype(np.float32)
    pr, seed, sid = 0.25, 424242, 5
    cfg = O.Config(n_layer=1, d_model=2, n_head=1, d_head=2, d_ff=1, vocab=2, seq_len=1, batch=1, dropout=pr)
    dA, dB, dR = dev(A, dtype), dev(B, dtype), dev(R, dtype)
    dbias = torch.from_numpy(bias).cuda()
    Cc = torch.zeros((M, N), dtype=dA.dtype, device="cuda")
    ok(L().ouro_op_gemm_dropout(stream(), dtype, 0, 0, M, N, K, p(dA), K, p(dB), N, p(Cc), N, p(dbias), p(dR), N,
                                pr, seed, sid, N, force))
    torch.cuda.synchronize()
    mask = O.dropout_mask(cfg, seed, sid, (M, N))
    ref = (host(dA) @ host(dB) + bias) * mask + host(dR)
    assert rel_err(host(Cc), ref) < TOL[dtype]


@pytest.mark.parametrize("dtype", [0, 1])
def test_colsum(dtype):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((333, 200)).astype(np.float32)
    dx_ = dev(x, dtype)
    out = torch.full((150,), 3.0, device="cuda")
    ok(L().ouro_op_colsum(stream(), dtype, p(dx_), 200, p(out), 333, 150))
    torch.cuda.synchronize()
    assert rel_err(host(out), host(dx_)[:, :150].sum(0)) < 1e-5


@pytest.mark.parametrize("dtype", [0, 1])
def test_embedding_gather_scatter(dtype):
    rng = np.random.default_rng(4)
    vocab, d, T, B = 50, 24, 7, 5
    N = B * T
    V = rng.standard_normal((vocab, d)).astype(np.float32)
    tok = rng.integers(0, vocab, N).astype(np.int32)
    tok[:6] = 3                                           # a hot row
    dV = dev(V, dtype)
    dtok = torch.from_numpy(tok).cuda()
    pe = rng.standard_normal((T, d)).astype(np.float32)
    dpe = torch.from_numpy(pe).cuda()
    tdt = torch.bfloat16 if dtype else torch.float32
    h = torch.zeros((N, d), dtype=tdt, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    ok(L().ouro_op_embed_fwd(stream(), dtype, p(dtok), p(dV), None, p(h), N, T, d, vocab, 1.0, p(flag)))
    torch.cuda.synchronize()
    assert torch.equal(h, dV[torch.from_numpy(tok.astype(np.int64)).cuda()])      # row selection is bit-exact
    ok(L().ouro_op_embed_fwd(stream(), dtype, p(dtok), p(dV), p(dpe), p(h), N, T, d, vocab, 1.5, p(flag)))
    torch.cuda.synchronize()
    ref = 1.5 * host(dV)[tok] + np.tile(pe, (B, 1))
    assert rel_err(host(h), ref) < (1e-6 if dtype == 0 else 4e-3)
    assert flag.item() == 0
    dh = rng.standard_normal((N, d)).astype(np.float32)
    ddh = dev(dh, dtype)
    dVi = torch.full((vocab, d), 9.0, device="cuda")
    ok(L().ouro_op_embed_bwd(stream(), dtype, p(dtok), p(ddh), p(dVi), N, d, vocab, 1.5))
    torch.cuda.synchronize()
    refg = np.zeros((vocab, d))
    np.add.at(refg, tok, 1.5 * host(ddh))
    assert rel_err(host(dVi), refg) < 1e-6
    assert np.all(host(dVi)[np.setdiff1d(np.arange(vocab), tok)] == 0)
    # out-of-range id: flagged, row skipped, nothing dereferenced
    tok2 = tok.copy(); tok2[2] = vocab; tok2[3] = -1
    dtok2 = torch.from_numpy(tok2).cuda()
    ok(L().ouro_op_embed_fwd(stream(), dtype, p(dtok2), p(dV), None, p(h), N, T, d, vocab, 1.0, p(flag)))
    torch.cuda.synchronize()
    assert flag.item() == 1 and np.all(host(h)[2:4] == 0)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("N,vocab", [(12, 256), (7, 1000), (5, 50257), (4, 32768), (3, 65536), (3, 65537), (6, 2056)])
def test_softmax_cross_entropy(dtype, N, vocab):
    rng = np.random.default_rng(N + vocab)
    logits = (rng.standard_normal((N, vocab)) * 3).astype(np.float32)
    tgt = rng.integers(0, vocab, N).astype(np.int32)
    ld = (vocab + 7) // 8 * 8                                  # padded rows, as the model lays them out
    tdt = torch.bfloat16 if dtype else torch.float32
    dl = torch.zeros((N, ld), dtype=tdt, device="cuda")
    dl[:, :vocab] = dev(logits, dtype)
    l64 = host(dl)[:, :vocab]                                  # the (rounded) logits both sides see
    dt = torch.from_numpy(tgt).cuda()
    G = torch.zeros((N, ld), dtype=tdt, device="cuda")
    lse = torch.zeros(N, device="cuda"); rl = torch.zeros(N, device="cuda"); loss = torch.zeros(1, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    ok(L().ouro_op_softmax_ce(stream(), dtype, p(dl), ld, p(dt), p(G), ld, p(lse), p(rl), p(loss), N, vocab, p(flag)))
    torch.cuda.synchronize()
    rloss, rlse = O.cross_entropy_fwd(l64, tgt)
    rG = O.cross_entropy_bwd(l64, rlse, tgt)
    assert abs(loss.item() - rloss) / rloss < 1e-5
    assert np.abs(host(lse) - rlse).max() < 1e-4
    assert rel_err(host(G)[:, :vocab], rG) < (1e-5 if dtype == 0 else 5e-3)
    assert flag.item() == 0
    # in place: G written over the logits
    dl2 = dl.clone()
    ok(L().ouro_op_softmax_ce(stream(), dtype, p(dl2), ld, p(dt), p(dl2), ld, p(lse), p(rl), p(loss), N, vocab, p(flag)))
    torch.cuda.synchronize()
    assert torch.equal(dl2[:, :vocab], G[:, :vocab])
    # zero logits: loss = ln(vocab) (uniform softmax)
    dl.zero_()
    ok(L().ouro_op_softmax_ce(stream(), dtype, p(dl), ld, p(dt), p(G), ld, p(lse), p(rl), p(loss), N, vocab, p(flag)))
    torch.cuda.synchronize()
    assert abs(loss.item() - math.log(vocab)) < 1e-5


@pytest.mark.parametrize("adam", [0, 1])
@pytest.mark.parametrize("n", [1, 7, 4096, 100003])
def test_update_kernel(adam, n):
    rng = np.random.default_rng(n + adam)
    w = rng.standard_normal(n).astype(np.float32)
    g0 = rng.standard_normal(n).astype(np.float32); g1 = rng.standard_normal(n).astype(np.float32)
    m = (rng.standard_normal(n) * 0.1).astype(np.float32); v = (rng.random(n) * 0.1).astype(np.float32)
    dw, dg0, dg1, dm, dv = (torch.from_numpy(x.copy()).cuda() for x in (w, g0, g1, m, v))
    sh = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    t = 5
    ok(L().ouro_op_update(stream(), p(dw), p(dm), p(dv), p(sh), p(dg0), 0.5, p(dg1), 0.5, n, adam, 0.01, 0.9, 0.999, 1e-8, t))
    torch.cuda.synchronize()
    cfg = O.Config(n_layer=1, d_model=8, n_head=2, d_head=4, d_ff=8, vocab=8, seq_len=2, batch=1, optimizer=adam)
    orc = O.Oracle.__new__(O.Oracle); orc.cfg = cfg; orc.t = t
    w64, m64, v64 = w.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    orc._apply(w64, 0.5 * g0.astype(np.float64) + 0.5 * g1.astype(np.float64), m64, v64, 0.01)
    assert rel_err(host(dw), w64) < 1e-6
    if adam:
        assert rel_err(host(dm), m64) < 1e-6 and rel_err(host(dv), v64) < 1e-6
    assert torch.equal(sh, dw.to(torch.bfloat16))            # bf16 copy = round-to-nearest-even of the master
    # zero gradient (null pointers) with zero moments leaves the weights bit-identical
    dw2 = torch.from_numpy(w.copy()).cuda(); z1 = torch.zeros(n, device="cuda"); z2 = torch.zeros(n, device="cuda")
    ok(L().ouro_op_update(stream(), p(dw2), p(z1), p(z2), None, None, 1.0, None, 0.0, n, adam, 0.01, 0.9, 0.999, 1e-8, 0))
    torch.cuda.synchronize()
    assert np.array_equal(dw2.cpu().numpy(), w) and not z1.any() and not z2.any()
