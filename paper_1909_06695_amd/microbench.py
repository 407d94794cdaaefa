"""Single-kernel timings through the C boundary (the commands behind profiles/).

  python -m paper_1909_06695_amd.microbench gemm tA tB M N K [iters]     one bf16 contraction
  python -m paper_1909_06695_amd.microbench layer d F tokens vocab        every contraction of a layer + LM head
  python -m paper_1909_06695_amd.microbench copy nbytes [iters]           plain device copy (PMC byte-counter scale)
"""
import ctypes as C
import sys

import torch

from . import binding


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def gemm(tA, tB, M, N, K, out_fp32=0, acc=0, epi=0, bias=False, res=False, iters=20, name=""):
    L = binding.lib()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    A = torch.randn((K, M) if tA else (M, K), device="cuda").to(torch.bfloat16)
    B = torch.randn((N, K) if tB else (K, N), device="cuda").to(torch.bfloat16)
    Cm = torch.zeros((M, N), device="cuda", dtype=torch.float32 if out_fp32 else torch.bfloat16)
    Z = torch.zeros((M, N), device="cuda", dtype=torch.bfloat16) if epi else None
    bi = torch.randn(N, device="cuda") if bias else None
    R = torch.randn((M, N), device="cuda").to(torch.bfloat16) if res else None

    def run():
        rc = L.ouro_op_gemm(st, 1, tA, tB, M, N, K, 1.0, _p(A), A.shape[1], _p(B), B.shape[1], _p(Cm), N, out_fp32, acc,
                            _p(bi), _p(R), N, epi, _p(Z), N, 0)
        binding.check(rc)

    for _ in range(3):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        run()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    print(f"{name:24s} tA={tA} tB={tB} M={M:6d} N={N:6d} K={K:6d} {us:9.1f} us {2.0 * M * N * K / us / 1e6:8.1f} TFLOP/s",
          flush=True)
    return us


def layer(d, F, n_tok, vocab):
    tot = 0.0
    tot += gemm(0, 0, n_tok, 3 * d, d, name="qkv fwd")
    tot += gemm(0, 0, n_tok, d, d, res=True, name="o fwd +res")
    tot += gemm(0, 0, n_tok, F, d, epi=1, bias=True, name="ffn1 fwd +bias+gelu")
    tot += gemm(0, 0, n_tok, d, F, bias=True, res=True, name="ffn2 fwd +bias+res")
    tot += gemm(0, 1, n_tok, F, d, epi=2, name="ffn2 dgrad *gelu'")
    tot += gemm(0, 1, n_tok, d, F, res=True, name="ffn1 dgrad +res")
    tot += gemm(0, 1, n_tok, d, d, name="o dgrad")
    tot += gemm(0, 1, n_tok, d, 3 * d, res=True, name="qkv dgrad +res")
    tot += gemm(1, 0, F, d, n_tok, out_fp32=1, acc=1, name="ffn2 wgrad")
    tot += gemm(1, 0, d, F, n_tok, out_fp32=1, acc=1, name="ffn1 wgrad")
    tot += gemm(1, 0, d, d, n_tok, out_fp32=1, acc=1, name="o wgrad")
    tot += gemm(1, 0, d, 3 * d, n_tok, out_fp32=1, acc=1, name="qkv wgrad")
    print(f"layer total {tot:.1f} us")
    gemm(0, 1, n_tok, vocab, d, iters=5, name="logits = h V^T")
    gemm(0, 0, n_tok, d, vocab, iters=5, name="dh = G V")
    gemm(1, 0, vocab, d, n_tok, out_fp32=1, iters=5, name="dVo = G^T h")


def copy(nbytes, iters=5):
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for _ in range(iters):
        b.copy_(a)
    torch.cuda.synchronize()


def main(argv):
    if argv and argv[0] == "gemm":
        tA, tB, M, N, K = (int(x) for x in argv[1:6])
        gemm(tA, tB, M, N, K, iters=int(argv[6]) if len(argv) > 6 else 20)
    elif argv and argv[0] == "layer":
        layer(*(int(x) for x in argv[1:5]))
    elif argv and argv[0] == "copy":
        copy(int(argv[1]), int(argv[2]) if len(argv) > 2 else 5)
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
