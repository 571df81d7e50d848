"""Which side should pay for the transposed operands of the weight gradient (dW = dY^T X, contraction over tokens)?

Two ways to give the MFMA its operands K-contiguous:
  (a) the kernel transposes bytes while it reads the staged tiles back from LDS (ds_read_b64_tr_b8) -- what
      jf_linear_wgrad does;
  (b) the producers also write transposed INT8 copies (dY^T, X^T with transposed scale grids, valid because blocks are
      square) and the product runs as the forward kernel on them.
This script times both routes of the same product (the results are bit-identical, which it checks) and what the
transposed copies cost where this library can write them (the quantizer), at the GPT-2-small MLP shape and at 8192^3.
Run from the repository root on the GPU: python -m microbench transposed_operands
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import paper_2403_12422_amd as jf  # noqa: E402


def timed_us(fn, reps):
    for _ in range(10):
        fn()
    torch.cuda.synchronize()
    best = 1e9
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps * 1e3)
    return best


def main():
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(240312422)
    for (N, C, D, B, reps) in ((4096, 768, 3072, 32, 300), (8192, 8192, 8192, 32, 20), (8192, 8192, 8192, 128, 20)):
        X = torch.randn((N, C), generator=gen, device=dev)
        G = torch.randn((N, D), generator=gen, device=dev) * 1e-3
        Xq, SX, XT, SXT = jf.jf_quantize_block(X, B, transposed_copy=True)
        Gq, SG, GT, SGT = jf.jf_quantize_block(G, B, transposed_copy=True)
        o1 = jf.jf_linear_wgrad(Gq, SG, Xq, SX, B)
        o2 = jf.jf_linear_fwd(GT, SGT, XT, SXT, B)          # (dY^T) (X^T)^T = dY^T X
        assert torch.equal(o1[0], o2[0]) and torch.equal(o1[1], o2[1])
        a = timed_us(lambda: jf.jf_linear_wgrad(Gq, SG, Xq, SX, B, out=o1), reps)
        b = timed_us(lambda: jf.jf_linear_fwd(GT, SGT, XT, SXT, B, out=o2), reps)
        oq = (torch.empty_like(Gq), torch.empty_like(SG))
        oqt = (torch.empty_like(Gq), torch.empty_like(SG), torch.empty_like(GT), torch.empty_like(SGT))
        qg = timed_us(lambda: jf.jf_quantize_block(G, B, out=oq), reps)
        qgt = timed_us(lambda: jf.jf_quantize_block(G, B, transposed_copy=True, out=oqt), reps)
        ox = (torch.empty_like(Xq), torch.empty_like(SX))
        oxt = (torch.empty_like(Xq), torch.empty_like(SX), torch.empty_like(XT), torch.empty_like(SXT))
        qx = timed_us(lambda: jf.jf_quantize_block(X, B, out=ox), reps)
        qxt = timed_us(lambda: jf.jf_quantize_block(X, B, transposed_copy=True, out=oxt), reps)
        print(f"tokens {N}, in {C}, out {D}, block {B}:")
        print(f"  weight gradient, bytes transposed on the way out of LDS      {a:9.1f} us")
        print(f"  same product from pre-transposed copies (forward kernel)      {b:9.1f} us   saves {a - b:7.1f} us")
        print(f"  quantizer of dY ({N} x {D}) without / with transposed copy    {qg:9.1f} / {qgt:9.1f} us   costs {qgt - qg:7.1f} us")
        print(f"  quantizer of X  ({N} x {C}) without / with transposed copy    {qx:9.1f} / {qxt:9.1f} us   costs {qxt - qx:7.1f} us")
        print(f"  net of writing both copies in the producers: {(a - b) - (qgt - qg) - (qxt - qx):+.1f} us per step "
              "(positive = producer-side copies would win)", flush=True)
        del X, G, Xq, XT, Gq, GT, o1, o2, oq, oqt, ox, oxt
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
