"""End-to-end use of the library on one synthetic layer, on one MI355X:

    python -m paper_2406_11235_amd.example [m n]

1. quantize: block LDL of a (synthetic) proxy Hessian, then BlockLDLQ with the tail-biting
   Viterbi quantizer as rounder (the paper's Algorithm 5), 2-bit 3INST;
2. infer: y = S_m V_m^T (W~ (V_n S_n x)) with the fused decode + matvec kernel and the two
   Hadamard transforms, checked against the dense product with the decoded weights.
The weights stand for an already incoherence-processed matrix W~ (i.i.d. Gaussian); torch is
used for memory and for the dense check only.
"""
import sys
import time

import torch

from . import (CODE_3INST, qtip_block_ldl, qtip_block_ldl_workspace, qtip_decode_matvec,
               qtip_dequantize, qtip_quantize_ldlq, qtip_quantize_ldlq_workspace, qtip_rht, qtip_rht_f32)


def largest_pow2_divisor(v, cap=16384):
    b = 1
    while v % (2 * b) == 0 and 2 * b <= cap:
        b *= 2
    return b


def main(m=1024, n=2048, seed=0):
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(seed)
    k, V, code = 2, 1, CODE_3INST
    W = torch.randn(m, n, device=dev, generator=g) * 1.2437            # the 3INST code's scale
    X = torch.randn(2 * n, n, dtype=torch.float64, device=dev, generator=g)
    X = 0.9 * X[:, :1] + 0.1 * X                                       # strongly correlated inputs
    H = X.T @ X / (2 * n) + 1e-3 * torch.eye(n, dtype=torch.float64, device=dev)

    # ---- quantize
    A = torch.empty(n, n, device=dev)
    ws = torch.empty(max(qtip_block_ldl_workspace(n), qtip_quantize_ldlq_workspace(m, n, k, V, m // 16)),
                     dtype=torch.uint8, device=dev)
    codes = torch.empty((m // 16) * (n // 16) * 8 * k, dtype=torch.int32, device=dev)
    What = torch.empty(m, n, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    qtip_block_ldl(H, n, 16, A, None, ws, ws.numel())
    qtip_quantize_ldlq(W, A, m, n, 16, k, V, code, None, codes, What, None, ws, ws.numel())
    torch.cuda.synchronize()
    t_quant = time.perf_counter() - t0
    E = (What - W).double()
    print(f"quantized {m} x {n} to {k} bits in {t_quant*1e3:.0f} ms; "
          f"mse/var {float((E**2).mean()) / 1.2437**2:.4f}, proxy loss {float(torch.trace(E @ H @ E.T)):.4g}")

    # ---- infer
    bn, bm = largest_pow2_divisor(n), largest_pow2_divisor(m)
    sn = (torch.randint(0, 2, (n,), device=dev, generator=g) * 2 - 1).to(torch.int8)
    sm = (torch.randint(0, 2, (m,), device=dev, generator=g) * 2 - 1).to(torch.int8)
    x = torch.randn(1, n, device=dev, generator=g).half()
    xt = torch.empty_like(x)
    z = torch.empty(m, device=dev)
    y = torch.empty(1, m, dtype=torch.float16, device=dev)
    qtip_rht(x, sn, n, bn, 1, 0, xt)                                   # x~ = V_n (S_n .* x)
    qtip_decode_matvec(codes, 16, k, V, code, None, m, n, xt, z)       # z = W~ x~
    qtip_rht_f32(z, sm, m, bm, 1, 1, y)                                # y = S_m .* (V_m^T z)
    Wd = torch.empty(m, n, dtype=torch.float16, device=dev)
    qtip_dequantize(codes, 16, k, V, code, None, m, n, Wd)
    torch.cuda.synchronize()
    assert torch.equal(Wd.float(), What), "decoded weights differ from the quantizer's"
    zref = Wd.double() @ xt.double().T
    err = float((z.double() - zref[:, 0]).abs().max() / zref.abs().max())
    print(f"decode + matvec against the dense product with the decoded weights: max rel err {err:.2e}")
    assert err < 2e-3
    return err


if __name__ == "__main__":
    args = [int(a) for a in sys.argv[1:3]]
    main(*args)
