"""GPU parity on seeded random shapes: every decode and product entry point against the
CPU oracle, over all codes, row lengths that select every wave count of the batch-1
kernel, row counts with and without a ragged last pair of tile rows, batch sizes on both
sides of every kernel switch, with and without the per-row scale.

Bars as in test_gpu_parity.py: decoded weights bit-exact; products within 2e-3 (1e-4
observed) of the fp64 oracle as max|y - y*| / max|y*|; the call that transforms its own
input gives the bits of the two separate calls.
"""
import numpy as np
import pytest

import oracle
import qtip_synth as synth
from parity_util import assert_products
from qtip_synth import CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB1, CODE_HYB2, CODE_LUT

pytestmark = pytest.mark.gpu

CODECS = [(CODE_3INST, 2, 1), (CODE_3INST, 3, 1), (CODE_3INST, 4, 1),
          (CODE_1MAD, 2, 1), (CODE_1MAD, 3, 1), (CODE_1MAD, 4, 1),
          (CODE_HYB, 2, 2), (CODE_HYB, 3, 2), (CODE_HYB, 4, 2),
          (CODE_HYB2, 2, 2), (CODE_HYB2, 3, 2), (CODE_HYB2, 4, 2),
          (CODE_HYB1, 2, 1), (CODE_HYB1, 3, 1), (CODE_HYB1, 4, 1),
          (CODE_LUT, 2, 1), (CODE_LUT, 3, 1), (CODE_LUT, 4, 1)]
BATCHES = [1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 64, 65, 100]
REL_TOL, OBSERVED_TOL = 2e-3, 1e-4
CASES_PER_SEED = 40


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / np.abs(ref).max())


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15])
def test_random_shapes(q, seed):
    import torch
    rng = np.random.default_rng(seed)
    for it in range(CASES_PER_SEED):
        code_id, k, V = CODECS[rng.integers(len(CODECS))]
        L = 14 if code_id == CODE_LUT else 16
        long_rows = rng.random() < 0.25
        m = 32 * int(rng.integers(1, 8 if long_rows else 30))
        if code_id != CODE_LUT and rng.random() < 0.5:
            m += 16
        n = 16 * int(rng.integers(1, 1900 if long_rows else 200))
        B = BATCHES[rng.integers(len(BATCHES))] if rng.random() < 0.7 else 1
        w = synth.Workload(f"random_{seed}_{it}", 9, it, m, n, code_id, k, V, 16, 16, B=B,
                           row_scale=bool(rng.random() < 0.5), L=L)
        inp = synth.make_inputs(w, seed=100000 * seed + it)
        case = f"seed {seed} case {it}: code {code_id} k={k} m={m} n={n} B={B} scale={w.row_scale}"
        print(case, flush=True)
        codes, lut, X, sc = dev(inp.codes), dev(inp.lut), dev(inp.X), dev(inp.row_scale)

        Wref = oracle.dequantize(inp.codes, L, k, V, code_id, m, n, inp.lut, tile=w.tile)
        Wd = torch.empty((m, n), dtype=torch.float16, device="cuda")
        q.qtip_dequantize(codes, L, k, V, code_id, lut, m, n, Wd)
        assert np.array_equal(Wd.cpu().numpy().view(np.uint16), Wref), case

        Y = torch.full((B, m), float("nan"), dtype=torch.float32, device="cuda")
        q.qtip_decode_matmat(codes, L, k, V, code_id, lut, m, n, X, B, sc, Y)
        assert_products(Y.cpu().numpy(), Wref, inp.X, inp.row_scale, code_id, inp.codes, k, context=case)
        if B > 1:
            continue

        y = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
        q.qtip_decode_matvec(codes, L, k, V, code_id, lut, m, n, X, y)
        assert_products(y.cpu().numpy().reshape(1, -1), Wref, inp.X, None, code_id, inp.codes, k, context=case)

        # steps 1 + 2 of the layer in one call; Hadamard block = the largest power of two
        # that divides n, at most 4096
        block = min(4096, n & -n)
        signs = rng.choice(np.array([-1, 1], dtype=np.int8), n)
        sg = dev(signs)
        xt = torch.empty((1, n), dtype=torch.float16, device="cuda")
        y2 = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
        q.qtip_rht(X, sg, n, block, 1, 0, xt)
        q.qtip_decode_matmat(codes, L, k, V, code_id, lut, m, n, xt, 1, sc, y2)
        y1 = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
        scratch = torch.empty(n, dtype=torch.float16, device="cuda")
        q.qtip_rht_decode_matvec(codes, L, k, V, code_id, lut, m, n, X, sg, block, sc, y1, scratch)
        assert np.array_equal(y1.cpu().numpy(), y2.cpu().numpy()), case
        xt_ref = oracle.rht(inp.X, signs, block, 0).astype(np.float16)   # the layer rounds x~ to fp16
        ref3 = oracle.matmat_dense(Wref, xt_ref, inp.row_scale)[0]
        assert rel_err(y1.cpu().numpy(), ref3) <= REL_TOL, case
