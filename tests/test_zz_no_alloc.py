"""qtip_rht_decode_matvec_noalloc (the entry point for callers that cannot allocate) against
qtip_rht_decode_matvec with a caller's scratch buffer: same kernels, so the same y bit for
bit, on two calls in a row, the second with a smaller input (the library's scratch still
holds the first call's longer vector), then once more on the small-layer form that needs no
scratch.  Also against the fp64 oracle at the products' bar."""
import numpy as np
import pytest

import oracle
import qtip_synth as synth
from qtip_synth import CODE_3INST, CODE_HYB

pytestmark = pytest.mark.gpu

REL_TOL = 2e-3


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


def layer_case(code_id, k, V, m, n, block, sub):
    w = synth.Workload(f"noalloc_{m}x{n}", 9, 900 + sub, m, n, code_id, k, V, block, 16, row_scale=True)
    return w, synth.make_inputs(w)


def run_both(q, w, inp):
    import torch
    args = (dev(inp.codes), 16, w.k, w.V, w.code_id, dev(inp.lut), w.m, w.n, dev(inp.X[0]), dev(inp.signs_n),
            w.block_n, dev(inp.row_scale))
    y_ref = torch.full((w.m,), float("nan"), dtype=torch.float32, device="cuda")
    xt = torch.empty(w.n, dtype=torch.float16, device="cuda")
    q.qtip_rht_decode_matvec(*args, y_ref, xt)
    y = torch.full((w.m,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_rht_decode_matvec_noalloc(*args, y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), y_ref.cpu().numpy()


def check_against_oracle(w, inp, y):
    Wref = oracle.dequantize(inp.codes, 16, w.k, w.V, w.code_id, w.m, w.n, inp.lut)
    xt = oracle.rht(inp.X[0], inp.signs_n, w.block_n, 0)
    # the product's reference takes the transformed vector as the kernel sees it: fp16
    ref = oracle.matmat_dense(Wref, xt.astype(np.float16), inp.row_scale)[0]
    err = float(np.abs(y - ref).max() / np.abs(ref).max())
    assert err <= REL_TOL, err


def test_two_calls_in_a_row_the_second_smaller(q):
    # both above 8192 inputs: the two-kernel form, through the library's own scratch
    for sub, (code_id, k, V, m, n, block) in enumerate([(CODE_3INST, 2, 1, 96, 16384, 4096),
                                                        (CODE_HYB, 4, 2, 48, 12288, 2048),
                                                        (CODE_3INST, 3, 1, 4112, 1024, 1024),   # m above 4096
                                                        (CODE_3INST, 2, 1, 64, 2048, 512)]):    # one launch, no scratch
        w, inp = layer_case(code_id, k, V, m, n, block, sub)
        y, y_ref = run_both(q, w, inp)
        assert np.all(np.isfinite(y))
        assert np.array_equal(y, y_ref), (m, n)
        check_against_oracle(w, inp, y)


def test_sizes_beyond_the_scratch_are_refused(q):
    import torch
    n = 65536 + 4096
    z = torch.zeros(n * 2, dtype=torch.int32, device="cuda")
    with pytest.raises(q.QtipError) as e:
        q.qtip_rht_decode_matvec_noalloc(z, 16, 2, 1, CODE_3INST, None, 16, n, z, z, 4096, None, z)
    assert e.value.code == -1 and "QTIP_NOALLOC_MAX_N" in str(e.value)
    # the largest size it takes
    w, inp = layer_case(CODE_3INST, 2, 1, 16, 65536, 4096, 7)
    y, y_ref = run_both(q, w, inp)
    assert np.array_equal(y, y_ref)
    # argument errors carry this entry point's name
    with pytest.raises(q.QtipError) as e:
        q.qtip_rht_decode_matvec_noalloc(z, 16, 2, 1, CODE_3INST, None, 16, 96, z, z, 64, None, z)
    assert e.value.code == -1 and "qtip_rht_decode_matvec_noalloc" in str(e.value)
