"""The bars the GPU products are held to, in one place.

REL_TOL is the stated bar: max|y - y*| / max|y*| <= 2e-3 against the fp64 product with the
oracle's fp16 code values.  OBSERVED_TOL (1e-4) is what fp32 accumulation of exact products
gives with margin; every kernel must meet it against the weights it contracts with:
  * all codes but 1MAD at batch 1: the fp16 code values themselves;
  * 1MAD at batch 1: Algorithm 1's unrounded quotient (s - 510) / 147.8 (the batch-1 kernel
    takes the affine map out of its loop and never rounds the quotient to fp16); against the
    fp16-rounded weights it then differs by the rounding of the weights, 2^-12 relative each,
    observed 2e-4 of the largest output on whole layers: UNROUNDED_TOL.
The element-wise form of the bar, |y - y*| <= 2e-3 |y*| + 2e-3 rms(y*), is asserted as well.
"""
import numpy as np

import oracle

REL_TOL = 2e-3
OBSERVED_TOL = 1e-4
UNROUNDED_TOL = 5e-4
CODE_1MAD = 0


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / np.abs(ref).max())


def assert_elementwise(got, ref):
    rms = float(np.sqrt((ref ** 2).mean()))
    excess = np.abs(got - ref) - (REL_TOL * np.abs(ref) + REL_TOL * rms)
    assert excess.max() <= 0.0, (float(excess.max()), int(excess.argmax()))


def takes_unrounded_weights(code_id, B):
    return code_id == CODE_1MAD and B == 1


def assert_products(got, Wref_bits, X, scale, code_id, codes=None, k=None, context=None):
    """got: (B, m) GPU outputs.  Wref_bits: the oracle's dense fp16 weights; X: (B, n) fp16;
    scale: per-row fp16 scale or None; codes, k: the stream, needed for 1MAD at batch 1."""
    got = np.asarray(got, dtype=np.float64)
    B = got.shape[0]
    ref = oracle.matmat_dense(Wref_bits, X, scale)
    err = rel_err(got, ref)
    if takes_unrounded_weights(code_id, B):
        m, n = Wref_bits.shape
        Wreal = oracle.dequantize_1mad_real(codes, k, m, n)
        ref_real = np.asarray(X, dtype=np.float16).astype(np.float64).reshape(B, n) @ Wreal.T
        if scale is not None:
            ref_real = ref_real * np.asarray(scale, dtype=np.float16).astype(np.float64)[None, :]
        err_real = rel_err(got, ref_real)
        assert err_real <= OBSERVED_TOL, (context, err_real)
        assert err <= REL_TOL and err <= UNROUNDED_TOL, (context, err)
    else:
        assert err <= REL_TOL and err <= OBSERVED_TOL, (context, err)
    assert_elementwise(got, ref)
    return err
