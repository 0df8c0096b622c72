"""GPU parity: every entry point of libqtip.so, called through the C ABI, against the
CPU oracle on the same seeded inputs.

Bars: decoded fp16 weights bit-exact; products within max relative error 2e-3 of
the fp64 oracle (fp32 accumulation), measured as max|y - y*| / max|y*|; the
Hadamard transform within fp16 rounding of the fp64 oracle.
"""
import numpy as np
import pytest

import oracle
import qtip_synth as synth
from parity_util import OBSERVED_TOL, REL_TOL, assert_products
from qtip_synth import CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB1, CODE_HYB2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def dev(a):
    import torch
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / np.abs(ref).max())


def run_dequantize(q, w, inp):
    import torch
    W = torch.empty((w.m, w.n), dtype=torch.float16, device="cuda")
    q.qtip_dequantize(dev(inp.codes), w.L, w.k, w.V, w.code_id, dev(inp.lut), w.m, w.n, W)
    torch.cuda.synchronize()
    return W.cpu().numpy().view(np.uint16)


def run_matmat(q, w, inp, use_matvec=False, scale=True):
    import torch
    Y = torch.full((w.B, w.m), float("nan"), dtype=torch.float32, device="cuda")
    codes, lut, X = dev(inp.codes), dev(inp.lut), dev(inp.X)
    sc = dev(inp.row_scale) if scale else None
    if use_matvec:
        assert w.B == 1 and sc is None
        q.qtip_decode_matvec(codes, w.L, w.k, w.V, w.code_id, lut, w.m, w.n, X, Y)
    else:
        q.qtip_decode_matmat(codes, w.L, w.k, w.V, w.code_id, lut, w.m, w.n, X, w.B, sc, Y)
    torch.cuda.synchronize()
    return Y.cpu().numpy().astype(np.float64)


ALL_CODECS = [(CODE_3INST, 2, 1), (CODE_3INST, 3, 1), (CODE_3INST, 4, 1),
              (CODE_1MAD, 2, 1), (CODE_1MAD, 3, 1), (CODE_1MAD, 4, 1),
              (CODE_HYB, 2, 2), (CODE_HYB, 3, 2), (CODE_HYB, 4, 2),
              (CODE_HYB2, 2, 2), (CODE_HYB2, 3, 2), (CODE_HYB2, 4, 2),
              (CODE_HYB1, 2, 1), (CODE_HYB1, 3, 1), (CODE_HYB1, 4, 1)]


def small_workload(code_id, k, V, m, n, B=1, row_scale=False, sub=0):
    return synth.Workload(f"small_{synth.CODE_NAMES[code_id]}_k{k}_{m}x{n}_b{B}", 9,
                          100 * code_id + 10 * k + sub, m, n, code_id, k, V, 16, 16, B=B,
                          row_scale=row_scale)


# ------------------------------------------------------------------ the codes

@pytest.mark.parametrize("code_id,V", [(CODE_1MAD, 1), (CODE_3INST, 1), (CODE_HYB, 2), (CODE_HYB2, 2), (CODE_HYB1, 1)])
def test_code_table_all_states_bit_exact(q, code_id, V):
    import torch
    rng = np.random.default_rng(42)
    lut = rng.standard_normal((512, 2)).astype(np.float16) if code_id in (CODE_HYB, CODE_HYB2) else None
    if code_id == CODE_HYB1:
        lut = rng.standard_normal(64).astype(np.float16)
    states = np.arange(65536, dtype=np.uint32)
    out = torch.zeros(65536 * V, dtype=torch.float16, device="cuda")
    q.qtip_decode_states(dev(states), 65536, 16, V, code_id, dev(lut), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16).reshape(65536, V)
    ref = oracle.codebook(16, V, code_id, lut).astype(np.float16).view(np.uint16)
    assert np.array_equal(got, ref)


def assert_batch1_weights(got, code_values, code_id, unrounded):
    """Weights brought out of the batch-1 kernel by one-hot activations.  Every code gives its
    fp16 code values exactly, except 1MAD, whose batch-1 kernel contracts with Algorithm 1's
    unrounded quotient: that must be the quotient to fp32 accuracy, and round to the code value."""
    if code_id != CODE_1MAD:
        assert np.array_equal(got, code_values)
        return
    real = unrounded()
    assert np.abs(got - real).max() <= 4e-7 * np.abs(real).max()
    assert np.array_equal(got.astype(np.float16).astype(np.float32), code_values)


def all_states_stream():
    """A 1024 x 256 matrix at k = 4, V = 1 whose streams carry every 16-bit state: tile t holds
    the 64 values 64 t .. 64 t + 63 as consecutive 16-bit pieces, which are the states of the
    sequence elements 0, 4, 8, ... (columns 0, 4, 8, 12 of every tile row)."""
    vals = np.arange(65536, dtype=np.uint32).reshape(1024, 32, 2)
    return (vals[:, :, 0] << 16) | vals[:, :, 1]           # MSB-first words: earlier piece in the high half


@pytest.mark.parametrize("code_id", [CODE_1MAD, CODE_3INST, CODE_HYB1])
def test_hot_loops_produce_the_code_values_for_every_state(q, code_id):
    """The batch-1 and the matrix-core kernels decode with instruction sequences of their own,
    not with the plain definitions behind qtip_decode_states and qtip_dequantize.  One-hot
    activations bring single weights out of them unchanged (w * 1 plus zeros, fp32): every
    one of the 2^16 states, through both kernels, must give exactly the oracle's code value."""
    import torch
    m, n, k = 1024, 256, 4
    rng = np.random.default_rng(77)
    lut = rng.standard_normal(64).astype(np.float16) if code_id == CODE_HYB1 else None
    codes = all_states_stream()
    Wref = oracle.dequantize(codes, 16, k, 1, code_id, m, n, lut).view(np.float16).astype(np.float32)
    C = oracle.codebook(16, 1, code_id, lut)[:, 0].astype(np.float32)
    cols = np.array([16 * J + c for J in range(16) for c in (0, 4, 8, 12)])
    # the construction does what it says: those columns hold all 2^16 code values, in order
    assert np.array_equal(Wref[:, cols].reshape(64, 16, 16, 4).transpose(0, 2, 1, 3).reshape(-1), C)
    X = np.zeros((64, n), dtype=np.float16)
    X[np.arange(64), cols] = 1.0
    dc, dl, dX = dev(codes), dev(lut), dev(X)
    Y = torch.full((64, m), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_decode_matmat(dc, 16, k, 1, code_id, dl, m, n, dX, 64, None, Y)
    y1 = torch.full((64, m), float("nan"), dtype=torch.float32, device="cuda")
    for b in range(64):
        q.qtip_decode_matvec(dc, 16, k, 1, code_id, dl, m, n, dX[b], y1[b])
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), Wref[:, cols].T)
    assert_batch1_weights(y1.cpu().numpy(), Wref[:, cols].T, code_id,
                          lambda: oracle.dequantize_1mad_real(codes, k, m, n)[:, cols].T)


@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
def test_hot_loops_produce_the_code_values_on_random_streams(q, code_id, k, V):
    """The same through every codec's own extraction (k = 2, 3, 4; V = 2 as well): random
    streams, one-hot activations for all 32 columns of a 512 x 32 matrix."""
    import torch
    m, n = 512, 32
    w = small_workload(code_id, k, V, m, n, sub=77)
    inp = synth.make_inputs(w)
    Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut).view(np.float16).astype(np.float32)
    X = np.eye(n, dtype=np.float16)
    dc, dl, dX = dev(inp.codes), dev(inp.lut), dev(X)
    Y = torch.full((n, m), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_decode_matmat(dc, 16, k, V, code_id, dl, m, n, dX, n, None, Y)
    y1 = torch.full((n, m), float("nan"), dtype=torch.float32, device="cuda")
    for b in range(n):
        q.qtip_decode_matvec(dc, 16, k, V, code_id, dl, m, n, dX[b], y1[b])
    torch.cuda.synchronize()
    assert np.array_equal(Y.cpu().numpy(), Wref.T)
    assert_batch1_weights(y1.cpu().numpy(), Wref.T, code_id,
                          lambda: oracle.dequantize_1mad_real(inp.codes, k, m, n).T)


# ----------------------------------------------------------------- dequantize

@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
@pytest.mark.parametrize("m,n", [(16, 16), (48, 1072), (160, 2064)])
def test_dequantize_small_bit_exact(q, code_id, k, V, m, n):
    w = small_workload(code_id, k, V, m, n)
    inp = synth.make_inputs(w)
    got = run_dequantize(q, w, inp)
    ref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
    assert np.array_equal(got, ref)


def test_dequantize_special_streams(q):
    # all-zero and all-one streams, and a single set bit that wraps around the tile end
    for code_id, k, V in [(CODE_3INST, 2, 1), (CODE_1MAD, 3, 1), (CODE_HYB, 4, 2), (CODE_HYB2, 2, 2)]:
        w = small_workload(code_id, k, V, 32, 32)
        inp = synth.make_inputs(w)
        for fill in (0, 0xFFFFFFFF):
            inp.codes[:] = fill
            ref = oracle.dequantize(inp.codes, 16, k, V, code_id, 32, 32, inp.lut)
            assert np.array_equal(run_dequantize(q, w, inp), ref)
        inp.codes[:] = 0
        inp.codes[:, 0] = 0x80000000     # first bit of each tile: seen by the last states
        inp.codes[:, -1] = 1             # last bit of each tile
        ref = oracle.dequantize(inp.codes, 16, k, V, code_id, 32, 32, inp.lut)
        assert np.array_equal(run_dequantize(q, w, inp), ref)


# ----------------------------------------------------------- matvec and matmat

@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
@pytest.mark.parametrize("m,n", [(16, 16), (48, 1072), (160, 4112)])
def test_matvec_small(q, code_id, k, V, m, n):
    w = small_workload(code_id, k, V, m, n)
    inp = synth.make_inputs(w)
    Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
    got = run_matmat(q, w, inp, use_matvec=True, scale=False)
    assert_products(got, Wref, inp.X, None, code_id, inp.codes, k)


@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
@pytest.mark.parametrize("B", [1, 3, 4, 8, 9, 15, 16, 17, 40, 64, 80])
def test_matmat_small_with_row_scale(q, code_id, k, V, B):
    m, n = 64, 1104
    w = small_workload(code_id, k, V, m, n, B=B, row_scale=True, sub=B)
    inp = synth.make_inputs(w)
    Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
    got = run_matmat(q, w, inp)
    assert_products(got, Wref, inp.X, inp.row_scale, code_id, inp.codes, k)
    assert_products(run_matmat(q, w, inp, scale=False), Wref, inp.X, None, code_id, inp.codes, k)


@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
@pytest.mark.parametrize("m,n,B", [(304, 1104, 16), (304, 4112, 33), (1040, 1104, 64), (272, 8208, 80)])
def test_matmat_large_batch_staged_activations(q, code_id, k, V, m, n, B):
    """Batches above 8 take the path that transposes activations through LDS: odd numbers of
    tile rows, row bands whose last step is partial (n/16 not a multiple of 4 per wave),
    ragged batch tails, and Y pre-filled with NaN by run_matmat."""
    w = small_workload(code_id, k, V, m, n, B=B, row_scale=True, sub=B + 1)
    inp = synth.make_inputs(w)
    Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
    ref = oracle.matmat_dense(Wref, inp.X, inp.row_scale)
    got = run_matmat(q, w, inp)
    err = rel_err(got, ref)
    assert err <= REL_TOL and err <= OBSERVED_TOL, err
    assert np.array_equal(run_matmat(q, w, inp), got)  # fixed summation order


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("n", [8192, 8208, 16400])
def test_hyb_long_rows_use_the_spread_table(q, k, n):
    """From 8192 columns on the HYB kernels read a table held in 16 copies (batch 1, and 9 to 16
    batch rows on the matrix cores); same weights, so the same bars, and the same bits as the
    one-copy kernel wherever the summation order is the same (batch 1)."""
    m = 48
    for B in (1, 9, 16):
        w = small_workload(CODE_HYB, k, 2, m, n, B=B, row_scale=B > 1, sub=60 + B)
        inp = synth.make_inputs(w)
        Wref = oracle.dequantize(inp.codes, 16, k, 2, CODE_HYB, m, n, inp.lut)
        ref = oracle.matmat_dense(Wref, inp.X, inp.row_scale)
        got = run_matmat(q, w, inp)
        err = rel_err(got, ref)
        assert err <= REL_TOL and err <= OBSERVED_TOL, (B, err)
        assert np.array_equal(run_matmat(q, w, inp), got)


def test_stacked_matrices_are_one_launch(q):
    """Matrices that share an input (q/k/v, up/gate: the matrix fusion of the paper's
    generation-speed runs) are stacked along the rows: tile rows are independent and contiguous in the code buffer, so the
    concatenated buffers are one valid matrix and one launch gives the concatenated outputs."""
    n = 2064
    parts, refs = [], []
    X = None
    for sub, m in enumerate((64, 16, 112)):
        w = small_workload(CODE_3INST, 2, 1, m, n, sub=40 + sub)
        inp = synth.make_inputs(w)
        X = inp.X if X is None else X
        inp.X = X
        parts.append(inp.codes)
        refs.append(run_matmat(q, w, inp, use_matvec=True, scale=False))
    w = small_workload(CODE_3INST, 2, 1, 192, n)
    inp = synth.make_inputs(w)
    inp.codes = np.concatenate(parts, axis=0)
    inp.X = X
    got = run_matmat(q, w, inp, use_matvec=True, scale=False)
    assert np.array_equal(got, np.concatenate(refs, axis=1))
    Wref = oracle.dequantize(inp.codes, 16, 2, 1, CODE_3INST, 192, n, None)
    assert rel_err(got, oracle.matmat_dense(Wref, X)) <= OBSERVED_TOL


FULL = ["cfg1_3inst_k2_1024x1024", "cfg2_3inst_k2_4096x4096", "cfg3_1mad_k2_14336x4096",
        "cfg3_1mad_k3_14336x4096", "cfg3_1mad_k4_14336x4096", "cfg3_1mad_k2_4096x14336",
        "cfg3_1mad_k3_4096x14336", "cfg3_1mad_k4_4096x14336", "cfg4_hyb_k2_8192x28672",
        "cfg5_hyb_k4_8192x8192_b1", "cfg5_hyb_k4_8192x8192_b4", "cfg5_hyb_k4_8192x8192_b16",
        "cfg5_hyb_k4_8192x8192_b64", "metric_3inst_k2_8192x28672", "next_hyb2_k2_8192x28672",
        "next_hyb1_k2_8192x28672"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_configs(q, name):
    """The configured shapes in the launch configuration the benchmark times: every decoded
    weight (bit patterns) and every output against the oracle's whole-matrix decode and its
    fp64 dense product."""
    import gc
    w = synth.WORKLOADS[name]
    inp = synth.make_inputs(w)
    ref_W = oracle.dequantize(inp.codes, 16, w.k, w.V, w.code_id, w.m, w.n, inp.lut)
    got_W = run_dequantize(q, w, inp)
    assert got_W.shape == ref_W.shape and np.array_equal(got_W, ref_W)
    del got_W
    got = run_matmat(q, w, inp)
    assert got.shape == (w.B, w.m) and np.all(np.isfinite(got))
    assert_products(got, ref_W, inp.X, inp.row_scale, w.code_id, inp.codes, w.k, context=name)
    del ref_W
    gc.collect()
    if w.B == 1 and not w.row_scale:
        got_mv = run_matmat(q, w, inp, use_matvec=True, scale=False)
        assert np.array_equal(got_mv, got)          # same kernel, deterministic


@pytest.mark.parametrize("code_id,k,V", [(CODE_3INST, 4, 1), (CODE_HYB, 4, 2)])
def test_offsets_beyond_32_bits(q, code_id, k, V):
    """98304 x 98304 at 4 bits: 4.8 GB of codes (byte offsets pass 2^32, word offsets 2^30),
    9.7e9 weights (element offsets pass 2^33).  The stream is drawn on the device; the oracle
    gets the tile rows of the sampled outputs, the last tile row among them, and decodes those
    rows one element at a time."""
    import torch
    m = n = 98304
    tn, nw = n // 16, 8 * k
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + code_id)
    codes = torch.randint(-2 ** 31, 2 ** 31 - 1, ((m // 16) * tn, nw), dtype=torch.int32, device="cuda",
                          generator=gen)
    rng = np.random.default_rng(77 + code_id)
    lut_h = rng.standard_normal((512, 2)).astype(np.float16) if code_id == CODE_HYB else None
    lut = dev(lut_h)
    X_h = rng.standard_normal((3, n)).astype(np.float16)
    X = dev(X_h)
    rows = np.array([5, 43690, 43691, 65535, 65536, 87381, m - 1])   # around 2^31 and 2^32 elements, and the end
    W = torch.empty((m, n), dtype=torch.float16, device="cuda")
    q.qtip_dequantize(codes, 16, k, V, code_id, lut, m, n, W)
    y = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_decode_matvec(codes, 16, k, V, code_id, lut, m, n, X[0], y)
    Y = torch.full((3, m), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_decode_matmat(codes, 16, k, V, code_id, lut, m, n, X, 3, None, Y)
    torch.cuda.synchronize()
    y_h, Y_h = y.cpu().numpy(), Y.cpu().numpy()
    assert np.all(np.isfinite(y_h)) and np.all(np.isfinite(Y_h))
    refs = []
    for i in rows:
        I, r = int(i) // 16, int(i) % 16
        band = codes[I * tn:(I + 1) * tn].cpu().numpy().view(np.uint32)        # this tile row's streams
        cols = list(range(0, n, 997)) + [n - 2, n - 1]
        want = np.array([oracle.decode_element(band, 16, k, V, code_id, n, r, j, lut_h) for j in cols],
                        dtype=np.uint16)
        got = W[int(i)].cpu().numpy().view(np.uint16)[cols]
        assert np.array_equal(got, want), i
        refs.append(oracle.decode_matmat_rows(band, 16, k, V, code_id, 16, n, X_h, [r], lut_h)[:, 0])
    ref = np.stack(refs, axis=1)                                                 # (3, len(rows))
    err = float(np.abs(Y_h[:, rows] - ref).max() / np.abs(ref).max())
    assert err <= REL_TOL and err <= OBSERVED_TOL, err
    err = float(np.abs(y_h[rows] - ref[0]).max() / np.abs(ref[0]).max())
    assert err <= REL_TOL and err <= OBSERVED_TOL, err


# ------------------------------------------------------------------ Hadamard

@pytest.mark.parametrize("block", [16, 32, 64, 256, 1024, 2048, 4096, 8192, 16384])
@pytest.mark.parametrize("side", [0, 1])
def test_rht_against_explicit_matrix(q, block, side):
    import torch
    rng = np.random.default_rng(block + side)
    nblk = 3 if block <= 4096 else 1
    batch = 2 if block <= 4096 else 1
    n = block * nblk
    x = rng.standard_normal((batch, n)).astype(np.float16)
    s = (rng.integers(0, 2, n) * 2 - 1).astype(np.int8)
    ref = oracle.rht(x, s, block, side)
    out = torch.zeros((batch, n), dtype=torch.float16, device="cuda")
    q.qtip_rht(dev(x), dev(s), n, block, batch, side, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # one fp16 rounding of an fp32 result
    assert np.all(np.abs(got - ref) <= 2.0 ** -11 * np.abs(ref) + 1e-5 * np.abs(ref).max())
    # fp32 input variant, and in-place operation of the fp16 variant
    out2 = torch.zeros((batch, n), dtype=torch.float16, device="cuda")
    q.qtip_rht_f32(dev(x.astype(np.float32)), dev(s), n, block, batch, side, out2)
    xin = dev(x)
    q.qtip_rht(xin, dev(s), n, block, batch, side, xin)
    torch.cuda.synchronize()
    assert torch.equal(out2, out) and torch.equal(xin, out)


@pytest.mark.parametrize("block,nblk", [(16, 517), (64, 131), (256, 43), (1024, 9), (2048, 3)])
def test_rht_many_small_blocks(q, block, nblk):
    """Blocks below 4096 share a workgroup (as many as make 4096 values): block counts that
    leave the last workgroup partly empty, both sides (11008 = 43 x 256 is a Llama width)."""
    import torch
    rng = np.random.default_rng(block + nblk)
    n = block * nblk
    x = rng.standard_normal((3, n)).astype(np.float16)
    s = (rng.integers(0, 2, n) * 2 - 1).astype(np.int8)
    for side in (0, 1):
        ref = oracle.rht(x, s, block, side)
        out = torch.full((3, n), float("nan"), dtype=torch.float16, device="cuda")
        q.qtip_rht(dev(x), dev(s), n, block, 3, side, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 2.0 ** -11 * np.abs(ref) + 1e-5 * np.abs(ref).max())


def test_full_layer_composition(q):
    """y = S_m V_m^T (scale .* (W~ (V_n S_n x))) on config 1, GPU end to end vs oracle."""
    import torch
    w = synth.WORKLOADS["cfg1_3inst_k2_1024x1024"]
    inp = synth.make_inputs(w)
    xt = torch.empty((1, w.n), dtype=torch.float16, device="cuda")
    q.qtip_rht(dev(inp.X), dev(inp.signs_n), w.n, w.block_n, 1, 0, xt)
    z = torch.empty((1, w.m), dtype=torch.float32, device="cuda")
    q.qtip_decode_matmat(dev(inp.codes), 16, w.k, w.V, w.code_id, None, w.m, w.n, xt, 1,
                         dev(inp.row_scale), z)
    y = torch.empty((1, w.m), dtype=torch.float16, device="cuda")
    q.qtip_rht_f32(z, dev(inp.signs_m), w.m, w.block_m, 1, 1, y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    # oracle, all in fp64 except where the method itself rounds (the fp16 activation)
    xt_ref = oracle.rht(inp.X, inp.signs_n, w.block_n, 0)
    Wd = oracle.dequantize(inp.codes, 16, w.k, w.V, w.code_id, w.m, w.n).view(np.float16)
    Wd = Wd.astype(np.float64)
    z_ref = (Wd @ xt_ref.reshape(-1)) * inp.row_scale.astype(np.float64)
    H = oracle.hadamard(w.block_m).astype(np.float64) / np.sqrt(w.block_m)
    y_ref = inp.signs_m * (H.T @ z_ref)
    assert rel_err(got, y_ref.reshape(1, -1)) <= REL_TOL
    # and the algebra of Section 2.1: the same as the dense product with
    # W = S_m V_m^T W~ V_n S_n
    Hn = oracle.hadamard(w.block_n).astype(np.float64) / np.sqrt(w.block_n)
    Wfull = (inp.signs_m[:, None] * (H.T @ (inp.row_scale.astype(np.float64)[:, None] * Wd))
             @ Hn) * inp.signs_n[None, :]
    y_dense = Wfull @ inp.X.astype(np.float64).reshape(-1)
    assert np.allclose(y_ref, y_dense, rtol=1e-9, atol=1e-9)


# ---------------------------------------------------------------- error paths

@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
@pytest.mark.parametrize("m,n,block", [(48, 1024, 256), (160, 4096, 4096), (32, 8192, 2048), (16, 16, 16),
                                       (32, 6144, 2048), (32, 12288, 4096), (4112, 64, 64)])
def test_rht_decode_matvec_equals_the_two_calls(q, code_id, k, V, m, n, block):
    """The call that transforms its own input: one launch up to n = 8192 and m = 4096 (every
    workgroup transforms x in LDS), two launches above; the same bits as qtip_rht followed by
    the product either way, and the oracle's layer within the bar."""
    import torch
    w = small_workload(code_id, k, V, m, n, row_scale=True, sub=3)
    inp = synth.make_inputs(w)
    rng = np.random.default_rng(n + m)
    signs = rng.choice(np.array([-1, 1], dtype=np.int8), n)
    codes, lut, X, sc, sg = dev(inp.codes), dev(inp.lut), dev(inp.X), dev(inp.row_scale), dev(signs)
    xt = torch.empty((1, n), dtype=torch.float16, device="cuda")
    y2 = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_rht(X, sg, n, block, 1, 0, xt)
    q.qtip_decode_matmat(codes, 16, k, V, code_id, lut, m, n, xt, 1, sc, y2)
    y1 = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
    two_launches = n > 8192 or m > 4096
    scratch = torch.empty(n, dtype=torch.float16, device="cuda") if two_launches else None
    q.qtip_rht_decode_matvec(codes, 16, k, V, code_id, lut, m, n, X, sg, block, sc, y1, scratch)
    torch.cuda.synchronize()
    assert np.array_equal(y1.cpu().numpy(), y2.cpu().numpy())
    Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
    xt_ref = oracle.rht(inp.X, signs, block, 0).astype(np.float16)      # the layer rounds x~ to fp16
    ref = oracle.matmat_dense(Wref, xt_ref, inp.row_scale)[0]
    err = np.abs(y1.cpu().numpy() - ref).max() / np.abs(ref).max()
    assert err <= REL_TOL, err
    if two_launches:
        with pytest.raises(q.QtipError):
            q.qtip_rht_decode_matvec(codes, 16, k, V, code_id, lut, m, n, X, sg, block, sc, y1, None)


def test_gpu_error_codes(q):
    import torch
    w = small_workload(CODE_3INST, 2, 1, 32, 32)
    inp = synth.make_inputs(w)
    codes, x = dev(inp.codes), dev(inp.X)
    y = torch.zeros(32, dtype=torch.float32, device="cuda")
    with pytest.raises(q.QtipError) as e:
        q.qtip_decode_matvec(codes, 16, 2, 1, CODE_3INST, None, 32, 24, x, y)
    assert e.value.code == -1
    with pytest.raises(q.QtipError) as e:
        q.qtip_decode_matvec(codes, 12, 2, 1, CODE_3INST, None, 32, 32, x, y)
    assert e.value.code == -2
    with pytest.raises(q.QtipError) as e:
        q.qtip_decode_matvec(codes, 16, 2, 2, CODE_HYB, None, 32, 32, x, y)
    assert e.value.code == -1
    # a misaligned code pointer is refused, not dereferenced
    with pytest.raises(q.QtipError):
        q.qtip_decode_matvec(codes.data_ptr() + 4, 16, 2, 1, CODE_3INST, None, 32, 32, x, y)
    torch.cuda.synchronize()
    q.qtip_decode_matvec(codes, 16, 2, 1, CODE_3INST, None, 32, 32, x, y)
    torch.cuda.synchronize()
    assert torch.isfinite(y).all()


def test_quantize_roundtrip_on_gpu(q):
    """Streams made by the host quantizer decode on the GPU to what it promised."""
    rng = np.random.default_rng(5)
    for code_id, k, V in [(CODE_3INST, 2, 1), (CODE_HYB, 2, 2)]:
        lut = rng.standard_normal((512, 2)).astype(np.float16) if code_id == CODE_HYB else None
        sd = oracle.codebook(16, V, code_id, lut).std()
        Wsrc = (rng.standard_normal((32, 32)) * sd).astype(np.float32)
        codes, mse = q.qtip_quantize(Wsrc, 32, 32, 16, k, V, code_id, lut)
        w = small_workload(code_id, k, V, 32, 32)
        inp = synth.make_inputs(w)
        inp.codes, inp.lut = codes, lut
        got = run_dequantize(q, w, inp).view(np.float16).astype(np.float64)
        assert abs(((got - Wsrc) ** 2).mean() - mse) < 1e-9
        assert mse / sd ** 2 < 0.09


# ------------------------------------------------------------ randomized shapes

def test_random_shapes_all_entry_points(q):
    """Seeded random (m, n, B, codec) cases: ragged tile counts, every wave-count variant."""
    rng = np.random.default_rng(20240611)
    for case in range(24):
        code_id, k, V = ALL_CODECS[int(rng.integers(0, len(ALL_CODECS)))]
        m = 16 * int(rng.integers(1, 12))
        n = 16 * int(rng.choice([1, 3, 7, 17, 33, 65, 129, 257, 1025]))
        B = int(rng.choice([1, 1, 2, 5, 16, 31, 33]))
        w = small_workload(code_id, k, V, m, n, B=B, row_scale=bool(case % 2), sub=case)
        inp = synth.make_inputs(w, seed=w.seed + 17 * case)
        Wref = oracle.dequantize(inp.codes, 16, k, V, code_id, m, n, inp.lut)
        assert np.array_equal(run_dequantize(q, w, inp), Wref), (case, m, n, k)
        assert_products(run_matmat(q, w, inp), Wref, inp.X, inp.row_scale, code_id, inp.codes, k,
                        context=(case, m, n, B, k))


def test_extreme_table_values_do_not_leak_into_dead_lanes(q):
    """HYB tables may hold infinities: lanes past the end of a ragged row must not add inf*0."""
    w = small_workload(CODE_HYB, 2, 2, 32, 16 * 19, B=1)
    inp = synth.make_inputs(w)
    inp.lut[7, 0] = np.float16(np.inf)          # one entry; find rows that never use it
    Wref = oracle.dequantize(inp.codes, 16, 2, 2, CODE_HYB, w.m, w.n, inp.lut)
    finite_rows = np.all(np.isfinite(Wref.view(np.float16)), axis=1)
    got = run_matmat(q, w, inp, use_matvec=True, scale=False)[0]
    assert np.all(np.isfinite(got[finite_rows]))
    inp.lut[7, 0] = np.float16(0.5)
    Wref = oracle.dequantize(inp.codes, 16, 2, 2, CODE_HYB, w.m, w.n, inp.lut)
    ref = oracle.matmat_dense(Wref, inp.X)
    assert rel_err(run_matmat(q, w, inp, use_matvec=True, scale=False), ref) <= OBSERVED_TOL


def test_stream_argument_is_honoured(q):
    import torch
    w = small_workload(CODE_3INST, 2, 1, 64, 512)
    inp = synth.make_inputs(w)
    s = torch.cuda.Stream()
    y = torch.zeros(w.m, dtype=torch.float32, device="cuda")
    codes, x = dev(inp.codes), dev(inp.X)
    torch.cuda.synchronize()
    q.qtip_decode_matvec(codes, 16, 2, 1, CODE_3INST, None, w.m, w.n, x, y, stream=s)
    s.synchronize()
    Wref = oracle.dequantize(inp.codes, 16, 2, 1, CODE_3INST, w.m, w.n)
    ref = oracle.matmat_dense(Wref, inp.X)[0]
    assert rel_err(y.cpu().numpy().astype(np.float64), ref) <= OBSERVED_TOL
