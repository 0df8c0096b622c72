"""GPU parity for the lookup-only code (L = 14, V = 1, a stored table of 2^14 fp16 values,
32 x 8 blocks): decode, batch-1 product, batched product on the matrix cores and the layer
call, through the C ABI, against the CPU oracle on the same seeded inputs.

Bars as for the other codes: decoded fp16 weights bit-exact; products within max relative
error 2e-3 of the fp64 oracle, measured as max|y - y*| / max|y*|."""
import numpy as np
import pytest

import oracle
import qtip_synth as synth
from qtip_synth import CODE_LUT

pytestmark = pytest.mark.gpu

REL_TOL = 2e-3
OBSERVED_TOL = 1e-4
TILE = (32, 8)


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


def workload(k, m, n, B=1, row_scale=False, sub=0):
    return synth.Workload(f"small_LUT14_k{k}_{m}x{n}_b{B}", 9, 400 + 10 * k + sub, m, n, CODE_LUT, k, 1, 16, 16,
                          B=B, row_scale=row_scale, L=14)


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


def ref_weights(w, inp):
    return oracle.dequantize(inp.codes, 14, w.k, 1, CODE_LUT, w.m, w.n, inp.lut, tile=TILE)


def test_every_state_reads_its_table_entry(q):
    import torch
    rng = np.random.default_rng(14)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    states = np.arange(1 << 14, dtype=np.uint32)
    out = torch.empty(1 << 14, dtype=torch.float16, device="cuda")
    q.qtip_decode_states(dev(states), states.size, 14, 1, CODE_LUT, dev(lut), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), lut.view(np.uint16))


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("m,n", [(32, 8), (96, 1080), (160, 2072)])
def test_dequantize_small_bit_exact(q, k, m, n):
    w = workload(k, m, n)
    inp = synth.make_inputs(w)
    assert np.array_equal(run_dequantize(q, w, inp), ref_weights(w, inp))


@pytest.mark.parametrize("k", [2, 3, 4])
def test_dequantize_special_streams(q, k):
    # all-zero and all-one streams, and single set bits around the block's end (the wrap)
    m, n = 32, 24
    w = workload(k, m, n)
    inp = synth.make_inputs(w)
    for fill in (0, 0xFFFFFFFF):
        inp.codes[:] = fill
        assert np.array_equal(run_dequantize(q, w, inp), ref_weights(w, inp))
    for word, bit in [(8 * k - 1, 0), (8 * k - 1, 5), (0, 31), (0, 20), (3, 16)]:
        inp.codes[:] = 0
        inp.codes[1, word] = np.uint32(1 << bit)
        assert np.array_equal(run_dequantize(q, w, inp), ref_weights(w, inp))


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("m,n", [(32, 8), (96, 1080), (160, 4104), (64, 16392)])
def test_matvec_small(q, k, m, n):
    w = workload(k, m, n)
    inp = synth.make_inputs(w)
    ref = oracle.matmat_dense(ref_weights(w, inp), inp.X)
    got = run_matmat(q, w, inp, use_matvec=True, scale=False)
    err = rel_err(got, ref)
    assert err <= REL_TOL and err <= OBSERVED_TOL, err
    assert np.array_equal(run_matmat(q, w, inp, use_matvec=True, scale=False), got)  # fixed summation order


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("B", [1, 2, 5, 16, 31, 32, 33, 64, 65, 130])
def test_matmat_small_with_row_scale(q, k, B):
    m, n = 96, 1112
    w = workload(k, m, n, B=B, row_scale=True, sub=B)
    inp = synth.make_inputs(w)
    Wref = ref_weights(w, inp)
    ref = oracle.matmat_dense(Wref, inp.X, inp.row_scale)
    got = run_matmat(q, w, inp)
    err = rel_err(got, ref)
    assert err <= REL_TOL and err <= OBSERVED_TOL, err
    assert rel_err(run_matmat(q, w, inp, scale=False), oracle.matmat_dense(Wref, inp.X)) <= OBSERVED_TOL


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("m,n,B", [(288, 1112, 16), (1056, 8, 7), (32, 4104, 40), (64, 8, 96)])
def test_matmat_ragged_shapes(q, k, m, n, B):
    """Waves with no blocks at all (n = 8), odd block counts per wave, ragged batch tails."""
    w = workload(k, m, n, B=B, row_scale=True, sub=B + 1)
    inp = synth.make_inputs(w)
    ref = oracle.matmat_dense(ref_weights(w, inp), inp.X, inp.row_scale)
    err = rel_err(run_matmat(q, w, inp), ref)
    assert err <= REL_TOL and err <= OBSERVED_TOL, err


def test_layer_call_equals_the_two_calls(q):
    import torch
    w = workload(2, 64, 2048, row_scale=True, sub=3)
    inp = synth.make_inputs(w)
    rng = np.random.default_rng(77)
    signs = rng.choice(np.array([-1, 1], dtype=np.int8), w.n)
    codes, lut, X, sc, sg = dev(inp.codes), dev(inp.lut), dev(inp.X), dev(inp.row_scale), dev(signs)
    xt = torch.empty((1, w.n), dtype=torch.float16, device="cuda")
    q.qtip_rht(X, sg, w.n, 512, 1, 0, xt)
    y2 = torch.empty((1, w.m), dtype=torch.float32, device="cuda")
    q.qtip_decode_matmat(codes, 14, 2, 1, CODE_LUT, lut, w.m, w.n, xt, 1, sc, y2)
    y1 = torch.full((w.m,), float("nan"), dtype=torch.float32, device="cuda")
    scratch = torch.empty(w.n, dtype=torch.float16, device="cuda")
    q.qtip_rht_decode_matvec(codes, 14, 2, 1, CODE_LUT, lut, w.m, w.n, X, sg, 512, sc, y1, scratch)
    torch.cuda.synchronize()
    assert np.array_equal(y1.cpu().numpy(), y2.cpu().numpy()[0])
    with pytest.raises(q.QtipError):  # this code always takes two launches
        q.qtip_rht_decode_matvec(codes, 14, 2, 1, CODE_LUT, lut, w.m, w.n, X, sg, 512, sc, y1, None)


def assert_products_match(got, ref):
    err = float(np.abs(got - ref).max() / np.abs(ref).max())
    assert err <= REL_TOL and err <= OBSERVED_TOL, err
    rms = float(np.sqrt((ref ** 2).mean()))
    excess = np.abs(got - ref) - (REL_TOL * np.abs(ref) + REL_TOL * rms)
    assert excess.max() <= 0.0, (float(excess.max()), int(excess.argmax()))


def test_full_size(q):
    """The 2-bit 8192 x 28672 shape in the launch configuration the benchmark times: every
    decoded weight and every output, batch 1 and batched on the matrix cores, against the
    oracle's whole-matrix decode and fp64 dense product."""
    import gc
    w = synth.WORKLOADS["next_lut14_k2_8192x28672"]
    inp = synth.make_inputs(w)
    ref_W = ref_weights(w, inp)
    got_W = run_dequantize(q, w, inp)
    assert np.array_equal(got_W, ref_W)
    del got_W
    ref = oracle.matmat_dense(ref_W, inp.X)
    got = run_matmat(q, w, inp)
    assert np.all(np.isfinite(got))
    assert_products_match(got, ref)
    # batched, on the matrix cores, same shape and weights
    w16 = synth.Workload("lut14_b16", 7, 0, w.m, w.n, CODE_LUT, 2, 1, 4096, 4096, B=16, L=14)
    inp16 = synth.make_inputs(w16)
    assert np.array_equal(inp16.codes, inp.codes) and np.array_equal(inp16.lut, inp.lut)
    ref = oracle.matmat_dense(ref_W, inp16.X)
    del ref_W
    gc.collect()
    got = run_matmat(q, w16, inp16)
    assert_products_match(got, ref)


def test_error_codes(q):
    import torch
    w = workload(2, 32, 64)
    inp = synth.make_inputs(w)
    codes, lut, X = dev(inp.codes), dev(inp.lut), dev(inp.X)
    Y = torch.empty((1, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(q.QtipError, match="L = 16"):
        q.qtip_decode_matvec(codes, 16, 2, 1, CODE_LUT, lut, 32, 64, X, Y)
    with pytest.raises(q.QtipError, match="lut"):
        q.qtip_decode_matvec(codes, 14, 2, 1, CODE_LUT, None, 32, 64, X, Y)
    with pytest.raises(q.QtipError, match="multiple of 32"):
        q.qtip_decode_matvec(codes, 14, 2, 1, CODE_LUT, lut, 16, 64, X, Y)
    with pytest.raises(q.QtipError, match="V = 2"):
        q.qtip_decode_matvec(codes, 14, 2, 2, CODE_LUT, lut, 32, 64, X, Y)
    with pytest.raises(q.QtipError, match="L = 14"):
        q.qtip_decode_matvec(codes, 14, 2, 1, synth.CODE_3INST, None, 32, 64, X, Y)
    H = torch.eye(32, dtype=torch.float64, device="cuda")
    A = torch.zeros((32, 32), dtype=torch.float32, device="cuda")
    ws = torch.empty(q.qtip_block_ldl_workspace(32), dtype=torch.uint8, device="cuda")
    with pytest.raises(q.QtipError, match="8 or 16"):
        q.qtip_block_ldl(H, 32, 12, A, None, ws, ws.numel())


# ------------------------------------------------------------------ quantizer

def run_quantize_gpu(q, W, k, lut, tiles_in_flight=None):
    import torch
    m, n = W.shape
    ntiles = (m // 32) * (n // 8)
    ws_bytes = q.qtip_quantize_gpu_workspace(k, 1, tiles_in_flight or ntiles)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_gpu(dev(np.ascontiguousarray(W, dtype=np.float32)), m, n, 14, k, 1, CODE_LUT, dev(lut), codes,
                        err, ws, ws_bytes)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32), err.cpu().numpy()


@pytest.mark.parametrize("k", [2, 3, 4])
def test_quantizer_streams_equal_the_binary32_oracle(q, k):
    """The search runs in binary32 with a fixed operation order, which the oracle repeats
    decision by decision (Section 2.3, Algorithm 4): streams and final values bit for bit."""
    rng = np.random.default_rng(1400 + k)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    C = oracle.codebook(14, 1, CODE_LUT, lut)
    m, n = 64, 16
    W = rng.standard_normal((m, n)).astype(np.float32)
    codes, err = run_quantize_gpu(q, W, k, lut)
    for I in range(m // 32):
        for J in range(n // 8):
            S = W[32 * I:32 * I + 32, 8 * J:8 * J + 8].reshape(-1)
            d, words = oracle.tailbiting_quantize_f32(S, 14, k, 1, C)
            assert np.array_equal(codes[I * (n // 8) + J], words), (I, J)
            assert err[I * (n // 8) + J] == d


def test_quantizer_degenerate_blocks_equal_the_binary32_oracle(q):
    """Blocks of zeros, of one constant, of weights 30 times the table's spread and with one
    outlier of 1e4: streams and final values bit for bit."""
    k = 2
    rng = np.random.default_rng(1450)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    C = oracle.codebook(14, 1, CODE_LUT, lut)
    outlier = rng.standard_normal((32, 8))
    outlier[rng.integers(32), rng.integers(8)] = 1e4
    blocks = [np.zeros((32, 8)), np.full((32, 8), 0.37), rng.standard_normal((32, 8)) * 30, outlier]
    W = np.concatenate(blocks, axis=1).astype(np.float32)
    codes, err = run_quantize_gpu(q, W, k, lut)
    for J in range(len(blocks)):
        d, words = oracle.tailbiting_quantize_f32(W[:, 8 * J:8 * J + 8].reshape(-1), 14, k, 1, C)
        assert np.array_equal(codes[J], words), J
        assert err[J] == d


def test_quantizer_roundtrip_and_distortion(q):
    """Weights that are decodable come back exactly; on Gaussian input every block's reported
    error is the binary64 distortion of its own stream, and the mean squared error agrees with
    the binary64 host search (equally good streams may differ, the distortion may not by more
    than binary32 rounding)."""
    rng = np.random.default_rng(1414)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    C = oracle.codebook(14, 1, CODE_LUT, lut)
    m, n, k = 64, 24, 2
    codes = rng.integers(0, 1 << 32, ((m // 32) * (n // 8), 8 * k), dtype=np.uint64).astype(np.uint32)
    W = oracle.dequantize(codes, 14, k, 1, CODE_LUT, m, n, lut, tile=TILE).view(np.float16).astype(np.float32)
    codes2, err = run_quantize_gpu(q, W, k, lut)
    assert np.all(err == 0.0)
    W2 = oracle.dequantize(codes2, 14, k, 1, CODE_LUT, m, n, lut, tile=TILE).view(np.float16).astype(np.float32)
    assert np.array_equal(W, W2)
    m, n = 128, 64   # 32 blocks, two batches of 20 and 12
    W = rng.standard_normal((m, n)).astype(np.float32)
    codes, err = run_quantize_gpu(q, W, k, lut, tiles_in_flight=20)
    tot = 0.0
    for I in range(m // 32):
        for J in range(n // 8):
            S = W[32 * I:32 * I + 32, 8 * J:8 * J + 8].reshape(-1).astype(np.float64)
            d = oracle.stream_distortion(codes[I * (n // 8) + J], S, 14, k, 1, C)
            assert abs(err[I * (n // 8) + J] - d) <= 1e-4 * d
            tot += d
    mse = tot / (m * n)
    _, mse_host = q.qtip_quantize(W, m, n, 14, k, 1, CODE_LUT, lut)
    assert abs(mse - mse_host) <= 2e-3 * mse_host, (mse, mse_host)
    # between Table 1's L = 16 random-table entry (0.068) and Table 2's L = 12 entry (0.0733), give or
    # take the noise of 8192 samples
    assert 0.066 < mse < 0.076, mse


# ------------------------------------------------------------------ BlockLDLQ, T_y = 8

def random_spd(rng, n, samples=None, corr=0.9):
    samples = samples or 4 * n
    base = rng.standard_normal((samples, 1))
    X = corr * base + (1 - corr) * rng.standard_normal((samples, n))
    X = X * rng.uniform(0.5, 2.0, n)[None, :]
    return X.T @ X / samples + 1e-3 * np.eye(n)


def run_block_ldl8(q, H):
    import torch
    n = H.shape[0]
    A = torch.full((n, n), float("nan"), dtype=torch.float32, device="cuda")
    D = torch.full((n // 8, 8, 8), float("nan"), dtype=torch.float64, device="cuda")
    wsb = q.qtip_block_ldl_workspace(n)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    q.qtip_block_ldl(dev(np.ascontiguousarray(H, dtype=np.float64)), n, 8, A, D, ws, wsb)
    torch.cuda.synchronize()
    return A.cpu().numpy(), D.cpu().numpy()


def run_ldlq(q, W, A, k, lut, tiles=None):
    import torch
    m, n = W.shape
    ntiles = (m // 32) * (n // 8)
    wsb = q.qtip_quantize_ldlq_workspace(m, n, k, 1, tiles or m // 32)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    What = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_ldlq(dev(np.ascontiguousarray(W, dtype=np.float32)), dev(np.ascontiguousarray(A, dtype=np.float32)),
                         m, n, 14, k, 1, CODE_LUT, dev(lut), codes, What, err, ws, wsb)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32), What.cpu().numpy(), err.cpu().numpy()


@pytest.mark.parametrize("n", [16, 48, 272])
def test_block_ldl_with_groups_of_8(q, n):
    rng = np.random.default_rng(800 + n)
    H = random_spd(rng, n)
    A, D = run_block_ldl8(q, H)
    Lm, Dref = oracle.block_ldl(H, 8)
    Aref = Lm - np.eye(n)
    assert np.all(np.isfinite(A)) and np.all(np.isfinite(D))
    for j in range(n // 8):
        assert np.all(A[8 * j:8 * j + 8, 8 * j:] == 0)
    assert np.abs(A - Aref).max() <= 1e-6 * max(1.0, np.abs(Aref).max())
    assert np.allclose(D, Dref, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("k", [2, 4])
def test_ldlq_streams_equal_the_oracle_loop(q, k):
    """Algorithm 5 with T_x = 32, T_y = 8: the same feedback matrix on both sides, streams,
    decoded weights and reported errors bit for bit."""
    rng = np.random.default_rng(900 + k)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    C = oracle.codebook(14, 1, CODE_LUT, lut)
    m, n = 64, 40
    W = rng.standard_normal((m, n)).astype(np.float32)
    Lm, _ = oracle.block_ldl(random_spd(rng, n), 8)
    A = (Lm - np.eye(n)).astype(np.float32)
    codes_ref, What_ref, xs = oracle.ldlq_quantize_f32(W, A, 14, k, 1, CODE_LUT, lut, tile=TILE)
    codes, What, err = run_ldlq(q, W, A, k, lut, tiles=1)
    assert np.array_equal(codes, codes_ref)
    assert np.array_equal(What, What_ref)
    tn = n // 8
    for t in range(codes.shape[0]):
        I, j = t // tn, t % tn
        d, _ = oracle.tailbiting_quantize_f32(xs[32 * I:32 * I + 32, 8 * j:8 * j + 8].reshape(-1), 14, k, 1, C)
        assert err[t] == d


def test_ldlq_lowers_the_proxy_loss(q):
    rng = np.random.default_rng(909)
    lut = rng.standard_normal(1 << 14).astype(np.float16)
    m, n = 128, 256
    W = rng.standard_normal((m, n)).astype(np.float32)
    H = random_spd(rng, n, corr=0.95)
    A, _ = run_block_ldl8(q, H)
    codes, What, err = run_ldlq(q, W, A, 2, lut)
    Wd = oracle.dequantize(codes, 14, 2, 1, CODE_LUT, m, n, lut, tile=TILE).view(np.float16).astype(np.float32)
    assert np.array_equal(What, Wd)
    _, What0, _ = run_ldlq(q, W, np.zeros((n, n), np.float32), 2, lut)
    loss = lambda Wh: np.trace((Wh - W).astype(np.float64) @ H @ (Wh - W).astype(np.float64).T)
    assert loss(What) < 0.7 * loss(What0)
