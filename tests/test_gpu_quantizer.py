"""GPU parity of qtip_quantize_gpu (Viterbi on the bitshift trellis, Section 2.3, made
tail-biting by Algorithm 4) against the CPU oracle.

The quantizer searches in binary32 with a fixed operation order, and the oracle has the
same recursion in binary32 (oracle.tailbiting_quantize_f32), so streams and final values
are compared bit for bit.  Larger runs are checked through what is unique: the reported
error of every tile equals the binary64 distortion of its own stream, and the mean
squared error agrees with the binary64 host quantizer and with Table 1.
"""
import numpy as np
import pytest

import oracle
import qtip_synth as synth
from qtip_synth import CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB1, CODE_HYB2

pytestmark = pytest.mark.gpu

ALL_CODECS = [(CODE_3INST, 2, 1), (CODE_3INST, 3, 1), (CODE_3INST, 4, 1),
              (CODE_1MAD, 2, 1), (CODE_1MAD, 3, 1), (CODE_1MAD, 4, 1),
              (CODE_HYB, 2, 2), (CODE_HYB, 3, 2), (CODE_HYB, 4, 2),
              (CODE_HYB2, 2, 2), (CODE_HYB2, 3, 2), (CODE_HYB2, 4, 2),
              (CODE_HYB1, 2, 1), (CODE_HYB1, 3, 1), (CODE_HYB1, 4, 1)]


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def make_lut(code_id, rng):
    if code_id == CODE_HYB1:
        return rng.standard_normal(64).astype(np.float16)
    return rng.standard_normal((512, 2)).astype(np.float16) if code_id in (CODE_HYB, CODE_HYB2) else None


def run_quantize_gpu(q, W, k, V, code_id, lut, tiles_in_flight=None):
    import torch
    m, n = W.shape
    ntiles = (m // 16) * (n // 16)
    ws_bytes = q.qtip_quantize_gpu_workspace(k, V, tiles_in_flight or ntiles)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    Wd = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).cuda()
    lutd = None if lut is None else torch.from_numpy(lut.view(np.uint16).astype(np.int16)).cuda()
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_gpu(Wd, m, n, 16, k, V, code_id, lutd, codes, err, ws, ws_bytes)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32), err.cpu().numpy()


def tile_sequence(W, I, J):
    return W[16 * I:16 * I + 16, 16 * J:16 * J + 16].reshape(-1)


@pytest.mark.parametrize("code_id,k,V", ALL_CODECS)
def test_streams_and_values_equal_the_binary32_oracle(q, code_id, k, V):
    rng = np.random.default_rng(3000 + 10 * code_id + k)
    lut = make_lut(code_id, rng)
    C = oracle.codebook(16, V, code_id, lut)
    m, n = 16, 32
    W = (rng.standard_normal((m, n)) * C.std()).astype(np.float32)
    # a workspace for one tile: the second tile goes through a second batch
    codes, err = run_quantize_gpu(q, W, k, V, code_id, lut, tiles_in_flight=1)
    for J in range(n // 16):
        d, words = oracle.tailbiting_quantize_f32(tile_sequence(W, 0, J), 16, k, V, C)
        assert np.array_equal(codes[J], words), (J, codes[J], words)
        assert err[J] == d


@pytest.mark.parametrize("code_id,k,V", [(CODE_3INST, 2, 1), (CODE_1MAD, 4, 1), (CODE_HYB, 3, 2), (CODE_HYB1, 2, 1)])
def test_degenerate_tiles_equal_the_binary32_oracle(q, code_id, k, V):
    """Tiles far from the Gaussian case: all zeros and a constant (many paths of nearly
    equal cost), weights 30 times the code's spread (every state far away), heavy tails,
    and one outlier of 1e4 among ordinary weights (costs near 1e8 beside costs near 1).
    Streams and final values bit for bit, as for ordinary tiles."""
    rng = np.random.default_rng(5000 + 10 * code_id + k)
    lut = make_lut(code_id, rng)
    C = oracle.codebook(16, V, code_id, lut)
    sd = C.std()
    outlier = rng.standard_normal((16, 16)) * sd
    outlier[rng.integers(16), rng.integers(16)] = 1e4
    tiles = [np.zeros((16, 16)), np.full((16, 16), 0.37 * sd), rng.standard_normal((16, 16)) * sd * 30,
             rng.standard_t(2, (16, 16)) * sd, outlier]
    W = np.concatenate(tiles, axis=1).astype(np.float32)
    codes, err = run_quantize_gpu(q, W, k, V, code_id, lut)
    for J in range(len(tiles)):
        d, words = oracle.tailbiting_quantize_f32(tile_sequence(W, 0, J), 16, k, V, C)
        assert np.array_equal(codes[J], words), (J, codes[J], words)
        assert err[J] == d


def test_decodable_weights_come_back_exactly(q):
    rng = np.random.default_rng(8)
    for code_id, k, V in [(CODE_3INST, 2, 1), (CODE_1MAD, 3, 1), (CODE_HYB, 2, 2), (CODE_HYB2, 4, 2)]:
        lut = make_lut(code_id, rng)
        m, n = 32, 48
        codes = rng.integers(0, 1 << 32, ((m // 16) * (n // 16), 8 * k), dtype=np.uint64).astype(np.uint32)
        W = oracle.dequantize(codes, 16, k, V, code_id, m, n, lut).view(np.float16).astype(np.float32)
        codes2, err = run_quantize_gpu(q, W, k, V, code_id, lut)
        assert np.all(err == 0.0)
        W2 = oracle.dequantize(codes2, 16, k, V, code_id, m, n, lut).view(np.float16).astype(np.float32)
        assert np.array_equal(W, W2)


@pytest.mark.parametrize("code_id,k,V,name", [(CODE_3INST, 2, 1, "3INST"), (CODE_1MAD, 2, 1, "1MAD"),
                                              (CODE_HYB, 2, 2, "HYB"), (CODE_HYB2, 2, 2, "HYB"),
                                              (CODE_HYB1, 2, 1, "HYB")])
def test_gaussian_matrix_properties_and_table1(q, golden, code_id, k, V, name):
    """256 tiles of i.i.d. Gaussian weights scaled to the code: every reported error is the
    true distortion of the tile's own (tail-biting) stream, the mean squared error matches
    the binary64 host quantizer, and it reproduces Table 1's 2-bit figure for the code."""
    t1 = {r[1]: float(r[2]) for r in golden("table_mse.txt") if r[0] == "table1"}
    rng = np.random.default_rng(4000 + code_id)
    # Table 1's HYB row uses a trained table; a table of Gaussian samples is a little worse
    lut = make_lut(code_id, rng)
    C = oracle.codebook(16, V, code_id, lut)
    sd = C.std()
    m, n = 64, 1024
    W = (rng.standard_normal((m, n)) * sd).astype(np.float32)
    codes, err = run_quantize_gpu(q, W, k, V, code_id, lut, tiles_in_flight=100)
    assert np.all(np.isfinite(err))
    tn = n // 16
    for t in range(0, codes.shape[0], 5):
        S = tile_sequence(W, t // tn, t % tn).astype(np.float64)
        true = oracle.stream_distortion(codes[t], S, 16, k, V, C)
        assert abs(err[t] - true) <= 2e-5 * true, (t, err[t], true)
    Wd = oracle.dequantize(codes, 16, k, V, code_id, m, n, lut).view(np.float16).astype(np.float64)
    mse = ((Wd - W) ** 2).mean()
    assert abs(err.astype(np.float64).sum() / (m * n) - mse) <= 1e-5 * mse
    _, mse_host = q.qtip_quantize(W, m, n, 16, k, V, code_id, lut)
    assert abs(mse - mse_host) <= 2e-4 * mse_host     # near-ties may pick other walks
    rel = mse / sd ** 2
    tol = 0.03 if code_id not in (CODE_HYB, CODE_HYB2, CODE_HYB1) else 0.12
    assert abs(rel / t1[name] - 1) < tol, (name, rel)
    assert rel > t1["DR"]


def test_quantize_gpu_error_codes(q):
    import torch
    W = torch.zeros((16, 16), dtype=torch.float32, device="cuda")
    codes = torch.zeros(16, dtype=torch.int32, device="cuda")
    need = q.qtip_quantize_gpu_workspace(2, 1, 1)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_gpu(W, 16, 16, 16, 2, 1, CODE_3INST, None, codes, None, None, need)
    assert e.value.code == -1
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_gpu(W, 16, 16, 16, 2, 1, CODE_3INST, None, codes, None, ws, need - 1)
    assert e.value.code == -1 and "workspace" in str(e.value)
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_gpu(W, 16, 16, 16, 2, 1, CODE_3INST, None, codes, None, ws.data_ptr() + 4, need)
    assert e.value.code == -1
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_gpu(W, 16, 16, 16, 5, 1, CODE_3INST, None, codes, None, ws, need)
    assert e.value.code == -2
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_gpu(W, 16, 16, 16, 2, 2, CODE_HYB, None, codes, None, ws, need)
    assert e.value.code == -1
    assert q.qtip_quantize_gpu_workspace(7, 1, 1) == 0
    # and a valid call right after the failures
    q.qtip_quantize_gpu(W, 16, 16, 16, 2, 1, CODE_3INST, None, codes, None, ws, need)
    torch.cuda.synchronize()
