"""GPU quantizer and BlockLDLQ against the binary64 oracle, by what the paper fixes.

Section 2.3 defines the quantizer as the minimum of the squared error over walks on the
trellis and Algorithm 4 as two such searches; Algorithm 5 defines the rounder's input x as
a plain sum.  None of that fixes a precision, so these tests do not look at which of two
nearly equal walks was taken: every GPU stream is scored in binary64 against the oracle's
binary64 searches (orc_viterbi, orc_tailbiting_quantize: Algorithm 4 as written), tile by
tile, and the GPU's x is compared with a binary64 feedback sum.

    free Viterbi optimum  <=  d(GPU stream)  <=  d(binary64 Algorithm 4) * (1 + 1e-4) + 1e-6

The lower bound holds for any valid stream (a tail-biting walk is a walk); the upper bound
says the binary32 search on the GPU lost nothing beyond rounding against the binary64 one.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
from qtip_synth import CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB1, CODE_HYB2, CODE_LUT

pytestmark = pytest.mark.gpu

REL, ABS = 1e-4, 1e-6
THREADS = 16

# (code, k, V, L, (T_x, T_y))
CODECS = [(c, k, 1, 16, (16, 16)) for c in (CODE_3INST, CODE_1MAD, CODE_HYB1) for k in (2, 3, 4)] + \
         [(c, k, 2, 16, (16, 16)) for c in (CODE_HYB, CODE_HYB2) for k in (2, 3, 4)] + \
         [(CODE_LUT, k, 1, 14, (32, 8)) for k in (2, 3, 4)]


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def make_lut(code_id, rng):
    if code_id == CODE_LUT:
        return rng.standard_normal(1 << 14).astype(np.float16)
    if code_id == CODE_HYB1:
        return rng.standard_normal(64).astype(np.float16)
    if code_id in (CODE_HYB, CODE_HYB2):
        return rng.standard_normal((512, 2)).astype(np.float16)
    return None


def tile_row(rng, sd, tile, gaussian=27):
    """One row of 32 blocks: `gaussian` i.i.d. Gaussian ones scaled to the code, then the
    degenerate ones (zeros, a constant, 30 sigma, heavy tails, one outlier of 1e4)."""
    outlier = rng.standard_normal(tile) * sd
    outlier[rng.integers(tile[0]), rng.integers(tile[1])] = 1e4
    blocks = [rng.standard_normal(tile) * sd for _ in range(gaussian)]
    blocks += [np.zeros(tile), np.full(tile, 0.37 * sd), rng.standard_normal(tile) * sd * 30,
               rng.standard_t(2, tile) * sd, outlier]
    return np.concatenate(blocks, axis=1).astype(np.float32)


def dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def lut_dev(lut):
    return None if lut is None else dev(lut.view(np.uint16).astype(np.int16))


def run_quantize_gpu(q, W, L, k, V, code_id, lut, tile):
    import torch
    m, n = W.shape
    ntiles = (m // tile[0]) * (n // tile[1])
    ws_bytes = q.qtip_quantize_gpu_workspace(k, V, ntiles)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_gpu(dev(W), m, n, L, k, V, code_id, lut_dev(lut), codes, err, ws, ws_bytes)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32), err.cpu().numpy()


def score_against_binary64(words, S, L, k, V, C):
    """(binary64 distortion of the stream, of the oracle's Algorithm 4, of the free optimum)."""
    S = np.asarray(S, dtype=np.float64)
    d_gpu = oracle.stream_distortion(words, S, L, k, V, C)
    d_alg4, _ = oracle.tailbiting_quantize(S, L, k, V, C)
    d_free, _ = oracle.viterbi(S, L, k, V, C)
    return d_gpu, d_alg4, d_free


def check_bounds(rows):
    for tag, d_gpu, d_alg4, d_free in rows:
        assert d_free <= d_alg4 * (1 + 1e-12) + 1e-12, tag       # the oracle's own order
        assert d_gpu >= d_free * (1 - 1e-12) - 1e-12, (tag, d_gpu, d_free)
        assert d_gpu <= d_alg4 * (1 + REL) + ABS, (tag, d_gpu, d_alg4)


@pytest.mark.parametrize("code_id,k,V,L,tile", CODECS)
def test_every_tile_is_as_good_as_the_binary64_search(q, code_id, k, V, L, tile):
    rng = np.random.default_rng(9100 + 10 * code_id + k)
    lut = make_lut(code_id, rng)
    C = oracle.codebook(L, V, code_id, lut)
    W = tile_row(rng, C.std(), tile)
    codes, err = run_quantize_gpu(q, W, L, k, V, code_id, lut, tile)
    ntiles = W.shape[1] // tile[1]
    assert codes.shape[0] == ntiles == 32

    def one(J):
        S = W[:, tile[1] * J:tile[1] * J + tile[1]].reshape(-1)
        return (J,) + score_against_binary64(codes[J], S, L, k, V, C)
    with ThreadPoolExecutor(THREADS) as ex:
        rows = list(ex.map(one, range(ntiles)))
    check_bounds(rows)
    # the error the kernel reports is the distortion of its own stream
    for J, d_gpu, _, _ in rows:
        assert abs(float(err[J]) - d_gpu) <= 1e-4 * d_gpu + 1e-6, (J, err[J], d_gpu)


def random_spd(rng, n, corr=0.9):
    samples = 4 * n
    base = rng.standard_normal((samples, 1))
    X = corr * base + (1 - corr) * rng.standard_normal((samples, n))
    X = X * rng.uniform(0.5, 2.0, n)[None, :]
    return X.T @ X / samples + 1e-3 * np.eye(n)


@pytest.mark.parametrize("code_id,k,V,L,tile", [(CODE_3INST, 2, 1, 16, (16, 16)), (CODE_1MAD, 3, 1, 16, (16, 16)),
                                                 (CODE_HYB, 2, 2, 16, (16, 16)), (CODE_HYB2, 2, 2, 16, (16, 16)),
                                                 (CODE_HYB1, 4, 1, 16, (16, 16)), (CODE_LUT, 2, 1, 14, (32, 8))])
def test_ldlq_feedback_and_rounding_against_binary64(q, code_id, k, V, L, tile):
    """Algorithm 5 on the GPU, checked without the binary32 oracle: the x that every column
    block was rounded from (the workspace's running sum) equals the binary64 sum
    W_j + (W - What)[:, later columns] A[later, j] formed from the GPU's own What, and every
    block's stream is as good a rounding of that x as the binary64 Algorithm 4 finds."""
    import torch
    rng = np.random.default_rng(9300 + 10 * code_id + k)
    lut = make_lut(code_id, rng)
    C = oracle.codebook(L, V, code_id, lut)
    Tx, Ty = tile
    m, n = 64, 96
    W = (rng.standard_normal((m, n)) * C.std()).astype(np.float32)
    Lm, _ = oracle.block_ldl(random_spd(rng, n), Ty)
    A = (Lm - np.eye(n)).astype(np.float32)
    ntiles = (m // Tx) * (n // Ty)
    wsb = q.qtip_quantize_ldlq_workspace(m, n, k, V, m // Tx)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    What = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_ldlq(dev(W), dev(A), m, n, L, k, V, code_id, lut_dev(lut), codes, What, err, ws, wsb)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy().view(np.uint32)
    What = What.cpu().numpy()
    err = err.cpu().numpy()
    # the first m x n floats of the workspace: x of every column block, as it was rounded
    x_gpu = ws[:m * n * 4].cpu().numpy().view(np.float32).reshape(m, n)

    W64, A64, What64 = W.astype(np.float64), A.astype(np.float64), What.astype(np.float64)
    x64 = np.empty((m, n))
    for j in range(n // Ty):
        lo, hi = Ty * j, Ty * j + Ty
        x64[:, lo:hi] = W64[:, lo:hi] + (W64[:, hi:] - What64[:, hi:]) @ A64[hi:, lo:hi]
    scale = np.abs(x64).max()
    assert np.abs(x_gpu - x64).max() <= 1e-5 * scale, np.abs(x_gpu - x64).max() / scale
    # What is the decode of the codes
    Wd = oracle.dequantize(codes, L, k, V, code_id, m, n, lut, tile=tile).view(np.float16).astype(np.float32)
    assert np.array_equal(What, Wd)

    tn = n // Ty

    def one(t):
        I, j = t // tn, t % tn
        S = x64[Tx * I:Tx * I + Tx, Ty * j:Ty * j + Ty].reshape(-1)
        return (t,) + score_against_binary64(codes[t], S, L, k, V, C)
    with ThreadPoolExecutor(THREADS) as ex:
        rows = list(ex.map(one, range(ntiles)))
    # x64 differs from the x the GPU rounded by binary32 rounding of the sum: give the
    # comparison that much room (|d(S) - d(S')| <= 2 sqrt(d) |S - S'| + |S - S'|^2)
    for t, d_gpu, d_alg4, d_free in rows:
        I, j = t // tn, t % tn
        dx = np.linalg.norm((x_gpu.astype(np.float64) - x64)[Tx * I:Tx * I + Tx, Ty * j:Ty * j + Ty])
        slack = 2 * np.sqrt(d_alg4) * dx + dx * dx
        assert d_gpu >= d_free * (1 - 1e-12) - 1e-12, (t, d_gpu, d_free)
        assert d_gpu <= d_alg4 * (1 + REL) + ABS + 2 * slack, (t, d_gpu, d_alg4, slack)
        assert abs(float(err[t]) - d_gpu) <= 1e-4 * d_gpu + 1e-6 + 2 * slack, (t, err[t], d_gpu)
