"""GPU parity of BlockLDLQ with the trellis quantizer as rounder (Algorithm 5):
qtip_block_ldl against the oracle's binary64 decomposition (floating point: tolerance),
qtip_quantize_ldlq against the oracle's loop given the same feedback matrix (the feedback
sum and the search are fixed-order binary32 on both sides: streams bit for bit)."""
import numpy as np
import pytest

import oracle
from qtip_synth import CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB1, CODE_HYB2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def random_spd(rng, n, corr=0.9):
    samples = 4 * n
    base = rng.standard_normal((samples, 1))
    X = corr * base + (1 - corr) * rng.standard_normal((samples, n))
    X = X * rng.uniform(0.5, 2.0, n)[None, :]
    return X.T @ X / samples + 1e-3 * np.eye(n)


def run_block_ldl(q, H):
    import torch
    n = H.shape[0]
    Hd = torch.from_numpy(np.ascontiguousarray(H, dtype=np.float64)).cuda()
    A = torch.full((n, n), float("nan"), dtype=torch.float32, device="cuda")
    D = torch.full((n // 16, 16, 16), float("nan"), dtype=torch.float64, device="cuda")
    wsb = q.qtip_block_ldl_workspace(n)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    q.qtip_block_ldl(Hd, n, 16, A, D, ws, wsb)
    torch.cuda.synchronize()
    return A.cpu().numpy(), D.cpu().numpy()


def run_ldlq(q, W, A, k, V, code_id, lut, tiles=None):
    import torch
    m, n = W.shape
    ntiles = (m // 16) * (n // 16)
    wsb = q.qtip_quantize_ldlq_workspace(m, n, k, V, tiles or m // 16)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    Wd = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).cuda()
    Ad = torch.from_numpy(np.ascontiguousarray(A, dtype=np.float32)).cuda()
    lutd = None if lut is None else torch.from_numpy(lut.view(np.uint16).astype(np.int16)).cuda()
    codes = torch.full((ntiles, 8 * k), -1, dtype=torch.int32, device="cuda")
    What = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    err = torch.full((ntiles,), float("nan"), dtype=torch.float32, device="cuda")
    q.qtip_quantize_ldlq(Wd, Ad, m, n, 16, k, V, code_id, lutd, codes, What, err, ws, wsb)
    torch.cuda.synchronize()
    return codes.cpu().numpy().view(np.uint32), What.cpu().numpy(), err.cpu().numpy()


@pytest.mark.parametrize("n", [16, 64, 272])
def test_block_ldl_matches_the_oracle(q, n):
    rng = np.random.default_rng(600 + n)
    H = random_spd(rng, n)
    A, D = run_block_ldl(q, H)
    Lm, Dref = oracle.block_ldl(H, 16)
    Aref = Lm - np.eye(n)
    assert np.all(np.isfinite(A)) and np.all(np.isfinite(D))
    for j in range(n // 16):
        assert np.all(A[16 * j:16 * j + 16, 16 * j:] == 0)          # zero on and above the diagonal blocks
    scale = max(1.0, np.abs(Aref).max())
    assert np.abs(A - Aref).max() <= 1e-6 * scale                     # binary32 output of a binary64 result
    assert np.allclose(D, Dref, rtol=1e-9, atol=1e-12)
    Lg = A.astype(np.float64) + np.eye(n)
    Dfull = np.zeros((n, n))
    for j in range(n // 16):
        Dfull[16 * j:16 * j + 16, 16 * j:16 * j + 16] = D[j]
    assert np.allclose(Lg @ Dfull @ Lg.T, H, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("code_id,k,V", [(CODE_3INST, 2, 1), (CODE_1MAD, 3, 1), (CODE_HYB, 2, 2), (CODE_HYB2, 2, 2),
                                          (CODE_HYB1, 2, 1)])
def test_ldlq_streams_equal_the_oracle_loop(q, code_id, k, V):
    rng = np.random.default_rng(700 + 10 * code_id + k)
    lut = rng.standard_normal((512, 2)).astype(np.float16) if code_id in (CODE_HYB, CODE_HYB2) else None
    if code_id == CODE_HYB1:
        lut = rng.standard_normal(64).astype(np.float16)
    C = oracle.codebook(16, V, code_id, lut)
    m, n = 32, 64
    W = (rng.standard_normal((m, n)) * C.std()).astype(np.float32)
    Lm, _ = oracle.block_ldl(random_spd(rng, n), 16)
    A = (Lm - np.eye(n)).astype(np.float32)
    codes_ref, What_ref, xs = oracle.ldlq_quantize_f32(W, A, 16, k, V, code_id, lut)
    # one tile in flight: each column block takes two batches of the quantizer
    codes, What, err = run_ldlq(q, W, A, k, V, code_id, lut, tiles=1)
    assert np.array_equal(codes, codes_ref)
    assert np.array_equal(What, What_ref)
    tn = n // 16
    for t in range(codes.shape[0]):
        I, j = t // tn, t % tn
        S = xs[16 * I:16 * I + 16, 16 * j:16 * j + 16].reshape(-1)
        d, _ = oracle.tailbiting_quantize_f32(S, 16, k, V, C)
        assert err[t] == d


def test_ldlq_lowers_the_proxy_loss_end_to_end(q):
    """Decomposition and loop both on the GPU, 3INST 2-bit, 128 x 256 with a strongly
    correlated Hessian: the proxy loss tr((What - W) H (What - W)^T) (Eq. 1) falls well below
    that of quantizing W directly, and What is the decode of the codes."""
    import torch
    rng = np.random.default_rng(99)
    m, n = 128, 256
    C = oracle.codebook(16, 1, CODE_3INST)
    W = (rng.standard_normal((m, n)) * C.std()).astype(np.float32)
    H = random_spd(rng, n, corr=0.95)
    A, D = run_block_ldl(q, H)
    codes, What, err = run_ldlq(q, W, A, 2, 1, CODE_3INST, None)
    Wd = oracle.dequantize(codes, 16, 2, 1, CODE_3INST, m, n).view(np.float16).astype(np.float32)
    assert np.array_equal(What, Wd)
    codes0, What0, _ = run_ldlq(q, W, np.zeros((n, n), np.float32), 2, 1, CODE_3INST, None)
    loss = lambda Wh: np.trace((Wh - W).astype(np.float64) @ H @ (Wh - W).astype(np.float64).T)
    assert loss(What) < 0.7 * loss(What0)
    # the identity behind Algorithm 5: proxy loss = sum over blocks of tr(eta_j D_j eta_j^T),
    # where ||eta||^2 per tile is the reported error; check the cheap consequence
    E = (What - W).astype(np.float64)
    eta = E @ (np.eye(n) + A.astype(np.float64))
    per_tile = (eta.reshape(m // 16, 16, n // 16, 16) ** 2).sum(axis=(1, 3)).reshape(-1)
    assert np.allclose(per_tile, err, rtol=2e-3, atol=1e-4)


def test_ldlq_error_codes(q):
    import torch
    W = torch.zeros((16, 32), dtype=torch.float32, device="cuda")
    A = torch.zeros((32, 32), dtype=torch.float32, device="cuda")
    H = torch.eye(32, dtype=torch.float64, device="cuda")
    codes = torch.zeros(32, dtype=torch.int32, device="cuda")
    need = q.qtip_quantize_ldlq_workspace(16, 32, 2, 1, 1)
    ws = torch.empty(max(need, q.qtip_block_ldl_workspace(32)), dtype=torch.uint8, device="cuda")
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_ldlq(W, None, 16, 32, 16, 2, 1, CODE_3INST, None, codes, None, None, ws, need)
    assert e.value.code == -1
    with pytest.raises(q.QtipError) as e:
        q.qtip_quantize_ldlq(W, A, 16, 32, 16, 2, 1, CODE_3INST, None, codes, None, None, ws, need - 1)
    assert e.value.code == -1 and "workspace" in str(e.value)
    with pytest.raises(q.QtipError) as e:
        q.qtip_block_ldl(H, 24, 16, A, None, ws, ws.numel())
    assert e.value.code == -1
    with pytest.raises(q.QtipError) as e:
        q.qtip_block_ldl(H, 32, 16, A, None, ws, 100)
    assert e.value.code == -1
    assert q.qtip_block_ldl_workspace(24) == 0 and q.qtip_quantize_ldlq_workspace(16, 32, 7, 1, 1) == 0
    q.qtip_block_ldl(H, 32, 16, A, None, ws, ws.numel())
    q.qtip_quantize_ldlq(W, A, 16, 32, 16, 2, 1, CODE_3INST, None, codes, None, None, ws, need)
    torch.cuda.synchronize()
    assert float(A.abs().max()) == 0.0          # H = I: no feedback


def test_example_quantize_then_infer(q):
    """The package's example: BlockLDLQ-quantize a synthetic layer on the GPU, then run the
    inference path on the result; the codes decode to the quantizer's What and the fused
    product agrees with the dense one."""
    from paper_2406_11235_amd import example
    assert example.main(256, 512, seed=3) < 2e-3
