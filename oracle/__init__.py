"""QTIP oracle -- TEST INFRASTRUCTURE ONLY.

ctypes front end of ``qtip_oracle.c``: a plain CPU statement of what the QTIP
inference path computes (arXiv 2406.11235), used by the tests, the smoke check
and the benchmark's cpu_baseline leg.  The product package never imports this
module and this module never imports the product package.

Every function takes and returns numpy arrays; fp16 values travel as uint16
bit patterns so that nothing is rounded on the way in or out.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qtip_oracle.c")
_LIB = os.path.join(_HERE, "libqtip_oracle.so")

CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB2, CODE_LUT, CODE_HYB1 = 0, 1, 2, 3, 4, 5


def _q(code_id, Q):
    """Index bits of the hash codes: 9 for HYB (Section 4.2), 6 for its V = 1 form."""
    return (6 if code_id == CODE_HYB1 else 9) if Q is None else Q


def build(force=False):
    """Compile the oracle with gcc (no fast-math, no FMA contraction).
    QTIP_ORACLE_LIBRARY names another build of the same source to load instead (the sanitizer
    leg of the tests builds one with -fsanitize=address,undefined)."""
    if os.environ.get("QTIP_ORACLE_LIBRARY"):
        return os.environ["QTIP_ORACLE_LIBRARY"]
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c = ctypes
        vp, i32, dbl = c.c_void_p, c.c_int, c.c_double
        L.orc_threads.restype = i32
        L.orc_f16_to_f64.restype = dbl
        L.orc_f16_to_f64.argtypes = [c.c_uint16]
        L.orc_f64_to_f16.restype = c.c_uint16
        L.orc_f64_to_f16.argtypes = [dbl]
        L.orc_stream_bit.restype = i32
        L.orc_stream_bit.argtypes = [vp, i32]
        L.orc_state.restype = c.c_uint32
        L.orc_state.argtypes = [vp, i32, i32, i32, i32]
        L.orc_code_1mad.restype = c.c_uint16
        L.orc_code_1mad.argtypes = [c.c_uint32]
        L.orc_code_1mad_real.restype = dbl
        L.orc_code_1mad_real.argtypes = [c.c_uint32]
        L.orc_dequantize_1mad_real.restype = i32
        L.orc_dequantize_1mad_real.argtypes = [vp, i32, i32, i32, vp]
        L.orc_code_3inst.restype = c.c_uint16
        L.orc_code_3inst.argtypes = [c.c_uint32]
        L.orc_code_hyb.restype = None
        L.orc_code_hyb.argtypes = [c.c_uint32, i32, vp, vp]
        L.orc_code_hyb2.restype = None
        L.orc_code_hyb2.argtypes = [c.c_uint32, i32, vp, vp]
        L.orc_code_hyb1.restype = c.c_uint16
        L.orc_code_hyb1.argtypes = [c.c_uint32, i32, vp]
        L.orc_codebook.restype = i32
        L.orc_codebook.argtypes = [i32, i32, i32, vp, i32, vp]
        L.orc_decode_sequence.restype = None
        L.orc_decode_sequence.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, vp]
        L.orc_decode_sequence_table.restype = None
        L.orc_decode_sequence_table.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.orc_dequantize.restype = i32
        L.orc_dequantize.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, vp]
        L.orc_dequantize_tiled.restype = i32
        L.orc_dequantize_tiled.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, vp]
        L.orc_decode_element_tiled.restype = c.c_uint16
        L.orc_decode_element_tiled.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, i32]
        L.orc_decode_matmat_rows_tiled.restype = None
        L.orc_decode_matmat_rows_tiled.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32, i32, vp,
                                                   i32, vp, vp, i32, vp]
        L.orc_decode_element.restype = c.c_uint16
        L.orc_decode_element.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, i32]
        L.orc_matmat_dense.restype = None
        L.orc_matmat_dense.argtypes = [vp, i32, i32, vp, i32, vp, vp]
        L.orc_decode_matmat_rows.restype = None
        L.orc_decode_matmat_rows.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, i32, vp,
                                             i32, vp, vp, i32, vp]
        L.orc_hadamard.restype = None
        L.orc_hadamard.argtypes = [i32, vp]
        L.orc_rht.restype = i32
        L.orc_rht.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.orc_viterbi.restype = dbl
        L.orc_viterbi.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp]
        L.orc_states_to_stream.restype = None
        L.orc_states_to_stream.argtypes = [vp, i32, i32, i32, vp]
        L.orc_tailbiting_quantize.restype = dbl
        L.orc_tailbiting_quantize.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.orc_viterbi_f32.restype = c.c_float
        L.orc_viterbi_f32.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp]
        L.orc_tailbiting_quantize_f32.restype = c.c_float
        L.orc_tailbiting_quantize_f32.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.orc_block_ldl.restype = i32
        L.orc_block_ldl.argtypes = [vp, i32, i32, vp, vp]
        L.orc_ldlq_feedback_f32.restype = None
        L.orc_ldlq_feedback_f32.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
        L.orc_stream_distortion.restype = dbl
        L.orc_stream_distortion.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.orc_exhaustive_tailbiting.restype = dbl
        L.orc_exhaustive_tailbiting.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.orc_exhaustive_walk.restype = dbl
        L.orc_exhaustive_walk.argtypes = [vp, i32, i32, i32, i32, vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a):
    """fp16 array or uint16 bit patterns -> contiguous uint16 bit patterns."""
    if a is None:
        return None
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return np.ascontiguousarray(a)


def _u32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint32, a.dtype
    return a


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def threads():
    return int(lib().orc_threads())


def f16_to_f64(h):
    return float(lib().orc_f16_to_f64(int(h)))


def f64_to_f16(v):
    return int(lib().orc_f64_to_f16(float(v)))


def stream_bit(words, i):
    return int(lib().orc_stream_bit(_p(_u32(words)), int(i)))


def state(words, nbits, L, kV, t):
    w = _u32(words)
    assert w.size * 32 >= nbits
    return int(lib().orc_state(_p(w), nbits, L, kV, t))


def code_1mad(x):
    return int(lib().orc_code_1mad(int(x)))


def code_1mad_real(x):
    """Algorithm 1's quotient (s - 510) / 147.8, unrounded (float64)."""
    return float(lib().orc_code_1mad_real(int(x)))


def dequantize_1mad_real(codes, k, m, n):
    """Dense 1MAD weights as Algorithm 1's unrounded quotients, float64 (m, n)."""
    codes = _u32(codes).reshape(-1)
    assert codes.size == (m // 16) * (n // 16) * 8 * k
    W = np.zeros((m, n), dtype=np.float64)
    rc = lib().orc_dequantize_1mad_real(_p(codes), k, m, n, _p(W))
    assert rc == 0
    return W


def code_3inst(x):
    return int(lib().orc_code_3inst(int(x)))


def code_hyb(x, lut, Q=9):
    lut = _u16(lut).reshape(-1)
    assert lut.size == 2 << Q
    out = np.zeros(2, dtype=np.uint16)
    lib().orc_code_hyb(int(x), Q, _p(lut), _p(out))
    return int(out[0]), int(out[1])


def code_hyb2(x, lut, Q=9):
    lut = _u16(lut).reshape(-1)
    assert lut.size == 2 << Q
    out = np.zeros(2, dtype=np.uint16)
    lib().orc_code_hyb2(int(x), Q, _p(lut), _p(out))
    return int(out[0]), int(out[1])


def code_hyb1(x, lut, Q=6):
    lut = _u16(lut).reshape(-1)
    assert lut.size == 1 << Q
    return int(lib().orc_code_hyb1(int(x), Q, _p(lut)))


def codebook(L, V, code_id, lut=None, Q=None):
    """C[2^L][V] as float64, by evaluating the code on every state."""
    lut = None if lut is None else _u16(lut).reshape(-1)
    C = np.zeros((1 << L, V), dtype=np.float64)
    rc = lib().orc_codebook(L, V, code_id, _p(lut), _q(code_id, Q), _p(C))
    assert rc == 0
    return C


def decode_sequence(words, T, L, k, V, code_id, lut=None, Q=None):
    w = _u32(words)
    assert w.size * 32 >= k * T
    lut = None if lut is None else _u16(lut).reshape(-1)
    out = np.zeros(T, dtype=np.uint16)
    lib().orc_decode_sequence(_p(w), T, L, k, V, code_id, _p(lut), _q(code_id, Q), _p(out))
    return out


def decode_sequence_table(words, T, L, k, V, C):
    w = _u32(words)
    assert w.size * 32 >= k * T
    C = _f64(C).reshape(1 << L, V)
    out = np.zeros(T, dtype=np.float64)
    st = np.zeros(T // V, dtype=np.uint32)
    lib().orc_decode_sequence_table(_p(w), T, L, k, V, _p(C), _p(out), _p(st))
    return out, st


def dequantize(codes, L, k, V, code_id, m, n, lut=None, Q=None, tile=(16, 16)):
    """Dense decoded weights as uint16 fp16 bit patterns, shape (m, n); tile = (T_x, T_y)."""
    Tx, Ty = tile
    codes = _u32(codes).reshape(-1)
    assert codes.size == (m // Tx) * (n // Ty) * 8 * k
    lut = None if lut is None else _u16(lut).reshape(-1)
    W = np.zeros((m, n), dtype=np.uint16)
    rc = lib().orc_dequantize_tiled(_p(codes), L, k, V, code_id, _p(lut), _q(code_id, Q), m, n, Tx, Ty, _p(W))
    assert rc == 0
    return W


def decode_element(codes, L, k, V, code_id, n, i, j, lut=None, Q=None, tile=(16, 16)):
    codes = _u32(codes).reshape(-1)
    lut = None if lut is None else _u16(lut).reshape(-1)
    return int(lib().orc_decode_element_tiled(_p(codes), L, k, V, code_id, _p(lut), _q(code_id, Q), n, tile[0], tile[1],
                                              i, j))


def matmat_dense(W, X, scale=None):
    """Y[b][i] = scale[i] * sum_j W[i][j] X[b][j] in fp64; fp16 inputs as bits."""
    W = _u16(W)
    m, n = W.shape
    X = _u16(X).reshape(-1, n)
    B = X.shape[0]
    scale = _u16(scale)
    Y = np.zeros((B, m), dtype=np.float64)
    lib().orc_matmat_dense(_p(W), m, n, _p(X), B, _p(scale), _p(Y))
    return Y


def decode_matmat_rows(codes, L, k, V, code_id, m, n, X, rows, lut=None, Q=None, scale=None, tile=(16, 16)):
    """fp64 outputs for the chosen rows only: shape (B, len(rows))."""
    codes = _u32(codes).reshape(-1)
    lut = None if lut is None else _u16(lut).reshape(-1)
    X = _u16(X).reshape(-1, n)
    B = X.shape[0]
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    scale = _u16(scale)
    Y = np.zeros((B, rows.size), dtype=np.float64)
    lib().orc_decode_matmat_rows_tiled(_p(codes), L, k, V, code_id, _p(lut), _q(code_id, Q), m, n, tile[0], tile[1],
                                       _p(X), B, _p(scale), _p(rows), rows.size, _p(Y))
    return Y


def hadamard(b):
    H = np.zeros((b, b), dtype=np.int8)
    lib().orc_hadamard(b, _p(H))
    return H


def rht(x, signs, block, side=0):
    """Random Hadamard transform of fp16 rows x (batch, n) -> float64."""
    x = _u16(x)
    x2 = x.reshape(1, -1) if x.ndim == 1 else x
    batch, n = x2.shape
    signs = np.ascontiguousarray(np.asarray(signs, dtype=np.int8))
    assert signs.size == n
    out = np.zeros((batch, n), dtype=np.float64)
    rc = lib().orc_rht(_p(np.ascontiguousarray(x2)), _p(signs), n, block, batch, side, _p(out))
    assert rc == 0, rc
    return out.reshape(x.shape)


def viterbi(S, L, k, V, C, first_top=-1, last_low=-1):
    S = _f64(S)
    T = S.size
    C = _f64(C).reshape(1 << L, V)
    st = np.zeros(T // V, dtype=np.uint32)
    d = lib().orc_viterbi(_p(S), T, L, k, V, _p(C), first_top, last_low, _p(st))
    return float(d), st


def states_to_stream(states, L, kV):
    st = _u32(states)
    G = st.size
    words = np.zeros((G * kV + 31) // 32, dtype=np.uint32)
    lib().orc_states_to_stream(_p(st), G, L, kV, _p(words))
    return words


def tailbiting_quantize(S, L, k, V, C):
    S = _f64(S)
    T = S.size
    C = _f64(C).reshape(1 << L, V)
    words = np.zeros((k * T + 31) // 32, dtype=np.uint32)
    d = lib().orc_tailbiting_quantize(_p(S), T, L, k, V, _p(C), _p(words))
    return float(d), words


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def viterbi_f32(S, L, k, V, C, first_top=-1, last_low=-1):
    """Viterbi with the value function in binary32 (see orc_viterbi_f32)."""
    S = _f32(S)
    T = S.size
    C = _f32(C).reshape(1 << L, V)
    st = np.zeros(T // V, dtype=np.uint32)
    d = lib().orc_viterbi_f32(_p(S), T, L, k, V, _p(C), first_top, last_low, _p(st))
    return np.float32(d), st


def tailbiting_quantize_f32(S, L, k, V, C):
    """Algorithm 4 with binary32 Viterbi calls; returns (final value as float32, words)."""
    S = _f32(S)
    T = S.size
    C = _f32(C).reshape(1 << L, V)
    words = np.zeros((k * T + 31) // 32, dtype=np.uint32)
    d = lib().orc_tailbiting_quantize_f32(_p(S), T, L, k, V, _p(C), _p(words))
    return np.float32(d), words


def stream_distortion(words, S, L, k, V, C):
    S = _f64(S)
    C = _f64(C).reshape(1 << L, V)
    return float(lib().orc_stream_distortion(_p(_u32(words)), _p(S), S.size, L, k, V, _p(C)))


def exhaustive_tailbiting(S, L, k, V, C):
    S = _f64(S)
    C = _f64(C).reshape(1 << L, V)
    w = np.zeros(1, dtype=np.uint32)
    d = lib().orc_exhaustive_tailbiting(_p(S), S.size, L, k, V, _p(C), _p(w))
    return float(d), w


def exhaustive_walk(S, L, k, V, C):
    S = _f64(S)
    C = _f64(C).reshape(1 << L, V)
    return float(lib().orc_exhaustive_walk(_p(S), S.size, L, k, V, _p(C)))


def block_ldl(H, g=16):
    """H = L D L^T, L unit block lower triangular, D block diagonal: returns (L, D blocks)."""
    H = _f64(H)
    n = H.shape[0]
    assert H.shape == (n, n) and n % g == 0
    Lm = np.zeros((n, n), dtype=np.float64)
    D = np.zeros((n // g, g, g), dtype=np.float64)
    rc = lib().orc_block_ldl(_p(H), n, g, _p(Lm), _p(D))
    assert rc == 0, rc
    return Lm, D


def ldlq_feedback_f32(W, E, A, j, g=16):
    W, E, A = _f32(W), _f32(E), _f32(A)
    m, n = W.shape
    x = np.zeros((m, g), dtype=np.float32)
    lib().orc_ldlq_feedback_f32(_p(W), _p(E), _p(A), m, n, g, j, _p(x))
    return x


def ldlq_quantize_f32(W, A, L, k, V, code_id, lut=None, rounder=None, tile=(16, 16), table=None):
    """Algorithm 5 with tile = (T_x, T_y): column blocks of T_y from the last to the first,
    feedback in binary32 (ldlq_feedback_f32), every T_x x T_y block of x rounded as one sequence
    by the binary32 tail-biting quantizer.  Returns (codes (tiles, 8k), What float32, x of every
    block).  `rounder(S) -> (value, words)` replaces the quantizer, `table` (2^L x V values) the
    code's own codebook (tests of the loop's identities on a small trellis)."""
    W, A = _f32(W), _f32(A)
    m, n = W.shape
    Tx, Ty = tile
    assert Tx * Ty == 256
    tn = n // Ty
    C = codebook(L, V, code_id, lut) if table is None else _f64(table).reshape(1 << L, V)
    codes = np.zeros(((m // Tx) * tn, 8 * k), dtype=np.uint32)
    What = np.zeros((m, n), dtype=np.float32)
    E = np.zeros((m, n), dtype=np.float32)
    xs = np.zeros((m, n), dtype=np.float32)
    for j in range(tn - 1, -1, -1):
        cols = slice(Ty * j, Ty * j + Ty)
        x = ldlq_feedback_f32(W, E, A, j, Ty)
        xs[:, cols] = x
        for I in range(m // Tx):
            S = x[Tx * I:Tx * I + Tx, :].reshape(-1)
            if rounder is None:
                _, words = tailbiting_quantize_f32(S, L, k, V, C)
            else:
                _, words = rounder(S)
            codes[I * tn + j] = words
            vals, _ = decode_sequence_table(words, 256, L, k, V, C)
            What[Tx * I:Tx * I + Tx, cols] = vals.reshape(Tx, Ty).astype(np.float32)
        E[:, cols] = W[:, cols] - What[:, cols]
    return codes, What, xs
