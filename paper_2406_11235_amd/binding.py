"""ctypes binding of libqtip.so: same names as include/qtip.h, argument marshalling only.

GPU entry points take torch tensors that already live on the device (or raw
integer device pointers) and enqueue on torch's current stream unless a stream is
given.  There is no fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import numpy as np

CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB2, CODE_LUT, CODE_HYB1 = 0, 1, 2, 3, 4, 5

_HERE = os.path.dirname(os.path.abspath(__file__))
# The environment variable QTIP_LIBRARY names another build of the same library to load instead
# (two builds compared on one box; the sanitizer build of the host code in tests/test_sanitizers.py).
_LIB_PATH = os.environ.get("QTIP_LIBRARY") or os.path.join(_HERE, "libqtip.so")
_lib = None

EXPORTS = ["qtip_rht", "qtip_rht_f32", "qtip_decode_matvec", "qtip_rht_decode_matvec",
           "qtip_rht_decode_matvec_noalloc", "qtip_decode_matmat",
           "qtip_dequantize", "qtip_decode_states", "qtip_quantize",
           "qtip_quantize_gpu_workspace", "qtip_quantize_gpu", "qtip_block_ldl_workspace",
           "qtip_block_ldl", "qtip_quantize_ldlq_workspace", "qtip_quantize_ldlq", "qtip_last_error",
           "qtip_version"]


class QtipError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"qtip error {code}: {message}")
        self.code = code


def library_path():
    return _LIB_PATH


def lib():
    """Load libqtip.so (built by paper_2406_11235_amd.build.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: run `python -m paper_2406_11235_amd.build` "
                "(there is no CPU fallback)")
        # torch ships its own HIP runtime; it must be the one libqtip.so binds to, or
        # the process ends up with two runtimes and the second one sees no device.
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        c = ctypes
        vp, i32 = c.c_void_p, c.c_int
        L.qtip_version.restype = i32
        L.qtip_version.argtypes = []
        L.qtip_last_error.restype = c.c_char_p
        L.qtip_last_error.argtypes = []
        L.qtip_rht.restype = i32
        L.qtip_rht.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp]
        L.qtip_rht_f32.restype = i32
        L.qtip_rht_f32.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp]
        L.qtip_decode_matvec.restype = i32
        L.qtip_decode_matvec.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, vp]
        L.qtip_rht_decode_matvec.restype = i32
        L.qtip_rht_decode_matvec.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
        L.qtip_rht_decode_matvec_noalloc.restype = i32
        L.qtip_rht_decode_matvec_noalloc.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp, i32, vp, vp, vp]
        L.qtip_decode_matmat.restype = i32
        L.qtip_decode_matmat.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, i32, vp, vp, vp]
        L.qtip_dequantize.restype = i32
        L.qtip_dequantize.argtypes = [vp, i32, i32, i32, i32, vp, i32, i32, vp, vp]
        L.qtip_decode_states.restype = i32
        L.qtip_decode_states.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.qtip_quantize.restype = i32
        L.qtip_quantize.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]
        L.qtip_quantize_gpu_workspace.restype = c.c_size_t
        L.qtip_quantize_gpu_workspace.argtypes = [i32, i32, c.c_long]
        L.qtip_quantize_gpu.restype = i32
        L.qtip_quantize_gpu.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp,
                                        c.c_size_t, vp]
        L.qtip_block_ldl_workspace.restype = c.c_size_t
        L.qtip_block_ldl_workspace.argtypes = [i32]
        L.qtip_block_ldl.restype = i32
        L.qtip_block_ldl.argtypes = [vp, i32, i32, vp, vp, vp, c.c_size_t, vp]
        L.qtip_quantize_ldlq_workspace.restype = c.c_size_t
        L.qtip_quantize_ldlq_workspace.argtypes = [i32, i32, i32, i32, c.c_long]
        L.qtip_quantize_ldlq.restype = i32
        L.qtip_quantize_ldlq.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                         c.c_size_t, vp]
        _lib = L
    return _lib


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc):
    if rc != 0:
        raise QtipError(rc, lib().qtip_last_error().decode())
    return rc


def qtip_version():
    return int(lib().qtip_version())


def qtip_last_error():
    return lib().qtip_last_error().decode()


def qtip_rht(x, signs, n, block, batch, side, out, stream=None):
    return _check(lib().qtip_rht(_ptr(x), _ptr(signs), n, block, batch, side, _ptr(out),
                                 _stream(stream)))


def qtip_rht_f32(x, signs, n, block, batch, side, out, stream=None):
    return _check(lib().qtip_rht_f32(_ptr(x), _ptr(signs), n, block, batch, side, _ptr(out),
                                     _stream(stream)))


def qtip_decode_matvec(codes, L, k, V, code_id, lut, m, n, x, y, stream=None):
    return _check(lib().qtip_decode_matvec(_ptr(codes), L, k, V, code_id, _ptr(lut), m, n,
                                           _ptr(x), _ptr(y), _stream(stream)))


def qtip_rht_decode_matvec(codes, L, k, V, code_id, lut, m, n, x, signs_n, block, row_scale, y,
                           xt_scratch=None, stream=None):
    return _check(lib().qtip_rht_decode_matvec(_ptr(codes), L, k, V, code_id, _ptr(lut), m, n, _ptr(x),
                                               _ptr(signs_n), block, _ptr(row_scale), _ptr(y),
                                               _ptr(xt_scratch), _stream(stream)))


def qtip_rht_decode_matvec_noalloc(codes, L, k, V, code_id, lut, m, n, x, signs_n, block, row_scale, y,
                                   stream=None):
    return _check(lib().qtip_rht_decode_matvec_noalloc(_ptr(codes), L, k, V, code_id, _ptr(lut), m, n, _ptr(x),
                                                       _ptr(signs_n), block, _ptr(row_scale), _ptr(y),
                                                       _stream(stream)))


def qtip_decode_matmat(codes, L, k, V, code_id, lut, m, n, X, B, row_scale, Y, stream=None):
    return _check(lib().qtip_decode_matmat(_ptr(codes), L, k, V, code_id, _ptr(lut), m, n,
                                           _ptr(X), B, _ptr(row_scale), _ptr(Y),
                                           _stream(stream)))


def qtip_dequantize(codes, L, k, V, code_id, lut, m, n, W, stream=None):
    return _check(lib().qtip_dequantize(_ptr(codes), L, k, V, code_id, _ptr(lut), m, n, _ptr(W),
                                        _stream(stream)))


def qtip_decode_states(states, count, L, V, code_id, lut, out, stream=None):
    return _check(lib().qtip_decode_states(_ptr(states), count, L, V, code_id, _ptr(lut),
                                           _ptr(out), _stream(stream)))


def qtip_quantize(W, m, n, L, k, V, code_id, lut=None):
    """Host quantizer: W float32 (m, n) numpy -> (codes uint32 (tiles, 8k), mse)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    assert W.shape == (m, n)
    if lut is not None:
        lut = np.ascontiguousarray(lut)
        assert lut.dtype in (np.float16, np.uint16) and lut.size == {CODE_LUT: 1 << 14, CODE_HYB1: 64}.get(code_id, 1024)
    codes = np.zeros((m * n // 256, 8 * k), dtype=np.uint32)  # one sequence per 256 weights
    mse = ctypes.c_double(0.0)
    _check(lib().qtip_quantize(_ptr(W), m, n, L, k, V, code_id, _ptr(lut), _ptr(codes),
                               ctypes.addressof(mse)))
    return codes, float(mse.value)


def qtip_quantize_gpu_workspace(k, V, tiles):
    return int(lib().qtip_quantize_gpu_workspace(k, V, tiles))


def qtip_quantize_gpu(W, m, n, L, k, V, code_id, lut, codes_out, tile_err, workspace,
                      workspace_bytes, stream=None):
    return _check(lib().qtip_quantize_gpu(_ptr(W), m, n, L, k, V, code_id, _ptr(lut),
                                          _ptr(codes_out), _ptr(tile_err), _ptr(workspace),
                                          workspace_bytes, _stream(stream)))


def qtip_block_ldl_workspace(n):
    return int(lib().qtip_block_ldl_workspace(n))


def qtip_block_ldl(H, n, g, A_out, D_out, workspace, workspace_bytes, stream=None):
    return _check(lib().qtip_block_ldl(_ptr(H), n, g, _ptr(A_out), _ptr(D_out), _ptr(workspace),
                                       workspace_bytes, _stream(stream)))


def qtip_quantize_ldlq_workspace(m, n, k, V, tiles):
    return int(lib().qtip_quantize_ldlq_workspace(m, n, k, V, tiles))


def qtip_quantize_ldlq(W, A, m, n, L, k, V, code_id, lut, codes_out, What_out, tile_err, workspace,
                       workspace_bytes, stream=None):
    return _check(lib().qtip_quantize_ldlq(_ptr(W), _ptr(A), m, n, L, k, V, code_id, _ptr(lut),
                                           _ptr(codes_out), _ptr(What_out), _ptr(tile_err),
                                           _ptr(workspace), workspace_bytes, _stream(stream)))
