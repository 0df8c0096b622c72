"""MI355X-native QTIP inference path: thin Python binding over libqtip.so.

All arithmetic runs in the HIP kernels behind the C ABI of include/qtip.h; this
package only marshals arguments.  torch is used for device memory and streams.
"""
from .binding import (CODE_1MAD, CODE_3INST, CODE_HYB, CODE_HYB2, CODE_LUT, CODE_HYB1, QtipError, lib, library_path,
                      qtip_decode_matmat, qtip_decode_matvec, qtip_decode_states,
                      qtip_dequantize, qtip_last_error, qtip_quantize, qtip_quantize_gpu,
                      qtip_quantize_gpu_workspace, qtip_block_ldl, qtip_block_ldl_workspace,
                      qtip_quantize_ldlq, qtip_quantize_ldlq_workspace, qtip_rht, qtip_rht_decode_matvec,
                      qtip_rht_decode_matvec_noalloc,
                      qtip_rht_f32,
                      qtip_version)

__all__ = ["CODE_1MAD", "CODE_3INST", "CODE_HYB", "CODE_HYB2", "CODE_LUT", "CODE_HYB1", "QtipError", "lib", "library_path",
           "qtip_decode_matmat", "qtip_decode_matvec", "qtip_decode_states", "qtip_dequantize",
           "qtip_last_error", "qtip_quantize", "qtip_quantize_gpu", "qtip_quantize_gpu_workspace",
           "qtip_block_ldl", "qtip_block_ldl_workspace", "qtip_quantize_ldlq", "qtip_quantize_ldlq_workspace",
           "qtip_rht", "qtip_rht_decode_matvec", "qtip_rht_decode_matvec_noalloc", "qtip_rht_f32", "qtip_version"]
