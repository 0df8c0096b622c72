// Launchers shared between the C-ABI entry points and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qtip {

hipError_t launch_dequantize(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                             int n, void *W, hipStream_t st);
hipError_t launch_matvec(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                         int n, const void *x, const void *scale, float *y, hipStream_t st);
hipError_t launch_matmat(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                         int n, const void *X, int B, const void *scale, float *Y, hipStream_t st);
// decode + matvec that computes the input-side transform V (S .* x) itself; n at most
// fused_rht_matvec_max_n().
int fused_rht_matvec_max_n();
hipError_t launch_rht_matvec(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                             int n, const void *x, const int8_t *signs, int block, const void *scale,
                             float *y, hipStream_t st);
hipError_t launch_decode_states(int code_id, const uint32_t *states, int count,
                                const uint32_t *lut, void *out, hipStream_t st);
hipError_t launch_rht(const void *x, bool x_is_f32, const int8_t *signs, int n, int block,
                      int batch, int side, void *out, hipStream_t st);

// The lookup-only code (qtip_lut14.hip): L = 14, V = 1, 32 x 8 blocks, lut = 2^14 fp16 values.
hipError_t launch_lut_dequantize(int k, const uint32_t *codes, const void *lut, int m, int n, void *W,
                                 hipStream_t st);
hipError_t launch_lut_matvec(int k, const uint32_t *codes, const void *lut, int m, int n, const void *x,
                             const void *scale, float *y, hipStream_t st);
hipError_t launch_lut_matmat(int k, const uint32_t *codes, const void *lut, int m, int n, const void *X,
                             int B, const void *scale, float *Y, hipStream_t st);
hipError_t launch_lut_decode_states(const uint32_t *states, int count, const void *lut, void *out,
                                    hipStream_t st);

// Host-only tail-biting Viterbi quantizer (qtip_quantize.cpp).
int quantize_host(const float *W, int m, int n, int L, int k, int V, int code_id, const uint16_t *lut,
                  uint32_t *codes_out, double *mse_out);

// GPU tail-biting Viterbi quantizer (qtip_viterbi.hip).  W is m x n with row stride ld
// (elements).  hipErrorInvalidValue if the workspace cannot hold one sequence.
size_t quantize_gpu_workspace(int k, int V, long tiles);
hipError_t launch_quantize_gpu(int k, int code_id, const float *W, int m, int n, int ld, const uint32_t *lut,
                               uint32_t *codes, float *tile_err, void *ws, size_t ws_bytes,
                               hipStream_t st);

// BlockLDLQ (qtip_ldlq.hip): block LDL decomposition in binary64 and Algorithm 5's loop.
size_t block_ldl_workspace(int n);
hipError_t launch_block_ldl(const double *H, int n, int g, float *A, double *Dout, void *ws, hipStream_t st);
size_t quantize_ldlq_workspace(int m, int n, int k, int V, long tiles);
hipError_t launch_quantize_ldlq(int k, int V, int code_id, const float *W, const float *A, int m, int n,
                                const uint32_t *lut, uint32_t *codes, float *What, float *tile_err,
                                void *ws, size_t ws_bytes, hipStream_t st);

}  // namespace qtip
