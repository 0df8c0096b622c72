// BlockLDLQ with the trellis quantizer as its rounder (Algorithm 5 of arXiv 2406.11235;
// T_x = T_y = 16 for the codes of Algorithms 1-3, T_x = 32 and T_y = 8 for the lookup-only
// code, whose smaller group size is the reason the paper gives for that shape; the comments
// below say 16 for T_y = G): the block LDL decomposition of the proxy Hessian and the loop over
// column blocks, last to first, that quantizes x = W_j + (W - What)_{>j} A_{>j,j} tile by
// tile with the GPU Viterbi quantizer and feeds the error of every finished block forward.
//
// Block LDL (H = L D L^T, L unit block lower triangular, D block diagonal, A = L - I) runs
// in binary64 on the device, right-looking, two launches per block column: a panel kernel
// (invert the 16x16 diagonal block, scale the column below it) and a trailing update on the
// lower triangle.  It is a one-off of n^3/3 multiply-adds per layer.
//
// The feedback sum is written so that a CPU reference can repeat it bit for bit, because
// what it feeds is a quantizer, whose decisions are not continuous: binary32, one fused
// multiply-add per term E[r][i] A[i][c], the terms taken block by block from the last
// column block down, ascending inside a block (the order in which a running sum that is
// updated after every finished block receives them).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qtip_device.h"
#include "qtip_internal.h"

namespace qtip {
namespace {

// G = T_y = block size of the decomposition = width of a sequence's block of the matrix

// ------------------------------------------------------------------ block LDL

__global__ void ldl_init_kernel(const double *__restrict__ H, double *__restrict__ S,
                                double *__restrict__ Lm, int n) {
    const size_t total = (size_t)n * n;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        S[idx] = H[idx];
        Lm[idx] = (idx / n == idx % n) ? 1.0 : 0.0;
    }
}

// Workgroup b of step j: b = 0 stores D_j; b > 0 computes L_ij = S_ij D_j^-1 for block row
// i = j + b.  Every workgroup inverts D_j itself (Gauss-Jordan in LDS, no pivoting: the
// block is symmetric positive definite).
template <int G>
__global__ __launch_bounds__(G * G) void ldl_panel_kernel(double *__restrict__ S, double *__restrict__ Lm,
                                                        int n, int j, double *__restrict__ Dout) {
    __shared__ double s_aug[G][2 * G + 1];
    __shared__ double s_t[G][G + 1];
    const int r = threadIdx.x / G, c = threadIdx.x % G;
    const int o = j * G;
    const double d = S[(size_t)(o + r) * n + o + c];
    s_aug[r][c] = d;
    s_aug[r][G + c] = r == c ? 1.0 : 0.0;
    if (blockIdx.x == 0 && Dout) Dout[((size_t)j * G + r) * G + c] = d;
    __syncthreads();
    for (int p = 0; p < G; p++) {
        const double piv = s_aug[p][p];
        __syncthreads();
        if (r == p) {
            s_aug[p][c] /= piv;
            s_aug[p][G + c] /= piv;
        }
        __syncthreads();
        const double f = s_aug[r][p];
        const double a0 = s_aug[p][c], a1 = s_aug[p][G + c];
        __syncthreads();
        if (r != p) {
            s_aug[r][c] -= f * a0;
            s_aug[r][G + c] -= f * a1;
        }
        __syncthreads();
    }
    if (blockIdx.x == 0) return;
    const int i0 = (j + blockIdx.x) * G;
    s_t[r][c] = S[(size_t)(i0 + r) * n + o + c];
    __syncthreads();
    double acc = 0.0;
#pragma unroll
    for (int q = 0; q < G; q++) acc += s_t[r][q] * s_aug[q][G + c];
    Lm[(size_t)(i0 + r) * n + o + c] = acc;
}

// S_ik -= L_ij (S_kj)^T for the blocks i >= k > j (D_j is symmetric, so L_ij D_j L_kj^T is
// L_ij times the transpose of the untouched S_kj = L_kj D_j).
template <int G>
__global__ __launch_bounds__(G * G) void ldl_update_kernel(double *__restrict__ S, const double *__restrict__ Lm,
                                                         int n, int j) {
    const int bi = j + 1 + blockIdx.y, bk = j + 1 + blockIdx.x;
    if (bk > bi) return;
    __shared__ double s_l[G][G + 1], s_s[G][G + 1];
    const int r = threadIdx.x / G, c = threadIdx.x % G;
    const int o = j * G;
    s_l[r][c] = Lm[(size_t)(bi * G + r) * n + o + c];
    s_s[r][c] = S[(size_t)(bk * G + r) * n + o + c];
    __syncthreads();
    double acc = 0.0;
#pragma unroll
    for (int q = 0; q < G; q++) acc += s_l[r][q] * s_s[c][q];
    S[(size_t)(bi * G + r) * n + bk * G + c] -= acc;
}

// A = L - I in binary32: the blocks strictly below the diagonal blocks, zero elsewhere.
__global__ void ldl_emit_kernel(const double *__restrict__ Lm, float *__restrict__ A, int n, int G) {
    const size_t total = (size_t)n * n;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int row = (int)(idx / n), col = (int)(idx % n);
        A[idx] = (row / G > col / G) ? (float)Lm[idx] : 0.f;
    }
}

// ------------------------------------------------------------------ Algorithm 5

// The feedback of Algorithm 5 as a running sum: X starts as W; when column block j is done,
// its error E_j = (W - What)[:, 16j:16j+16] is fed to every column before it,
//     X[r][c] += sum_{i in block j, ascending} E_j[r][i] A[16 j + i][c],   c < 16 j,
// one fused multiply-add per term.  When block j's turn comes, X[:, 16j:16j+16] is its x.
// Per element the terms arrive by blocks from the last one down and ascending inside a
// block: that order is the definition both sides use.  A thread owns one column and 8 rows:
// 16 values of A in registers, the rows' errors are wave-uniform.
constexpr int UPD_ROWS = 8;
template <int G>
__global__ __launch_bounds__(256) void ldlq_update_kernel(const float *__restrict__ Eslab,
                                                          const float *__restrict__ A, int m, int n, int j,
                                                          float *__restrict__ X) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int r0 = blockIdx.y * UPD_ROWS;
    if (c >= j * G) return;
    float a[G];
#pragma unroll
    for (int i = 0; i < G; i++) a[i] = A[(size_t)(j * G + i) * n + c];
#pragma unroll
    for (int rr = 0; rr < UPD_ROWS; rr++) {
        const int r = r0 + rr;
        if (r >= m) break;
        float acc = X[(size_t)r * n + c];
#pragma unroll
        for (int i = 0; i < G; i++) acc = __builtin_fmaf(Eslab[(size_t)r * G + i], a[i], acc);
        X[(size_t)r * n + c] = acc;
    }
}

__global__ void ldlq_copy_kernel(const float *__restrict__ src, float *__restrict__ dst, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// After block j is quantized: its error slab E_j and What from the decoded slab, and the
// slab's codes and errors to their places in the matrix's tile order.
// (TX x G is the block that is one sequence, so the slab holds m / TX of them.)
template <int G, int TX>
__global__ __launch_bounds__(256) void ldlq_finish_kernel(const float *__restrict__ W,
                                                          const half_t *__restrict__ slab,
                                                          const uint32_t *__restrict__ slab_codes,
                                                          const float *__restrict__ slab_err, int m, int n,
                                                          int j, int nwords, float *__restrict__ Eslab,
                                                          float *__restrict__ What,
                                                          uint32_t *__restrict__ codes,
                                                          float *__restrict__ tile_err) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int r = idx / G, c = idx % G;
    if (r >= m) return;
    const float w = (float)slab[(size_t)r * G + c];
    const size_t at = (size_t)r * n + j * G + c;
    Eslab[(size_t)r * G + c] = W[at] - w;
    if (What) What[at] = w;
    const int tn = n / G;
    if (idx < (m / TX) * nwords) {
        const int I = idx / nwords, wd = idx % nwords;
        codes[((size_t)I * tn + j) * nwords + wd] = slab_codes[idx];
    }
    if (tile_err && idx < m / TX) tile_err[(size_t)idx * tn + j] = slab_err[idx];
}

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

}  // namespace

size_t block_ldl_workspace(int n) { return 2 * align256((size_t)n * n * sizeof(double)); }

template <int G>
static hipError_t block_ldl_t(const double *H, int n, float *A, double *Dout, void *ws, hipStream_t st) {
    double *S = (double *)ws;
    double *Lm = (double *)((char *)ws + align256((size_t)n * n * sizeof(double)));
    const int nb = n / G;
    hipLaunchKernelGGL(ldl_init_kernel, dim3(1024), dim3(256), 0, st, H, S, Lm, n);
    for (int j = 0; j < nb; j++) {
        hipLaunchKernelGGL(ldl_panel_kernel<G>, dim3(nb - j), dim3(G * G), 0, st, S, Lm, n, j, Dout);
        if (j + 1 < nb)
            hipLaunchKernelGGL(ldl_update_kernel<G>, dim3(nb - j - 1, nb - j - 1), dim3(G * G), 0, st, S,
                               (const double *)Lm, n, j);
    }
    hipLaunchKernelGGL(ldl_emit_kernel, dim3(1024), dim3(256), 0, st, (const double *)Lm, A, n, G);
    return hipGetLastError();
}

hipError_t launch_block_ldl(const double *H, int n, int g, float *A, double *Dout, void *ws, hipStream_t st) {
    return g == 8 ? block_ldl_t<8>(H, n, A, Dout, ws, st) : block_ldl_t<16>(H, n, A, Dout, ws, st);
}

// Workspace of the loop: the running sum X (m x n), the error slab (m x G), the decoded
// slab (fp16 m x G), the slab's codes and errors, then the Viterbi quantizer's own workspace.
static size_t ldlq_fixed_bytes(int m, int n, int k, int G, int TX) {
    return align256((size_t)m * n * 4) + align256((size_t)m * G * 4) + align256((size_t)m * G * 2) +
           align256((size_t)(m / TX) * 8 * k * 4) + align256((size_t)(m / TX) * 4);
}

// (sized for 16 x 16 blocks, which is also enough for 32 x 8)
size_t quantize_ldlq_workspace(int m, int n, int k, int V, long tiles) {
    if (tiles > m / 16) tiles = m / 16;
    return ldlq_fixed_bytes(m, n, k, 16, 16) + quantize_gpu_workspace(k, V, tiles);
}

template <int G, int TX>
static hipError_t quantize_ldlq_t(int k, int code_id, const float *W, const float *A, int m, int n,
                                  const uint32_t *lut, uint32_t *codes, float *What, float *tile_err,
                                  void *ws, size_t ws_bytes, hipStream_t st) {
    char *p = (char *)ws;
    float *X = (float *)p;
    p += align256((size_t)m * n * 4);
    float *Eslab = (float *)p;
    p += align256((size_t)m * G * 4);
    half_t *slab = (half_t *)p;
    p += align256((size_t)m * G * 2);
    uint32_t *slab_codes = (uint32_t *)p;
    p += align256((size_t)(m / TX) * 8 * k * 4);
    float *slab_err = (float *)p;
    p += align256((size_t)(m / TX) * 4);
    const size_t fixed = ldlq_fixed_bytes(m, n, k, G, TX);
    if (ws_bytes <= fixed) return hipErrorInvalidValue;
    const size_t qbytes = ws_bytes - fixed;
    const int nwords = 8 * k;
    const dim3 egrid((m * G + 255) / 256);
    hipLaunchKernelGGL(ldlq_copy_kernel, dim3(1024), dim3(256), 0, st, W, X, (size_t)m * n);
    for (int j = n / G - 1; j >= 0; j--) {
        // column block j of X is complete: quantize it in place (row stride n)
        hipError_t e = launch_quantize_gpu(k, code_id, X + (size_t)j * G, m, G, n, lut, slab_codes, slab_err, p,
                                           qbytes, st);
        if (e != hipSuccess) return e;
        e = launch_dequantize(k, code_id, slab_codes, lut, m, G, slab, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((ldlq_finish_kernel<G, TX>), egrid, dim3(256), 0, st, W, (const half_t *)slab,
                           (const uint32_t *)slab_codes, (const float *)slab_err, m, n, j, nwords, Eslab, What,
                           codes, tile_err);
        if (j > 0)
            hipLaunchKernelGGL(ldlq_update_kernel<G>, dim3((j * G + 255) / 256, (m + UPD_ROWS - 1) / UPD_ROWS),
                               dim3(256), 0, st, (const float *)Eslab, A, m, n, j, X);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_quantize_ldlq(int k, int V, int code_id, const float *W, const float *A, int m, int n,
                                const uint32_t *lut, uint32_t *codes, float *What, float *tile_err,
                                void *ws, size_t ws_bytes, hipStream_t st) {
    (void)V;
    if (code_id == CODE_LUT)
        return quantize_ldlq_t<8, 32>(k, code_id, W, A, m, n, lut, codes, What, tile_err, ws, ws_bytes, st);
    return quantize_ldlq_t<16, 16>(k, code_id, W, A, m, n, lut, codes, What, tile_err, ws, ws_bytes, st);
}

}  // namespace qtip
