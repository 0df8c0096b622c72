// Random Hadamard transform of activations (Section 2.1 of arXiv 2406.11235):
// a block-diagonal fast Walsh-Hadamard transform with +-1 sign vectors.
//
// One workgroup transforms one block of one batch row.  The log2(block) butterfly
// stages run four at a time on 16 values held in registers; between such rounds
// the values are exchanged through LDS, each round owning a different group of
// four index bits.  Arithmetic is fp32; the 1/sqrt(block) scale and the fp16
// rounding happen once, at the final store.
#include "qtip_device.h"
#include "qtip_internal.h"

namespace qtip {

template <int Q>
__device__ __forceinline__ void butterflies(float (&v)[16]) {
#pragma unroll
    for (int h = 1; h < (1 << Q); h <<= 1)
#pragma unroll
        for (int e = 0; e < 16; e++)
            if ((e & h) == 0) {
                float a = v[e], b = v[e | h];
                v[e] = a + b;
                v[e | h] = a - b;
            }
}

// Element index of register e of unit u in a round that owns index bits
// [lo, lo + q): the low q bits of e are those bits, the rest of e extends u.
__device__ __forceinline__ int rht_index(int u, int e, int lo, int q) {
    const int rest = (u << (4 - q)) | (e >> q);
    const int el = e & ((1 << q) - 1);
    return ((rest >> lo) << (lo + q)) | (el << lo) | (rest & ((1 << lo) - 1));
}

template <typename TIN>
__global__ __launch_bounds__(256) void rht_kernel(const TIN *__restrict__ x,
                                                  const int8_t *__restrict__ signs, int n, int p,
                                                  int side, half_t *__restrict__ out) {
    extern __shared__ float s_v[];
    const int b = 1 << p;
    const size_t base = (size_t)blockIdx.y * n + (size_t)blockIdx.x * b;
    const int8_t *sg = signs + (size_t)blockIdx.x * b;
    const float inv = 1.0f / sqrtf((float)b);
    const int units = b >> 4;
    for (int lo = 0; lo < p; lo += 4) {
        const int q = min(4, p - lo);
        const bool first = lo == 0, last = lo + q == p;
        for (int u = threadIdx.x; u < units; u += 256) {
            float v[16];
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int idx = rht_index(u, e, lo, q);
                if (first) {
                    float t = (float)x[base + idx];
                    v[e] = side == 0 ? t * (float)sg[idx] : t;
                } else {
                    v[e] = s_v[idx];
                }
            }
            if (q == 4) butterflies<4>(v);
            else if (q == 3) butterflies<3>(v);
            else if (q == 2) butterflies<2>(v);
            else butterflies<1>(v);
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int idx = rht_index(u, e, lo, q);
                if (last) {
                    float t = v[e] * inv;
                    if (side != 0) t *= (float)sg[idx];
                    out[base + idx] = (half_t)t;
                } else {
                    s_v[idx] = v[e];
                }
            }
        }
        __syncthreads();
    }
}

hipError_t launch_rht(const void *x, bool x_is_f32, const int8_t *signs, int n, int block,
                      int batch, int side, void *out, hipStream_t st) {
    int p = 0;
    while ((1 << p) < block) p++;
    dim3 grid(n / block, batch);
    const size_t lds = (size_t)block * sizeof(float);
    if (x_is_f32)
        hipLaunchKernelGGL((rht_kernel<float>), grid, dim3(256), lds, st, (const float *)x, signs,
                           n, p, side, (half_t *)out);
    else
        hipLaunchKernelGGL((rht_kernel<half_t>), grid, dim3(256), lds, st, (const half_t *)x, signs,
                           n, p, side, (half_t *)out);
    return hipGetLastError();
}

}  // namespace qtip
