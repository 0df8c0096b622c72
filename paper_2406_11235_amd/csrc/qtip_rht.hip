// Random Hadamard transform of activations (Section 2.1 of arXiv 2406.11235):
// a block-diagonal fast Walsh-Hadamard transform with +-1 sign vectors.
//
// One workgroup transforms one block of one batch row with rht_block (qtip_rht_device.h).
#include "qtip_device.h"
#include "qtip_internal.h"
#include "qtip_rht_device.h"

namespace qtip {

// PT > 0 fixes log2(block) at compile time; PT == 0 takes it from the argument.
template <typename TIN, int PT>
__global__ __launch_bounds__(256) void rht_kernel(const TIN *__restrict__ x,
                                                  const int8_t *__restrict__ signs, int n, int prt,
                                                  int side, half_t *__restrict__ out) {
    extern __shared__ float s_v[];
    const int b = 1 << (PT > 0 ? PT : prt);
    const size_t base = (size_t)blockIdx.y * n + (size_t)blockIdx.x * b;
    half_t *o = out + base;
    rht_block<TIN, PT>(x + base, signs + (size_t)blockIdx.x * b, prt, side, s_v, threadIdx.x, 256,
                       [o](int idx, half_t v) { o[idx] = v; });
}

hipError_t launch_rht(const void *x, bool x_is_f32, const int8_t *signs, int n, int block,
                      int batch, int side, void *out, hipStream_t st) {
    int p = 0;
    while ((1 << p) < block) p++;
    dim3 grid(n / block, batch);
    const size_t lds = (size_t)rht_lds_floats(block) * sizeof(float);
#define QTIP_RHT_LAUNCH(T, PT)                                                                   \
    hipLaunchKernelGGL((rht_kernel<T, PT>), grid, dim3(256), lds, st, (const T *)x, signs, n, p, \
                       side, (half_t *)out)
#define QTIP_RHT_BY_P(T)                                  \
    switch (p) {                                          \
        case 10: QTIP_RHT_LAUNCH(T, 10); break;           \
        case 11: QTIP_RHT_LAUNCH(T, 11); break;           \
        case 12: QTIP_RHT_LAUNCH(T, 12); break;           \
        case 13: QTIP_RHT_LAUNCH(T, 13); break;           \
        default: QTIP_RHT_LAUNCH(T, 0); break;            \
    }
    if (x_is_f32) {
        QTIP_RHT_BY_P(float);
    } else {
        QTIP_RHT_BY_P(half_t);
    }
    return hipGetLastError();
}

}  // namespace qtip
