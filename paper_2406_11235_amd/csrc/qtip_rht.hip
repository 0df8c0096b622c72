// Random Hadamard transform of activations (Section 2.1 of arXiv 2406.11235):
// a block-diagonal fast Walsh-Hadamard transform with +-1 sign vectors.
//
// One workgroup of 256 threads transforms one block of 4096 or more values of one batch
// row, or as many smaller blocks as make 4096 values (a thread holds 16 values per round),
// with rht_block (qtip_rht_device.h).
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
    const int p = PT > 0 ? PT : prt;
    const int b = 1 << p;
    // groups of b/16 threads, one block each, when the block is below 4096
    const int gthreads = b >= 4096 ? 256 : b >> 4;
    const int group = threadIdx.x / gthreads, gtid = threadIdx.x % gthreads;
    const int blk = blockIdx.x * (256 / gthreads) + group;
    const bool active = (size_t)blk * b < (size_t)n;
    const size_t base = (size_t)blockIdx.y * n + (active ? (size_t)blk * b : 0);
    half_t *o = out + base;
    rht_block<TIN, PT>(x + base, signs + (active ? (size_t)blk * b : 0), prt, side,
                       s_v + group * rht_lds_floats(b), gtid, gthreads, active,
                       [o](int idx, half_t v) { o[idx] = v; });
}

hipError_t launch_rht(const void *x, bool x_is_f32, const int8_t *signs, int n, int block,
                      int batch, int side, void *out, hipStream_t st) {
    int p = 0;
    while ((1 << p) < block) p++;
    const int per_wg = block >= 4096 ? 1 : 4096 / block;  // blocks per workgroup
    dim3 grid((n / block + per_wg - 1) / per_wg, batch);
    const size_t lds = (size_t)rht_lds_floats(block) * per_wg * sizeof(float);
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
