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

// LDS slot of element idx: one pad word per 32 keeps the stride-16 and stride-256
// access patterns of the exchange rounds down to two-way bank conflicts.
// (Blocks above 8192 would not fit 64 KiB with the padding and go without.)
__device__ __forceinline__ int rht_slot(int idx, int padmask) {
    return idx + ((idx >> 5) & padmask);
}

// 16 consecutive inputs of one thread as floats (first round: idx = 16u + e).
__device__ __forceinline__ void load16(const half_t *p, float (&v)[16]) {
    const uint4 a = reinterpret_cast<const uint4 *>(p)[0], b = reinterpret_cast<const uint4 *>(p)[1];
    const uint32_t r[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 8; i++) {
        half2_t h = as_half2(r[i]);
        v[2 * i] = (float)h.x;
        v[2 * i + 1] = (float)h.y;
    }
}
__device__ __forceinline__ void load16(const float *p, float (&v)[16]) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const float4 t = reinterpret_cast<const float4 *>(p)[i];
        v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
    }
}
// 16 consecutive +-1 signs applied through the sign bit.
__device__ __forceinline__ void apply_signs16(const int8_t *sg, float (&v)[16]) {
    const uint4 t = *reinterpret_cast<const uint4 *>(sg);
    const uint32_t r[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int e = 0; e < 16; e++) {
        const uint32_t neg = (r[e >> 2] >> (8 * (e & 3) + 7)) & 1u;  // sign bit of the int8
        v[e] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, v[e]) ^ (neg << 31));
    }
}

// PT > 0 fixes log2(block) at compile time (index arithmetic folds away);
// PT == 0 takes it from the argument.
template <typename TIN, int PT>
__global__ __launch_bounds__(256) void rht_kernel(const TIN *__restrict__ x,
                                                  const int8_t *__restrict__ signs, int n, int prt,
                                                  int side, half_t *__restrict__ out) {
    extern __shared__ float s_v[];
    const int p = PT > 0 ? PT : prt;
    const int b = 1 << p;
    const size_t base = (size_t)blockIdx.y * n + (size_t)blockIdx.x * b;
    const int8_t *sg = signs + (size_t)blockIdx.x * b;
    const float inv = 1.0f / sqrtf((float)b);
    const int units = b >> 4;
    const int padmask = b <= 8192 ? -1 : 0;
#pragma unroll
    for (int lo = 0; lo < (PT > 0 ? PT : 16); lo += 4) {
        if (lo >= p) break;
        const int q = min(4, p - lo);
        const bool first = lo == 0, last = lo + q == p;
        for (int u = threadIdx.x; u < units; u += 256) {
            float v[16];
            if (first) {
                // block >= 16, so the first round always owns bits 0..3: idx = 16u + e
                load16(x + base + 16 * u, v);
                if (side == 0) apply_signs16(sg + 16 * u, v);
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) v[e] = s_v[rht_slot(rht_index(u, e, lo, q), padmask)];
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
                    s_v[rht_slot(idx, padmask)] = v[e];
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
    const size_t lds = (size_t)(block <= 8192 ? block + (block >> 5) + 1 : block) * sizeof(float);
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
