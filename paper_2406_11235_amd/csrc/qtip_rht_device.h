// Device-side core of the random Hadamard transform (Section 2.1 of arXiv 2406.11235):
// one block of a block-diagonal fast Walsh-Hadamard transform with +-1 signs, done by all
// threads of a workgroup.  The log2(block) butterfly stages run four at a time on 16
// values held in registers; between such rounds the values are exchanged through LDS,
// each round owning a different group of four index bits.  Arithmetic is fp32; the
// 1/sqrt(block) scale and the fp16 rounding happen once, at the final store.  Used by the
// stand-alone kernel and by the decode + matvec kernel that transforms its own input.
#pragma once
#include "qtip_device.h"

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

// One block of 2^p values: x (global) -> store(idx, fp16 value).  A group of `nthreads`
// threads (`tid` = 0 .. nthreads-1) works on one block; several groups of a workgroup may
// work on different blocks, each with its own s_v, as long as EVERY thread of the workgroup
// makes the call with the same p: it synchronizes the workgroup after every round, the last
// included.  Threads with active = false only take part in the synchronization.  PT > 0 fixes p at compile time (index arithmetic folds away); PT == 0 takes it
// from the argument.  sg: the block's signs.  side 0: V (S .* x); side 1: S .* (V^T x).
// s_v: LDS scratch of 2^p floats, plus one per 32 when 2^p <= 8192.
template <typename TIN, int PT, typename STORE>
__device__ __forceinline__ void rht_block(const TIN *__restrict__ x, const int8_t *__restrict__ sg, int prt,
                                          int side, float *s_v, int tid, int nthreads, bool active,
                                          STORE store) {
    const int p = PT > 0 ? PT : prt;
    const int b = 1 << p;
    // 2^(-p/2) as an exact power of two times the correctly rounded 1/sqrt(2): the same bits
    // whether p is known at compile time or not (a run-time 1/sqrtf is not exactly rounded)
    const float inv = ((p & 1) ? 0.70710678118654752440f : 1.0f) *
                      __builtin_bit_cast(float, (uint32_t)(127 - (p >> 1)) << 23);
    const int units = b >> 4;
    const int padmask = b <= 8192 ? -1 : 0;
#pragma unroll
    for (int lo = 0; lo < (PT > 0 ? PT : 16); lo += 4) {
        if (lo >= p) break;
        const int q = min(4, p - lo);
        const bool first = lo == 0, last = lo + q == p;
        for (int u = active ? tid : units; u < units; u += nthreads) {
            float v[16];
            if (first) {
                // block >= 16, so the first round always owns bits 0..3: idx = 16u + e
                load16(x + 16 * u, v);
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
                    // Keep the fp32 product and the fp16 rounding apart: left alone, the
                    // compiler merges them into one v_fma_mixlo_f16 (a single rounding) in
                    // some instantiations and not in others, and the last fp16 bit differs.
                    asm volatile("" : "+v"(t));
                    store(idx, (half_t)t);
                } else {
                    s_v[rht_slot(idx, padmask)] = v[e];
                }
            }
        }
        __syncthreads();
    }
}

// LDS floats rht_block needs for a block of `block` values.
__host__ __device__ constexpr int rht_lds_floats(int block) {
    return block <= 8192 ? block + (block >> 5) + 1 : block;
}

}  // namespace qtip
