// Decode kernels for the lookup-only code (the appendix on lookup-only codes of arXiv
// 2406.11235): L = 14, V = 1, a stored table of 2^14 fp16 values, and T_x = 32, T_y = 8, so a
// sequence of 256 weights is a 32 x 8 block (32 outputs, 8 inputs).
//
// Two things that the paper counts against this code on the GPUs it names are different
// on this chip.  The table is 32 KiB and a CU has 160 KiB of LDS, so every workgroup simply
// keeps a copy of its own.  And T_x = 32 is the row count of the 32x32x16 matrix-core
// instruction: two neighbouring blocks (J, J+1) of a block row are its 32 x 16 A operand, with
// lane (row i, half s) holding exactly block row i of block J + s, eight weights that sit
// next to each other in the stream.
//
// The work split is that of the 16 x 16 kernels: a workgroup owns one block row I (32 outputs),
// its waves take contiguous ranges of J and meet in LDS at the end.
#include "qtip_device.h"
#include "qtip_internal.h"

namespace qtip {
namespace {

constexpr int LUT_L = 14;
constexpr int LUT_STATES = 1 << LUT_L;
constexpr int LUT_TX = 32, LUT_TY = 8;

__device__ __forceinline__ void stage_table(const uint16_t *__restrict__ lut, uint16_t *s_tab, int nthreads) {
    const uint4 *src = reinterpret_cast<const uint4 *>(lut);
    uint4 *dst = reinterpret_cast<uint4 *>(s_tab);
    for (int i = threadIdx.x; i < LUT_STATES * 2 / 16; i += nthreads) dst[i] = src[i];
}

// Byte offset (2 * state) in the table of the weight whose state starts P bits into w.
template <int NW>
__device__ __forceinline__ uint32_t table_offset(const uint32_t (&w)[NW], int P) {
    // the 14 state bits end up in bits 14..1
    if (P < 17) return (w[0] >> (17 - P)) & 0x7FFEu;
    return window32(w, P - 17) & 0x7FFEu;
}
// The same for the two weights at P and P + 16 from one 32-bit window.
template <int NW>
__device__ __forceinline__ void table_offset_pair(const uint32_t (&w)[NW], int P, uint32_t &a, uint32_t &b) {
    if (P == 0) {
        a = (w[0] >> 17) & 0x7FFEu;
        b = (w[0] >> 1) & 0x7FFEu;
    } else {
        const uint32_t A = window32(w, P - 1);  // state(P) in bits 30..17, state(P + 16) in bits 14..1
        a = (A >> 16) & 0x7FFEu;
        b = A & 0x7FFEu;
    }
}
__device__ __forceinline__ half_t table_at(const uint16_t *tab, uint32_t byte_offset) {
    return *reinterpret_cast<const half_t *>(reinterpret_cast<const char *>(tab) + byte_offset);
}

// Table offsets of all weights of a lane: WL = 32 WPL / K weights from bit 0 of w.
template <int K, int WL, int NW>
__device__ __forceinline__ void lane_offsets(const uint32_t (&w)[NW], uint32_t (&off)[WL]) {
    if constexpr (K == 2 || K == 4) {
        constexpr int G = 16 / K;  // weights 16 bits apart share a window
#pragma unroll
        for (int base = 0; base < WL; base += 2 * G)
#pragma unroll
            for (int j = 0; j < G; j++) table_offset_pair(w, (base + j) * K, off[base + j], off[base + j + G]);
    } else {
#pragma unroll
        for (int c = 0; c < WL; c++) off[c] = table_offset(w, c * K);
    }
}

// ---------------------------------------------------------------- dequantize

template <int K>
__global__ __launch_bounds__(256) void lut_dequantize_kernel(const uint32_t *__restrict__ codes,
                                                             const uint16_t *__restrict__ lut, int tn,
                                                             long ntiles, half_t *__restrict__ W) {
    constexpr int WPL = Geo<K>::WPL, LPT = Geo<K>::LPT;
    constexpr int WL = WPL * 32 / K, RL = WL / LUT_TY;
    constexpr int TPW = 64 / LPT;
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long tile = wave * TPW + lane / LPT;
    const bool valid = tile < ntiles;
    const int q = lane & (LPT - 1);
    const Words<K> r = load_words<K>(codes, valid ? tile : ntiles - 1, q);
    uint32_t w[WPL + 1];
#pragma unroll
    for (int i = 0; i < WPL; i++) w[i] = r.v[i];
    w[WPL] = __shfl(w[0], (lane & ~(LPT - 1)) | ((q + 1) & (LPT - 1)), 64);
    if (!valid) return;
    const long I = tile / tn, J = tile % tn;
    const size_t n = (size_t)tn * LUT_TY;
    uint32_t off[WL];
    lane_offsets<K, WL>(w, off);
#pragma unroll
    for (int rr = 0; rr < RL; rr++) {
        uint32_t h[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const half2_t p = {table_at(lut, off[8 * rr + 2 * c]), table_at(lut, off[8 * rr + 2 * c + 1])};
            h[c] = as_u32(p);
        }
        *reinterpret_cast<uint4 *>(W + (size_t)(LUT_TX * I + q * RL + rr) * n + LUT_TY * J) =
            uint4{h[0], h[1], h[2], h[3]};
    }
}

__global__ void lut_decode_states_kernel(const uint32_t *__restrict__ states, int count,
                                         const uint16_t *__restrict__ lut, uint16_t *__restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = lut[states[i] & (LUT_STATES - 1)];
}

// ------------------------------------------------------- decode + matvec (B = 1)

template <int K, int NW>
__global__ __launch_bounds__(NW * 64) void lut_matvec_kernel(const uint32_t *__restrict__ codes,
                                                             const uint16_t *__restrict__ lut, int tn,
                                                             const half_t *__restrict__ x,
                                                             const half_t *__restrict__ scale,
                                                             float *__restrict__ y) {
    constexpr int WPL = Geo<K>::WPL, LPT = Geo<K>::LPT;
    constexpr int WL = WPL * 32 / K, RL = WL / LUT_TY;  // weights and block rows per lane
    constexpr int TPI = 64 / LPT;                       // blocks per wave per step
    __shared__ __attribute__((aligned(16))) uint16_t s_tab[LUT_STATES];
    __shared__ float s_part[NW][LUT_TX];
    stage_table(lut, s_tab, NW * 64);
    __syncthreads();
    const int I = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane / LPT, q = lane & (LPT - 1);
    const int chunk = ((tn + NW * TPI - 1) / (NW * TPI)) * TPI;
    const int J0 = wave * chunk;
    const int Jend = min(tn, J0 + chunk);
    float acc[RL];
#pragma unroll
    for (int rr = 0; rr < RL; rr++) acc[rr] = 0.f;

    // software pipeline over two alternating operand sets, as in the 16 x 16 kernel
    struct Operands {
        Words<K> w;
        uint4 xv;
    };
    auto issue = [&](Operands &o, int Jb) {
        const int Jc = min(Jb + g, Jend - 1);  // lanes past the end re-read the last block
        o.w = load_words<K>(codes, (size_t)I * tn + Jc, q);
        o.xv = *reinterpret_cast<const uint4 *>(x + LUT_TY * Jc);
    };
    auto compute = [&](const Operands &o, int Jb) {
        uint32_t w[WPL + 1];
#pragma unroll
        for (int i = 0; i < WPL; i++) w[i] = o.w.v[i];
        w[WPL] = __shfl(w[0], (lane & ~(LPT - 1)) | ((q + 1) & (LPT - 1)), 64);  // tail-biting wrap
        if (Jb + g < Jend) {
            const uint32_t xv[4] = {o.xv.x, o.xv.y, o.xv.z, o.xv.w};
            uint32_t off[WL];
            lane_offsets<K, WL>(w, off);
#pragma unroll
            for (int rr = 0; rr < RL; rr++)
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const half2_t p = {table_at(s_tab, off[8 * rr + 2 * c]), table_at(s_tab, off[8 * rr + 2 * c + 1])};
                    acc[rr] = __builtin_amdgcn_fdot2(p, as_half2(xv[c]), acc[rr], false);
                }
        }
    };
    Operands opA, opB;
    if (J0 < Jend) issue(opA, J0);
    for (int Jb = J0; Jb < Jend; Jb += 2 * TPI) {
        if (Jb + TPI < Jend) issue(opB, Jb + TPI);
        compute(opA, Jb);
        if (Jb + TPI < Jend) {
            if (Jb + 2 * TPI < Jend) issue(opA, Jb + 2 * TPI);
            compute(opB, Jb + TPI);
        }
    }
    // lanes with equal q hold partial sums of the same rows: add over g
#pragma unroll
    for (int rr = 0; rr < RL; rr++)
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1) acc[rr] += __shfl_xor(acc[rr], off, 64);
    if (g == 0) {
#pragma unroll
        for (int rr = 0; rr < RL; rr++) s_part[wave][q * RL + rr] = acc[rr];
    }
    __syncthreads();
    if (threadIdx.x < LUT_TX) {
        float s = 0.f;
#pragma unroll
        for (int wv = 0; wv < NW; wv++) s += s_part[wv][threadIdx.x];
        const int row = LUT_TX * I + threadIdx.x;
        if (scale) s *= (float)scale[row];
        y[row] = s;
    }
}

// ------------------------------------------- decode + batched product on MFMA
//
// v_mfma_f32_32x32x16_f16, D = A * B.  A wave step covers the two blocks (I, J0), (I, J0 + 1):
//   lane l = (row i = l % 32, half s = l / 32) decodes block row i of block J0 + s: 8 weights,
//   one A operand; the B operand of lane (j = l % 32, s) is X[b0 + j][8 (J0 + s) .. + 7], one
//   16-byte load.  A and B pair contraction slots by (s, element), so the order in which the
//   hardware numbers them does not matter.  D element e of lane l is output row
//   32 I + 8 (e / 4) + 4 (l / 32) + e % 4 for batch row b0 + l % 32.
typedef float float16_t __attribute__((ext_vector_type(16)));

template <int K, int NB, int NW>
__global__ __launch_bounds__(NW * 64) void lut_matmat_kernel(const uint32_t *__restrict__ codes,
                                                             const uint16_t *__restrict__ lut, int tn,
                                                             int m, const half_t *__restrict__ X, int B,
                                                             const half_t *__restrict__ scale,
                                                             float *__restrict__ Y) {
    constexpr int NWORDS = 8 * K;
    __shared__ __attribute__((aligned(16))) uint16_t s_tab[LUT_STATES];
    __shared__ float s_part[NW - 1][NB][16][64];
    stage_table(lut, s_tab, NW * 64);
    __syncthreads();
    const int I = blockIdx.x;
    const int b0 = blockIdx.y * (32 * NB);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 31, s = lane >> 5;
    const size_t n = (size_t)tn * LUT_TY;
    const int chunk = ((tn + NW * 2 - 1) / (NW * 2)) * 2;
    const int J0 = wave * chunk;
    const int Jend = min(tn, J0 + chunk);
    // block row i starts 8 K i bits into the block; its 8 K + 14 - K bits lie in two words
    const int bit = 8 * K * i, w0 = bit >> 5, sh = bit & 31;

    float16_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[nb][e] = 0.f;

    uint32_t wn[2];
    half8_t xn[NB];
    auto issue = [&](int Jb) {
        const int J = min(Jb + s, Jend - 1);  // a half past the end re-reads the last block
        const uint32_t *tile = codes + ((size_t)I * tn + J) * NWORDS;
        wn[0] = stream_load(tile + w0);
        wn[1] = stream_load(tile + (w0 + 1) % NWORDS);  // wraps inside the block (tail-biting)
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
            const int b = b0 + 32 * nb + i;
            xn[nb] = *reinterpret_cast<const half8_t *>(X + (size_t)min(b, B - 1) * n + LUT_TY * J);
        }
    };
    // Three stages in flight: the stream words and activations of step t + 2 are being loaded,
    // the table reads of step t + 1 are issued before the matrix-core instruction of step t,
    // so that the LDS and the matrix cores work at the same time inside one wave.
    auto decode = [&](half8_t &a, half8_t (&xb)[NB], int Jb) {
        const uint64_t both = (((uint64_t)wn[0] << 32) | wn[1]) << sh;
        const uint32_t w[2] = {(uint32_t)(both >> 32), (uint32_t)both};
        const bool live = Jb + s < Jend;
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
            xb[nb] = xn[nb];
            if (!live || b0 + 32 * nb + i >= B) xb[nb] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};  // dead half / batch row
        }
        if (Jb + 2 < Jend) issue(Jb + 2);
#pragma unroll
        for (int c = 0; c < 8; c++) a[c] = table_at(s_tab, table_offset(w, c * K));
    };
    half8_t a1, x1[NB];
    if (J0 < Jend) {
        issue(J0);
        decode(a1, x1, J0);
    }
    for (int Jb = J0; Jb < Jend; Jb += 2) {
        const half8_t a = a1;
        half8_t xb[NB];
#pragma unroll
        for (int nb = 0; nb < NB; nb++) xb[nb] = x1[nb];
        if (Jb + 2 < Jend) decode(a1, x1, Jb + 2);
#pragma unroll
        for (int nb = 0; nb < NB; nb++) acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xb[nb], acc[nb], 0, 0, 0);
    }
    if (wave > 0) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int e = 0; e < 16; e++) s_part[wave - 1][nb][e][lane] = acc[nb][e];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
            const int b = b0 + 32 * nb + i;
            if (b >= B) continue;
#pragma unroll
            for (int e4 = 0; e4 < 4; e4++) {
                float4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    v[e] = acc[nb][4 * e4 + e];
#pragma unroll
                    for (int wv = 0; wv < NW - 1; wv++) v[e] += s_part[wv][nb][4 * e4 + e][lane];
                }
                const int orow = LUT_TX * I + 8 * e4 + 4 * s;
                if (scale) {
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] *= (float)scale[orow + e];
                }
                *reinterpret_cast<float4_t *>(Y + (size_t)b * m + orow) = v;
            }
        }
    }
}

// The same for more than 16 batch rows.  The B operand puts neighbouring lanes on different
// batch rows, i.e. different cache lines, which the texture path serves at a fraction of the
// rate of a load whose neighbouring lanes read neighbouring addresses.  Here a wave loads its
// activations line by line instead, for four steps at once (8 lanes = the 128 bytes one
// batch row has under eight blocks), and transposes them through a private piece of LDS, as
// the 16 x 16 kernel does.
template <int K, int NB, int NW>
__global__ __launch_bounds__(NW * 64) void lut_matmat_staged_kernel(const uint32_t *__restrict__ codes,
                                                                    const uint16_t *__restrict__ lut, int tn,
                                                                    int m, const half_t *__restrict__ X, int B,
                                                                    const half_t *__restrict__ scale,
                                                                    float *__restrict__ Y) {
    constexpr int NWORDS = 8 * K;
    constexpr int ROWS = 32 * NB, NQ = ROWS / 8, XST = 144;  // rows padded to 144 bytes (banks)
    constexpr int PART_BYTES = (NW - 1) * NB * 16 * 64 * 4, STAGE_BYTES = NW * ROWS * XST;
    __shared__ __attribute__((aligned(16))) uint16_t s_tab[LUT_STATES];
    // one buffer, used twice: the waves' staging regions in the loop, the partial sums after it
    __shared__ __attribute__((aligned(16))) char s_buf[PART_BYTES > STAGE_BYTES ? PART_BYTES : STAGE_BYTES];
    float(*s_part)[NB][16][64] = reinterpret_cast<float(*)[NB][16][64]>(s_buf);
    stage_table(lut, s_tab, NW * 64);
    __syncthreads();
    const int I = blockIdx.x;
    const int b0 = blockIdx.y * ROWS;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 31, s = lane >> 5;
    const int lr = lane >> 3, ch = lane & 7;
    char *const stage = s_buf + wave * (ROWS * XST);
    const size_t n = (size_t)tn * LUT_TY;
    const int chunk = ((tn + NW * 8 - 1) / (NW * 8)) * 8;
    const int J0 = wave * chunk;
    const int Jend = min(tn, J0 + chunk);
    const int bit = 8 * K * i, w0 = bit >> 5, sh = bit & 31;

    float16_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[nb][e] = 0.f;

    uint32_t wn[2];
    half8_t xq[NQ];  // piece ch of batch rows b0 + 8 q + lr, for the eight blocks from Jm on
    auto load_x = [&](int Jm) {
        const int Jx = min(Jm + ch, Jend - 1);
#pragma unroll
        for (int q = 0; q < NQ; q++) {
            const int b = b0 + 8 * q + lr;
            xq[q] = *reinterpret_cast<const half8_t *>(X + (size_t)min(b, B - 1) * n + LUT_TY * Jx);
        }
    };
    auto issue_w = [&](int Jb) {
        const int J = min(Jb + s, Jend - 1);  // a half past the end re-reads the last block
        const uint32_t *tile = codes + ((size_t)I * tn + J) * NWORDS;
        wn[0] = stream_load(tile + w0);
        wn[1] = stream_load(tile + (w0 + 1) % NWORDS);  // wraps inside the block (tail-biting)
    };
    auto decode = [&](half8_t &a) {
        const uint64_t both = (((uint64_t)wn[0] << 32) | wn[1]) << sh;
        const uint32_t w[2] = {(uint32_t)(both >> 32), (uint32_t)both};
#pragma unroll
        for (int c = 0; c < 8; c++) a[c] = table_at(s_tab, table_offset(w, c * K));
    };
    auto wave_sync = [] {  // the LDS operations of one wave complete in order; keep the compiler in line
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    half8_t a1;
    if (J0 < Jend) {
        load_x(J0);
        issue_w(J0);
        decode(a1);
        if (J0 + 2 < Jend) issue_w(J0 + 2);
    }
    for (int Jm = J0; Jm < Jend; Jm += 8) {
#pragma unroll
        for (int q = 0; q < NQ; q++) *reinterpret_cast<half8_t *>(stage + (8 * q + lr) * XST + 16 * ch) = xq[q];
        wave_sync();
        if (Jm + 8 < Jend) load_x(Jm + 8);
#pragma unroll
        for (int sub = 0; sub < 4; sub++) {
            const int Jb = Jm + 2 * sub;
            if (Jb < Jend) {  // the same for the whole wave
                const half8_t a = a1;
                const bool live = Jb + s < Jend;
                half8_t xb[NB];
#pragma unroll
                for (int nb = 0; nb < NB; nb++) {
                    xb[nb] = *reinterpret_cast<const half8_t *>(stage + (32 * nb + i) * XST + 16 * (2 * sub + s));
                    if (!live) xb[nb] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};  // this half has no block
                }
                if (Jb + 2 < Jend) {
                    decode(a1);
                    if (Jb + 4 < Jend) issue_w(Jb + 4);
                }
#pragma unroll
                for (int nb = 0; nb < NB; nb++)
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xb[nb], acc[nb], 0, 0, 0);
            }
        }
        wave_sync();  // all reads of this round before the next round's writes
    }
    __syncthreads();  // the staging regions become the partial sums
    if (wave > 0) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++)
#pragma unroll
            for (int e = 0; e < 16; e++) s_part[wave - 1][nb][e][lane] = acc[nb][e];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
            const int b = b0 + 32 * nb + i;
            if (b >= B) continue;
#pragma unroll
            for (int e4 = 0; e4 < 4; e4++) {
                float4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    v[e] = acc[nb][4 * e4 + e];
#pragma unroll
                    for (int wv = 0; wv < NW - 1; wv++) v[e] += s_part[wv][nb][4 * e4 + e][lane];
                }
                const int orow = LUT_TX * I + 8 * e4 + 4 * s;
                if (scale) {
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] *= (float)scale[orow + e];
                }
                *reinterpret_cast<float4_t *>(Y + (size_t)b * m + orow) = v;
            }
        }
    }
}

}  // namespace

// ------------------------------------------------------------------ launchers

hipError_t launch_lut_dequantize(int k, const uint32_t *codes, const void *lut, int m, int n, void *W,
                                 hipStream_t st) {
    const long ntiles = (long)(m / LUT_TX) * (n / LUT_TY);
    const uint16_t *tab = (const uint16_t *)lut;
#define QTIP_LUT_DQ(K)                                                                                   \
    {                                                                                                    \
        constexpr int TPW = 64 / Geo<K>::LPT;                                                            \
        const long waves = (ntiles + TPW - 1) / TPW;                                                     \
        hipLaunchKernelGGL((lut_dequantize_kernel<K>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, \
                           st, codes, tab, n / LUT_TY, ntiles, (half_t *)W);                             \
    }
    if (k == 2) QTIP_LUT_DQ(2) else if (k == 3) QTIP_LUT_DQ(3) else QTIP_LUT_DQ(4)
#undef QTIP_LUT_DQ
    return hipGetLastError();
}

hipError_t launch_lut_decode_states(const uint32_t *states, int count, const void *lut, void *out,
                                    hipStream_t st) {
    hipLaunchKernelGGL(lut_decode_states_kernel, dim3((count + 255) / 256), dim3(256), 0, st, states, count,
                       (const uint16_t *)lut, (uint16_t *)out);
    return hipGetLastError();
}

template <int K>
static hipError_t lut_matvec_t(const uint32_t *codes, const uint16_t *tab, int m, int n, const void *x,
                               const void *scale, float *y, hipStream_t st) {
    constexpr int TPI = 64 / Geo<K>::LPT;
    const int tm = m / LUT_TX, tn = n / LUT_TY;
    const int steps = (tn + TPI - 1) / TPI;
    // every workgroup first copies the table (32 KiB), so few large workgroups
    if (steps >= 32)
        hipLaunchKernelGGL((lut_matvec_kernel<K, 16>), dim3(tm), dim3(1024), 0, st, codes, tab, tn,
                           (const half_t *)x, (const half_t *)scale, y);
    else
        hipLaunchKernelGGL((lut_matvec_kernel<K, 8>), dim3(tm), dim3(512), 0, st, codes, tab, tn,
                           (const half_t *)x, (const half_t *)scale, y);
    return hipGetLastError();
}

hipError_t launch_lut_matvec(int k, const uint32_t *codes, const void *lut, int m, int n, const void *x,
                             const void *scale, float *y, hipStream_t st) {
    const uint16_t *tab = (const uint16_t *)lut;
    if (k == 2) return lut_matvec_t<2>(codes, tab, m, n, x, scale, y, st);
    if (k == 3) return lut_matvec_t<3>(codes, tab, m, n, x, scale, y, st);
    return lut_matvec_t<4>(codes, tab, m, n, x, scale, y, st);
}

template <int K>
static hipError_t lut_matmat_t(const uint32_t *codes, const uint16_t *tab, int m, int n, const void *X, int B,
                               const void *scale, float *Y, hipStream_t st) {
    const int tm = m / LUT_TX, tn = n / LUT_TY;
    // a workgroup owns 32 outputs, so there are few workgroups: many waves each
    if (B <= 16)  // few distinct batch rows: load the B operand directly
        hipLaunchKernelGGL((lut_matmat_kernel<K, 1, 16>), dim3(tm, 1), dim3(1024), 0, st, codes, tab, tn, m,
                           (const half_t *)X, B, (const half_t *)scale, Y);
    else if (B <= 32)
        hipLaunchKernelGGL((lut_matmat_staged_kernel<K, 1, 16>), dim3(tm, 1), dim3(1024), 0, st, codes, tab, tn,
                           m, (const half_t *)X, B, (const half_t *)scale, Y);
    else
        hipLaunchKernelGGL((lut_matmat_staged_kernel<K, 2, 8>), dim3(tm, (B + 63) / 64), dim3(512), 0, st,
                           codes, tab, tn, m, (const half_t *)X, B, (const half_t *)scale, Y);
    return hipGetLastError();
}

hipError_t launch_lut_matmat(int k, const uint32_t *codes, const void *lut, int m, int n, const void *X,
                             int B, const void *scale, float *Y, hipStream_t st) {
    const uint16_t *tab = (const uint16_t *)lut;
    if (k == 2) return lut_matmat_t<2>(codes, tab, m, n, X, B, scale, Y, st);
    if (k == 3) return lut_matmat_t<3>(codes, tab, m, n, X, B, scale, Y, st);
    return lut_matmat_t<4>(codes, tab, m, n, X, B, scale, Y, st);
}

}  // namespace qtip
