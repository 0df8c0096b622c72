// Decode kernels for gfx950: dequantize, fused decode + matrix-vector product on
// the vector ALUs, and fused decode + batched product on the matrix cores.
//
// Work split (all three): one workgroup owns one tile row I (16 output rows)
// and walks the tiles (I, J) along the input dimension, so outputs are written
// once by their owner and no atomics or zero-filled buffers are needed.  The
// waves of a workgroup take contiguous J ranges and their partial sums meet in
// LDS at the end.
#include "qtip_device.h"
#include "qtip_internal.h"
#include "qtip_rht_device.h"

namespace qtip {

// The same plus the first word of the next lane of the same tile (cyclically: the
// tail-biting wrap of Section 3.2).
template <int K>
__device__ __forceinline__ void load_tile_words(const uint32_t *__restrict__ codes, size_t tile,
                                                int lane, uint32_t (&w)[Geo<K>::WPL + 1]) {
    constexpr int WPL = Geo<K>::WPL, LPT = Geo<K>::LPT;
    const int q = lane & (LPT - 1);
    const Words<K> r = load_words<K>(codes, tile, q);
#pragma unroll
    for (int i = 0; i < WPL; i++) w[i] = r.v[i];
    w[WPL] = __shfl(w[0], (lane & ~(LPT - 1)) | ((q + 1) & (LPT - 1)), 64);
}

// Decode tile row rr (0..RPL-1) of this lane: 16 fp16 weights as 8 pairs.
template <int K, int V, int CODE, int NWD>
__device__ __forceinline__ void decode_row(const uint32_t (&w)[NWD], int rr,
                                           const uint32_t *lut, half2_t (&out)[8]) {
#pragma unroll
    for (int c = 0; c < 8; c++) {
        if constexpr (V == 2) {
            uint32_t st = window16(w, rr * 16 * K + c * 2 * K);
            out[c] = CODE == CODE_HYB2 ? code_hyb2(st, lut) : code_hyb(st, lut);
        } else {
            uint32_t s0 = window16(w, rr * 16 * K + (2 * c) * K);
            uint32_t s1 = window16(w, rr * 16 * K + (2 * c + 1) * K);
            half2_t h;
            if constexpr (CODE == CODE_HYB1) {
                h.x = code_hyb1(s0, reinterpret_cast<const uint16_t *>(lut));
                h.y = code_hyb1(s1, reinterpret_cast<const uint16_t *>(lut));
            } else if constexpr (CODE == CODE_3INST) {
                h.x = code_3inst(s0);
                h.y = code_3inst(s1);
            } else {
                h.x = code_1mad(s0);
                h.y = code_1mad(s1);
            }
            out[c] = h;
        }
    }
}

__device__ __forceinline__ void stage_lut(const uint32_t *__restrict__ lut, uint32_t *s_lut) {
    for (int i = threadIdx.x; i < (1 << HYB_Q); i += blockDim.x) s_lut[i] = lut[i];
    __syncthreads();
}

// ---------------------------------------------------------------- dequantize

template <int K, int V, int CODE>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint32_t *__restrict__ codes,
                                                         const uint32_t *__restrict__ lut,
                                                         int tn, long ntiles,
                                                         half_t *__restrict__ W) {
    constexpr int WPL = Geo<K>::WPL, LPT = Geo<K>::LPT, RPL = Geo<K>::RPL;
    constexpr int TPW = 64 / LPT;  // tiles per wave per step
    __shared__ uint32_t s_lut[1 << HYB_Q];
    if constexpr (code_is_hyb(CODE)) stage_lut(lut, s_lut);
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long tile = wave * TPW + lane / LPT;
    const bool valid = tile < ntiles;
    uint32_t w[WPL + 1];
    load_tile_words<K>(codes, valid ? tile : ntiles - 1, lane, w);
    if (!valid) return;
    const long I = tile / tn, J = tile % tn;
    const int q = lane & (LPT - 1);
    const size_t n = (size_t)tn * 16;
#pragma unroll
    for (int rr = 0; rr < RPL; rr++) {
        half2_t h[8];
        decode_row<K, V, CODE>(w, rr, code_is_hyb(CODE) ? s_lut : lut, h);
        uint4 lo = {as_u32(h[0]), as_u32(h[1]), as_u32(h[2]), as_u32(h[3])};
        uint4 hi = {as_u32(h[4]), as_u32(h[5]), as_u32(h[6]), as_u32(h[7])};
        uint4 *dst = reinterpret_cast<uint4 *>(W + (size_t)(16 * I + q * RPL + rr) * n + 16 * J);
        dst[0] = lo;
        dst[1] = hi;
    }
}

// -------------------------------------------------------- decode one state each

template <int CODE>
__global__ void decode_states_kernel(const uint32_t *__restrict__ states, int count,
                                     const uint32_t *__restrict__ lut, half_t *__restrict__ out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    uint32_t st = states[i] & 0xFFFFu;
    if constexpr (code_is_hyb(CODE)) {
        half2_t h = CODE == CODE_HYB2 ? code_hyb2(st, lut) : code_hyb(st, lut);
        out[2 * i] = h.x;
        out[2 * i + 1] = h.y;
    } else if constexpr (CODE == CODE_HYB1) {
        out[i] = code_hyb1(st, reinterpret_cast<const uint16_t *>(lut));
    } else if constexpr (CODE == CODE_3INST) {
        out[i] = code_3inst(st);
    } else {
        out[i] = code_1mad(st);
    }
}

// ------------------------------------------------------- decode + matvec (B = 1)

// A value of the lane `off` lanes away (lane ^ off), any off < 64.
__device__ __forceinline__ float lane_xor(float v, int lane, int off) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ off) << 2, __builtin_bit_cast(int, v)));
}
// v + the value of the lane N places further round this lane's row of 16 (a DPP row rotate).
template <int N> __device__ __forceinline__ float add_row_ror(float v) {
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xF, 0xF, false));
}
// The end of the batch-1 kernels: lane = g * LPT + q holds RPL partial sums, rows q * RPL + rr
// of the tile row, and the 64 / LPT lanes with the same q are to be added up.  Over lane bits 5
// and 4 the lanes trade sums instead of each adding all of them: a lane hands the partner the
// rows the partner keeps and adds what it gets to the rows it keeps itself, so the number of
// sums per lane halves with every exchange (three cross-lane reads at RPL = 4, two at RPL = 2,
// where adding everything everywhere takes sixteen and six); the lane bits below 4 are summed
// with row rotates inside the vector ALU.  On return acc[0] is the whole sum for row
// q * RPL + (return value), the same in all lanes that differ only in the lane bits below 4
// that belong to g.
template <int LPT, int RPL>
__device__ __forceinline__ int reduce_over_tile_groups(float (&acc)[RPL], int lane) {
    static_assert((LPT == 4 && RPL == 4) || (LPT == 8 && RPL == 2), "tile geometries of Geo<K>");
    const bool b5 = lane & 32, b4 = lane & 16;
    float v;
    if constexpr (RPL == 4) {
        // bit 5 clear keeps rows 0 and 1, set keeps rows 2 and 3
        const float r0 = lane_xor(b5 ? acc[0] : acc[2], lane, 32), r1 = lane_xor(b5 ? acc[1] : acc[3], lane, 32);
        const float v0 = (b5 ? acc[2] : acc[0]) + r0, v1 = (b5 ? acc[3] : acc[1]) + r1;
        // bit 4 clear keeps the first of the two, set the second
        v = (b4 ? v1 : v0) + lane_xor(b4 ? v0 : v1, lane, 16);
        v = add_row_ror<8>(v);
        v = add_row_ror<4>(v);
        acc[0] = v;
        return (b5 ? 2 : 0) + (b4 ? 1 : 0);
    } else {
        v = (b5 ? acc[1] : acc[0]) + lane_xor(b5 ? acc[0] : acc[1], lane, 32);
        v += lane_xor(v, lane, 16);
        v = add_row_ror<8>(v);
        acc[0] = v;
        return b5 ? 1 : 0;
    }
}

// FUSED: x is the untransformed activation and the workgroup first computes the input-side
// random Hadamard transform V (S .* x) of Section 2.1 into LDS itself (every workgroup the
// whole vector: at most 8192 values, about 2 us, against a kernel launch and the gap to
// the next dependent kernel, which cost more for layers this small), with the arithmetic
// of the stand-alone transform, so that the result is the same bit for bit.
constexpr int FUSED_MAX_N = 8192;

// SPREAD: the HYB codes' table in 16 copies (see RowDotHyb); it costs 64 KiB of LDS and their
// filling per workgroup, and pays on long rows.  (Eight waves per SIMD, i.e. at most 64
// registers: the loop needs no more, and a second workgroup per CU is worth more than the few
// values that spill around it.)
// (The V = 1 hash code keeps a whole tile's table reads in flight and needs more registers; the
// kernel that transforms its own input runs with at most one workgroup per CU, four waves per
// SIMD, and may take the registers that leaves it.)
template <int K, int V, int CODE, int NW, bool FUSED, bool SPREAD = false, bool WIDE = false>
__global__ __launch_bounds__(NW * 64, (CODE == CODE_HYB1 || FUSED) ? 4 : 8) void matvec_kernel(const uint32_t *__restrict__ codes,
                                                         const uint32_t *__restrict__ lut,
                                                         int tn, const half_t *__restrict__ x,
                                                         const int8_t *__restrict__ signs, int log2_block,
                                                         const half_t *__restrict__ scale,
                                                         float *__restrict__ y) {
    constexpr int WPL = MvGeo<K, WIDE>::WPL, LPT = MvGeo<K, WIDE>::LPT, RPL = MvGeo<K, WIDE>::RPL;
    constexpr int TPI = 64 / LPT;  // tiles per wave per iteration
    __shared__ __attribute__((aligned(16))) uint32_t s_lut[code_lds_words(CODE, SPREAD)];
    __shared__ float s_part[NW][16];
    __shared__ __attribute__((aligned(16))) half_t s_x[FUSED ? FUSED_MAX_N : 8];
    // room for FUSED_MAX_N values in blocks of any size, each block with its padding
    __shared__ float s_v[FUSED ? FUSED_MAX_N + FUSED_MAX_N / 32 + FUSED_MAX_N / 16 : 1];
    if constexpr (FUSED) {
        // groups of threads take one block each (a thread holds 16 values per round)
        const int b = 1 << log2_block, n = 16 * tn;
        const int gthreads = min(NW * 64, b >> 4);
        const int groups = min(NW * 64 / gthreads, FUSED_MAX_N / b);  // what s_v holds
        const int group = threadIdx.x / gthreads, gtid = threadIdx.x % gthreads;
        for (int o0 = 0; o0 < n; o0 += groups * b) {
            const int o = o0 + group * b;
            const bool active = group < groups && o < n;
            half_t *dst = s_x + (active ? o : 0);
            rht_block<half_t, 0>(x + (active ? o : 0), signs + (active ? o : 0), log2_block, 0,
                                 s_v + (active ? group : 0) * rht_lds_floats(b), gtid, gthreads, active,
                                 [dst](int idx, half_t v) { dst[idx] = v; });
        }
    }
    stage_code_table<CODE, SPREAD>(lut, s_lut, NW * 64);
    typename RowDotFor<K, CODE, SPREAD>::type rd;
    rd.init(s_lut);
    const int I = blockIdx.x;
    // the wave's number as a scalar: its tile range and the loop over it then live in scalar
    // registers and the loop control costs no vector instructions
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int g = lane / LPT, q = lane & (LPT - 1);
    const int chunk = ((tn + NW * TPI - 1) / (NW * TPI)) * TPI;
    const int J0 = wave * chunk;
    const int Jend = min(tn, J0 + chunk);
    // this tile row's words: a uniform base, so that a lane's address is base + 32-bit offset
    const uint32_t *__restrict__ row_codes = codes + (size_t)I * tn * (8 * K);
    float acc[RPL];
#pragma unroll
    for (int rr = 0; rr < RPL; rr++) acc[rr] = 0.f;

    // Software pipeline: the loads of step i+1 are in flight while step i is decoded.
    // Two operand sets alternate (the loop body is two steps), so nothing is copied
    // (3-4 % on the computed codes, measured against the copying form on one box).
    struct Operands {
        WordsN<WPL> w;
        uint4 xa, xb;
    };
    auto issue = [&](Operands &o, int Jb) {
        const uint32_t Jc = min(Jb + g, Jend - 1);  // lanes past the end re-read the last tile
        // (byte offsets in 32 bits from uniform bases: the loads take them as they are)
        o.w = load_words_at<WPL>(row_codes, Jc * (32 * K) + q * (4 * WPL));
        if constexpr (FUSED) {
            const uint4 *xp = reinterpret_cast<const uint4 *>(s_x + 16 * Jc);
            o.xa = xp[0];
            o.xb = xp[1];
        } else {
            const uint4 *xp = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(x) + (size_t)(Jc * 32u));
            o.xa = xp[0];
            o.xb = xp[1];
        }
    };
    auto compute = [&](const Operands &o, int Jb) {
        uint32_t w[WPL + 1];
#pragma unroll
        for (int i = 0; i < WPL; i++) w[i] = o.w.v[i];
        // first word of the next lane of the same tile, cyclically (tail-biting wrap)
        w[WPL] = __shfl(w[0], (lane & ~(LPT - 1)) | ((q + 1) & (LPT - 1)), 64);
        if (Jb + g < Jend) {
            uint32_t xv[8] = {o.xa.x, o.xa.y, o.xa.z, o.xa.w, o.xb.x, o.xb.y, o.xb.z, o.xb.w};
            rd.prep_x(xv);
            rd.run_tile(w, xv, acc);
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
    rd.finish(acc);
    // lanes with equal q hold partial sums of the same rows: add over g
    const int rr_mine = reduce_over_tile_groups<LPT, RPL>(acc, lane);
    if ((g & (16 / LPT - 1)) == 0) s_part[wave][q * RPL + rr_mine] = acc[0];
    __syncthreads();
    if (threadIdx.x < 16) {
        float s = 0.f;
#pragma unroll
        for (int wv = 0; wv < NW; wv++) s += s_part[wv][threadIdx.x];
        const int row = 16 * I + threadIdx.x;
        if (scale) s *= (float)scale[row];
        y[row] = s;
    }
}

// ------------------------------------------- decode + batched product on MFMA
//
// v_mfma_f32_16x16x32_f16, D = A * B, with the decoded weights as A and the
// activations as B.  A wave step covers four tiles (I, J0..J0+3) of one tile row:
//   lane l = (row i = l % 16, slot s = l / 16) decodes the whole tile row i of tile
//   J0 + s: 16 weights = 8 packed registers, the A operands of two MFMAs (columns
//   0..7 and 8..15 of the tile);
//   the matching B operand of lane (j = l % 16, s) is X[b0 + j][16 (J0+s) + 8h .. +7],
//   one 16-byte load; A and B pair contraction slots by (s, element), so the order
//   in which the hardware numbers them does not matter;
//   D[4 (l / 16) + r][l % 16] = output row 16 I + 4 (l/16) + r for batch row b0 + l % 16.
// A wave owns R = 2 neighbouring tile rows so that every B operand it loads feeds
// two MFMAs; NB groups of 16 batch rows share every decoded weight.  The waves of
// a workgroup split the tiles of the row band and meet in LDS.
// The B operand puts neighbouring lanes on different batch rows, that is on different
// cache lines, and the texture path serves such a 16-byte-per-lane load at a fraction
// of the rate of one whose neighbouring lanes read neighbouring addresses.  With few
// distinct batch rows that does not matter; at larger batch (STAGE) a wave loads its
// activations line by line (8 lanes = the 128 bytes that one batch row has under the
// four tiles of a step) and transposes them through a private piece of LDS.

// The words that hold tile row i (16 K bits from bit 16 K i) and the 16 - K V bits
// after it, brought to bit offset 0; indices wrap inside the tile (tail-biting).
template <int K>
__device__ __forceinline__ void load_row_words(const uint32_t *__restrict__ tile, int i,
                                               uint32_t (&w)[3]) {
    constexpr int NWORDS = 8 * K;
    const int bit = 16 * K * i;
    const int w0 = bit >> 5;
    w[0] = stream_load(tile + w0);
    w[1] = stream_load(tile + (w0 + 1) % NWORDS);
    w[2] = (K == 2) ? 0u : stream_load(tile + (w0 + 2) % NWORDS);
}
template <int K>
__device__ __forceinline__ void align_row_words(int i, uint32_t (&w)[3]) {
    if constexpr (K == 3) {
        if (i & 1) {  // odd rows start in the middle of a word
            w[0] = __builtin_amdgcn_alignbit(w[0], w[1], 16);
            w[1] = __builtin_amdgcn_alignbit(w[1], w[2], 16);
            w[2] <<= 16;
        }
    }
}

// SPREAD: the HYB table in 16 copies, as in the batch-1 kernel (64 KiB: only next to the
// small partial-sum buffer of NB = 1).
template <int K, int V, int CODE, int NB, int NW, bool STAGE, bool SPREAD = false>
__global__ __launch_bounds__(NW * 64) void matmat_kernel(const uint32_t *__restrict__ codes,
                                                         const uint32_t *__restrict__ lut,
                                                         int tm, int tn, const half_t *__restrict__ X,
                                                         int B, const half_t *__restrict__ scale,
                                                         float *__restrict__ Y) {
    constexpr int R = 2;
    constexpr int NWORDS = 8 * K;
    __shared__ __attribute__((aligned(16))) uint32_t s_lut[code_lds_words(CODE, SPREAD)];
    // one buffer, used twice: in the loop each wave's staging region (SR batch rows at a
    // time, 128 bytes each, padded to 144 so that the row-wise writes and the
    // column-wise reads both spread over the banks), after it the partial sums
    constexpr int SR = NB >= 2 ? 32 : 16, NH = 16 * NB / SR, XST = 144;
    constexpr int PART_FLOATS = (NW - 1) * R * NB * 256;
    constexpr int STAGE_FLOATS = STAGE ? NW * SR * XST / 4 : 0;
    __shared__ __attribute__((aligned(16))) float s_buf[PART_FLOATS > STAGE_FLOATS ? PART_FLOATS : STAGE_FLOATS];
    float(*s_part)[R][NB][4][64] = reinterpret_cast<float(*)[R][NB][4][64]>(s_buf);
    stage_code_table<CODE, SPREAD>(lut, s_lut, NW * 64);
    RowDecode<K, CODE, SPREAD> rdec;
    rdec.init(s_lut);
    const int I0 = blockIdx.x * R;
    const int b0 = blockIdx.y * (16 * NB);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = lane & 15, s = lane >> 4;
    const size_t n = (size_t)tn * 16;
    const int m = tm * 16;
    const int chunk = ((tn + NW * 4 - 1) / (NW * 4)) * 4;
    const int J0 = wave * chunk;
    const int Jend = min(tn, J0 + chunk);
    const bool row_ok[R] = {true, I0 + 1 < tm};

    float4_t acc[R][NB];
#pragma unroll
    for (int r = 0; r < R; r++)
#pragma unroll
        for (int nb = 0; nb < NB; nb++) acc[r][nb] = float4_t{0.f, 0.f, 0.f, 0.f};

    // software pipeline: operands of step t+1 are loaded while step t runs
    uint32_t wn[R][3];
    half8_t xn[NB][2];  // STAGE: piece (lane % 8) of batch rows 8 q + lane / 8, q = 2 nb + h
    const int lr = lane >> 3, ch = lane & 7;
    char *const stage = reinterpret_cast<char *>(s_buf) + wave * (SR * XST);
    auto issue = [&](int Jb) {
        const int J = min(Jb + s, Jend - 1);  // slots past the end re-read the last tile
#pragma unroll
        for (int r = 0; r < R; r++) {
            const int I = row_ok[r] ? I0 + r : I0;
            load_row_words<K>(codes + ((size_t)I * tn + J) * NWORDS, i, wn[r]);
        }
        if constexpr (STAGE) {
            const int Jx = min(Jb + (ch >> 1), Jend - 1);
#pragma unroll
            for (int q = 0; q < 2 * NB; q++) {
                const int b = b0 + 8 * q + lr;
                xn[q >> 1][q & 1] = *reinterpret_cast<const half8_t *>(
                    X + (size_t)min(b, B - 1) * n + 16 * Jx + 8 * (ch & 1));
            }
        } else {
#pragma unroll
            for (int nb = 0; nb < NB; nb++) {
                const int b = b0 + 16 * nb + i;
                const half_t *xp = X + (size_t)min(b, B - 1) * n + 16 * J;
                xn[nb][0] = *reinterpret_cast<const half8_t *>(xp);
                xn[nb][1] = *reinterpret_cast<const half8_t *>(xp + 8);
            }
        }
    };
    if (J0 < Jend) issue(J0);
    for (int Jb = J0; Jb < Jend; Jb += 4) {
        uint32_t w[R][3];
        half8_t xb[NB][2];
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int t = 0; t < 3; t++) w[r][t] = wn[r][t];
        const bool live = Jb + s < Jend;
        if constexpr (STAGE) {
            // The lanes of the wave exchange data through LDS without a workgroup barrier:
            // the LDS operations of one wave complete in order, and the fences keep the
            // compiler from moving them across each other.
#pragma unroll
            for (int hf = 0; hf < NH; hf++) {
#pragma unroll
                for (int qq = 0; qq < SR / 8; qq++) {
                    const int q = hf * (SR / 8) + qq;
                    *reinterpret_cast<half8_t *>(stage + (8 * qq + lr) * XST + 16 * ch) = xn[q >> 1][q & 1];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int nbb = 0; nbb < SR / 16; nbb++)
#pragma unroll
                    for (int h = 0; h < 2; h++)
                        xb[hf * (SR / 16) + nbb][h] = *reinterpret_cast<const half8_t *>(
                            stage + (16 * nbb + i) * XST + 16 * (2 * s + h));
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
            const bool bok = live && (b0 + 16 * nb + i < B);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                if constexpr (!STAGE) xb[nb][h] = xn[nb][h];
                if (!bok) xb[nb][h] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};  // dead slot / batch row
            }
        }
        if (Jb + 4 < Jend) issue(Jb + 4);
#pragma unroll
        for (int r = 0; r < R; r++) {
            align_row_words<K>(i, w[r]);
            uint32_t hrow[8];
            rdec.run(w[r], 0, hrow);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const half8_t a = __builtin_bit_cast(
                    half8_t, u32x4{hrow[4 * h], hrow[4 * h + 1], hrow[4 * h + 2], hrow[4 * h + 3]});
#pragma unroll
                for (int nb = 0; nb < NB; nb++)
                    acc[r][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xb[nb][h], acc[r][nb], 0, 0, 0);
            }
        }
    }
    if constexpr (STAGE) __syncthreads();  // the staging regions become the partial sums
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int nb = 0; nb < NB; nb++)
#pragma unroll
                for (int e = 0; e < 4; e++) s_part[wave - 1][r][nb][e][lane] = acc[r][nb][e];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int r = 0; r < R; r++) {
            if (!row_ok[r]) continue;
#pragma unroll
            for (int nb = 0; nb < NB; nb++) {
                const int b = b0 + 16 * nb + i;
                if (b >= B) continue;
                float4_t v = acc[r][nb];
#pragma unroll
                for (int wv = 0; wv < NW - 1; wv++)
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] += s_part[wv][r][nb][e][lane];
                const int orow = 16 * (I0 + r) + 4 * s;
                if (scale) {
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] *= (float)scale[orow + e];
                }
                *reinterpret_cast<float4_t *>(Y + (size_t)b * m + orow) = v;
            }
        }
    }
}

// ------------------------------------------------------------------ launchers

template <int K, int V, int CODE>
static hipError_t launch_dequantize_t(const uint32_t *codes, const uint32_t *lut, int m, int n,
                                      void *W, hipStream_t st) {
    const long ntiles = (long)(m / 16) * (n / 16);
    constexpr int TPW = 64 / Geo<K>::LPT;
    const long waves = (ntiles + TPW - 1) / TPW;
    const long blocks = (waves + 3) / 4;
    hipLaunchKernelGGL((dequantize_kernel<K, V, CODE>), dim3((unsigned)blocks), dim3(256), 0, st,
                       codes, lut, n / 16, ntiles, (half_t *)W);
    return hipGetLastError();
}

// Waves per workgroup for the batch-1 kernel.  A workgroup owns one tile row, so the
// grid has m/16 workgroups and NW decides both how many waves the chip gets and how
// many steps each wave runs: few steps leave a wave's start-up and reduction exposed,
// few waves leave SIMDs idle or the vector ALU short of waves to interleave.
// Measured by kernel durations from the profiler's trace (for kernels this short a loop
// of launches from the host times the host): as many waves as there are steps, up to 16,
// is best everywhere: 4096 x 4096 (16 steps) 6.0 us with 8 waves, 5.4 with 16; 14336 x 4096
// 11.6 -> 11.3.  The kernel that transforms its own input takes the same count, so that it
// adds its partial sums in the same order and gives the same bits as the two separate calls.
static int pick_matvec_waves(int steps_per_row) {
    if (steps_per_row >= 16) return 16;
    if (steps_per_row >= 8) return 8;
    if (steps_per_row >= 4) return 4;
    return 2;
}

// The 16-copy HYB table: from which row length on it pays for the 64 KiB each workgroup fills
// (measured: 8192 x 28672 29.9 -> 22.5 us at k = 2, 8192 x 8192 10.0 -> 9.6, 14336 x 4096 10.0 ->
// 12.0).  The two-sign-flip form is bound by its vector instructions and gains nothing.
static bool pick_hyb_spread(int code, int n) {
    return code == CODE_HYB && n >= 8192;
}

template <int K, int V, int CODE>
static hipError_t launch_matvec_t(const uint32_t *codes, const uint32_t *lut, int m, int n,
                                  const void *x, const int8_t *signs, int log2_block, const void *scale,
                                  float *y, hipStream_t st) {
    constexpr int TPI = 64 / Geo<K>::LPT;
    const int tm = m / 16, tn = n / 16;
    const int steps = (tn + TPI - 1) / TPI;
    const int nw = pick_matvec_waves(steps);
    const bool spread = pick_hyb_spread(CODE, n);
    // signs != null: x is untransformed and the kernel transforms it itself (n <= FUSED_MAX_N)
#define QTIP_MV_LAUNCH4(NW, FUSED, SPREAD, WIDE)                                                            \
    hipLaunchKernelGGL((matvec_kernel<K, V, CODE, NW, FUSED, SPREAD, WIDE>), dim3(tm), dim3(NW * 64), 0, st, \
                       codes, lut, tn, (const half_t *)x, signs, log2_block, (const half_t *)scale, y)
#define QTIP_MV_LAUNCH(NW, WIDE)                                \
    if (signs)                                                  \
        QTIP_MV_LAUNCH4(NW, true, false, WIDE);                 \
    else if (code_is_hyb(CODE) && spread)                       \
        QTIP_MV_LAUNCH4(NW, false, code_is_hyb(CODE), WIDE);    \
    else                                                        \
        QTIP_MV_LAUNCH4(NW, false, false, WIDE)
    // Four rows per lane at k = 3 and 4 (MvGeo<K, true>: steps of 16 tiles) where 16 waves still have a
    // step each and the row splits into such steps as evenly as into the narrow ones (measured, k = 4:
    // 14336 x 4096 12.44 -> 11.38 us, 8192 x 8192 HYB 10.64 -> 10.38; 4096 x 14336, 896 tiles = 3.5 wide
    // steps per wave, 11.76 -> 12.10 us, so it keeps the narrow form).  The choice depends on the row
    // length alone, so the kernel that transforms its own input makes the same one.
    if constexpr (K != 2) {
        constexpr int WTPI = 64 / MvGeo<K, true>::LPT;
        const int wsteps = (tn + WTPI - 1) / WTPI;
        if (wsteps >= 16 && 2 * ((wsteps + 15) / 16) <= (steps + nw - 1) / nw) {
            QTIP_MV_LAUNCH(16, true);
            return hipGetLastError();
        }
    }
    switch (nw) {
        case 2: QTIP_MV_LAUNCH(2, false); break;
        case 4: QTIP_MV_LAUNCH(4, false); break;
        case 16: QTIP_MV_LAUNCH(16, false); break;
        default: QTIP_MV_LAUNCH(8, false); break;
    }
#undef QTIP_MV_LAUNCH
#undef QTIP_MV_LAUNCH4
    return hipGetLastError();
}

template <int K, int V, int CODE>
static hipError_t launch_matmat_t(const uint32_t *codes, const uint32_t *lut, int m, int n,
                                  const void *X, int B, const void *scale, float *Y,
                                  hipStream_t st) {
    constexpr int NW = 8;
    const int groups = (B + 15) / 16;
    const int tm = m / 16, tn = n / 16;
    const dim3 block(NW * 64);
    const half_t *Xh = (const half_t *)X, *sc = (const half_t *)scale;
    constexpr bool HYB = CODE == CODE_HYB;
    // (measured: the 16 table copies pay at 9 to 16 batch rows, 8192 x 8192 13.1 -> 12.3 us and
    // 8192 x 28672 35 -> 31 us, and make no difference below)
    const bool spread = HYB && pick_hyb_spread(CODE, n);
    if (groups == 1 && B <= 8) {  // few distinct batch rows: load the B operand directly
        hipLaunchKernelGGL((matmat_kernel<K, V, CODE, 1, NW, false>), dim3((tm + 1) / 2, 1), block, 0,
                           st, codes, lut, tm, tn, Xh, B, sc, Y);
    } else if (groups == 1) {
        if (spread)
            hipLaunchKernelGGL((matmat_kernel<K, V, CODE, 1, NW, true, HYB>), dim3((tm + 1) / 2, 1), block, 0,
                               st, codes, lut, tm, tn, Xh, B, sc, Y);
        else
            hipLaunchKernelGGL((matmat_kernel<K, V, CODE, 1, NW, true>), dim3((tm + 1) / 2, 1), block, 0,
                               st, codes, lut, tm, tn, Xh, B, sc, Y);
    } else if (groups == 2) {
        hipLaunchKernelGGL((matmat_kernel<K, V, CODE, 2, NW, true>), dim3((tm + 1) / 2, 1), block, 0,
                           st, codes, lut, tm, tn, Xh, B, sc, Y);
    } else {
        hipLaunchKernelGGL((matmat_kernel<K, V, CODE, 4, NW, true>), dim3((tm + 1) / 2, (groups + 3) / 4),
                           block, 0, st, codes, lut, tm, tn, Xh, B, sc, Y);
    }
    return hipGetLastError();
}

#define QTIP_DISPATCH(FN, ...)                                                         \
    do {                                                                               \
        if (code_id == CODE_HYB1) {                                                    \
            if (k == 2) return FN<2, 1, CODE_HYB1>(__VA_ARGS__);                       \
            if (k == 3) return FN<3, 1, CODE_HYB1>(__VA_ARGS__);                       \
            return FN<4, 1, CODE_HYB1>(__VA_ARGS__);                                   \
        } else if (code_id == CODE_HYB2) {                                             \
            if (k == 2) return FN<2, 2, CODE_HYB2>(__VA_ARGS__);                       \
            if (k == 3) return FN<3, 2, CODE_HYB2>(__VA_ARGS__);                       \
            return FN<4, 2, CODE_HYB2>(__VA_ARGS__);                                   \
        } else if (code_id == CODE_HYB) {                                              \
            if (k == 2) return FN<2, 2, CODE_HYB>(__VA_ARGS__);                        \
            if (k == 3) return FN<3, 2, CODE_HYB>(__VA_ARGS__);                        \
            return FN<4, 2, CODE_HYB>(__VA_ARGS__);                                    \
        } else if (code_id == CODE_3INST) {                                            \
            if (k == 2) return FN<2, 1, CODE_3INST>(__VA_ARGS__);                      \
            if (k == 3) return FN<3, 1, CODE_3INST>(__VA_ARGS__);                      \
            return FN<4, 1, CODE_3INST>(__VA_ARGS__);                                  \
        } else {                                                                       \
            if (k == 2) return FN<2, 1, CODE_1MAD>(__VA_ARGS__);                       \
            if (k == 3) return FN<3, 1, CODE_1MAD>(__VA_ARGS__);                       \
            return FN<4, 1, CODE_1MAD>(__VA_ARGS__);                                   \
        }                                                                              \
    } while (0)

hipError_t launch_dequantize(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                             int n, void *W, hipStream_t st) {
    if (code_id == CODE_LUT) return launch_lut_dequantize(k, codes, lut, m, n, W, st);
    QTIP_DISPATCH(launch_dequantize_t, codes, lut, m, n, W, st);
}

hipError_t launch_matvec(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                         int n, const void *x, const void *scale, float *y, hipStream_t st) {
    if (code_id == CODE_LUT) return launch_lut_matvec(k, codes, lut, m, n, x, scale, y, st);
    QTIP_DISPATCH(launch_matvec_t, codes, lut, m, n, x, (const int8_t *)nullptr, 0, scale, y, st);
}

int fused_rht_matvec_max_n() { return FUSED_MAX_N; }

hipError_t launch_rht_matvec(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                             int n, const void *x, const int8_t *signs, int block, const void *scale,
                             float *y, hipStream_t st) {
    int log2_block = 0;
    while ((1 << log2_block) < block) log2_block++;
    QTIP_DISPATCH(launch_matvec_t, codes, lut, m, n, x, signs, log2_block, scale, y, st);
}

hipError_t launch_matmat(int k, int code_id, const uint32_t *codes, const uint32_t *lut, int m,
                         int n, const void *X, int B, const void *scale, float *Y,
                         hipStream_t st) {
    if (code_id == CODE_LUT) return launch_lut_matmat(k, codes, lut, m, n, X, B, scale, Y, st);
    QTIP_DISPATCH(launch_matmat_t, codes, lut, m, n, X, B, scale, Y, st);
}

hipError_t launch_decode_states(int code_id, const uint32_t *states, int count,
                                const uint32_t *lut, void *out, hipStream_t st) {
    const int blocks = (count + 255) / 256;
    if (code_id == CODE_LUT) return launch_lut_decode_states(states, count, lut, out, st);
    if (code_id == CODE_HYB1)
        hipLaunchKernelGGL((decode_states_kernel<CODE_HYB1>), dim3(blocks), dim3(256), 0, st, states,
                           count, lut, (half_t *)out);
    else if (code_id == CODE_HYB2)
        hipLaunchKernelGGL((decode_states_kernel<CODE_HYB2>), dim3(blocks), dim3(256), 0, st, states,
                           count, lut, (half_t *)out);
    else if (code_id == CODE_HYB)
        hipLaunchKernelGGL((decode_states_kernel<CODE_HYB>), dim3(blocks), dim3(256), 0, st, states,
                           count, lut, (half_t *)out);
    else if (code_id == CODE_3INST)
        hipLaunchKernelGGL((decode_states_kernel<CODE_3INST>), dim3(blocks), dim3(256), 0, st,
                           states, count, lut, (half_t *)out);
    else
        hipLaunchKernelGGL((decode_states_kernel<CODE_1MAD>), dim3(blocks), dim3(256), 0, st,
                           states, count, lut, (half_t *)out);
    return hipGetLastError();
}

}  // namespace qtip
