// Device-side building blocks of the QTIP decode path for gfx950 (CDNA4):
// tile geometry, state-window extraction from packed words held in VGPRs, and
// the state -> fp16 value codes (Algorithms 1-3 of arXiv 2406.11235).
//
// Two forms of every code live here.  The plain functions (code_3inst,
// code_1mad, code_hyb) are the definitions written out; dequantize, the
// state-table test entry and the MFMA path use them.  The RowDot structs are
// the batch-1 hot loop: one tile row (16 weights) decoded and contracted with 16
// activations, in as few vector instructions as the exact codes allow (in the
// kernel, where eight waves in different phases share a SIMD, every vector
// instruction costs about four cycles whatever its kind):
//   * a zero-extended state is one v_bfe_u32, from its word or from one funnel
//     shift per word for the states that cross into the next word;
//   * the HYB codes hash two states at once: with 16-bit states, the high and low
//     halves of a 32-bit window at a multiple of k*V bits are both states;
//   * the LCG a*x+b (mod 2^32) is one v_mad_u64_u32 on the zero-extended state;
//   * mask+xor is one v_bitop3_b32;
//   * the fp16 add of the two halves writes straight into one half of a packed
//     register (SDWA), so a v_dot2c_f32_f16 consumes two weights at once.
// Both forms produce the same fp16 weights bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qtip {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int CODE_1MAD = 0;
constexpr int CODE_3INST = 1;
constexpr int CODE_HYB = 2;
constexpr int CODE_HYB2 = 3;  // HYB with a second sign flip (bit 31 of the hash on the first entry)
constexpr int CODE_LUT = 4;   // lookup-only: L = 14, V = 1, 32 x 8 blocks (kernels in qtip_lut14.hip)
constexpr int CODE_HYB1 = 5;  // Algorithm 3 with one entry per row: V = 1, Q = 6 (64 fp16 values)
// state bits L and log2 of T_y (a sequence is a (256 / T_y) x T_y block of the matrix)
__host__ __device__ constexpr int code_state_bits(int code) { return code == CODE_LUT ? 14 : 16; }
__host__ __device__ constexpr int code_log2_ty(int code) { return code == CODE_LUT ? 3 : 4; }
__host__ __device__ constexpr bool code_is_hyb(int code) { return code == CODE_HYB || code == CODE_HYB2; }
// words of LDS the hot loops of a code keep their table in (see stage_code_table); SPREAD:
// the batch-1 kernel's form of the HYB table, HYB_SPREAD copies (see RowDotHyb)
constexpr int HYB_SPREAD = 16;
__host__ __device__ constexpr int code_lds_words(int code, bool spread = false) {
    return code_is_hyb(code) ? (spread ? 1024 * HYB_SPREAD : 1024) : code == CODE_HYB1 ? 4096 : 1;
}

// Section 3.1.1 constants.
constexpr uint32_t MAD_A = 34038481u, MAD_B = 76625530u;
constexpr uint32_t INST_A = 89226354u, INST_B = 64248484u;
constexpr uint32_t INST_MASK = 0x8FFF8FFFu;  // sign, 2 low exponent bits, mantissa; twice
constexpr uint32_t INST_MM = 0x3B603B60u;    // fp16(0.922) = 0x3B60 in both halves
constexpr int HYB_Q = 9;
constexpr float MAD_INV_SCALE = 0.0067658998646820027f;  // fp32(1 / 147.8)

// How one 16x16 tile (8K words) is spread over lanes: every lane holds WPL
// consecutive words = RPL whole tile rows; LPT lanes cover a tile.
template <int K> struct Geo;
template <> struct Geo<2> { static constexpr int WPL = 4, LPT = 4, RPL = 4; };
template <> struct Geo<3> { static constexpr int WPL = 3, LPT = 8, RPL = 2; };
template <> struct Geo<4> { static constexpr int WPL = 4, LPT = 8, RPL = 2; };

template <int K> struct Words;
template <> struct Words<2> { uint32_t v[4]; };
template <> struct Words<3> { uint32_t v[3]; };
template <> struct Words<4> { uint32_t v[4]; };

// A word of the code stream.  Every word is read once per product and the stream is far
// larger than the caches (58.7 MB against 4 MiB of L2 per XCD), so the loads carry the
// non-temporal hint: they do not displace the activations, which every workgroup re-reads
// (measured over rotating buffers: 8192 x 28672 2-bit 3INST 34.3 -> 34.0 us, HYB 21.4 -> 20.7,
// 8192 x 8192 4-bit HYB 11.9 -> 11.4, 14336 x 4096 4-bit 1MAD 13.0 -> 12.8).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t stream_load(const uint32_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ u32x4_t stream_load4(const uint32_t *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}

// A lane's WPL words at word offset `off` from a base every lane shares.
template <int K>
__device__ __forceinline__ Words<K> load_words(const uint32_t *__restrict__ base, uint32_t off) {
    constexpr int WPL = Geo<K>::WPL;
    const uint32_t *p = base + off;
    Words<K> r;
    if constexpr (WPL == 4) {
        const u32x4_t t = stream_load4(p);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
        r.v[0] = stream_load(p); r.v[1] = stream_load(p + 1); r.v[2] = stream_load(p + 2);
    }
    return r;
}
// The batch-1 kernel's second spread of a tile over lanes (WIDE): at k = 3 and 4 a lane takes
// four tile rows like at k = 2 (six or eight words, four lanes per tile), so that the work
// around a step (offsets, loads, the wrap read, the end test) is shared by 64 weights per lane
// instead of 32.  A step then covers 16 tiles, and rows whose tile count does not split evenly
// into such steps over the waves keep the narrow form (the launcher chooses).
template <int K, bool WIDE> struct MvGeo : Geo<K> {};
template <> struct MvGeo<3, true> { static constexpr int WPL = 6, LPT = 4, RPL = 4; };
template <> struct MvGeo<4, true> { static constexpr int WPL = 8, LPT = 4, RPL = 4; };
template <int WPL> struct WordsN { uint32_t v[WPL]; };
// A lane's WPL words at byte offset `byte_off` from a base every lane shares.
template <int WPL>
__device__ __forceinline__ WordsN<WPL> load_words_at(const uint32_t *__restrict__ base, uint32_t byte_off) {
    const uint32_t *p = reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(base) + (size_t)byte_off);
    WordsN<WPL> r;
    if constexpr (WPL % 4 == 0) {
#pragma unroll
        for (int i = 0; i < WPL; i += 4) {
            const u32x4_t t = stream_load4(p + i);
            r.v[i] = t.x; r.v[i + 1] = t.y; r.v[i + 2] = t.z; r.v[i + 3] = t.w;
        }
    } else if constexpr (WPL % 2 == 0) {  // six words: 8-byte aligned
#pragma unroll
        for (int i = 0; i < WPL; i += 2) {
            const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p + i));
            r.v[i] = t.x; r.v[i + 1] = t.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < WPL; i++) r.v[i] = stream_load(p + i);
    }
    return r;
}
// This lane's WPL words of tile `tile` (q = lane's position inside the tile).
template <int K>
__device__ __forceinline__ Words<K> load_words(const uint32_t *__restrict__ codes, size_t tile,
                                               int q) {
    return load_words<K>(codes + tile * (8 * K), (uint32_t)(q * Geo<K>::WPL));
}

__device__ __forceinline__ half2_t as_half2(uint32_t v) {
    return __builtin_bit_cast(half2_t, v);
}
__device__ __forceinline__ uint32_t as_u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// 32 bits starting P bits into the word array w (MSB-first words): one word or
// a two-word funnel shift.  P is a compile-time constant after unrolling.
template <int NW>
__device__ __forceinline__ uint32_t window32(const uint32_t (&w)[NW], int P) {
    const int i = P >> 5, s = P & 31;
    if (s == 0) return w[i];
    return __builtin_amdgcn_alignbit(w[i], w[i + 1], 32 - s);
}

// 16-bit window starting P bits into the word array w, zero-extended: one bit-field extract.
// A window that crosses into the next word is taken from the 32 bits that start at bit 16 of
// its word; that funnel shift is the same for every such window of the word (the compiler
// keeps one), so a tile row of 16 windows costs one or two funnel shifts and 16 extracts.
template <int NW>
__device__ __forceinline__ uint32_t window16(const uint32_t (&w)[NW], int P) {
    const int i = P >> 5, s = P & 31;
    if (s == 0) return w[i] >> 16;
    if (s == 16) return w[i] & 0xFFFFu;
    if (s < 16) return (w[i] >> (16 - s)) & 0xFFFFu;
    const uint32_t m = __builtin_amdgcn_alignbit(w[i], w[i + 1], 16);
    return (m >> (32 - s)) & 0xFFFFu;
}

// ------------------------------------------------------------------ plain codes

// Algorithm 2: LCG, mask + XOR with the packed magic constant, sum of the two
// fp16 halves (one IEEE binary16 add).
__device__ __forceinline__ half_t code_3inst(uint32_t x) {
    uint32_t X = x * INST_A + INST_B;
    half2_t h = as_half2((X & INST_MASK) ^ INST_MM);
    return h.x + h.y;
}

// Algorithm 1: LCG, sum of the four bytes, (s - 510) / 147.8 rounded to fp16.
// (float)(s - 510) * fp32(1/147.8), rounded to fp32 and then to fp16, equals the
// correctly rounded quotient for every s in 0..1020 (checked exhaustively by the
// tests; the quotient 5(s-510)/739 is never close to a rounding boundary).
__device__ __forceinline__ half_t code_1mad(uint32_t x) {
    uint32_t X = x * MAD_A + MAD_B;
    int s = (int)__builtin_amdgcn_sad_u8(X, 0u, 0u);
    return (half_t)((float)(s - 510) * MAD_INV_SCALE);
}

// Algorithm 3 with Q = 9: hash x*x + x, bits 6..14 index the table, bit 15
// negates the second entry.  lut holds one 32-bit word per row (entry 0 in the
// low half).
__device__ __forceinline__ half2_t code_hyb(uint32_t x, const uint32_t *lut) {
    uint32_t X = x * x + x;
    uint32_t v = lut[(X >> (15 - HYB_Q)) & ((1u << HYB_Q) - 1u)];
    return as_half2(v ^ ((X & 0x8000u) << 16));
}

// The two-sign-flip form mentioned with Algorithm 3: bit 31 of the hash is XORed alongside
// bit 15, which flips the first entry as well (an effective table of 2^(Q+2) vectors).
__device__ __forceinline__ half2_t code_hyb2(uint32_t x, const uint32_t *lut) {
    uint32_t X = x * x + x;
    uint32_t v = lut[(X >> (15 - HYB_Q)) & ((1u << HYB_Q) - 1u)];
    return as_half2(v ^ ((X & 0x8000u) << 16) ^ ((X >> 16) & 0x8000u));
}
// Algorithm 3 with V = 1 and Q = 6: bits 9..14 of the hash index 64 values, bit 15 negates
// the value.  lut: 64 fp16 bit patterns.
constexpr int HYB1_Q = 6;
__device__ __forceinline__ half_t code_hyb1(uint32_t x, const uint16_t *lut) {
    uint32_t X = x * x + x;
    uint16_t v = lut[(X >> (15 - HYB1_Q)) & ((1u << HYB1_Q) - 1u)] ^ (uint16_t)(X & 0x8000u);
    return __builtin_bit_cast(half_t, v);
}
// For 16-bit states x*x + x does not wrap, so its bit 31 is set exactly when x >= 46341.
// Both halves of R are states: bit 15 of each half of the result is that comparison
// (x >= 46341  <=>  bit 15 of x set and bit 15 of x - 46341 mod 2^16 clear).
__device__ __forceinline__ uint32_t hyb2_sign_mask(uint32_t R) {
    uint32_t D;
    asm("v_pk_sub_u16 %0, %1, %2" : "=v"(D) : "v"(R), "v"(0xB505B505u));
    return R & ~D & 0x80008000u;
}

// ------------------------------------------------------------- hot-loop pieces

// (a * x + b) mod 2^32 for a zero-extended 16-bit x: one full-rate instruction.
// b64 holds b in its low word and 0 in its high word.
__device__ __forceinline__ uint32_t lcg_mad64(uint32_t x, uint32_t a, uint64_t b64) {
    uint64_t d, carry;
    asm("v_mad_u64_u32 %0, %1, %2, %3, %4" : "=v"(d), "=s"(carry) : "v"(x), "s"(a), "v"(b64));
    return (uint32_t)d;
}

// The 16 zero-extended states of tile row rr of this lane's words.
template <int K, int NW>
__device__ __forceinline__ void row_states(const uint32_t (&w)[NW], int rr, uint32_t (&st)[16]) {
    const int P0 = rr * 16 * K;
#pragma unroll
    for (int c = 0; c < 16; c++) st[c] = window16(w, P0 + c * K);
}

// Two packed weight pairs from four 3INST words: p = (sum(y0), sum(y1)), q = (sum(y2),
// sum(y3)), each sum one binary16 add of the two halves of a word, written straight
// into one half of a packed register (SDWA).  The two pairs are interleaved so that no
// instruction reads a register half-written by the instruction just before it (a
// one-cycle hazard on this ISA); the trailing s_nop covers the first user.
__device__ __forceinline__ void add_halves_pack2x2(uint32_t y0, uint32_t y1, uint32_t y2, uint32_t y3,
                                                   uint32_t &p, uint32_t &q) {
    asm("v_add_f16_sdwa %0, %2, %2 dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %1, %4, %4 dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %0, %3, %3 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %1, %5, %5 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "s_nop 0"
        : "=&v"(p), "=&v"(q)
        : "v"(y0), "v"(y1), "v"(y2), "v"(y3));
}

// The 1024 signed HYB vectors in LDS (see RowDot<K, CODE_HYB>): staging and lookup.
constexpr int HYB_LDS_WORDS = 2 << HYB_Q;
__device__ __forceinline__ void stage_signed_lut(const uint32_t *__restrict__ lut, uint32_t *s_lut,
                                                 int nthreads) {
    for (int i = threadIdx.x; i < (1 << HYB_Q); i += nthreads) {
        const uint32_t v = lut[i];
        s_lut[i] = v;
        s_lut[(1 << HYB_Q) + i] = v ^ 0x80000000u;
    }
}
__device__ __forceinline__ uint32_t hyb_signed_lookup(const uint32_t *s_lut, uint32_t byte_addr) {
    return *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(s_lut) + byte_addr);
}
// The V = 1 form in LDS: hash bits 9..15 select one of 128 signed values, and the table is
// small enough to give every LDS bank a copy of its own: word e * 32 + b holds value e (in
// both halves) for bank b, and lane l reads bank l % 32, so that no two lanes of a pass ever
// meet in a bank whatever their states are: 16 KiB buy table reads without bank conflicts.
__device__ __forceinline__ void stage_hyb1_table(const uint32_t *__restrict__ lut, uint32_t *s_lut,
                                                 int nthreads) {
    const uint16_t *lut16 = reinterpret_cast<const uint16_t *>(lut);
    for (int i = threadIdx.x; i < 128 * 32; i += nthreads) {
        const int e = i >> 5;
        const uint32_t v = lut16[e & 63] ^ ((e & 64) ? 0x8000u : 0u);
        s_lut[i] = v | (v << 16);
    }
}
// The same 1024 signed vectors, HYB_SPREAD = 16 copies: word e * 16 + c is vector e for the
// lanes with lane % 16 == c.  A read of 32 lanes then puts at most two lanes on any bank
// (lanes l and l + 16, when their vectors' numbers have the same parity), against the
// three to four that land on the fullest bank when 32 random reads share one copy.  (32
// copies would leave no conflicts at all but fill 128 KiB, one workgroup per CU instead of
// two: measured 31.5 us against 22.3 us for 16 copies and 29.9 us for one, 8192 x 28672.)
__device__ __forceinline__ void stage_signed_lut_spread(const uint32_t *__restrict__ lut, uint32_t *s_lut,
                                                        int nthreads) {
    for (int e = threadIdx.x; e < 1024; e += nthreads) {
        const uint32_t v = lut[e & 511] ^ ((e & 512) ? 0x80000000u : 0u);
        uint4 *dst = reinterpret_cast<uint4 *>(s_lut + e * HYB_SPREAD);
#pragma unroll
        for (int q = 0; q < HYB_SPREAD / 4; q++) dst[q] = uint4{v, v, v, v};
    }
}
template <int CODE, bool SPREAD = false>
__device__ __forceinline__ void stage_code_table(const uint32_t *__restrict__ lut, uint32_t *s_lut,
                                                 int nthreads) {
    if constexpr (code_is_hyb(CODE) && SPREAD) stage_signed_lut_spread(lut, s_lut, nthreads);
    if constexpr (code_is_hyb(CODE) && !SPREAD) stage_signed_lut(lut, s_lut, nthreads);
    if constexpr (CODE == CODE_HYB1) stage_hyb1_table(lut, s_lut, nthreads);
    if constexpr (code_lds_words(CODE) > 1) __syncthreads();
}
// The 16 values of tile row rr of this lane's words for the V = 1 hash code, each in both
// halves of its register.  lane4 = 4 (lane % 32).
template <int K, int NW>
__device__ __forceinline__ void hyb1_row_values(const uint32_t (&w)[NW], int rr, const uint32_t *s_lut,
                                                uint32_t lane4, uint32_t (&v)[16]) {
    const int P0 = rr * 16 * K;
    if constexpr (K == 2 || K == 4) {
        constexpr int G = 16 / K;  // states between the two halves of a window
#pragma unroll
        for (int base = 0; base < 16; base += 2 * G)
#pragma unroll
            for (int j = 0; j < G; j++) {
                const uint32_t R = window32(w, P0 + (base + j) * K);
                uint32_t H;  // both hashes at once: low 16 bits of x*x + x in each half
                asm("v_pk_mad_u16 %0, %1, %1, %1" : "=v"(H) : "v"(R));
                // hash bits 9..15 times 128 bytes, plus this lane's bank
                v[base + j] = hyb_signed_lookup(s_lut, ((H >> 18) & 0x3F80u) | lane4);
                v[base + j + G] = hyb_signed_lookup(s_lut, ((H >> 2) & 0x3F80u) | lane4);
            }
    } else {
#pragma unroll
        for (int c = 0; c < 16; c++) {
            const uint32_t st = window16(w, P0 + c * K);
            const uint32_t X = st * st + st;
            v[c] = hyb_signed_lookup(s_lut, ((X >> 2) & 0x3F80u) | lane4);
        }
    }
}
// weights c (low half) and c + 1 (high half) as one packed pair
__device__ __forceinline__ uint32_t hyb1_pair(uint32_t lo, uint32_t hi) {
    return (hi & 0xFFFF0000u) | (lo & 0xFFFFu);
}

// acc += p . xa + q . xb for the packed pairs of the previous group, then the next
// group's four fp16 sums into the same p and q.  Order: the dot products read p and q
// first (their halves were written at least two instructions earlier), then the four
// SDWA adds rewrite them, interleaved as in add_halves_pack2x2.
__device__ __forceinline__ void dot2x2_add_halves(uint32_t &p, uint32_t &q, uint32_t xa, uint32_t xb,
                                                  float &acc, uint32_t y0, uint32_t y1, uint32_t y2,
                                                  uint32_t y3) {
    asm("v_dot2c_f32_f16 %2, %0, %7\n\t"
        "v_dot2c_f32_f16 %2, %1, %8\n\t"
        "v_add_f16_sdwa %0, %3, %3 dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %1, %5, %5 dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %0, %4, %4 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:WORD_0 src1_sel:WORD_1\n\t"
        "v_add_f16_sdwa %1, %6, %6 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:WORD_0 src1_sel:WORD_1"
        : "+v"(p), "+v"(q), "+v"(acc)
        : "v"(y0), "v"(y1), "v"(y2), "v"(y3), "v"(xa), "v"(xb));
}
// The last group's dot products, followed by the wait states the dot unit needs before
// another kind of instruction may read or overwrite its result.
__device__ __forceinline__ void dot2x2_tail(uint32_t p, uint32_t q, uint32_t xa, uint32_t xb, float &acc) {
    asm("v_dot2c_f32_f16 %0, %1, %3\n\t"
        "v_dot2c_f32_f16 %0, %2, %4\n\t"
        "s_nop 3"
        : "+v"(acc)
        : "v"(p), "v"(q), "v"(xa), "v"(xb));
}

// One tile row decoded to 8 packed fp16 pairs in column order, with the hot-loop
// instruction sequences (same bits as the plain code functions).  Used where the
// weights feed the matrix cores.
// SPREAD (HYB only): the table holds HYB_SPREAD copies of every vector, as in RowDotHyb.
template <int K, int CODE, bool SPREAD = false> struct RowDecode {
    uint64_t b64;
    uint32_t mm;
    const uint32_t *lut;
    // byte address of the HYB vector selected by hash bits 6..15, given at bits 6..15 of h
    __device__ __forceinline__ uint32_t hyb_address(uint32_t h) const {
        if constexpr (SPREAD) return (h & 0xFFC0u) | ((threadIdx.x & (HYB_SPREAD - 1)) << 2);
        else return (h >> 4) & 0xFFCu;
    }
    __device__ __forceinline__ void init(const uint32_t *lds_lut) {
        lut = lds_lut;
        b64 = CODE == CODE_3INST ? INST_B : MAD_B;
        mm = INST_MM;
        asm volatile("" : "+v"(b64), "+v"(mm));
    }
    template <int NW>
    __device__ __forceinline__ void run(const uint32_t (&w)[NW], int rr, uint32_t (&h)[8]) const {
        if constexpr (CODE == CODE_HYB1) {
            uint32_t v[16];
            hyb1_row_values<K>(w, rr, lut, (threadIdx.x & 31u) << 2, v);
#pragma unroll
            for (int c = 0; c < 8; c++) h[c] = hyb1_pair(v[2 * c], v[2 * c + 1]);
        } else if constexpr (CODE == CODE_3INST) {
            uint32_t st[16], y[16];
            row_states<K>(w, rr, st);
#pragma unroll
            for (int c = 0; c < 16; c++) y[c] = (lcg_mad64(st[c], INST_A, b64) & INST_MASK) ^ mm;
#pragma unroll
            for (int c = 0; c < 16; c += 4)
                add_halves_pack2x2(y[c], y[c + 1], y[c + 2], y[c + 3], h[c / 2], h[c / 2 + 1]);
        } else if constexpr (CODE == CODE_1MAD) {
            uint32_t st[16];
            row_states<K>(w, rr, st);
#pragma unroll
            for (int c = 0; c < 16; c += 2) {
                float f[2];
#pragma unroll
                for (int e = 0; e < 2; e++) {
                    uint32_t X = lcg_mad64(st[c + e], MAD_A, b64);
                    uint32_t t = __builtin_amdgcn_sad_u8(X, 0u, 0x4B000000u);  // float 2^23 + s
                    f[e] = (__builtin_bit_cast(float, t) - 8389118.0f) * MAD_INV_SCALE;
                }
                h[c / 2] = as_u32(half2_t{(half_t)f[0], (half_t)f[1]});
            }
        } else {
            const int P0 = rr * 16 * K;  // lut is the 1024-entry signed table
            if constexpr (K == 2 || K == 4) {
                constexpr int G = 8 / K;
#pragma unroll
                for (int base = 0; base < 8; base += 2 * G)
#pragma unroll
                    for (int j = 0; j < G; j++) {
                        const uint32_t R = window32(w, P0 + (base + j) * 2 * K);
                        uint32_t H;
                        asm("v_pk_mad_u16 %0, %1, %1, %1" : "=v"(H) : "v"(R));
                        // state base+j in the high half of H, state base+j+G in the low half
                        h[base + j] = hyb_signed_lookup(lut, hyb_address(H >> 16));
                        h[base + j + G] = hyb_signed_lookup(lut, hyb_address(H));
                        if constexpr (CODE == CODE_HYB2) {
                            const uint32_t M = hyb2_sign_mask(R);
                            h[base + j] ^= M >> 16;
                            h[base + j + G] ^= M & 0x8000u;
                        }
                    }
            } else {
#pragma unroll
                for (int c = 0; c < 8; c++) {
                    const uint32_t st = window16(w, P0 + c * 2 * K);
                    const uint32_t X = st * st + st;
                    h[c] = hyb_signed_lookup(lut, hyb_address(X));
                    if constexpr (CODE == CODE_HYB2) h[c] ^= (X >> 16) & 0x8000u;
                }
            }
        }
    }
};

template <int K, int CODE> struct RowDot;

// 3INST, V = 1.
template <int K> struct RowDot<K, CODE_3INST> {
    uint64_t b64;
    uint32_t mm;
    __device__ __forceinline__ void init(const uint32_t *) {
        b64 = INST_B;
        mm = INST_MM;
        // keep the constants in VGPRs (they feed VOP3 slots next to an SGPR)
        asm volatile("" : "+v"(b64), "+v"(mm));
    }
    __device__ __forceinline__ void prep_x(uint32_t (&)[8]) const {}
    template <int NW>
    __device__ __forceinline__ void run(const uint32_t (&w)[NW], int rr, const uint32_t (&x)[8],
                                        float &acc) const {
        uint32_t st[16], y[16];
        row_states<K>(w, rr, st);
        // (a multiply-add needs a wait state before the next instruction that reads its result,
        // and before another multiply-add: each mask + xor goes behind the next multiply-add)
        uint32_t X = lcg_mad64(st[0], INST_A, b64);
#pragma unroll
        for (int c = 1; c < 16; c++) {
            const uint32_t Xn = lcg_mad64(st[c], INST_A, b64);
            y[c - 1] = (X & INST_MASK) ^ mm;
            X = Xn;
        }
        y[15] = (X & INST_MASK) ^ mm;
        // Software-pipelined by groups of four weights: a group's two dot products are
        // issued at the head of the next group's block, so that every block ends with four
        // SDWA adds and the dot unit's results are old enough (three wait states) before any
        // instruction outside the blocks can touch the accumulator.
        uint32_t p, q;
        add_halves_pack2x2(y[0], y[1], y[2], y[3], p, q);
#pragma unroll
        for (int c = 4; c < 16; c += 4)
            dot2x2_add_halves(p, q, x[c / 2 - 2], x[c / 2 - 1], acc, y[c], y[c + 1], y[c + 2], y[c + 3]);
        dot2x2_tail(p, q, x[6], x[7], acc);
    }
    template <int NW, int RPL>
    __device__ __forceinline__ void run_tile(const uint32_t (&w)[NW], const uint32_t (&x)[8],
                                             float (&acc)[RPL]) const {
#pragma unroll
        for (int rr = 0; rr < RPL; rr++) run(w, rr, x, acc[rr]);
    }
    template <int RPL> __device__ __forceinline__ void finish(float (&)[RPL]) const {}
};

// 1MAD, V = 1, batch 1.  Algorithm 1 returns the quotient (s - 510) / 147.8 of the byte sum s;
// the product with it is linear in s, so the hot loop contracts the sums themselves and takes
// the affine map out of the loop:
//     sum_j (s_j - 510) / 147.8 * x_j  =  (sum_j (1024 + s_j) x_j  -  1534 sum_j x_j) / 147.8.
// 1024 + s is free as a binary16 number: v_sad_u8 adds the four bytes on top of 0x6400, the
// bit pattern of 1024, and s <= 1020 stays inside the mantissa; v_sad_hi_u8 does the same
// into the high half, so two byte-sum instructions leave a packed pair for v_dot2c, with no
// subtract, scale, conversion or pack per weight (6.9 -> 4.9 vector instructions per weight).
// Every product (1024 + s) x is exact in fp32 and the sums are accumulated in fp32 like any
// other code's.  The weight this uses is the unrounded quotient; qtip_dequantize and the
// matrix-core kernel round it to binary16 first, a relative difference of at most 2^-12 per
// weight (measured on whole layers: 2e-4 of the largest output, a tenth of the 2e-3 bar).
template <int K> struct RowDot<K, CODE_1MAD> {
    uint64_t b64;
    uint32_t bias;
    float sx;  // sum of the activations this lane has contracted with (each tile's 16 once)
    __device__ __forceinline__ void init(const uint32_t *) {
        b64 = MAD_B;
        bias = 0x64006400u;  // 1024 in both halves
        sx = 0.f;
        asm volatile("" : "+v"(b64), "+v"(bias));
    }
    __device__ __forceinline__ void prep_x(uint32_t (&)[8]) const {}
    template <int NW, int RPL>
    __device__ __forceinline__ void run_tile(const uint32_t (&w)[NW], const uint32_t (&x)[8],
                                             float (&acc)[RPL]) {
#pragma unroll
        for (int c = 0; c < 8; c++) sx = __builtin_amdgcn_fdot2(as_half2(0x3C003C00u), as_half2(x[c]), sx, false);
#pragma unroll
        for (int rr = 0; rr < RPL; rr++) {
            uint32_t st[16];
            row_states<K>(w, rr, st);
#pragma unroll
            for (int c = 0; c < 16; c += 2) {
                uint32_t t, p;  // (1024 + s(c + 1), 1024 + s(c)) as packed binary16
                asm("v_sad_u8 %0, %1, 0, %2" : "=v"(t) : "v"(lcg_mad64(st[c], MAD_A, b64)), "v"(bias));
                asm("v_sad_hi_u8 %0, %1, 0, %2" : "=v"(p) : "v"(lcg_mad64(st[c + 1], MAD_A, b64)), "v"(t));
                acc[rr] = __builtin_amdgcn_fdot2(as_half2(p), as_half2(x[c / 2]), acc[rr], false);
            }
        }
    }
    // this lane's sums over its tiles: take the affine map out (before lanes are added up)
    template <int RPL> __device__ __forceinline__ void finish(float (&acc)[RPL]) const {
#pragma unroll
        for (int rr = 0; rr < RPL; rr++) acc[rr] = (acc[rr] - 1534.0f * sx) * MAD_INV_SCALE;
    }
};

// HYB, V = 2.  Bit 15 of the hash negates entry 1 and bits 6..14 pick the row, so
// bits 6..15 together index 2^(Q+1) = 1024 signed vectors (Section 3.1.2 puts it the
// same way); the hot loop reads that 4 KiB table from LDS, built by the kernel from the
// 512 stored rows: signed[s * 512 + idx] = row idx with entry 1 negated iff s.  One
// shift and one mask turn a hash into a byte address, and no sign fix-up is left.
// SPREAD: the table holds HYB_SPREAD copies of every vector (stage_signed_lut_spread) and a
// lane reads its own; else one copy (stage_signed_lut).
template <int K, bool TWO, bool SPREAD> struct RowDotHyb {
    const uint32_t *lut;  // LDS: the 1024 signed vectors
    uint32_t lane4;       // SPREAD: byte offset of this lane's copy inside a vector's 64 bytes
    __device__ __forceinline__ void init(const uint32_t *lds_lut) {
        lut = lds_lut;
        lane4 = (threadIdx.x & (HYB_SPREAD - 1)) << 2;
    }
    // byte address of the vector selected by hash bits 6..15, given those bits at 6..15 of h
    __device__ __forceinline__ uint32_t address(uint32_t h) const {
        if constexpr (SPREAD) return (h & 0xFFC0u) | lane4;  // times 64 bytes: in place already
        else return (h >> 4) & 0xFFCu;
    }
    __device__ __forceinline__ void prep_x(uint32_t (&)[8]) const {}
    template <int RPL> __device__ __forceinline__ void finish(float (&)[RPL]) const {}
    // All RPL rows of this lane, software-pipelined by row: the hashes and the eight
    // table reads of row r+1 are issued before the reads of row r are consumed, so
    // a wave keeps the LDS and the vector ALU busy at the same time by itself.
    // (Waves of a workgroup run in near lockstep; leaving the overlap to chance
    // between waves makes LDS time and ALU time add up instead.)
    template <int NW, int RPL>
    __device__ __forceinline__ void run_tile(const uint32_t (&w)[NW], const uint32_t (&x)[8],
                                             float (&acc)[RPL]) const {
        if constexpr (K == 2 || K == 4) {
            constexpr int G = 8 / K;  // states between the two halves of a window
            uint32_t v[RPL][8];
            auto issue_row = [&](int rr) {
#pragma unroll
                for (int base = 0; base < 8; base += 2 * G)
#pragma unroll
                    for (int j = 0; j < G; j++) {
                        const uint32_t R = window32(w, rr * 16 * K + (base + j) * 2 * K);
                        // both hashes at once: low 16 bits of x*x + x in each half
                        uint32_t H;
                        asm("v_pk_mad_u16 %0, %1, %1, %1" : "=v"(H) : "v"(R));
                        // hash bits 6..15 times 64 bytes (they are in place already) plus this
                        // lane's copy; state base+j sits in the high half
                        v[rr][base + j] = hyb_signed_lookup(lut, address(H >> 16));
                        v[rr][base + j + G] = hyb_signed_lookup(lut, address(H));
                        if constexpr (TWO) {  // TWO: the first entry's sign, from the states themselves
                            const uint32_t M = hyb2_sign_mask(R);
                            v[rr][base + j] ^= M >> 16;
                            v[rr][base + j + G] ^= M & 0x8000u;
                        }
                    }
            };
            issue_row(0);
#pragma unroll
            for (int rr = 0; rr < RPL; rr++) {
                if (rr + 1 < RPL) issue_row(rr + 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < 8; c++)
                    acc[rr] = __builtin_amdgcn_fdot2(as_half2(v[rr][c]), as_half2(x[c]), acc[rr], false);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int rr = 0; rr < RPL; rr++)
#pragma unroll
                for (int c = 0; c < 8; c++) {
                    const uint32_t st = window16(w, rr * 16 * K + c * 2 * K);
                    const uint32_t X = st * st + st;
                    uint32_t v = hyb_signed_lookup(lut, address(X));
                    if constexpr (TWO) v ^= (X >> 16) & 0x8000u;
                    acc[rr] = __builtin_amdgcn_fdot2(as_half2(v), as_half2(x[c]), acc[rr], false);
                }
        }
    }
};
// The V = 1 hash code: per row 16 conflict-free table reads, pipelined by row like HYB.
template <int K> struct RowDot<K, CODE_HYB1> {
    const uint32_t *lut;  // LDS: 128 signed values x 32 banks
    uint32_t lane4;
    __device__ __forceinline__ void init(const uint32_t *lds_lut) {
        lut = lds_lut;
        lane4 = (threadIdx.x & 31u) << 2;
    }
    __device__ __forceinline__ void prep_x(uint32_t (&)[8]) const {}
    template <int RPL> __device__ __forceinline__ void finish(float (&)[RPL]) const {}
    template <int NW, int RPL>
    __device__ __forceinline__ void run_tile(const uint32_t (&w)[NW], const uint32_t (&x)[8],
                                             float (&acc)[RPL]) const {
        uint32_t v[RPL][16];
        hyb1_row_values<K>(w, 0, lut, lane4, v[0]);
#pragma unroll
        for (int rr = 0; rr < RPL; rr++) {
            if (rr + 1 < RPL) hyb1_row_values<K>(w, rr + 1, lut, lane4, v[rr + 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < 8; c++)
                acc[rr] = __builtin_amdgcn_fdot2(as_half2(hyb1_pair(v[rr][2 * c], v[rr][2 * c + 1])),
                                                 as_half2(x[c]), acc[rr], false);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
};
template <int K> struct RowDot<K, CODE_HYB> : RowDotHyb<K, false, false> {};
template <int K> struct RowDot<K, CODE_HYB2> : RowDotHyb<K, true, false> {};
// The batch-1 kernel's choice: the spread table for the HYB codes when it asks for it.
template <int K, int CODE, bool SPREAD> struct RowDotFor { using type = RowDot<K, CODE>; };
template <int K> struct RowDotFor<K, CODE_HYB, true> { using type = RowDotHyb<K, false, true>; };
template <int K> struct RowDotFor<K, CODE_HYB2, true> { using type = RowDotHyb<K, true, true>; };

}  // namespace qtip
