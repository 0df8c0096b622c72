// Device-side building blocks of the QTIP decode path for gfx950 (CDNA4):
// tile geometry, state-window extraction from packed words held in VGPRs, and
// the state -> fp16 value codes (Algorithms 1-3 of arXiv 2406.11235).
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

// Section 3.1.1 constants.
constexpr uint32_t MAD_A = 34038481u, MAD_B = 76625530u;
constexpr uint32_t INST_A = 89226354u, INST_B = 64248484u;
constexpr uint32_t INST_MASK = 0x8FFF8FFFu;  // sign, 2 low exponent bits, mantissa; twice
constexpr uint32_t INST_MM = 0x3B603B60u;    // fp16(0.922) = 0x3B60 in both halves
constexpr int HYB_Q = 9;

// How one 16x16 tile (8K words) is spread over lanes: every lane holds WPL
// consecutive words = RPL whole tile rows; LPT lanes cover a tile.
template <int K> struct Geo;
template <> struct Geo<2> { static constexpr int WPL = 4, LPT = 4, RPL = 4; };
template <> struct Geo<3> { static constexpr int WPL = 3, LPT = 8, RPL = 2; };
template <> struct Geo<4> { static constexpr int WPL = 4, LPT = 8, RPL = 2; };

__device__ __forceinline__ half2_t as_half2(uint32_t v) {
    return __builtin_bit_cast(half2_t, v);
}
__device__ __forceinline__ uint32_t as_u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// 16-bit window starting P bits into the word array w (P is a compile-time
// constant after unrolling; words are MSB-first, so a window is a right shift
// of one word or of a two-word funnel).
template <int NW>
__device__ __forceinline__ uint32_t window16(const uint32_t (&w)[NW], int P) {
    const int i = P >> 5, s = P & 31;
    if (s <= 16) return (w[i] >> (16 - s)) & 0xFFFFu;
    return __builtin_amdgcn_alignbit(w[i], w[i + 1], 48 - s) & 0xFFFFu;
}

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
    return (half_t)((float)(s - 510) * 0.0067658998646820027f);
}

// Algorithm 3 with Q = 9: hash x*x + x, bits 6..14 index the table, bit 15
// negates the second entry.  lut holds one 32-bit word per row (entry 0 in the
// low half); `stride` words separate consecutive rows (1 = plain table).
__device__ __forceinline__ half2_t code_hyb(uint32_t x, const uint32_t *lut, int stride = 1) {
    uint32_t X = x * x + x;
    uint32_t v = lut[((X >> (15 - HYB_Q)) & ((1u << HYB_Q) - 1u)) * stride];
    return as_half2(v ^ ((X & 0x8000u) << 16));
}

}  // namespace qtip
