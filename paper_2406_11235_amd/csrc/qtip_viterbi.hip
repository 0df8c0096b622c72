// GPU quantizer: the Viterbi algorithm on the (L, k, V) bitshift trellis (Section 2.3 of
// arXiv 2406.11235: value function and update rule; Section 3.1: edge rule), made
// tail-biting by Algorithm 4, one T_x x T_y block = one length-256 sequence (Section 4), for
// the computed codes of Algorithms 1-3 (L = 16, 16 x 16 blocks) and the lookup-only code of
// the appendix (L = 14, 32 x 8 blocks; the text below says 16 and 1024, read L and 2^L / 64).
//
// Layout on the chip.  One workgroup of NT = 1024 threads owns one sequence and keeps the
// whole value function, 2^16 binary32 numbers, in registers: thread `tid` holds the 64
// states y = NT r + tid (half of the 128 registers a thread has at four waves per SIMD;
// the code values take most of the other half).  The bitshift structure makes that layout communication-free
// for the minimum: the 2^kV predecessors of y all end in the top 16-kV bits of y, so
// states with a common "prefix" hi = y >> kV share one minimum, and the predecessors
// p 2^(16-kV) + hi of a prefix have the same low 10 bits, i.e. live in one thread
// (kV <= 6; for kV = 8 they are spread over four threads, which meet in LDS; for kV <= 3 a
// thread instead owns whole (predecessor, child) squares of states, see VitGeo).  A step is
//   phase 1: every thread takes the minimum and arg-minimum over the predecessors of
//            its prefixes, publishes the minima in LDS (2^(16-kV) floats, 64 KiB at
//            kV = 2) and stores the arg-minima, kV bits each, packed into one or two
//            words per thread and step, to the back-pointer workspace in HBM;
//   phase 2: every thread reads the minimum of each of its states' prefixes back from
//            LDS and adds the squared error of the state's code value.
// Code values never change, so they sit in registers as packed fp16 (V = 1); for the
// HYB code a state only selects one of 1024 signed table rows (2048 with two sign flips), so
// each step first builds their squared errors in LDS and states carry a row number.
// A second, tiny kernel walks the back-pointers (one thread per sequence: the walk is a
// chain of dependent loads, so it is run over a whole batch of sequences at once).
// Algorithm 4 is forward / walk-to-the-middle / constrained forward / full walk.
//
// Arithmetic (fixed, so that a CPU reference can repeat every decision): binary32,
//   e_j = C[y][j] - s[V t + j];
//   V = 1: value = fma(e_0, e_0, min)            (the first step: e_0 e_0)
//   V = 2: value = min + fma(e_1, e_1, e_0 e_0)  (the error comes from a per-step table)
// with exactly these roundings (the file is compiled without contraction).
// Minima take the lowest predecessor on ties, the final state the lowest state.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qtip_device.h"
#include "qtip_internal.h"

#pragma clang fp contract(off)

namespace qtip {
namespace {

constexpr int VT_T = 256;    // sequence length (one T_x x T_y block)
constexpr int VT_REGS = 64;  // states per thread

// LB = L, the number of state bits: 16 (NT = 1024 threads per sequence) for the codes of
// Algorithms 1-3, 14 (NT = 256) for the lookup-only code.
template <int KV, int LB>
struct VitGeo {
    static constexpr int NT = (1 << LB) / VT_REGS;  // threads per sequence
    static constexpr int OV = LB - KV;              // bits two consecutive states share
    static constexpr int NP = 1 << OV;              // prefixes = minima per step
    static constexpr int NC = 1 << KV;              // predecessors per prefix
    static constexpr bool LOCAL = NP >= NT;         // predecessors of a prefix in one thread
    static constexpr int NB1 = LOCAL ? NP / NT : 1;     // prefixes per thread
    // back-pointers: kV bits per prefix, FPW whole fields per word, PWT words per thread
    static constexpr int FPW = 32 / KV;
    static constexpr int PWT = (NB1 + FPW - 1) / FPW;
    // kV <= 3: a thread can own, for a few values "mid" of the middle L - 2 kV bits of the
    // state, all 2^kV x 2^kV states (p, mid, c).  Then the predecessors of a prefix (mid, c)
    // are still its own registers, and so are all 2^kV children of a prefix it reads back, so
    // one LDS read serves 2^kV states and a thread's minima are contiguous in LDS (16-byte
    // LDS operations).  SJ = mids per thread: mid = SJ tid + j.
    static constexpr bool SLOT = KV <= 3;
    static constexpr int SJ = SLOT ? VT_REGS / (NC * NC) : 1;
    // kV = 2, 1024 threads: the back-pointer of a prefix is kept as the three outcomes of the
    // comparisons that found its minimum (v1 < v0, v3 < v2, min23 < min01) instead of the
    // index they imply: a comparison's lane mask goes straight into the packed word as the
    // carry of an add (word = 2 word + carry), and no instruction ever forms the index.  16
    // prefixes x 3 bits are two words per thread and step: prefix f is bits 3 (f % 8) ..
    // + 2 of word f / 8, comparison outcomes in the order above from bit 2 down.
    static constexpr bool RAW3 = KV == 2 && NT == 1024;
    static constexpr int PW = RAW3 ? 2 * NT : SLOT ? NT : LOCAL ? NT * PWT : NP;  // back-pointer words per step
};

__host__ __device__ constexpr int vit_max(int a, int b) { return a > b ? a : b; }

// Minimum of val[base + j stride], j = 0 .. COUNT-1, and the lowest j that attains it.
// CH independent compare-select chains (j = c mod CH) run interleaved, so that the wait
// states between a compare and the selects reading its mask are filled, and are merged
// at the end; ties go to the lower j at every stage.  All indices fold to constants once
// the callers' loops are unrolled.
template <int COUNT, int CH>
__device__ __forceinline__ void argmin_regs(const float (&val)[VT_REGS], int base, int stride, float &bv,
                                            uint32_t &bj) {
    float cv[CH];
    uint32_t cj[CH];
#pragma unroll
    for (int c = 0; c < CH; c++) {
        cv[c] = val[base + c * stride];
        cj[c] = (uint32_t)c;
    }
#pragma unroll
    for (int j = CH; j < COUNT; j++) {
        const int c = j % CH;
        const float v = val[base + j * stride];
        const bool lt = v < cv[c];
        cv[c] = lt ? v : cv[c];
        cj[c] = lt ? (uint32_t)j : cj[c];
    }
    bv = cv[0];
    bj = cj[0];
#pragma unroll
    for (int c = 1; c < CH; c++) {
        const bool better = cv[c] < bv || (cv[c] == bv && cj[c] < bj);
        bv = better ? cv[c] : bv;
        bj = better ? cj[c] : bj;
    }
}

// The same minimum and arg-minimum for COUNT a power of two, as a tournament: the values go
// through v_min_f32 (no select waits on a compare), and the index never exists as a number:
// every comparison leaves a 64-lane mask in scalar registers, the masks of the winner's path
// are combined there (scalar and/or, which issue beside the vector instructions), and
// bits[b] ends up as the lane mask of index bit b.  Left wins on ties at every level, which
// is the lowest index, as in argmin_regs.
template <int N>
__device__ __forceinline__ float argmin_tournament(const float (&val)[VT_REGS], int base, int stride, int lo,
                                                   uint64_t *bits) {
    if constexpr (N == 1) {
        return val[base + lo * stride];
    } else {
        constexpr int H = N / 2;
        constexpr int LOGH = H == 1 ? 0 : H == 2 ? 1 : H == 4 ? 2 : 3;
        uint64_t bl[4], br[4];
        const float a = argmin_tournament<H>(val, base, stride, lo, bl);
        const float b = argmin_tournament<H>(val, base, stride, lo + H, br);
        const uint64_t lt = __ballot(b < a);
#pragma unroll
        for (int i = 0; i < LOGH; i++) bits[i] = (lt & br[i]) | (~lt & bl[i]);
        bits[LOGH] = lt;
        // (as an instruction: the builtin first "canonicalizes" both operands, one extra
        // instruction each, against signalling NaNs that cannot occur here)
        float m;
        asm("v_min_f32 %0, %1, %2" : "=v"(m) : "v"(a), "v"(b));
        return m;
    }
}
// lt = b < a; word = 2 word + lt; m = min(a, b): the comparison's mask is consumed as the carry
// of the add that follows it (ties: lt = 0, the left operand, as everywhere).
__device__ __forceinline__ void compare_shift_min(float a, float b, uint32_t &word, float &m) {
    asm("v_cmp_lt_f32 vcc, %3, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc\n\tv_min_f32 %1, %2, %3"
        : "+v"(word), "=v"(m)
        : "v"(a), "v"(b)
        : "vcc");
}
// word = 2 word + (this lane's bit of mask): one add-with-carry.
__device__ __forceinline__ void shift_in_bit(uint32_t &word, uint64_t mask) {
    uint64_t carry_out;
    asm("v_addc_co_u32_e64 %0, %1, %0, %0, %2" : "+v"(word), "=s"(carry_out) : "s"(mask));
}

// rotate = 1: the sequence rotated by T/2 (Algorithm 4's first call).  overlap != null:
// the first state's top 16-kV bits and the last state's low 16-kV bits are forced to
// overlap[slot] (its second call).  Sequence `slot` of the batch is tile tile0 + slot.
template <int KV, int V, int CODE>
// (four waves per SIMD, i.e. at most 128 registers, also where a workgroup is only four waves)
__global__ __launch_bounds__((VitGeo<KV, code_state_bits(CODE)>::NT), 4) void viterbi_forward_kernel(
    const float *__restrict__ W, int n, int tn, long tile0, const uint32_t *__restrict__ lut, int rotate,
    const uint32_t *__restrict__ overlap, uint32_t *__restrict__ ptrs, uint32_t *__restrict__ final_state,
    float *__restrict__ final_value) {
    using Geo = VitGeo<KV, code_state_bits(CODE)>;
    constexpr int NP = Geo::NP, NC = Geo::NC, NB1 = Geo::NB1, PW = Geo::PW, VT_NT = Geo::NT;
    constexpr int LTY = code_log2_ty(CODE), TY = 1 << LTY, TX = VT_T >> LTY;  // the block is TX x TY
    constexpr int G = VT_T / V;
    constexpr bool HYB = code_is_hyb(CODE);
    constexpr int ROWS = CODE == CODE_HYB2 ? 2048 : 1024;  // signed table rows a state can select
    // The per-step error table is read at random (one read per state and step), so it is kept
    // in DCOPY copies: word row * DCOPY + c belongs to the lanes with lane % DCOPY == c, and a
    // 32-lane pass finds at most four lanes on four banks instead of 32 on 32 (the fullest
    // bank then holds about 2 reads instead of 3.5).
    constexpr int DCOPY = 8;
    static_assert(HYB == (V == 2), "V = 2 is the HYB code");
    // LDS: minima (or, for kV = 8, per-thread partial minima, their predecessors and the
    // 256 minima), reused for the final reduction; then the HYB error table
    constexpr int BEST_FLOATS = Geo::LOCAL ? vit_max(NP, 2 * VT_NT) : 2 * VT_NT + NP;
    __shared__ __attribute__((aligned(16))) float s_mem[BEST_FLOATS + VT_T + (HYB ? ROWS * DCOPY : 0)];
    float *const s_best = s_mem;
    float *const s_seq = s_mem + BEST_FLOATS;      // the sequence
    float *const s_D = s_mem + BEST_FLOATS + VT_T;  // HYB only
    const float *const s_Dmine = s_D + (threadIdx.x & (DCOPY - 1));

    const int tid = threadIdx.x;
    const int slot = blockIdx.x;
    const long tile = tile0 + slot;
    const int I = (int)(tile / tn), J = (int)(tile % tn);

    static_assert(VT_NT >= VT_T, "one thread per sequence element");
    if (tid < VT_T) {
        const int s = rotate ? ((tid + VT_T / 2) & (VT_T - 1)) : tid;
        s_seq[tid] = W[(size_t)(TX * I + (s >> LTY)) * n + TY * J + (s & (TY - 1))];
    }
    __syncthreads();
    auto seq = [&](int u) -> float { return s_seq[u]; };
    // the state held in register r: NT r + tid, or (p, SJ tid + j, c) with r = (p SJ + j) NC + c;
    // increasing in r either way
    auto state_of = [&](int r) -> uint32_t {
        if constexpr (Geo::SLOT) {
            const int p = r / (Geo::SJ * NC), j = (r / NC) % Geo::SJ, c = r % NC;
            return ((uint32_t)p << Geo::OV) | ((uint32_t)(tid * Geo::SJ + j) << KV) | (uint32_t)c;
        } else {
            return (uint32_t)(r * VT_NT + tid);
        }
    };

    // code values of this thread's states
    half2_t cpk[HYB ? 1 : VT_REGS / 2];
    uint32_t ipk[HYB ? VT_REGS / 2 : 1];
#pragma unroll
    for (int r = 0; r < VT_REGS; r++) {
        const uint32_t y = state_of(r);
        if constexpr (HYB) {
            const uint32_t X = y * y + y;
            uint32_t row = (X >> (15 - HYB_Q)) & 1023u;  // table index and sign bit
            if constexpr (CODE == CODE_HYB2) row |= (X >> 31) << 10;  // second sign bit
            // kept as the byte offset of the row's error in the per-step table
            if (r & 1)
                ipk[r >> 1] |= (row * 4 * DCOPY) << 16;
            else
                ipk[r >> 1] = row * 4 * DCOPY;
        } else {
            if constexpr (CODE == CODE_LUT)
                cpk[r >> 1][r & 1] = reinterpret_cast<const half_t *>(lut)[y];
            else if constexpr (CODE == CODE_HYB1)
                cpk[r >> 1][r & 1] = code_hyb1(y, reinterpret_cast<const uint16_t *>(lut));
            else
                cpk[r >> 1][r & 1] = CODE == CODE_3INST ? code_3inst(y) : code_1mad(y);
        }
    }
    // (opaque to the compiler from here on, or it recomputes the codes inside the loop
    // instead of keeping them)
#pragma unroll
    for (int r2 = 0; r2 < VT_REGS / 2; r2++) {
        if constexpr (HYB) {
            asm volatile("" : "+v"(ipk[r2]));
        } else {
            uint32_t cw = as_u32(cpk[r2]);
            asm volatile("" : "+v"(cw));
            cpk[r2] = as_half2(cw);
        }
    }
    // squared error of table row `row` against (s0, s1)
    auto hyb_error = [&](int row, float s0, float s1) -> float {
        const half2_t c = as_half2(lut[row & 511]);
        const float c0 = (row & 1024) ? -(float)c.x : (float)c.x;
        const float c1 = (row & 512) ? -(float)c.y : (float)c.y;
        const float e0 = c0 - s0, e1 = c1 - s1;
        return __builtin_fmaf(e1, e1, e0 * e0);
    };
    auto store_error = [&](int row, float e) {  // all copies of one row: 16-byte stores
        float4_t *dst = reinterpret_cast<float4_t *>(s_D + row * DCOPY);
#pragma unroll
        for (int q = 0; q < DCOPY / 4; q++) dst[q] = float4_t{e, e, e, e};
    };
    // New values of states 2 r2 and 2 r2 + 1 of this thread (they share a packed register)
    // from the minima b0, b1 of their prefixes: fma(e, e, b) for V = 1, b + table entry for
    // HYB.  The unpacking is pinned here (volatile asm): hoisted out of the step loop it turns
    // the 32 packed registers into 64 and the loop starts spilling, and the reloads cost far
    // more than the unpacking (the waves run in lockstep between barriers, so nothing hides
    // their latency).  For V = 1 the conversion and the subtraction are one v_fma_mix_f32,
    // (float)c * 1.0 - s: an exact product and one rounding, the same bits as c - s.
    auto update2 = [&](int r2, float s0, float b0, float b1, float &v0, float &v1) {
        if constexpr (HYB) {
            uint32_t o0, o1;  // byte offsets of the two rows' errors in the per-step table
            asm volatile("v_and_b32 %0, 0xffff, %2\n\tv_lshrrev_b32 %1, 16, %2"
                         : "=&v"(o0), "=v"(o1)
                         : "v"(ipk[r2]));
            // (s_Dmine = the table shifted by this lane's copy)
            v0 = b0 + *reinterpret_cast<const float *>(reinterpret_cast<const char *>(s_Dmine) + o0);
            v1 = b1 + *reinterpret_cast<const float *>(reinterpret_cast<const char *>(s_Dmine) + o1);
        } else {
            const uint32_t cw = as_u32(cpk[r2]);
            float e0, e1;
            asm volatile("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,0]"
                         : "=v"(e0) : "v"(cw), "v"(s0));
            asm volatile("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
                         : "=v"(e1) : "v"(cw), "v"(s0));
            v0 = __builtin_fmaf(e0, e0, b0);
            v1 = __builtin_fmaf(e1, e1, b1);
        }
    };
    // One state at a time (V = 1): the form the kV <= 3 layout runs fastest with (measured;
    // the loops differ only in how the compiler schedules around the pinned instructions).
    auto update1 = [&](int r, float s0, float b) -> float {
        const uint32_t cw = as_u32(cpk[r >> 1]);
        float e;
        if (r & 1)
            asm volatile("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
                         : "=v"(e) : "v"(cw), "v"(s0));
        else
            asm volatile("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,0]"
                         : "=v"(e) : "v"(cw), "v"(s0));
        return __builtin_fmaf(e, e, b);
    };

    const float INF = __builtin_inff();
    const bool constrained = overlap != nullptr;
    const uint32_t O = constrained ? overlap[slot] : 0u;

    float val[VT_REGS];
    {
        const float s0 = seq(0), s1 = V == 2 ? seq(1) : 0.f;
        if constexpr (HYB) {
#pragma unroll
            for (int j = tid; j < ROWS; j += VT_NT) store_error(j, hyb_error(j, s0, s1));
            __syncthreads();
        }
#pragma unroll
        for (int r2 = 0; r2 < VT_REGS / 2; r2++) {
            float d[2];
            update2(r2, s0, 0.f, 0.f, d[0], d[1]);  // the first step has no predecessors
#pragma unroll
            for (int h = 0; h < 2; h++)
                val[2 * r2 + h] = (constrained && (state_of(2 * r2 + h) >> KV) != O) ? INF : d[h];
        }
        if constexpr (HYB) __syncthreads();
    }

    uint32_t *const my_ptrs = ptrs + (size_t)slot * G * PW;
    for (int t = 1; t < G; t++) {
        if constexpr (HYB) {
#pragma unroll
            for (int j = tid; j < ROWS; j += VT_NT) store_error(j, hyb_error(j, seq(V * t), seq(V * t + 1)));
        }
        if constexpr (Geo::SLOT) {
            // prefix hi = (SJ tid + j) NC + c; its predecessors are registers (p SJ + j) NC + c
            constexpr int F = Geo::SJ * NC;  // prefixes per thread, contiguous in hi
            float bests[F];
            uint32_t word = 0;
            // The tournament form pays where the waves of a CU are in different phases of the
            // step (several small workgroups per CU, L = 14: 1.06 -> 0.97 us per sequence): its
            // scalar instructions then overlap other waves' vector work.  With one 16-wave
            // workgroup per CU all waves reach this point together, the scalar unit (one per
            // CU) becomes the queue, and the select chains are faster (4.69 against 4.91 us).
            if constexpr (Geo::RAW3) {
                uint32_t words[2] = {0u, 0u};
#pragma unroll
                for (int f = F - 1; f >= 0; f--) {
                    float m01, m23;
                    compare_shift_min(val[f], val[f + F], words[f >> 3], m01);
                    compare_shift_min(val[f + 2 * F], val[f + 3 * F], words[f >> 3], m23);
                    compare_shift_min(m01, m23, words[f >> 3], bests[f]);
                    if ((f & 3) == 0) __builtin_amdgcn_sched_barrier(0);
                }
                my_ptrs[(size_t)t * PW + VT_NT + tid] = words[1];
                word = words[0];
            } else if constexpr (VT_NT <= 256) {
                // prefixes from the last to the first and bits from the top down, so that prefix
                // f ends up in bits f kV .. f kV + kV - 1 of the word
#pragma unroll
                for (int f = F - 1; f >= 0; f--) {
                    uint64_t bits[4];
                    bests[f] = argmin_tournament<NC>(val, f, F, 0, bits);
#pragma unroll
                    for (int b = KV - 1; b >= 0; b--) shift_in_bit(word, bits[b]);
                    if ((f & 3) == 0) __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int f = 0; f < F; f++) {
                    uint32_t bp;
                    argmin_regs<NC, 1>(val, f, F, bests[f], bp);
                    word |= bp << (f * KV);
                    if ((f & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
            // A thread's F minima are one row of F floats.  Written as they stand, the 16-byte
            // stores of neighbouring lanes would be a whole row apart and land on two of the
            // eight 16-byte bank groups; with 16 floats per row the four pieces of row T are
            // therefore kept rotated by (T / 2) % 4 places, which spreads eight lanes over all
            // eight groups both here and where the rows are read back, four prefixes at a time.
#pragma unroll
            for (int f = 0; f < F; f += 4) {
                const int piece = F == 16 ? ((f >> 2) + (tid >> 1)) & 3 : f >> 2;
                *reinterpret_cast<float4_t *>(&s_best[tid * F + 4 * piece]) =
                    float4_t{bests[f], bests[f + 1], bests[f + 2], bests[f + 3]};
            }
            my_ptrs[(size_t)t * PW + tid] = word;
        } else if constexpr (Geo::LOCAL) {
            // prefix hi = NT h + tid; its predecessors p 2^OV + hi are registers p NB1 + h
            uint32_t word[Geo::PWT];
#pragma unroll
            for (int w = 0; w < Geo::PWT; w++) word[w] = 0;
#pragma unroll
            for (int h = 0; h < NB1; h++) {
                float bv;
                uint32_t bp;
                argmin_regs<NC, (NB1 >= 4 || NC < 8) ? 1 : 4 / NB1>(val, h, NB1, bv, bp);
                s_best[h * VT_NT + tid] = bv;
                word[h / Geo::FPW] |= bp << ((h % Geo::FPW) * KV);
                // a few chains at a time: enough to fill the wait states between a compare
                // and the selects that use its mask, few enough to stay in registers
                if ((h & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int w = 0; w < Geo::PWT; w++) my_ptrs[(size_t)t * PW + w * VT_NT + tid] = word[w];
        } else {
            // prefix hi = tid % NP; this thread holds predecessors p = (VT_NT/NP) r + tid / NP
            constexpr int Q = VT_NT / NP;
            float bv;
            uint32_t br;
            argmin_regs<VT_REGS, 4>(val, 0, 1, bv, br);
            float *s_pv = s_best;
            uint32_t *s_pp = reinterpret_cast<uint32_t *>(s_best + VT_NT);
            s_pv[tid] = bv;
            s_pp[tid] = br * Q + (uint32_t)(tid / NP);
            __syncthreads();
            if (tid < NP) {
                bv = s_pv[tid];
                uint32_t bp = s_pp[tid];
#pragma unroll
                for (int q = 1; q < Q; q++) {
                    const float v = s_pv[q * NP + tid];
                    const uint32_t p = s_pp[q * NP + tid];
                    const bool better = v < bv || (v == bv && p < bp);
                    bv = better ? v : bv;
                    bp = better ? p : bp;
                }
                s_best[2 * VT_NT + tid] = bv;
                my_ptrs[(size_t)t * PW + tid] = bp;
            }
        }
        __syncthreads();
        const float *best_mine = (Geo::LOCAL ? s_best : s_best + 2 * VT_NT) + (tid >> KV);
        // (read after the barrier, so that the errors are not computed, and kept in
        // registers that are not there, before the minima)
        const float s0 = HYB ? 0.f : seq(t);
        if constexpr (Geo::SLOT) {
            // states (p, mid, c') follow prefix (p, mid): one read per (p, j) serves NC states
#pragma unroll
            for (int p = 0; p < NC; p++) {
                float b[Geo::SJ];
                if constexpr (Geo::SJ == 4) {
                    // prefixes p NP/NC + 4 tid .. + 3 are piece tid % 4 of row T = p NT/4 + tid / 4,
                    // kept at place (tid % 4 + T / 2) % 4 of that row (p NT/8 is a multiple of 4)
                    static_assert(Geo::SJ * NC == 16 && (VT_NT / 8) % 4 == 0, "row rotation");
                    const int place = ((tid & 3) + (tid >> 3)) & 3;
                    const float4_t t4 =
                        *reinterpret_cast<const float4_t *>(&s_best[p * (NP / NC) + (tid & ~3) * 4 + place * 4]);
                    b[0] = t4[0], b[1] = t4[1], b[2] = t4[2], b[3] = t4[3];
                } else {
#pragma unroll
                    for (int j = 0; j < Geo::SJ; j++) b[j] = s_best[p * (NP / NC) + tid * Geo::SJ + j];
                }
#pragma unroll
                for (int j = 0; j < Geo::SJ; j++)
#pragma unroll
                    for (int c = 0; c < NC; c++) {
                        const int r = (p * Geo::SJ + j) * NC + c;
                        val[r] = update1(r, s0, b[j]);
                    }
                if (((p * Geo::SJ) & 1) == 1 || Geo::SJ > 1) __builtin_amdgcn_sched_barrier(0);
            }
        } else
        // eight states at a time: the register file has no room for 64 loads in flight
#pragma unroll
        for (int r0 = 0; r0 < VT_REGS; r0 += 8) {
#pragma unroll
            for (int r = r0; r < r0 + 8; r += 2) {
                // prefixes of states NT r + tid and NT (r + 1) + tid; written so that the
                // addresses are one base register plus constants
                const float b0 = best_mine[r * (VT_NT >> KV)], b1 = best_mine[(r + 1) * (VT_NT >> KV)];
                update2(r / 2, s0, b0, b1, val[r], val[r + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    }

    // the best allowed final state, lowest state on ties
    float bv = INF;
    uint32_t by = 0xFFFFFFFFu;
#pragma unroll
    for (int r = 0; r < VT_REGS; r++) {
        const uint32_t y = state_of(r);
        const bool ok = !constrained || (y & (uint32_t)(NP - 1)) == O;
        if (ok && val[r] < bv) {
            bv = val[r];
            by = y;
        }
    }
    float *s_rv = s_best;
    uint32_t *s_ry = reinterpret_cast<uint32_t *>(s_best + VT_NT);
    s_rv[tid] = bv;
    s_ry[tid] = by;
    __syncthreads();
    for (int stride = VT_NT / 2; stride > 0; stride >>= 1) {
        if (tid < stride) {
            const float v = s_rv[tid + stride];
            const uint32_t y = s_ry[tid + stride];
            if (v < s_rv[tid] || (v == s_rv[tid] && y < s_ry[tid])) {
                s_rv[tid] = v;
                s_ry[tid] = y;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        final_state[slot] = s_ry[0];
        final_value[slot] = s_rv[0];
    }
}

// One thread per sequence walks the back-pointers from the final state.
// pass 1: down to step G/2 - 1, whose low 16-kV bits are the overlap of Algorithm 4.
// pass 2: the whole walk; step t contributes the top kV bits of its state as stream bits
// t kV .. (t+1) kV - 1 (first bit = most significant bit of word 0).
template <int KV, int V, int LB>
__global__ __launch_bounds__(64) void viterbi_backtrace_kernel(
    const uint32_t *__restrict__ ptrs, const uint32_t *__restrict__ final_state,
    const float *__restrict__ final_value, int count, int pass, uint32_t *__restrict__ overlap,
    uint32_t *__restrict__ codes, float *__restrict__ tile_err, long tile0) {
    using Geo = VitGeo<KV, LB>;
    constexpr int OV = Geo::OV, NP = Geo::NP, NC = Geo::NC, PW = Geo::PW, VT_NT = Geo::NT;
    constexpr int G = VT_T / V, NWORDS = KV * G / 32;
    const int slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= count) return;
    const uint32_t *my_ptrs = ptrs + (size_t)slot * G * PW;
    uint32_t arg = final_state[slot];
    uint32_t words[NWORDS];
#pragma unroll
    for (int w = 0; w < NWORDS; w++) words[w] = 0;
    const int stop = pass == 1 ? G / 2 - 1 : 0;
    for (int t = G - 1;; t--) {
        if (pass == 2) {
            const uint32_t top = arg >> OV;
            for (int b = 0; b < KV; b++) {
                const int pos = t * KV + b;
                if ((top >> (KV - 1 - b)) & 1u) words[pos >> 5] |= 1u << (31 - (pos & 31));
            }
        }
        if (t == stop) break;
        const uint32_t hi = arg >> KV;
        uint32_t p;
        if constexpr (Geo::RAW3) {
            const uint32_t f = hi % 16;  // prefix hi is prefix f of thread hi / 16
            const uint32_t word = my_ptrs[(size_t)t * PW + (f >> 3) * VT_NT + hi / 16];
            const uint32_t bits = (word >> (3 * (f & 7))) & 7u;  // (v1 < v0, v3 < v2, min23 < min01)
            p = (bits & 1u) ? 2u + ((bits >> 1) & 1u) : (bits >> 2);
        } else if constexpr (Geo::SLOT) {
            constexpr uint32_t F = Geo::SJ * NC;  // prefix hi is field hi % F of thread hi / F
            const uint32_t word = my_ptrs[(size_t)t * PW + hi / F];
            p = (word >> ((hi % F) * KV)) & (uint32_t)(NC - 1);
        } else if constexpr (Geo::LOCAL) {
            const uint32_t h = hi / VT_NT;
            const uint32_t word = my_ptrs[(size_t)t * PW + (h / Geo::FPW) * VT_NT + (hi & (VT_NT - 1))];
            p = (word >> ((h % Geo::FPW) * KV)) & (uint32_t)(NC - 1);
        } else {
            p = my_ptrs[(size_t)t * PW + hi];
        }
        arg = (p << OV) | hi;
    }
    if (pass == 1) {
        overlap[slot] = arg & (uint32_t)(NP - 1);
    } else {
        uint32_t *out = codes + (size_t)(tile0 + slot) * NWORDS;
#pragma unroll
        for (int w = 0; w < NWORDS; w++) out[w] = words[w];
        if (tile_err) tile_err[tile0 + slot] = final_value[slot];
    }
}

// Workspace for `tiles` sequences in flight: three words per sequence (final state,
// overlap, final value), then the back-pointers.
template <int KV, int V, int LB>
constexpr size_t per_tile_bytes() {
    return (size_t)(VT_T / V) * VitGeo<KV, LB>::PW * sizeof(uint32_t);
}
constexpr size_t VT_HEAD_ALIGN = 256;

size_t head_bytes(long tiles) {
    const size_t b = (size_t)tiles * 3 * sizeof(uint32_t);
    return (b + VT_HEAD_ALIGN - 1) / VT_HEAD_ALIGN * VT_HEAD_ALIGN;
}

template <int KV, int V, int CODE>
hipError_t quantize_gpu_t(const float *W, int m, int n, int ld, const uint32_t *lut, uint32_t *codes,
                          float *tile_err, void *ws, size_t ws_bytes, hipStream_t st) {
    constexpr int LB = code_state_bits(CODE), VT_NT = VitGeo<KV, LB>::NT;
    constexpr int TY = 1 << code_log2_ty(CODE), TX = VT_T / TY;
    const int tn = n / TY;
    const long ntiles = (long)(m / TX) * tn;
    // the largest batch the workspace holds
    long cap = (long)(ws_bytes / per_tile_bytes<KV, V, LB>());  // upper bound, trimmed below
    if (cap > ntiles) cap = ntiles;
    while (cap > 0 && head_bytes(cap) + (size_t)cap * per_tile_bytes<KV, V, LB>() > ws_bytes) cap--;
    if (cap <= 0) return hipErrorInvalidValue;
    uint32_t *final_state = (uint32_t *)ws;
    uint32_t *overlap = final_state + cap;
    float *final_value = (float *)(overlap + cap);
    uint32_t *ptrs = (uint32_t *)((char *)ws + head_bytes(cap));
    for (long tile0 = 0; tile0 < ntiles; tile0 += cap) {
        const int cnt = (int)(ntiles - tile0 < cap ? ntiles - tile0 : cap);
        const dim3 bgrid((cnt + 63) / 64);
        hipLaunchKernelGGL((viterbi_forward_kernel<KV, V, CODE>), dim3(cnt), dim3(VT_NT), 0, st, W, ld, tn,
                           tile0, lut, 1, (const uint32_t *)nullptr, ptrs, final_state, final_value);
        hipLaunchKernelGGL((viterbi_backtrace_kernel<KV, V, LB>), bgrid, dim3(64), 0, st, ptrs, final_state,
                           final_value, cnt, 1, overlap, codes, tile_err, tile0);
        hipLaunchKernelGGL((viterbi_forward_kernel<KV, V, CODE>), dim3(cnt), dim3(VT_NT), 0, st, W, ld, tn,
                           tile0, lut, 0, (const uint32_t *)overlap, ptrs, final_state, final_value);
        hipLaunchKernelGGL((viterbi_backtrace_kernel<KV, V, LB>), bgrid, dim3(64), 0, st, ptrs, final_state,
                           final_value, cnt, 2, overlap, codes, tile_err, tile0);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

size_t quantize_gpu_workspace(int k, int V, long tiles) {
    const int kV = k * V;
    size_t pw;
    switch (kV) {
        // (sized for L = 16; the lookup-only code, L = 14, needs a quarter of it)
        case 2: pw = VitGeo<2, 16>::PW; break;
        case 3: pw = VitGeo<3, 16>::PW; break;
        case 4: pw = VitGeo<4, 16>::PW; break;
        case 6: pw = VitGeo<6, 16>::PW; break;
        default: pw = VitGeo<8, 16>::PW; break;
    }
    return head_bytes(tiles) + (size_t)tiles * (VT_T / V) * pw * sizeof(uint32_t);
}

hipError_t launch_quantize_gpu(int k, int code_id, const float *W, int m, int n, int ld, const uint32_t *lut,
                               uint32_t *codes, float *tile_err, void *ws, size_t ws_bytes,
                               hipStream_t st) {
    if (code_id == CODE_HYB1) {
        if (k == 2) return quantize_gpu_t<2, 1, CODE_HYB1>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<3, 1, CODE_HYB1>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<4, 1, CODE_HYB1>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    } else if (code_id == CODE_LUT) {
        if (k == 2) return quantize_gpu_t<2, 1, CODE_LUT>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<3, 1, CODE_LUT>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<4, 1, CODE_LUT>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    } else if (code_id == CODE_HYB2) {
        if (k == 2) return quantize_gpu_t<4, 2, CODE_HYB2>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<6, 2, CODE_HYB2>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<8, 2, CODE_HYB2>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    } else if (code_id == CODE_HYB) {
        if (k == 2) return quantize_gpu_t<4, 2, CODE_HYB>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<6, 2, CODE_HYB>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<8, 2, CODE_HYB>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    } else if (code_id == CODE_3INST) {
        if (k == 2) return quantize_gpu_t<2, 1, CODE_3INST>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<3, 1, CODE_3INST>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<4, 1, CODE_3INST>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    } else {
        if (k == 2) return quantize_gpu_t<2, 1, CODE_1MAD>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        if (k == 3) return quantize_gpu_t<3, 1, CODE_1MAD>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
        return quantize_gpu_t<4, 1, CODE_1MAD>(W, m, n, ld, lut, codes, tile_err, ws, ws_bytes, st);
    }
}

}  // namespace qtip
