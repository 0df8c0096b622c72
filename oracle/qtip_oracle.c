/*
 * QTIP oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow CPU statement of what the QTIP inference path computes
 * (arXiv 2406.11235), written from the paper so that the GPU library can be
 * checked against something that shares no code with it.  Only the tests,
 * the smoke check and the benchmark's "cpu_baseline" leg may call this file;
 * the product library never does.
 *
 * What is here, and the passage each part follows:
 *   - fp16 <-> fp64 conversion in software (IEEE 754 binary16, RNE);
 *   - the packed bitstream and the L-bit state window of the bitshift
 *     trellis (Section 3.1; Figure 1; tail-biting wrap, Section 3.2);
 *   - the state -> value codes 1MAD (Algorithm 1), 3INST (Algorithm 2) and
 *     HYB (Algorithm 3), its two-sign-flip form and its V = 1 form, plus a plain table code
 *     C[2^L][V] (Section 2.3) and the lookup-only code of the appendix on
 *     lookup-only codes (a stored fp16 table of 2^L entries, V = 1);
 *   - decode of a tile and of a whole matrix (Section 4: a T_x x T_y
 *     block is one sequence; Algorithm 5's reshape gives the order), for
 *     16 x 16 tiles and, in the _tiled functions, any T_x T_y = 256;
 *   - dense fp64 matrix-vector / matrix-matrix product with the decoded
 *     weights;
 *   - the random Hadamard transform with an explicit Sylvester matrix
 *     (Section 2.1);
 *   - the Viterbi algorithm on the bitshift trellis (Section 2.3), the
 *     tail-biting approximation (Algorithm 4) and exhaustive searches for
 *     tiny problems; the same two in binary32, operation by operation, for
 *     checking a single-precision quantizer decision by decision;
 *   - the quantizer's outer loop, BlockLDLQ with the trellis quantizer as its
 *     rounder (Algorithm 5): block LDL decomposition and the feedback step.
 *
 * Storage convention (the paper fixes only the logical bit order, through
 * Figure 1: the first stored bit is the most significant bit of the first
 * state).  A sequence of T weights is nbits = k*T bits.  Logical bit i lives
 * in 32-bit word i/32 at bit position 31-(i%32).  A matrix is a row-major
 * array of 16x16 tiles, tile (I,J) at index I*(n/16)+J, each tile k*T/32
 * words.  Sequence element s of a tile is matrix element (16I + s/16,
 * 16J + s%16); with T_x x T_y tiles, (T_x I + s/T_y, T_y J + s%T_y).
 *
 * Parity pins live in tests/test_oracle_pins.py.  Unpinned by the paper and
 * fixed by this build's reading: which HYB entry the sign bit flips (the
 * text's "second entry"), the physical word packing, and the per-row scale.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_CODE_1MAD 0
#define ORC_CODE_3INST 1
#define ORC_CODE_HYB 2
#define ORC_CODE_HYB2 3
#define ORC_CODE_LUT 4 /* lookup-only: the value of a state is table entry [state] */
#define ORC_CODE_HYB1 5 /* Algorithm 3 with V = 1 (the Q = 6 one-dimensional table of Section 4.3's remark) */

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ fp16 */

/* IEEE binary16 bit pattern -> its exact real value. */
double orc_f16_to_f64(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 31;
    int f = h & 1023;
    double v;
    if (e == 31)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -24); /* subnormal: f * 2^-24 */
    else
        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* Real value -> nearest binary16, ties to even. */
uint16_t orc_f64_to_f16(double v) {
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return 0x7E00u;
    if (a >= 65520.0) return sign | 0x7C00u; /* at or above max + half ulp */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: spacing 2^-24; nearbyint rounds to even */
        double q = nearbyint(ldexp(a, 24));
        return sign | (uint16_t)q; /* q == 1024 is the smallest normal */
    }
    int e2;
    (void)frexp(a, &e2); /* a = fr * 2^e2, fr in [0.5, 1) */
    int E = e2 - 1;      /* a in [2^E, 2^(E+1)) */
    double r = nearbyint(ldexp(a, 10 - E)); /* in [1024, 2048] */
    if (r == 2048.0) {
        r = 1024.0;
        E += 1;
    }
    if (E > 15) return sign | 0x7C00u;
    return sign | (uint16_t)((E + 15) << 10) | (uint16_t)((int)r - 1024);
}

/* ------------------------------------------------- stream and state window */

/* Logical bit i of a sequence's packed words (MSB-first inside a word). */
int orc_stream_bit(const uint32_t *words, int i) {
    return (int)((words[i >> 5] >> (31 - (i & 31))) & 1u);
}

void orc_stream_set_bit(uint32_t *words, int i, int bit) {
    uint32_t mask = 1u << (31 - (i & 31));
    if (bit)
        words[i >> 5] |= mask;
    else
        words[i >> 5] &= ~mask;
}

/*
 * State of group t (0-based): the L bits at cyclic positions t*kV ... t*kV+L-1
 * of the nbits-bit sequence, first bit most significant (Section 3.1, with
 * the paper's 1-based positions shifted to 0-based; positions past the end
 * wrap to the start because the sequence is tail-biting, Section 3.2).
 * Read one bit at a time.
 */
uint32_t orc_state(const uint32_t *words, int nbits, int L, int kV, int t) {
    uint32_t s = 0;
    for (int i = 0; i < L; i++) {
        int p = (t * kV + i) % nbits;
        s = s * 2u + (uint32_t)orc_stream_bit(words, p);
    }
    return s;
}

/* --------------------------------------------------------------- the codes */

/* Algorithm 1 ("1MAD"), a = 34038481, b = 76625530; output rounded to fp16. */
uint16_t orc_code_1mad(uint32_t x) {
    uint32_t X = 34038481u * x + 76625530u; /* uint32 arithmetic is mod 2^32 */
    int s = (int)(X & 255u) + (int)((X >> 8) & 255u) + (int)((X >> 16) & 255u) +
            (int)((X >> 24) & 255u);
    double w = ((double)s - 510.0) / 147.8;
    return orc_f64_to_f16(w);
}

/*
 * Algorithm 1 as printed: the value it returns is the quotient (s - 510) / 147.8 itself; the
 * paper names no storage type for it.  orc_code_1mad above is this value rounded to fp16.
 */
double orc_code_1mad_real(uint32_t x) {
    uint32_t X = 34038481u * x + 76625530u;
    int s = (int)(X & 255u) + (int)((X >> 8) & 255u) + (int)((X >> 16) & 255u) +
            (int)((X >> 24) & 255u);
    return ((double)s - 510.0) / 147.8;
}

/* Algorithm 2 ("3INST"), a = 89226354, b = 64248484, m = fp16(0.922). */
uint16_t orc_code_3inst(uint32_t x) {
    uint32_t X = 89226354u * x + 64248484u;
    uint32_t m16 = orc_f64_to_f16(0.922);
    uint32_t mm = (m16 << 16) + m16;
    /* keep sign, low two exponent bits and the mantissa of each half */
    uint32_t mask = 0x8FFF8FFFu; /* b1000111111111111 twice */
    uint32_t Y = (X & mask) ^ mm;
    double m1 = orc_f16_to_f64((uint16_t)(Y & 0xFFFFu));
    double m2 = orc_f16_to_f64((uint16_t)((Y >> 16) & 0xFFFFu));
    /* the sum of two binary16 numbers is exact in binary64, so one rounding */
    return orc_f64_to_f16(m1 + m2);
}

/*
 * Algorithm 3 ("HYB"): hash x*x + x, Q index bits taken from bit 15-Q upward,
 * bit 15 of the hash flips the sign of the second looked-up entry.
 * lut holds 2^Q pairs of fp16 bit patterns, entry v of row idx at lut[2*idx+v].
 */
void orc_code_hyb(uint32_t x, int Q, const uint16_t *lut, uint16_t out[2]) {
    uint32_t X = x * x + x;
    uint32_t idx = (X >> (15 - Q)) & ((1u << Q) - 1u);
    out[0] = lut[2 * idx + 0];
    out[1] = lut[2 * idx + 1];
    if ((X >> 15) & 1u) out[1] ^= 0x8000u;
}

/*
 * The two-sign-flip form of Algorithm 3 (Section 3.1.2 notes it as a free
 * extension that the paper's numbers do not use): bit 31 of the hash is XORed
 * alongside bit 15, so each of the two looked-up entries gets a sign of its
 * own and a state selects one of 2^(Q+2) vectors.  Reading: bit 15 keeps the
 * second entry, as in orc_code_hyb; bit 31 takes the first.
 */
void orc_code_hyb2(uint32_t x, int Q, const uint16_t *lut, uint16_t out[2]) {
    uint32_t X = x * x + x;
    uint32_t idx = (X >> (15 - Q)) & ((1u << Q) - 1u);
    out[0] = lut[2 * idx + 0];
    out[1] = lut[2 * idx + 1];
    if ((X >> 31) & 1u) out[0] ^= 0x8000u;
    if ((X >> 15) & 1u) out[1] ^= 0x8000u;
}

/*
 * Algorithm 3 with V = 1 (the paper names it with Q = 6 as a fit for hardware
 * with a 64-entry table lookup): the same hash, Q index bits from bit 15-Q
 * upward into a table of 2^Q single fp16 values, and bit 15 of the hash flips
 * the sign of the looked-up value (with one entry per row, "the second entry"
 * of the V = 2 form can only be the entry itself).
 */
uint16_t orc_code_hyb1(uint32_t x, int Q, const uint16_t *lut) {
    uint32_t X = x * x + x;
    uint32_t idx = (X >> (15 - Q)) & ((1u << Q) - 1u);
    uint16_t v = lut[idx];
    if ((X >> 15) & 1u) v ^= 0x8000u;
    return v;
}

/* One state -> V fp16 values for the given code. */
static void orc_code_eval(int code_id, uint32_t state, const uint16_t *lut, int Q,
                          uint16_t *out) {
    if (code_id == ORC_CODE_1MAD)
        out[0] = orc_code_1mad(state);
    else if (code_id == ORC_CODE_3INST)
        out[0] = orc_code_3inst(state);
    else if (code_id == ORC_CODE_HYB2)
        orc_code_hyb2(state, Q, lut, out);
    else if (code_id == ORC_CODE_LUT)
        out[0] = lut[state]; /* Section 2.3's plain table, 2^L fp16 entries (V = 1) */
    else if (code_id == ORC_CODE_HYB1)
        out[0] = orc_code_hyb1(state, Q, lut);
    else
        orc_code_hyb(state, Q, lut, out);
}

/* Full codebook C[2^L][V] as doubles (used by the quantizer functions). */
int orc_codebook(int L, int V, int code_id, const uint16_t *lut, int Q, double *C) {
    if ((code_id == ORC_CODE_HYB || code_id == ORC_CODE_HYB2) ? V != 2 : V != 1) return -1;
    for (uint32_t x = 0; x < (1u << L); x++) {
        uint16_t v[2];
        orc_code_eval(code_id, x, lut, Q, v);
        for (int j = 0; j < V; j++) C[(size_t)x * V + j] = orc_f16_to_f64(v[j]);
    }
    return 0;
}

/* ------------------------------------------------------------------ decode */

/*
 * Decode one sequence of T weights: group t gives weights V*t ... V*t+V-1.
 * out receives T fp16 bit patterns.
 */
void orc_decode_sequence(const uint32_t *words, int T, int L, int k, int V, int code_id,
                         const uint16_t *lut, int Q, uint16_t *out) {
    int nbits = k * T;
    for (int t = 0; t < T / V; t++) {
        uint32_t st = orc_state(words, nbits, L, k * V, t);
        uint16_t v[2];
        orc_code_eval(code_id, st, lut, Q, v);
        for (int j = 0; j < V; j++) out[V * t + j] = v[j];
    }
}

/* Same with an explicit table codebook C[2^L][V] of doubles (Section 2.3). */
void orc_decode_sequence_table(const uint32_t *words, int T, int L, int k, int V,
                               const double *C, double *out, uint32_t *states) {
    int nbits = k * T;
    for (int t = 0; t < T / V; t++) {
        uint32_t st = orc_state(words, nbits, L, k * V, t);
        if (states) states[t] = st;
        for (int j = 0; j < V; j++) out[V * t + j] = C[(size_t)st * V + j];
    }
}

/*
 * Decode a whole m x n matrix stored as Tx x Ty tiles (Tx rows of the output
 * dimension, Ty columns of the input dimension, Tx Ty = 256; Section 4) into
 * dense row-major fp16 bit patterns W[m][n] (no row scale).  Tile (I, J) is
 * sequence I (n/Ty) + J; its element s is matrix element (Tx I + s / Ty,
 * Ty J + s % Ty), the order Algorithm 5's reshape of an m x Ty slab gives.
 */
int orc_dequantize_tiled(const uint32_t *codes, int L, int k, int V, int code_id,
                         const uint16_t *lut, int Q, int m, int n, int Tx, int Ty, uint16_t *W) {
    if (Tx * Ty != 256 || m % Tx || n % Ty) return -1;
    const int T = 256;
    int wpt = k * T / 32; /* words per tile */
    int tn = n / Ty;
#pragma omp parallel for schedule(static)
    for (int I = 0; I < m / Tx; I++) {
        uint16_t seq[256];
        for (int J = 0; J < tn; J++) {
            const uint32_t *tile = codes + ((size_t)I * tn + J) * wpt;
            orc_decode_sequence(tile, T, L, k, V, code_id, lut, Q, seq);
            for (int s = 0; s < T; s++)
                W[(size_t)(Tx * I + s / Ty) * n + (Ty * J + s % Ty)] = seq[s];
        }
    }
    return 0;
}

/*
 * The 1MAD matrix with Algorithm 1's unrounded quotients as weights (16 x 16 tiles, L = 16,
 * V = 1), dense row-major doubles: the reference for products that do not go through fp16
 * weights.  Same stream walk and placement as orc_dequantize_tiled.
 */
int orc_dequantize_1mad_real(const uint32_t *codes, int k, int m, int n, double *W) {
    if (m % 16 || n % 16) return -1;
    const int T = 256, L = 16;
    int wpt = k * T / 32;
    int tn = n / 16;
#pragma omp parallel for schedule(static)
    for (int I = 0; I < m / 16; I++)
        for (int J = 0; J < tn; J++) {
            const uint32_t *tile = codes + ((size_t)I * tn + J) * wpt;
            for (int s = 0; s < T; s++)
                W[(size_t)(16 * I + s / 16) * n + (16 * J + s % 16)] =
                    orc_code_1mad_real(orc_state(tile, k * T, L, k, s));
        }
    return 0;
}

int orc_dequantize(const uint32_t *codes, int L, int k, int V, int code_id,
                   const uint16_t *lut, int Q, int m, int n, uint16_t *W) {
    return orc_dequantize_tiled(codes, L, k, V, code_id, lut, Q, m, n, 16, 16, W);
}

/* Decoded weight (i, j) alone, straight from the stream. */
uint16_t orc_decode_element_tiled(const uint32_t *codes, int L, int k, int V, int code_id,
                                  const uint16_t *lut, int Q, int n, int Tx, int Ty, int i, int j) {
    const int T = 256;
    int wpt = k * T / 32;
    const uint32_t *tile = codes + ((size_t)(i / Tx) * (n / Ty) + (j / Ty)) * wpt;
    int s = Ty * (i % Tx) + (j % Ty);
    uint32_t st = orc_state(tile, k * T, L, k * V, s / V);
    uint16_t v[2];
    orc_code_eval(code_id, st, lut, Q, v);
    return v[s % V];
}

uint16_t orc_decode_element(const uint32_t *codes, int L, int k, int V, int code_id,
                            const uint16_t *lut, int Q, int n, int i, int j) {
    return orc_decode_element_tiled(codes, L, k, V, code_id, lut, Q, n, 16, 16, i, j);
}

/* ------------------------------------------------------------ dense product */

/*
 * Y[b][i] = scale[i] * sum_j W[i][j] * X[b][j], everything in fp64.
 * W, X and scale are fp16 bit patterns; scale may be NULL (no scale).
 */
void orc_matmat_dense(const uint16_t *W, int m, int n, const uint16_t *X, int B,
                      const uint16_t *scale, double *Y) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; i++) {
        for (int b = 0; b < B; b++) {
            double acc = 0.0;
            for (int j = 0; j < n; j++)
                acc += orc_f16_to_f64(W[(size_t)i * n + j]) *
                       orc_f16_to_f64(X[(size_t)b * n + j]);
            if (scale) acc *= orc_f16_to_f64(scale[i]);
            Y[(size_t)b * m + i] = acc;
        }
    }
}

/*
 * The same product for a chosen set of output rows, decoding each needed
 * weight on its own: Y[b][r] for r in rows[0..nrows).  Y is B x nrows.
 */
void orc_decode_matmat_rows_tiled(const uint32_t *codes, int L, int k, int V, int code_id,
                                  const uint16_t *lut, int Q, int m, int n, int Tx, int Ty,
                                  const uint16_t *X, int B, const uint16_t *scale, const int *rows,
                                  int nrows, double *Y) {
    (void)m;
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < nrows; r++) {
        int i = rows[r];
        double *wrow = (double *)malloc(sizeof(double) * (size_t)n);
        for (int j = 0; j < n; j++)
            wrow[j] = orc_f16_to_f64(
                orc_decode_element_tiled(codes, L, k, V, code_id, lut, Q, n, Tx, Ty, i, j));
        for (int b = 0; b < B; b++) {
            double acc = 0.0;
            for (int j = 0; j < n; j++) acc += wrow[j] * orc_f16_to_f64(X[(size_t)b * n + j]);
            if (scale) acc *= orc_f16_to_f64(scale[i]);
            Y[(size_t)b * nrows + r] = acc;
        }
        free(wrow);
    }
}

void orc_decode_matmat_rows(const uint32_t *codes, int L, int k, int V, int code_id,
                            const uint16_t *lut, int Q, int m, int n, const uint16_t *X,
                            int B, const uint16_t *scale, const int *rows, int nrows,
                            double *Y) {
    orc_decode_matmat_rows_tiled(codes, L, k, V, code_id, lut, Q, m, n, 16, 16, X, B, scale, rows,
                                 nrows, Y);
}

/* ---------------------------------------------------------------- Hadamard */

/* Sylvester construction: H_1 = [1], H_2b = [[H_b, H_b], [H_b, -H_b]]. */
void orc_hadamard(int b, int8_t *H) {
    H[0] = 1;
    for (int s = 1; s < b; s *= 2)
        for (int i = 0; i < s; i++)
            for (int j = 0; j < s; j++) {
                int8_t v = H[(size_t)i * b + j];
                H[(size_t)i * b + (j + s)] = v;
                H[(size_t)(i + s) * b + j] = v;
                H[(size_t)(i + s) * b + (j + s)] = (int8_t)-v;
            }
}

/*
 * Random Hadamard transform of `batch` vectors of length n in blocks of b
 * (n a multiple of b, b a power of two), V = H_b / sqrt(b) (Section 2.1):
 *   side 0 (input side):  out = V (S .* x)      per block
 *   side 1 (output side): out = S .* (V^T x)    per block
 * x is fp16 bit patterns, signs are +1/-1, out is fp64.
 */
int orc_rht(const uint16_t *x, const int8_t *signs, int n, int b, int batch, int side,
            double *out) {
    if (b <= 0 || (b & (b - 1)) || n % b) return -1;
    int8_t *H = (int8_t *)malloc((size_t)b * b);
    if (!H) return -2;
    orc_hadamard(b, H);
    double inv = 1.0 / sqrt((double)b);
    for (int r = 0; r < batch; r++)
        for (int blk = 0; blk < n / b; blk++) {
            const uint16_t *xb = x + (size_t)r * n + (size_t)blk * b;
            const int8_t *sb = signs + (size_t)blk * b;
            double *ob = out + (size_t)r * n + (size_t)blk * b;
#pragma omp parallel for schedule(static)
            for (int i = 0; i < b; i++) {
                double acc = 0.0;
                for (int j = 0; j < b; j++) {
                    double xv = orc_f16_to_f64(xb[j]);
                    if (side == 0)
                        acc += H[(size_t)i * b + j] * (sb[j] * xv);
                    else
                        acc += H[(size_t)j * b + i] * xv; /* transpose */
                }
                acc *= inv;
                if (side != 0) acc *= sb[i];
                ob[i] = acc;
            }
        }
    free(H);
    return 0;
}

/* ----------------------------------------------------------------- Viterbi */

/*
 * Viterbi on the (L,k,V) bitshift trellis (Section 2.3 value function and
 * update rule; Section 3.1 edge rule: i -> j iff j = (i*2^kV mod 2^L) + c).
 * S has T values, grouped V at a time; C is the codebook [2^L][V].
 * first_top >= 0 forces the top L-kV bits of the first state; last_low >= 0
 * forces the low L-kV bits of the last state (Algorithm 4's second call).
 * Ties go to the lowest state index.  states_out gets the T/V walk states.
 * Returns the total squared error, or -1 on allocation failure.
 */
double orc_viterbi(const double *S, int T, int L, int k, int V, const double *C,
                   int first_top, int last_low, uint32_t *states_out) {
    int kV = k * V;
    int G = T / V;
    uint32_t NS = 1u << L;
    uint32_t nin = 1u << kV; /* incoming edges per node */
    int ov = L - kV;         /* overlap width */
    uint32_t ovmask = (1u << ov) - 1u;
    double *val = (double *)malloc(sizeof(double) * NS);
    double *nxt = (double *)malloc(sizeof(double) * NS);
    uint32_t *back = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)NS * G);
    if (!val || !nxt || !back) {
        free(val);
        free(nxt);
        free(back);
        return -1.0;
    }
    /* t = 1: any start state (or only those with the forced top bits) */
    for (uint32_t y = 0; y < NS; y++) {
        double d = 0.0;
        for (int j = 0; j < V; j++) {
            double e = C[(size_t)y * V + j] - S[j];
            d += e * e;
        }
        if (first_top >= 0 && (y >> kV) != (uint32_t)first_top) d = INFINITY;
        val[y] = d;
    }
    for (int t = 1; t < G; t++) {
        for (uint32_t y = 0; y < NS; y++) {
            /* predecessors x of y: low L-kV bits of x = top L-kV bits of y */
            double best = INFINITY;
            uint32_t arg = 0;
            for (uint32_t p = 0; p < nin; p++) {
                uint32_t x = (p << ov) | (y >> kV);
                if (val[x] < best) {
                    best = val[x];
                    arg = x;
                }
            }
            double d = 0.0;
            for (int j = 0; j < V; j++) {
                double e = C[(size_t)y * V + j] - S[V * t + j];
                d += e * e;
            }
            nxt[y] = best + d;
            back[(size_t)t * NS + y] = arg;
        }
        double *tmp = val;
        val = nxt;
        nxt = tmp;
    }
    double best = INFINITY;
    uint32_t arg = 0;
    for (uint32_t y = 0; y < NS; y++) {
        if (last_low >= 0 && (y & ovmask) != (uint32_t)last_low) continue;
        if (val[y] < best) {
            best = val[y];
            arg = y;
        }
    }
    for (int t = G - 1; t >= 0; t--) {
        states_out[t] = arg;
        if (t > 0) arg = back[(size_t)t * NS + arg];
    }
    free(val);
    free(nxt);
    free(back);
    return best;
}

/*
 * Walk states -> stream bits: group t contributes the top kV bits of its
 * state, i.e. stream bits t*kV ... (t+1)*kV-1.  For a tail-biting walk this
 * is the whole k*T-bit sequence.
 */
void orc_states_to_stream(const uint32_t *states, int G, int L, int kV, uint32_t *words) {
    int nwords = (G * kV + 31) / 32;
    memset(words, 0, sizeof(uint32_t) * (size_t)nwords);
    for (int t = 0; t < G; t++)
        for (int i = 0; i < kV; i++) {
            int bit = (int)((states[t] >> (L - 1 - i)) & 1u);
            orc_stream_set_bit(words, t * kV + i, bit);
        }
}

/*
 * Algorithm 4: rotate right by T/2, Viterbi, read the L-kV bit overlap at the
 * junction between rotated positions T/2 and T/2+1 (1-based; the original
 * sequence's last and first group), then Viterbi on the original sequence
 * with that overlap forced at both ends.  Writes k*T stream bits; returns the
 * squared error of the tail-biting reconstruction.
 */
double orc_tailbiting_quantize(const double *S, int T, int L, int k, int V, const double *C,
                               uint32_t *words) {
    int kV = k * V;
    int G = T / V;
    int ov = L - kV;
    int half = T / 2; /* floor(T/2); callers use T with V | T/2 */
    double *Sr = (double *)malloc(sizeof(double) * (size_t)T);
    uint32_t *st = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)G);
    if (!Sr || !st) {
        free(Sr);
        free(st);
        return -1.0;
    }
    for (int i = 0; i < T; i++) Sr[(i + half) % T] = S[i];
    orc_viterbi(Sr, T, L, k, V, C, -1, -1, st);
    /* group half/V - 1 (0-based) is the original's last, group half/V its first */
    uint32_t O = st[half / V - 1] & ((1u << ov) - 1u);
    double d = orc_viterbi(S, T, L, k, V, C, (int)O, (int)O, st);
    orc_states_to_stream(st, G, L, kV, words);
    free(Sr);
    free(st);
    return d;
}

/*
 * The same Viterbi recursion carried in binary32, for checking a quantizer
 * that keeps its value function in single precision: the paper does not fix
 * the precision of the search, and a different precision can decide
 * near-ties differently, so both sides take the decisions in this one.
 * The operations, each correctly rounded to binary32, are exactly these (the
 * file is built with contraction off; fmaf is the fused multiply-add):
 *   e_j = C[y][j] - S[V t + j];
 *   V = 1: value(y) = fmaf(e_0, e_0, min over predecessors)   (first step: e_0*e_0)
 *   V = 2: value(y) = (min over predecessors) + fmaf(e_1, e_1, e_0*e_0)
 * (the form a GPU takes: one fused operation per state for V = 1, a per-step
 * table of the 2^(Q+1) possible errors for the V = 2 codes).
 * Minima and ties are as in orc_viterbi.  V <= 2.
 */
float orc_viterbi_f32(const float *S, int T, int L, int k, int V, const float *C,
                      int first_top, int last_low, uint32_t *states_out) {
    int kV = k * V;
    int G = T / V;
    uint32_t NS = 1u << L;
    uint32_t nin = 1u << kV;
    int ov = L - kV;
    uint32_t ovmask = (1u << ov) - 1u;
    float *val = (float *)malloc(sizeof(float) * NS);
    float *nxt = (float *)malloc(sizeof(float) * NS);
    uint32_t *back = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)NS * G);
    if (!val || !nxt || !back || V > 2) {
        free(val);
        free(nxt);
        free(back);
        return -1.0f;
    }
    for (int t = 0; t < G; t++) {
        for (uint32_t y = 0; y < NS; y++) {
            float e0 = C[(size_t)y * V] - S[V * t];
            float d = e0 * e0;
            if (V == 2) {
                float e1 = C[(size_t)y * V + 1] - S[V * t + 1];
                d = fmaf(e1, e1, d);
            }
            if (t == 0) {
                if (first_top >= 0 && (y >> kV) != (uint32_t)first_top) d = INFINITY;
                nxt[y] = d;
                continue;
            }
            float best = INFINITY;
            uint32_t arg = 0;
            for (uint32_t p = 0; p < nin; p++) {
                uint32_t x = (p << ov) | (y >> kV);
                if (val[x] < best) {
                    best = val[x];
                    arg = x;
                }
            }
            nxt[y] = V == 1 ? fmaf(e0, e0, best) : best + d;
            back[(size_t)t * NS + y] = arg;
        }
        float *tmp = val;
        val = nxt;
        nxt = tmp;
    }
    float best = INFINITY;
    uint32_t arg = 0;
    for (uint32_t y = 0; y < NS; y++) {
        if (last_low >= 0 && (y & ovmask) != (uint32_t)last_low) continue;
        if (val[y] < best) {
            best = val[y];
            arg = y;
        }
    }
    for (int t = G - 1; t >= 0; t--) {
        states_out[t] = arg;
        if (t > 0) arg = back[(size_t)t * NS + arg];
    }
    free(val);
    free(nxt);
    free(back);
    return best;
}

/* Algorithm 4 with the binary32 recursion above in both of its Viterbi calls. */
float orc_tailbiting_quantize_f32(const float *S, int T, int L, int k, int V, const float *C,
                                  uint32_t *words) {
    int kV = k * V;
    int G = T / V;
    int ov = L - kV;
    int half = T / 2;
    float *Sr = (float *)malloc(sizeof(float) * (size_t)T);
    uint32_t *st = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)G);
    if (!Sr || !st) {
        free(Sr);
        free(st);
        return -1.0f;
    }
    for (int i = 0; i < T; i++) Sr[(i + half) % T] = S[i];
    orc_viterbi_f32(Sr, T, L, k, V, C, -1, -1, st);
    uint32_t O = st[half / V - 1] & ((1u << ov) - 1u);
    float d = orc_viterbi_f32(S, T, L, k, V, C, (int)O, (int)O, st);
    orc_states_to_stream(st, G, L, kV, words);
    free(Sr);
    free(st);
    return d;
}

/* Squared error of the cyclic decode of `words` against S (table code). */
double orc_stream_distortion(const uint32_t *words, const double *S, int T, int L, int k,
                             int V, const double *C) {
    double d = 0.0;
    for (int t = 0; t < T / V; t++) {
        uint32_t st = orc_state(words, k * T, L, k * V, t);
        for (int j = 0; j < V; j++) {
            double e = C[(size_t)st * V + j] - S[V * t + j];
            d += e * e;
        }
    }
    return d;
}

/*
 * Exhaustive search over every cyclic k*T-bit stream (k*T <= 24): the optimal
 * tail-biting distortion.  best_words may be NULL.
 */
double orc_exhaustive_tailbiting(const double *S, int T, int L, int k, int V,
                                 const double *C, uint32_t *best_words) {
    int nbits = k * T;
    if (nbits > 24) return -1.0;
    double best = INFINITY;
    uint32_t w[1];
    for (uint32_t code = 0; code < (1u << nbits); code++) {
        w[0] = code << (32 - nbits); /* bit 0 of the stream = MSB of the word */
        double d = orc_stream_distortion(w, S, T, L, k, V, C);
        if (d < best) {
            best = d;
            if (best_words) best_words[0] = w[0];
        }
    }
    return best;
}

/*
 * Exhaustive search over every walk (free start state, 2^kV choices per later
 * step): what Viterbi without constraints must find.  Needs
 * L + (T/V-1)*kV <= 24.
 */
double orc_exhaustive_walk(const double *S, int T, int L, int k, int V, const double *C) {
    int kV = k * V;
    int G = T / V;
    int total = L + (G - 1) * kV;
    if (total > 24) return -1.0;
    double best = INFINITY;
    for (uint32_t code = 0; code < (1u << total); code++) {
        /* the walk's open (not tail-biting) stream is `total` bits long */
        double d = 0.0;
        for (int t = 0; t < G; t++) {
            uint32_t st = (code >> (total - L - t * kV)) & ((1u << L) - 1u);
            for (int j = 0; j < V; j++) {
                double e = C[(size_t)st * V + j] - S[V * t + j];
                d += e * e;
            }
        }
        if (d < best) best = d;
    }
    return best;
}

/* --------------------------------------------------- BlockLDLQ (Algorithm 5) */

/*
 * g-block LDL decomposition of a symmetric positive definite H (Algorithm 5,
 * second line, g = T_y): H = L D L^T with L unit block lower triangular
 * (identity g x g blocks on its diagonal) and D block diagonal.  Plain
 * right-looking elimination in binary64: D_j is the current diagonal block,
 * L_ij = S_ij D_j^-1 below it, and the trailing matrix loses L_ij D_j L_kj^T.
 * D_j^-1 by Gauss-Jordan with row pivoting.  H, L: n x n row-major (L full,
 * zeros above the diagonal blocks); D: (n/g) blocks of g x g.  0 or -1.
 */
int orc_block_ldl(const double *H, int n, int g, double *Lout, double *Dout) {
    if (n % g) return -1;
    int nb = n / g;
    double *S = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *inv = (double *)malloc(sizeof(double) * (size_t)g * g);
    double *aug = (double *)malloc(sizeof(double) * (size_t)g * 2 * g);
    if (!S || !inv || !aug) {
        free(S);
        free(inv);
        free(aug);
        return -1;
    }
    memcpy(S, H, sizeof(double) * (size_t)n * n);
    memset(Lout, 0, sizeof(double) * (size_t)n * n);
    for (int i = 0; i < n; i++) Lout[(size_t)i * n + i] = 1.0;
    for (int j = 0; j < nb; j++) {
        int o = j * g;
        for (int r = 0; r < g; r++)
            for (int c = 0; c < g; c++) {
                double v = S[(size_t)(o + r) * n + o + c];
                Dout[((size_t)j * g + r) * g + c] = v;
                aug[r * 2 * g + c] = v;
                aug[r * 2 * g + g + c] = r == c ? 1.0 : 0.0;
            }
        for (int c = 0; c < g; c++) {
            int piv = c;
            for (int r = c + 1; r < g; r++)
                if (fabs(aug[r * 2 * g + c]) > fabs(aug[piv * 2 * g + c])) piv = r;
            if (aug[piv * 2 * g + c] == 0.0) {
                free(S);
                free(inv);
                free(aug);
                return -1;
            }
            if (piv != c)
                for (int q = 0; q < 2 * g; q++) {
                    double t = aug[c * 2 * g + q];
                    aug[c * 2 * g + q] = aug[piv * 2 * g + q];
                    aug[piv * 2 * g + q] = t;
                }
            double d = aug[c * 2 * g + c];
            for (int q = 0; q < 2 * g; q++) aug[c * 2 * g + q] /= d;
            for (int r = 0; r < g; r++) {
                if (r == c) continue;
                double f = aug[r * 2 * g + c];
                for (int q = 0; q < 2 * g; q++) aug[r * 2 * g + q] -= f * aug[c * 2 * g + q];
            }
        }
        for (int r = 0; r < g; r++)
            for (int c = 0; c < g; c++) inv[r * g + c] = aug[r * 2 * g + g + c];
        /* L_ij = S_ij D_j^-1 for the rows below the block */
        for (int i = o + g; i < n; i++)
            for (int c = 0; c < g; c++) {
                double acc = 0.0;
                for (int q = 0; q < g; q++) acc += S[(size_t)i * n + o + q] * inv[q * g + c];
                Lout[(size_t)i * n + o + c] = acc;
            }
        /* trailing update: S_ik -= L_ij D_j L_kj^T = L_ij (S_kj)^T (D_j symmetric) */
#pragma omp parallel for schedule(static)
        for (int i = o + g; i < n; i++)
            for (int kk = o + g; kk < n; kk++) {
                double acc = 0.0;
                for (int q = 0; q < g; q++) acc += Lout[(size_t)i * n + o + q] * S[(size_t)kk * n + o + q];
                S[(size_t)i * n + kk] -= acc;
            }
    }
    free(S);
    free(inv);
    free(aug);
    return 0;
}

/*
 * The feedback step of Algorithm 5 for column block j (g = T_y columns):
 *   x = W[:, jg:(j+1)g] + (W - What)[:, (j+1)g:] A[(j+1)g:, jg:(j+1)g]
 * (A = L - I is zero on and above its diagonal blocks, so the block's own
 * columns drop out of the paper's slice jT_y: ).  Binary32, in one fixed
 * order so that a GPU implementation can be followed decision by decision:
 * start from W[r][jg+c] and add the terms E[r][i] * A[i][jg+c], one fused
 * multiply-add each, taking the column blocks from the last one down to
 * j+1 and the columns i inside a block in ascending order.  (The paper gives
 * no order; this is the order in which a sum that is updated every time a
 * block is finished receives its terms.)
 * E = W - What (m x n), A n x n, x m x g, all row-major float.
 */
void orc_ldlq_feedback_f32(const float *W, const float *E, const float *A, int m, int n, int g,
                           int j, float *x) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < m; r++)
        for (int c = 0; c < g; c++) {
            float acc = W[(size_t)r * n + j * g + c];
            for (int b = n / g - 1; b > j; b--)
                for (int i = b * g; i < (b + 1) * g; i++)
                    acc = fmaf(E[(size_t)r * n + i], A[(size_t)i * n + j * g + c], acc);
            x[(size_t)r * g + c] = acc;
        }
}

