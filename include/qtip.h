/*
 * qtip.h -- C ABI of the MI355X (gfx950) QTIP inference library.
 *
 * QTIP (arXiv 2406.11235) stores a weight matrix W~ (m outputs x n inputs, already
 * conjugated by random Hadamard transforms) as trellis-coded bitstreams: every
 * 16 x 16 block of W~ is one length-256 sequence quantized with an (L, k, V)
 * "bitshift" trellis (Section 3.1), stored tail-biting in exactly 256*k bits
 * (Section 3.2), and mapped from L-bit states to values by a computed code
 * (1MAD, 3INST: Section 3.1.1, Algorithms 1-2) or a hash + small lookup table
 * (HYB: Section 3.1.2, Algorithm 3).  Inference decodes the stream on the fly
 * and multiplies by the Hadamard-transformed activation (Section 2.1).
 *
 * DATA FORMATS (shared by every call)
 *   codes   uint32 words, DEVICE memory unless stated otherwise.  The matrix is a
 *           row-major array of 16x16 tiles; tile (I, J) (I over outputs, J over
 *           inputs) starts at word (I*(n/16) + J) * 8k and holds 8k words =
 *           256*k bits.  Logical stream bit i of a tile is bit 31-(i%32) of word
 *           i/32, so the first stored bit is the most significant bit of the
 *           first state (Figure 1).  Must be 16-byte aligned.
 *   state   group t (t = 0 .. 256/V - 1) of a tile has the L-bit state made of
 *           stream bits t*k*V ... t*k*V+L-1, first bit most significant, positions
 *           taken modulo 256*k (tail-biting wrap).
 *   order   group t decodes to sequence elements V*t ... V*t+V-1; sequence element
 *           s of tile (I, J) is W~[16I + s/16][16J + s%16] (the row-major reshape
 *           of a T_x x T_y block in Algorithm 5).
 *   lut     HYB only: 2^9 x 2 fp16 values, DEVICE memory, entry v of row idx at
 *           half-word 2*idx + v.  Bit 15 of the hash negates entry v = 1 (the
 *           "second entry" of Section 3.1.2).  4-byte aligned.
 *   fp16    IEEE binary16, passed as void*.
 *   QTIP_CODE_HYB1: lut is 64 fp16 values, DEVICE memory, 4-byte aligned; L = 16, V = 1.
 *   QTIP_CODE_LUT (the lookup-only code of the appendix on lookup-only codes) differs in
 *           three places: L = 14; the sequence of 256 weights is a 32 x 8 block
 *           (T_x = 32 outputs, T_y = 8 inputs), so the matrix is a row-major array of
 *           32 x 8 blocks, block (I, J) at word (I*(n/8) + J) * 8k, its element s at
 *           W~[32I + s/8][8J + s%8]; lut is the code itself, 2^14 fp16 values, DEVICE
 *           memory, 16-byte aligned, the value of state x at half-word x.
 *
 * SUPPORTED PARAMETERS
 *   code_id QTIP_CODE_1MAD / QTIP_CODE_3INST with L = 16, V = 1 and k in {2, 3, 4};
 *   QTIP_CODE_HYB and QTIP_CODE_HYB2 (Q = 9) with L = 16, V = 2 and k in {2, 3, 4};
 *   QTIP_CODE_HYB1 (Q = 6) with L = 16, V = 1 and k in {2, 3, 4}; m and n
 *   multiples of 16.  QTIP_CODE_LUT with L = 14, V = 1 and k in {2, 3, 4}; m a multiple of
 *   32, n of 8.  Anything else returns QTIP_EUNSUPPORTED / QTIP_EINVAL.
 *   Sizes: m, n and batch sizes are ints; every offset into codes, weights, activations
 *   and outputs is formed in 64 bits, so buffers may pass 4 GiB (checked on 98304 x 98304
 *   at 4 bits); only the position inside one tile row's code stream is kept in 32 bits,
 *   which limits n to QTIP_MAX_N = 2^28 (above it: QTIP_EINVAL).  The calls that record nothing but kernel launches (all of the GPU entry
 *   points) may be captured into a HIP graph.
 *
 * OWNERSHIP, STREAMS, ERRORS
 *   The caller owns every buffer.  GPU entry points take device pointers, enqueue
 *   their kernels on `stream` (a hipStream_t passed as void*; NULL = the default
 *   stream) and return without synchronizing.  The library allocates no device
 *   memory and keeps no state besides a thread-local error string.  Every call
 *   returns 0 (QTIP_OK) or a negative error code and never throws or aborts;
 *   qtip_last_error() describes the last failure on the calling thread.
 *   Buffers must not overlap unless a call says it allows it.
 */
#ifndef QTIP_H
#define QTIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QTIP_VERSION 100

#define QTIP_OK 0
#define QTIP_EINVAL (-1)       /* null pointer, bad size or alignment           */
#define QTIP_EUNSUPPORTED (-2) /* (L, k, V, code_id) outside the supported set  */
#define QTIP_EHIP (-3)         /* HIP runtime / launch failure                  */
#define QTIP_ENOMEM (-4)       /* host allocation failed (qtip_quantize)        */

#define QTIP_MAX_N (1 << 28) /* largest number of columns any entry point takes */

#define QTIP_CODE_1MAD 0  /* Algorithm 1 */
#define QTIP_CODE_3INST 1 /* Algorithm 2 */
#define QTIP_CODE_HYB 2   /* Algorithm 3, Q = 9, one sign flip */
#define QTIP_CODE_HYB2 3  /* the same with bit 31 of the hash also XORed (Section 3.1.2): the first
                             entry gets a sign of its own; for L = 16 that bit is set exactly when
                             the state is at least 46341 */
#define QTIP_CODE_HYB1 5  /* Algorithm 3 with one entry per row: L = 16, V = 1, Q = 6 (Section 4.3's remark
                             on hardware with a 64-entry table lookup): bits 9..14 of the hash index
                             64 fp16 values, bit 15 negates the value */
#define QTIP_CODE_LUT 4   /* lookup-only code (appendix on lookup-only codes): L = 14, V = 1, the value
                             of a state is entry [state] of a stored table; T_x = 32, T_y = 8 */

/*
 * Random Hadamard transform of activations (Section 2.1: W~ = V_m S_m W S_n V_n^T,
 * so the layer computes y = S_m V_m^T (W~ (V_n S_n x))).  V is the orthogonal
 * block-diagonal Walsh-Hadamard matrix H_block / sqrt(block) in natural
 * (Sylvester) order; n must be a multiple of block, block a power of two in
 * [16, 16384].
 *   side 0 (input side):   out = V (S .* x)    for each of the `batch` rows of x
 *   side 1 (output side):  out = S .* (V^T x)
 * x: device, batch x n row-major, fp16 (qtip_rht) or fp32 (qtip_rht_f32, for
 * feeding the fp32 result of a multiply straight into the output-side transform).
 * signs: device, n int8 values, each +1 or -1.  out_f16: device, batch x n fp16.
 * out may alias x in qtip_rht.  x, signs and out must be 16-byte aligned.
 * Arithmetic is fp32, rounded once to fp16.
 */
int qtip_rht(const void *x_f16, const int8_t *signs, int n, int block, int batch, int side,
             void *out_f16, void *stream);
int qtip_rht_f32(const float *x_f32, const int8_t *signs, int n, int block, int batch,
                 int side, void *out_f16, void *stream);

/*
 * Fused decode + matrix-vector product, batch 1 (Sections 3.1, 3.1.1-3.1.2 and 4:
 * decode each tile's bitstream to fp16 weights and contract with the activation):
 *   y[i] = sum_j W~[i][j] * x[j],   i < m, j < n.
 * x_f16: device, n fp16 (normally the output of qtip_rht side 0).  y: device, m
 * fp32, overwritten.  The weights are exactly the fp16 values of qtip_dequantize and
 * every product is accumulated in fp32, with one exception: QTIP_CODE_1MAD at batch 1
 * contracts with the quotient (s - 510) / 147.8 that Algorithm 1 returns, not with its
 * fp16 rounding (the sum over j of (s_j - 510) x_j is formed first and divided once), so y
 * differs from the product with the fp16 values by the rounding of the weights: at most
 * 2^-12 relative per weight, about 2e-4 of the largest output on whole layers, against the
 * fp64 product with the unrounded quotients about 1e-6.  lut_f16 is NULL unless the code
 * has a table (QTIP_CODE_HYB, QTIP_CODE_HYB2, QTIP_CODE_HYB1, QTIP_CODE_LUT).
 */
int qtip_decode_matvec(const uint32_t *codes, int L, int k, int V, int code_id,
                       const void *lut_f16, int m, int n, const void *x_f16, float *y,
                       void *stream);

/*
 * Batched form: Y[b][i] = row_scale[i] * sum_j W~[i][j] * X[b][j], b < B.
 * X_f16: device, B x n row-major fp16.  Y: device, B x m row-major fp32,
 * overwritten.  row_scale_f16: device, m fp16, or NULL for no scale.  B >= 1.
 * B = 1 runs the batch-1 kernel on the vector ALUs (for QTIP_CODE_1MAD with the unrounded
 * quotient, as qtip_decode_matvec); every B >= 2 runs on the matrix cores
 * (MFMA) with the decoded 16x16 tile as one operand (Section 4: T_x = T_y = 16 matches a
 * 16x16 matrix-multiply tile; with QTIP_CODE_LUT two neighbouring 32 x 8 blocks are the
 * 32 x 16 operand of the 32x32x16 instruction).  Y must be 16-byte aligned (and m a multiple
 * of 16, as everywhere): outputs are stored four at a time.
 */
int qtip_decode_matmat(const uint32_t *codes, int L, int k, int V, int code_id,
                       const void *lut_f16, int m, int n, const void *X_f16, int B,
                       const void *row_scale_f16, float *Y, void *stream);

/*
 * The input side of a whole layer in one call: y = row_scale .* (W~ (V (S_n .* x))),
 * i.e. qtip_rht(side 0, batch 1) followed by the batch-1 product, with the same
 * arithmetic and therefore the same y bit for bit.  For n <= 8192 and m <= 4096 it is ONE
 * kernel launch: every workgroup transforms x itself, in LDS, before it starts on its tile
 * row (about 2 us of redundant work per workgroup against a kernel launch plus the gap
 * before a dependent kernel, which is what bounds layers of this size: 4096 x 4096 goes
 * from 14.9 to 8.9 us per call).  Larger layers have several workgroups per CU and would
 * redo the transform too often: there the call enqueues the two kernels and needs
 * xt_scratch (device, n fp16, 16-byte aligned; may be NULL otherwise) for the transformed
 * vector (QTIP_CODE_LUT always takes this two-kernel form: its workgroups fill their LDS
 * with the table).  Together with qtip_rht_f32(side 1) on y a small layer is two launches.
 *   x_f16: device, n fp16, untransformed.  signs_n: device, n int8 in {+1,-1}.
 *   block: Hadamard block (as qtip_rht).  row_scale_f16: device m fp16 or NULL.
 */
int qtip_rht_decode_matvec(const uint32_t *codes, int L, int k, int V, int code_id,
                           const void *lut_f16, int m, int n, const void *x_f16,
                           const int8_t *signs_n, int block, const void *row_scale_f16, float *y,
                           void *xt_scratch_f16, void *stream);

/*
 * qtip_rht_decode_matvec for callers that cannot bring a scratch buffer and must not cause an
 * allocation: code recorded under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments without xt_scratch, same kernels, same y bit for bit.
 * The transformed activation of the two-kernel form lives in a buffer of the library's own, a
 * static device array of QTIP_NOALLOC_MAX_N fp16 values (128 KiB, held on every GPU the
 * library is used on until the process ends); n above QTIP_NOALLOC_MAX_N is QTIP_EINVAL.
 * The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library
 * routine): the array's device address is looked up once per device, on the first call
 * there (QTIP_EHIP if that fails).  The buffer is written before it is read in every call,
 * so nothing is cleared.  All calls on one GPU share it: two calls that overlap on one GPU
 * (different streams, or graphs replayed concurrently) race and give wrong results; calls
 * ordered on one stream are safe.
 */
#define QTIP_NOALLOC_MAX_N 65536
int qtip_rht_decode_matvec_noalloc(const uint32_t *codes, int L, int k, int V, int code_id,
                                   const void *lut_f16, int m, int n, const void *x_f16,
                                   const int8_t *signs_n, int block, const void *row_scale_f16,
                                   float *y, void *stream);

/*
 * Decode only (for testing): W_f16[i][j] = W~[i][j], device, m x n row-major fp16,
 * no row scale.  Bit-exact with the definitions of Algorithms 1-3.
 */
int qtip_dequantize(const uint32_t *codes, int L, int k, int V, int code_id,
                    const void *lut_f16, int m, int n, void *W_f16, void *stream);

/*
 * Decode the code function alone on a list of states (for testing):
 * out_f16[V*i + v] = code(states[i])[v].  states: device, count uint32 values
 * below 2^L.  out_f16: device, count*V fp16.
 */
int qtip_decode_states(const uint32_t *states, int count, int L, int V, int code_id,
                       const void *lut_f16, void *out_f16, void *stream);

/*
 * CPU quantizer, used to make valid inputs and to validate; never on the timed
 * path.  ALL pointers are HOST memory.  Each 16x16 tile of W (m x n row-major
 * fp32; each 32 x 8 block with QTIP_CODE_LUT) is quantized as one sequence with the
 * Viterbi algorithm on the bitshift trellis (Section 2.3) made tail-biting by
 * Algorithm 4, under squared error.  codes_out receives m*n/256 * 8k words in the
 * format above.  mse_out (may be NULL) receives the mean squared error of the
 * reconstruction.  lut_f16 is a host copy of the code's table (NULL for the computed
 * codes).  Binary64 search.  Starts one worker thread per tile up to
 * std::thread::hardware_concurrency() (all host cores; there is no way to ask for fewer) and
 * joins them before it returns.
 */
int qtip_quantize(const float *W, int m, int n, int L, int k, int V, int code_id,
                  const void *lut_f16, uint32_t *codes_out, double *mse_out);

/*
 * GPU quantizer: the same problem as qtip_quantize -- every 16x16 tile of W
 * quantized as one sequence by the Viterbi algorithm on the bitshift trellis
 * (Section 2.3), made tail-biting by Algorithm 4, under squared error against the
 * code's values (Algorithms 1-3) -- run on the device, one workgroup per tile with
 * the 2^16-entry value function held in registers.  (QTIP_CODE_LUT: every 32 x 8 block,
 * 2^14 states; read 32 x 8 for 16 x 16 below.)
 *   W:          device, m x n row-major fp32.
 *   lut_f16:    device table of the code (NULL for the computed codes).
 *   codes_out:  device, (m/16)*(n/16)*8k words, the format above.
 *   tile_err:   device, (m/16)*(n/16) floats, or NULL: the final value of the
 *               search for each tile = its squared reconstruction error, as
 *               accumulated in binary32.
 *   workspace:  device, 256-byte aligned, workspace_bytes long; holds the
 *               back-pointers of the tiles in flight.  Any size from
 *               qtip_quantize_gpu_workspace(k, V, 1) up works; tiles are processed
 *               in batches of as many as fit, so give it
 *               qtip_quantize_gpu_workspace(k, V, t) for t of a few thousand (about
 *               2 MiB per tile at k = 2, V = 1, 1 MiB at k = 3 or 4, 0.5 MiB or less at
 *               V = 2; sized for L = 16,
 *               QTIP_CODE_LUT uses a quarter of it) to keep the device full.
 *               Contents are scratch.
 * The search runs in binary32 with fixed roundings (e = c - s; V = 1: value =
 * fma(e, e, minimum over predecessors); V = 2: value = minimum + fma(e1, e1, e0*e0)),
 * lowest predecessor and lowest final state on ties; the paper does not fix a
 * precision.  Streams therefore equal a binary32 CPU search bit for bit, and may
 * differ from a binary64 search where two walks tie to within rounding.
 * Enqueues on `stream` and returns without synchronizing.
 */
size_t qtip_quantize_gpu_workspace(int k, int V, long tiles);
int qtip_quantize_gpu(const float *W, int m, int n, int L, int k, int V, int code_id,
                      const void *lut_f16, uint32_t *codes_out, float *tile_err, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * Block LDL decomposition of a proxy Hessian (Algorithm 5, second and third lines, with
 * T_y = g): H = L D L^T, L unit block lower triangular with g x g identity blocks on
 * its diagonal, D block diagonal; the feedback matrix is A = L - I.  g is 16 (the codes of
 * Algorithms 1-3) or 8 (the lookup-only code); n a multiple of 16.
 *   H:       device, n x n row-major binary64, symmetric positive definite (only its
 *            lower triangle is read).  If it is not positive definite the results
 *            hold non-finite values; no error is raised.
 *   A_out:   device, n x n row-major fp32: L - I (zero on and above the diagonal blocks).
 *   D_out:   device, (n/g) x g x g binary64, or NULL: the diagonal blocks of D.
 *   workspace: device, 256-byte aligned, qtip_block_ldl_workspace(n) bytes (two n x n
 *            binary64 matrices); contents are scratch.
 * Binary64 throughout; 2 n/g + 2 kernel launches on `stream`, no synchronization.
 */
size_t qtip_block_ldl_workspace(int n);
int qtip_block_ldl(const double *H, int n, int g, float *A_out, double *D_out, void *workspace,
                   size_t workspace_bytes, void *stream);

/*
 * The quantizer inside BlockLDLQ (Algorithm 5; written here for T_x = T_y = 16; with the
 * lookup-only code read 32 x 8 blocks, column blocks of 8 and A from qtip_block_ldl with
 * g = 8): for column blocks j from the last to the first,
 *     x = W[:, 16j:16j+16] + (W - What)[:, 16j+16:] A[16j+16:, 16j:16j+16],
 * every 16x16 block of x quantized as one sequence by the tail-biting Viterbi quantizer
 * (as qtip_quantize_gpu, same arithmetic), What[:, 16j:16j+16] = its decode.
 *   W: device m x n fp32.  A: device n x n fp32 from qtip_block_ldl (only the blocks
 *   below the diagonal blocks are read).  codes_out: as qtip_quantize_gpu.
 *   What_out: device m x n fp32 or NULL: the decoded weights.  tile_err: device,
 *   (m/16)*(n/16) floats or NULL: squared error of every tile against its x.
 *   workspace: 256-byte aligned; qtip_quantize_ldlq_workspace(m, n, k, V, t) bytes keep
 *   t tiles of a column block in flight (a block has m/16 tiles; t = m/16 is the most
 *   that helps; any t >= 1 works; the size is computed for 16 x 16 blocks and covers 32 x 8).
 * The feedback sum is binary32, one fused multiply-add per term, column blocks from the last
 * one down and ascending inside a block, so that the input of the quantizer is reproducible.
 * The workspace holds a running m x n fp32 sum besides the quantizer's own: on return its
 * first m*n floats are x of Algorithm 5, row-major, every column block as it was rounded.
 */
size_t qtip_quantize_ldlq_workspace(int m, int n, int k, int V, long tiles);
int qtip_quantize_ldlq(const float *W, const float *A, int m, int n, int L, int k, int V, int code_id,
                       const void *lut_f16, uint32_t *codes_out, float *What_out, float *tile_err,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Message for the last error on this thread ("" if none). Never NULL. */
const char *qtip_last_error(void);

/* QTIP_VERSION of the built library. */
int qtip_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QTIP_H */
