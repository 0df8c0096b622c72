// extern "C" entry points of include/qtip.h: argument validation, error strings,
// and dispatch to the kernel launchers.  Nothing here touches the data.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "../../include/qtip.h"
#include "qtip_internal.h"

namespace {

bool is_hyb(int code_id) { return code_id == QTIP_CODE_HYB || code_id == QTIP_CODE_HYB2; }
bool is_lut(int code_id) { return code_id == QTIP_CODE_LUT; }
bool has_table(int code_id) { return is_hyb(code_id) || is_lut(code_id) || code_id == QTIP_CODE_HYB1; }

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(const char *what, hipError_t e) {
    return fail(QTIP_EHIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Scratch of qtip_rht_decode_matvec_noalloc: the transformed activation between its two
// kernels.  One copy per GPU, at an address of its own on each; the name below is only a
// host-side handle, the device address comes from hipGetSymbolAddress (noalloc_scratch()).
static __device__ __align__(256) unsigned char scratch[QTIP_NOALLOC_MAX_N * 2];
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device (looked up once per device), or nullptr
// with the error string set.
void *noalloc_scratch(const char *fn) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        hip_fail(fn, e);
        return nullptr;
    }
    if (dev < 0 || dev >= MAX_DEVICES) {
        fail(QTIP_EHIP, "%s: device index %d is outside the %d this library keeps scratch for", fn, dev, MAX_DEVICES);
        return nullptr;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            hip_fail(fn, e);
            return nullptr;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing threads store the same address
    }
    return p;
}

// The (L, k, V, code) combinations that are built, the table the HYB codes need, and the
// matrix shape: shared by every call that reads or writes a code stream.
int check_code(const char *fn, int L, int k, int V, int code_id, const void *lut, int m, int n) {
    if (code_id != QTIP_CODE_1MAD && code_id != QTIP_CODE_3INST && code_id != QTIP_CODE_HYB &&
        code_id != QTIP_CODE_HYB2 && code_id != QTIP_CODE_LUT && code_id != QTIP_CODE_HYB1)
        return fail(QTIP_EUNSUPPORTED, "%s: unknown code_id %d", fn, code_id);
    const int wantL = is_lut(code_id) ? 14 : 16;
    if (L != wantL)
        return fail(QTIP_EUNSUPPORTED, "%s: L = %d (code %d is built for L = %d)", fn, L, code_id, wantL);
    if (k < 2 || k > 4) return fail(QTIP_EUNSUPPORTED, "%s: k = %d (supported: 2, 3, 4)", fn, k);
    const int wantV = is_hyb(code_id) ? 2 : 1;
    if (V != wantV)
        return fail(QTIP_EUNSUPPORTED, "%s: V = %d (code %d needs V = %d)", fn, V, code_id, wantV);
    if (has_table(code_id) && !lut) return fail(QTIP_EINVAL, "%s: code %d needs a lut", fn, code_id);
    if (lut && !aligned(lut, is_lut(code_id) ? 16 : 4))
        return fail(QTIP_EINVAL, "%s: lut must be %d-byte aligned", fn, is_lut(code_id) ? 16 : 4);
    // a sequence is a T_x x T_y block of the matrix: 32 x 8 for the lookup-only code, else 16 x 16
    const int tx = is_lut(code_id) ? 32 : 16, ty = is_lut(code_id) ? 8 : 16;
    if (m <= 0 || n <= 0 || m % tx || n % ty)
        return fail(QTIP_EINVAL, "%s: m = %d must be a positive multiple of %d, n = %d of %d", fn, m, tx, n, ty);
    // the kernels address the code stream of one tile row with 32-bit byte offsets (n k / 2 bytes)
    if (n > QTIP_MAX_N) return fail(QTIP_EINVAL, "%s: n = %d is above QTIP_MAX_N = %d", fn, n, QTIP_MAX_N);
    return QTIP_OK;
}

// The same for calls that read a code stream.
int check_codec(const char *fn, const void *codes, int L, int k, int V, int code_id,
                const void *lut, int m, int n) {
    if (!codes) return fail(QTIP_EINVAL, "%s: codes is NULL", fn);
    if (int rc = check_code(fn, L, k, V, code_id, lut, m, n)) return rc;
    if (!aligned(codes, 16)) return fail(QTIP_EINVAL, "%s: codes must be 16-byte aligned", fn);
    return QTIP_OK;
}

int rht_common(const char *fn, const void *x, bool f32, const int8_t *signs, int n, int block,
               int batch, int side, void *out, void *stream) {
    if (!x || !signs || !out) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (block < 16 || block > 16384 || (block & (block - 1)))
        return fail(QTIP_EINVAL, "%s: block = %d must be a power of two in [16, 16384]", fn, block);
    if (n <= 0 || n % block) return fail(QTIP_EINVAL, "%s: n = %d is not a multiple of block %d", fn, n, block);
    if (batch < 1 || batch > 65535) return fail(QTIP_EINVAL, "%s: batch = %d out of range", fn, batch);
    if (side != 0 && side != 1) return fail(QTIP_EINVAL, "%s: side = %d must be 0 or 1", fn, side);
    if (!aligned(x, 16) || !aligned(signs, 16) || !aligned(out, 16))
        return fail(QTIP_EINVAL, "%s: x, signs and out must be 16-byte aligned", fn);
    hipError_t e = qtip::launch_rht(x, f32, signs, n, block, batch, side, out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

}  // namespace

extern "C" {

int qtip_version(void) { return QTIP_VERSION; }

const char *qtip_last_error(void) { return g_err; }

int qtip_rht(const void *x_f16, const int8_t *signs, int n, int block, int batch, int side,
             void *out_f16, void *stream) {
    return rht_common("qtip_rht", x_f16, false, signs, n, block, batch, side, out_f16, stream);
}

int qtip_rht_f32(const float *x_f32, const int8_t *signs, int n, int block, int batch, int side,
                 void *out_f16, void *stream) {
    if ((const void *)x_f32 == (const void *)out_f16 && x_f32)
        return fail(QTIP_EINVAL, "qtip_rht_f32: out must not alias x");
    return rht_common("qtip_rht_f32", x_f32, true, signs, n, block, batch, side, out_f16, stream);
}

int qtip_decode_matvec(const uint32_t *codes, int L, int k, int V, int code_id, const void *lut_f16,
                       int m, int n, const void *x_f16, float *y, void *stream) {
    const char *fn = "qtip_decode_matvec";
    if (int rc = check_codec(fn, codes, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (!x_f16 || !y) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (!aligned(x_f16, 16)) return fail(QTIP_EINVAL, "%s: x must be 16-byte aligned", fn);
    hipError_t e = qtip::launch_matvec(k, code_id, codes, (const uint32_t *)lut_f16, m, n, x_f16,
                                       nullptr, y, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

int qtip_rht_decode_matvec(const uint32_t *codes, int L, int k, int V, int code_id, const void *lut_f16,
                           int m, int n, const void *x_f16, const int8_t *signs_n, int block,
                           const void *row_scale_f16, float *y, void *xt_scratch_f16, void *stream) {
    const char *fn = "qtip_rht_decode_matvec";
    if (int rc = check_codec(fn, codes, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (!x_f16 || !signs_n || !y) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (block < 16 || block > 16384 || (block & (block - 1)))
        return fail(QTIP_EINVAL, "%s: block = %d must be a power of two in [16, 16384]", fn, block);
    if (n % block) return fail(QTIP_EINVAL, "%s: n = %d is not a multiple of block %d", fn, n, block);
    if (!aligned(x_f16, 16) || !aligned(signs_n, 16))
        return fail(QTIP_EINVAL, "%s: x and signs must be 16-byte aligned", fn);
    hipError_t e;
    // one launch pays while there is at most one workgroup (tile row) per CU; with more, every
    // CU would redo the transform several times over
    if (!is_lut(code_id) && n <= qtip::fused_rht_matvec_max_n() && m <= 16 * 256) {
        e = qtip::launch_rht_matvec(k, code_id, codes, (const uint32_t *)lut_f16, m, n, x_f16, signs_n, block,
                                    row_scale_f16, y, (hipStream_t)stream);
    } else {
        if (!xt_scratch_f16 || !aligned(xt_scratch_f16, 16))
            return fail(QTIP_EINVAL,
                        "%s: n = %d above %d, m = %d above 4096 or the lookup-only code: xt_scratch (n fp16, "
                        "16-byte aligned) is needed", fn, n, qtip::fused_rht_matvec_max_n(), m);
        e = qtip::launch_rht(x_f16, false, signs_n, n, block, 1, 0, xt_scratch_f16, (hipStream_t)stream);
        if (e == hipSuccess)
            e = qtip::launch_matvec(k, code_id, codes, (const uint32_t *)lut_f16, m, n, xt_scratch_f16,
                                    row_scale_f16, y, (hipStream_t)stream);
    }
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

int qtip_rht_decode_matvec_noalloc(const uint32_t *codes, int L, int k, int V, int code_id,
                                   const void *lut_f16, int m, int n, const void *x_f16,
                                   const int8_t *signs_n, int block, const void *row_scale_f16, float *y,
                                   void *stream) {
    const char *fn = "qtip_rht_decode_matvec_noalloc";
    if (n > QTIP_NOALLOC_MAX_N)
        return fail(QTIP_EINVAL, "%s: n = %d is above QTIP_NOALLOC_MAX_N = %d, the size of the library's own "
                    "scratch; use qtip_rht_decode_matvec with a buffer of the caller's", fn, n, QTIP_NOALLOC_MAX_N);
    void *xt = noalloc_scratch(fn);
    if (!xt) return QTIP_EHIP;
    const int rc = qtip_rht_decode_matvec(codes, L, k, V, code_id, lut_f16, m, n, x_f16, signs_n, block,
                                          row_scale_f16, y, xt, stream);
    if (rc != QTIP_OK) {  // same checks, this entry point's name in the message
        char msg[sizeof(g_err)];
        snprintf(msg, sizeof(msg), "%s", g_err);
        const char *colon = strchr(msg, ':');
        fail(rc, "%s%s", fn, colon ? colon : msg);
    }
    return rc;
}

int qtip_decode_matmat(const uint32_t *codes, int L, int k, int V, int code_id, const void *lut_f16,
                       int m, int n, const void *X_f16, int B, const void *row_scale_f16, float *Y,
                       void *stream) {
    const char *fn = "qtip_decode_matmat";
    if (int rc = check_codec(fn, codes, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (!X_f16 || !Y) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (B < 1 || B > 65535 * 64) return fail(QTIP_EINVAL, "%s: B = %d out of range", fn, B);
    if (!aligned(X_f16, 16) || !aligned(Y, 16))
        return fail(QTIP_EINVAL, "%s: X and Y must be 16-byte aligned", fn);
    hipError_t e;
    if (B == 1)
        e = qtip::launch_matvec(k, code_id, codes, (const uint32_t *)lut_f16, m, n, X_f16,
                                row_scale_f16, Y, (hipStream_t)stream);
    else
        e = qtip::launch_matmat(k, code_id, codes, (const uint32_t *)lut_f16, m, n, X_f16, B,
                                row_scale_f16, Y, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

int qtip_dequantize(const uint32_t *codes, int L, int k, int V, int code_id, const void *lut_f16,
                    int m, int n, void *W_f16, void *stream) {
    const char *fn = "qtip_dequantize";
    if (int rc = check_codec(fn, codes, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (!W_f16) return fail(QTIP_EINVAL, "%s: W is NULL", fn);
    if (!aligned(W_f16, 16)) return fail(QTIP_EINVAL, "%s: W must be 16-byte aligned", fn);
    hipError_t e = qtip::launch_dequantize(k, code_id, codes, (const uint32_t *)lut_f16, m, n, W_f16,
                                           (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

int qtip_decode_states(const uint32_t *states, int count, int L, int V, int code_id,
                       const void *lut_f16, void *out_f16, void *stream) {
    const char *fn = "qtip_decode_states";
    if (!states || !out_f16) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (count < 0) return fail(QTIP_EINVAL, "%s: count = %d", fn, count);
    if (int rc = check_code(fn, L, /*k=*/2, V, code_id, lut_f16, 32, 16)) return rc;  // no k, no shape
    if (count == 0) return QTIP_OK;
    hipError_t e = qtip::launch_decode_states(code_id, states, count, (const uint32_t *)lut_f16,
                                              out_f16, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

int qtip_quantize(const float *W, int m, int n, int L, int k, int V, int code_id,
                  const void *lut_f16, uint32_t *codes_out, double *mse_out) {
    const char *fn = "qtip_quantize";
    if (!W || !codes_out) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (int rc = check_code(fn, L, k, V, code_id, lut_f16, m, n)) return rc;
    int rc;
    try {
        rc = qtip::quantize_host(W, m, n, L, k, V, code_id, (const uint16_t *)lut_f16, codes_out, mse_out);
    } catch (const std::bad_alloc &) {
        return fail(QTIP_ENOMEM, "%s: out of host memory", fn);
    } catch (...) {
        return fail(QTIP_ENOMEM, "%s: host failure", fn);
    }
    if (rc != 0) return fail(QTIP_ENOMEM, "%s: worker failed (out of host memory?)", fn);
    return QTIP_OK;
}

size_t qtip_quantize_gpu_workspace(int k, int V, long tiles) {
    if (k < 2 || k > 4 || (V != 1 && V != 2) || tiles <= 0) return 0;
    return qtip::quantize_gpu_workspace(k, V, tiles);
}

int qtip_quantize_gpu(const float *W, int m, int n, int L, int k, int V, int code_id,
                      const void *lut_f16, uint32_t *codes_out, float *tile_err, void *workspace,
                      size_t workspace_bytes, void *stream) {
    const char *fn = "qtip_quantize_gpu";
    if (!W || !codes_out || !workspace) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (int rc = check_code(fn, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (((uintptr_t)W | (uintptr_t)codes_out | (uintptr_t)tile_err) % 4 || (uintptr_t)workspace % 256)
        return fail(QTIP_EINVAL, "%s: W, codes_out, tile_err need 4-byte, workspace 256-byte alignment", fn);
    if (workspace_bytes < qtip::quantize_gpu_workspace(k, V, 1))
        return fail(QTIP_EINVAL, "%s: workspace of %zu bytes cannot hold one tile (%zu needed)", fn,
                    workspace_bytes, qtip::quantize_gpu_workspace(k, V, 1));
    hipError_t e = qtip::launch_quantize_gpu(k, code_id, W, m, n, n, (const uint32_t *)lut_f16, codes_out,
                                             tile_err, workspace, workspace_bytes, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

size_t qtip_block_ldl_workspace(int n) {
    if (n <= 0 || n % 16) return 0;
    return qtip::block_ldl_workspace(n);
}

int qtip_block_ldl(const double *H, int n, int g, float *A_out, double *D_out, void *workspace,
                   size_t workspace_bytes, void *stream) {
    const char *fn = "qtip_block_ldl";
    if (!H || !A_out || !workspace) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (g != 8 && g != 16) return fail(QTIP_EINVAL, "%s: g = %d must be 8 or 16", fn, g);
    if (n <= 0 || n % 16) return fail(QTIP_EINVAL, "%s: n = %d must be a positive multiple of 16", fn, n);
    if ((uintptr_t)H % 8 || (uintptr_t)D_out % 8 || (uintptr_t)A_out % 4 || (uintptr_t)workspace % 256)
        return fail(QTIP_EINVAL, "%s: H, D_out need 8-byte, A_out 4-byte, workspace 256-byte alignment", fn);
    if (workspace_bytes < qtip::block_ldl_workspace(n))
        return fail(QTIP_EINVAL, "%s: workspace of %zu bytes, %zu needed", fn, workspace_bytes,
                    qtip::block_ldl_workspace(n));
    hipError_t e = qtip::launch_block_ldl(H, n, g, A_out, D_out, workspace, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

size_t qtip_quantize_ldlq_workspace(int m, int n, int k, int V, long tiles) {
    if (k < 2 || k > 4 || (V != 1 && V != 2) || tiles <= 0 || m <= 0 || n <= 0 || m % 16 || n % 8) return 0;
    return qtip::quantize_ldlq_workspace(m, n, k, V, tiles);
}

int qtip_quantize_ldlq(const float *W, const float *A, int m, int n, int L, int k, int V, int code_id,
                       const void *lut_f16, uint32_t *codes_out, float *What_out, float *tile_err,
                       void *workspace, size_t workspace_bytes, void *stream) {
    const char *fn = "qtip_quantize_ldlq";
    if (!W || !A || !codes_out || !workspace) return fail(QTIP_EINVAL, "%s: NULL pointer", fn);
    if (int rc = check_code(fn, L, k, V, code_id, lut_f16, m, n)) return rc;
    if (((uintptr_t)W | (uintptr_t)A | (uintptr_t)codes_out | (uintptr_t)What_out | (uintptr_t)tile_err) % 4 ||
        (uintptr_t)workspace % 256)
        return fail(QTIP_EINVAL, "%s: arrays need 4-byte, workspace 256-byte alignment", fn);
    if (workspace_bytes < qtip::quantize_ldlq_workspace(m, n, k, V, 1))
        return fail(QTIP_EINVAL, "%s: workspace of %zu bytes, at least %zu needed", fn, workspace_bytes,
                    qtip::quantize_ldlq_workspace(m, n, k, V, 1));
    hipError_t e = qtip::launch_quantize_ldlq(k, V, code_id, W, A, m, n, (const uint32_t *)lut_f16, codes_out,
                                              What_out, tile_err, workspace, workspace_bytes,
                                              (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(fn, e);
    return QTIP_OK;
}

}  // extern "C"
