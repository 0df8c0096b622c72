// Host-only stand-ins for the kernel launchers, for the sanitizer build of the library's host
// code (argument checks in qtip_api.hip, the host quantizer qtip_quantize.cpp): they launch
// nothing and report success, so that every path of the entry points up to the launch runs
// under AddressSanitizer / UndefinedBehaviorSanitizer on a machine without a GPU.
#include "qtip_internal.h"

extern "C" const char *hipGetErrorString(hipError_t) { return "stub"; }
extern "C" hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
extern "C" hipError_t hipGetSymbolAddress(void **p, const void *symbol) { *p = const_cast<void *>(symbol); return hipSuccess; }

namespace qtip {

hipError_t launch_dequantize(int, int, const uint32_t *, const uint32_t *, int, int, void *, hipStream_t) { return hipSuccess; }
hipError_t launch_matvec(int, int, const uint32_t *, const uint32_t *, int, int, const void *, const void *, float *, hipStream_t) { return hipSuccess; }
hipError_t launch_matmat(int, int, const uint32_t *, const uint32_t *, int, int, const void *, int, const void *, float *, hipStream_t) { return hipSuccess; }
int fused_rht_matvec_max_n() { return 8192; }
hipError_t launch_rht_matvec(int, int, const uint32_t *, const uint32_t *, int, int, const void *, const int8_t *, int, const void *, float *, hipStream_t) { return hipSuccess; }
hipError_t launch_decode_states(int, const uint32_t *, int, const uint32_t *, void *, hipStream_t) { return hipSuccess; }
hipError_t launch_rht(const void *, bool, const int8_t *, int, int, int, int, void *, hipStream_t) { return hipSuccess; }
hipError_t launch_lut_dequantize(int, const uint32_t *, const void *, int, int, void *, hipStream_t) { return hipSuccess; }
hipError_t launch_lut_matvec(int, const uint32_t *, const void *, int, int, const void *, const void *, float *, hipStream_t) { return hipSuccess; }
hipError_t launch_lut_matmat(int, const uint32_t *, const void *, int, int, const void *, int, const void *, float *, hipStream_t) { return hipSuccess; }
hipError_t launch_lut_decode_states(const uint32_t *, int, const void *, void *, hipStream_t) { return hipSuccess; }
size_t quantize_gpu_workspace(int k, int V, long tiles) { return (size_t)tiles * 4096 * k * V; }
hipError_t launch_quantize_gpu(int, int, const float *, int, int, int, const uint32_t *, uint32_t *, float *, void *, size_t, hipStream_t) { return hipSuccess; }
size_t block_ldl_workspace(int n) { return 2 * (size_t)n * n * sizeof(double); }
hipError_t launch_block_ldl(const double *, int, int, float *, double *, void *, hipStream_t) { return hipSuccess; }
size_t quantize_ldlq_workspace(int m, int n, int k, int V, long tiles) { return (size_t)m * n * 4 + quantize_gpu_workspace(k, V, tiles); }
hipError_t launch_quantize_ldlq(int, int, int, const float *, const float *, int, int, const uint32_t *, uint32_t *, float *, float *, void *, size_t, hipStream_t) { return hipSuccess; }

}  // namespace qtip
