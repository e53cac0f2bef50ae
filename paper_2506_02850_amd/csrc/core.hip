// Error reporting, host-side quota arithmetic (Eq. 6-7) and the calibration copy kernel.
#include <math.h>
#include <string.h>

#include "common.h"

namespace metok {

char* error_buffer() {
    static thread_local char buf[512] = {0};
    return buf;
}

void clear_error() { error_buffer()[0] = 0; }

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(METOK_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return METOK_OK;
}

int ceil_ratio(double x) { return static_cast<int>(ceil(x - 1e-9)); }

// One 16-byte non-temporal load and store per thread: the fastest plain copy measured on MI355X
// (6.5 TB/s read + write; more loads in flight per thread are slower).
__global__ __launch_bounds__(256) void copy16_kernel(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src, size_t n) {
    const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace metok

using namespace metok;

extern "C" const char* metok_last_error(void) { return error_buffer(); }

extern "C" int metok_version(void) { return 100; }

extern "C" int metok_retention_quotas(int level, double r, double alpha, int64_t n_key_orig, int64_t n_non_orig,
                                      int32_t quota_out[2]) {
    clear_error();
    if (level < 0 || level > 3) return fail(METOK_ERR_INVALID_ARG, "level must be 0..3, got %d", level);
    if (!(r > 0.0 && r <= 1.0) || !(alpha > 0.0 && alpha <= 1.0))
        return fail(METOK_ERR_INVALID_ARG, "need 0 < r <= 1 and 0 < alpha <= 1 (r=%g alpha=%g)", r, alpha);
    if (n_key_orig < 0 || n_non_orig < 0 || n_key_orig > INT32_MAX || n_non_orig > INT32_MAX || !quota_out)
        return fail(METOK_ERR_INVALID_ARG, "token counts must fit int32 and quota_out must not be NULL");
    // Eq. 6: 1, r, r^2, 0.  Eq. 7: 1, alpha r, 0, 0.  Ratios refer to the counts that entered the LLM.
    const double key_ratio[4] = {1.0, r, r * r, 0.0};
    const double non_ratio[4] = {1.0, alpha * r, 0.0, 0.0};
    int64_t qk = ceil_ratio(key_ratio[level] * static_cast<double>(n_key_orig));
    int64_t qn = ceil_ratio(non_ratio[level] * static_cast<double>(n_non_orig));
    quota_out[0] = static_cast<int32_t>(qk > n_key_orig ? n_key_orig : qk);
    quota_out[1] = static_cast<int32_t>(qn > n_non_orig ? n_non_orig : qn);
    return METOK_OK;
}

extern "C" int metok_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
    clear_error();
    if (!dst || !src || (bytes & 15u) || !aligned16(dst) || !aligned16(src))
        return fail(METOK_ERR_INVALID_ARG, "calib copy needs 16-byte aligned pointers and size");
    if (bytes == 0) return METOK_OK;
    size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 0x7fffffffu) return fail(METOK_ERR_INVALID_ARG, "calib copy too large");
    hipLaunchKernelGGL(copy16_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<u32x4_t*>(dst), static_cast<const u32x4_t*>(src), n);
    return check_launch("calib copy");
}
