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

KernelTrace& kernel_trace() {
    static thread_local KernelTrace t = {METOK_TRACE_NONE, nullptr, nullptr};
    return t;
}

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

extern "C" int metok_trace_kernel(int kernel, void* ev_begin, void* ev_end) {
    clear_error();
    if (kernel < METOK_TRACE_NONE || kernel > METOK_TRACE_MOVE_ROWS) return fail(METOK_ERR_INVALID_ARG, "unknown kernel id %d", kernel);
    KernelTrace& t = kernel_trace();
    if (kernel == METOK_TRACE_NONE || !ev_begin || !ev_end) { t.kernel = METOK_TRACE_NONE; t.begin = nullptr; t.end = nullptr; return METOK_OK; }
    t.kernel = kernel; t.begin = static_cast<hipEvent_t>(ev_begin); t.end = static_cast<hipEvent_t>(ev_end);
    return METOK_OK;
}

extern "C" int metok_preset(int model, metok_params* out) {
    clear_error();
    // Appendix "Implementation Details": one setting per base model
    static const metok_params presets[4] = {METOK_PRESET_LLAVA_OV_0_5B, METOK_PRESET_LLAVA_OV_7B, METOK_PRESET_LONGVA_7B,
                                            METOK_PRESET_VILA_13B};
    if (!out) return fail(METOK_ERR_INVALID_ARG, "out is NULL");
    if (model < 0 || model > 3) return fail(METOK_ERR_INVALID_ARG, "unknown model %d", model);
    *out = presets[model];
    return METOK_OK;
}

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

extern "C" int metok_account(const int32_t* event_len, const uint8_t* event_is_key, int k, int grid_h, int grid_w,
                             double alpha, double beta, int s1, int s2, int pool_edge, double r,
                             const int32_t layers_h[3], int n_layers, int64_t n_text, metok_account_t* out) {
    clear_error();
    if (!event_len || !event_is_key || !layers_h || !out) return fail(METOK_ERR_INVALID_ARG, "NULL pointer argument");
    if (k < 1 || grid_h < 1 || grid_w < 1 || s1 < 1 || s2 < 1 || n_text < 0)
        return fail(METOK_ERR_INVALID_ARG, "k, grid and strides must be positive, n_text non-negative");
    if (!(alpha > 0.0 && alpha <= 1.0) || !(beta > 0.0 && beta <= 1.0) || !(r > 0.0 && r <= 1.0))
        return fail(METOK_ERR_INVALID_ARG, "need 0 < alpha, beta, r <= 1");
    if (pool_edge != METOK_POOL_FLOOR && pool_edge != METOK_POOL_CEIL) return fail(METOK_ERR_INVALID_ARG, "unknown pool_edge %d", pool_edge);
    if (n_layers < 1 || n_layers > METOK_MAX_LAYERS) return fail(METOK_ERR_INVALID_ARG, "n_layers must be in [1, %d]", METOK_MAX_LAYERS);
    if (!(0 <= layers_h[0] && layers_h[0] <= layers_h[1] && layers_h[1] <= layers_h[2]))
        return fail(METOK_ERR_INVALID_ARG, "pruning layers must be non-negative and ascending");
    const int gmax = grid_h > grid_w ? grid_h : grid_w;
    auto rows = [&](double s) -> int64_t {
        int v = ceil_ratio(s);
        v = v < 1 ? 1 : (v > gmax ? gmax : v);
        auto side = [&](int g) { return pool_edge == METOK_POOL_FLOOR ? (g / v > 1 ? g / v : 1) : (g + v - 1) / v; };
        return static_cast<int64_t>(side(grid_h)) * side(grid_w);
    };
    const int64_t rows_kk = rows(s1), rows_kn = rows(s2), rows_nk = rows(s1 / alpha), rows_nn = rows(s2 / alpha);
    int64_t key = 0, non = 0, frames = 0;
    for (int j = 0; j < k; ++j) {
        const int64_t n = event_len[j];
        if (n < 1) return fail(METOK_ERR_INVALID_ARG, "event_len[%d] = %lld: every event has at least one frame", j, (long long)n);
        int64_t n_kf = ceil_ratio(beta * static_cast<double>(n));       // key frames of the event (Sec. 3.2.1)
        n_kf = n_kf > n ? n : n_kf;
        if (event_is_key[j]) key += n_kf * rows_kk + (n - n_kf) * rows_kn;
        else                 non += n_kf * rows_nk + (n - n_kf) * rows_nn;
        frames += n;
    }
    if (key > INT32_MAX || non > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "token counts must fit int32");
    out->tokens_encoder = frames * grid_h * grid_w;
    out->tokens_llm = key + non;
    out->tokens_key = key;
    out->tokens_non = non;
    const double key_ratio[4] = {1.0, r, r * r, 0.0}, non_ratio[4] = {1.0, alpha * r, 0.0, 0.0};      // Eq. 6-7
    for (int level = 0; level < 4; ++level) {
        int64_t qk = ceil_ratio(key_ratio[level] * static_cast<double>(key)), qn = ceil_ratio(non_ratio[level] * static_cast<double>(non));
        out->level_tokens[level] = (qk > key ? key : qk) + (qn > non ? non : qn);
    }
    int64_t prefill = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int level = (l >= layers_h[0]) + (l >= layers_h[1]) + (l >= layers_h[2]);
        prefill += out->level_tokens[level] + n_text;
    }
    out->prefill_token_layers = prefill;
    out->kv_token_layers_full = static_cast<int64_t>(n_layers) * (key + non + n_text);
    out->kv_token_layers_stage2 = prefill;
    // Sec. 3.3: layers below l_1 keep every row, the others the text rows only
    const int64_t l1 = layers_h[0] < n_layers ? layers_h[0] : n_layers;
    out->kv_token_layers_stage3 = l1 * (key + non + n_text) + (n_layers - l1) * n_text;
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
