// C ABI of the fptq library: argument validation, shape dispatch, error text.
// Every entry point validates first and launches afterwards, so a failing call writes nothing.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "fptq_common.h"
#include "fptq_testing.h"

namespace fptq {

static thread_local char g_err[256] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

static int hip_fail(const char *what, hipError_t e)
{
    set_error("%s: %s", what, hipGetErrorString(e));
    return FPTQ_ERR_HIP;
}

static const int64_t MAX_ELEMS = (int64_t)1 << 40;
// INT32 accumulation is exact while 64 K < 2^31 (|q w| <= 64); with a zero point the epilogue forms
// acc - z * sum_k w, at most 128 K in magnitude.
static const int64_t MAX_K = ((int64_t)1 << 25) - 1, MAX_K_ZERO_POINT = ((int64_t)1 << 24) - 1;

// ---- per-device state.  Filled once per device under a lock; readers take the lock-free path afterwards.
static DeviceInfo g_devices[MAX_DEVICES];
static std::atomic<bool> g_device_ready[MAX_DEVICES];
static std::mutex g_device_mutex;

hipError_t device_info(const DeviceInfo **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_device_ready[dev].load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_device_mutex);
        if (!g_device_ready[dev].load(std::memory_order_relaxed)) {
            DeviceInfo info = {};
            info.device = dev;
            int cus = 0;
            if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
            info.cus = cus > 0 ? cus : DEFAULT_CUS;
            if ((e = gemm_device_init(&info)) != hipSuccess) return e;
            if ((e = hadamard_device_init(dev)) != hipSuccess) return e;
            g_devices[dev] = info;
            g_device_ready[dev].store(true, std::memory_order_release);
        }
    }
    *out = &g_devices[dev];
    return hipSuccess;
}

int device_cus_or_default()
{
    const DeviceInfo *info;
    if (device_info(&info) != hipSuccess) {
        (void)hipGetLastError();     // a host-only query without a device must not leave a sticky error behind
        return DEFAULT_CUS;
    }
    return info->cus;
}

static int check_dims(const char *fn, int64_t a, int64_t b, const char *an, const char *bn)
{
    if (a < 1 || b < 1 || a > MAX_ELEMS / b) {
        set_error("%s: bad shape %s=%lld %s=%lld", fn, an, (long long)a, bn, (long long)b);
        return FPTQ_ERR_SHAPE;
    }
    return FPTQ_OK;
}

static int check_align(const char *fn, const void *p, unsigned a, const char *name)
{
    if (reinterpret_cast<uintptr_t>(p) & (a - 1)) {
        set_error("%s: %s must be %u-byte aligned", fn, name, a);
        return FPTQ_ERR_ALIGN;
    }
    return FPTQ_OK;
}

// The few-token kernel serves M <= 32 and, for matrices of fewer than 10240 channels, M <= 64; above that, or
// whenever a prefill tile shape is forced, the MFMA GEMM runs: its 64 x 64 and 128 x 64 tiles with four K groups
// are faster from 65 tokens on everywhere, and from 33 tokens on wide matrices (measured over cold weights at 64
// tokens, best few-token launch shape against the MFMA kernel: 6144 x 4096 7.0 us against 9.1, 4096 x 14336 13.9
// against 19.5, but 28672 x 4096 19.1 against 15.9 and 22016 x 4096 16.7 against 14.4, with 10240 to 15360
// channels about even; at 80 tokens 4096 x 14336 22.1 against 17.0).
static bool few_token_shape(int64_t M, int64_t N) { return M <= 32 || (M <= 64 && N < 10240); }

typedef hipError_t (*linear_fn)(const uint8_t *, const uint8_t *, int64_t, int64_t, int64_t, float, const float *,
                                const float *, int, const int32_t *, uint16_t *, int32_t *, hipStream_t);

static int linear_common(const char *fn, linear_fn force, const void *xq, const void *wq, int64_t M, int64_t N,
                         int64_t K, float s_a, const float *s_w, const float *d, int zp, const int32_t *wsum, void *y,
                         int32_t *acc, void *stream, void *workspace = nullptr, int64_t workspace_bytes = 0)
{
    if (!xq || !wq || !s_w || !y) {
        set_error("%s: NULL pointer", fn);
        return FPTQ_ERR_NULL;
    }
    int rc;
    if ((rc = check_dims(fn, M, K, "M", "K")) || (rc = check_dims(fn, N, K, "N", "K")) ||
        (rc = check_dims(fn, M, N, "M", "N")))
        return rc;
    if (!(s_a > 0.0f) || !std::isfinite(s_a)) {
        set_error("%s: s_a must be finite and > 0", fn);
        return FPTQ_ERR_VALUE;
    }
    if ((rc = check_align(fn, xq, 16, "xq_packed")) || (rc = check_align(fn, wq, 16, "w_packed")) ||
        (rc = check_align(fn, y, 16, "y_bf16")) || (rc = check_align(fn, acc, 16, "acc_dbg")) ||
        (rc = check_align(fn, s_w, 4, "s_w")) || (rc = check_align(fn, d, 4, "row_out_scale")) ||
        (rc = check_align(fn, wsum, 4, "w_row_sum")))
        return rc;
    if (zp < -8 || zp > 7 || (zp != 0 && !wsum)) {
        set_error("%s: zero_point must be in [-8, 7] and needs w_row_sum", fn);
        return FPTQ_ERR_VALUE;
    }
    if (K > (zp != 0 ? MAX_K_ZERO_POINT : MAX_K)) {
        set_error("%s: K=%lld exceeds %lld, the longest sum INT32 holds exactly%s", fn, (long long)K,
                  (long long)(zp != 0 ? MAX_K_ZERO_POINT : MAX_K), zp != 0 ? " with a zero point" : "");
        return FPTQ_ERR_SHAPE;
    }
    if (zp == 0) wsum = nullptr;
    if ((rc = check_align(fn, workspace, 256, "workspace"))) return rc;
    if (workspace_bytes < 0) {
        set_error("%s: negative workspace_bytes", fn);
        return FPTQ_ERR_SIZE;
    }
    linear_fn f = force ? force : (few_token_shape(M, N) && forced_gemm_tile() == 0 ? launch_linear_decode : launch_linear_mfma);
    hipError_t e;
    if (f == launch_linear_mfma && workspace)
        e = launch_linear_mfma_ws((const uint8_t *)xq, (const uint8_t *)wq, M, N, K, s_a, s_w, d, zp, wsum, (uint16_t *)y, acc,
                                  (int32_t *)workspace, workspace_bytes, (hipStream_t)stream);
    else
        e = f((const uint8_t *)xq, (const uint8_t *)wq, M, N, K, s_a, s_w, d, zp, wsum, (uint16_t *)y, acc, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail(fn, e);
}

}  // namespace fptq

using namespace fptq;

extern "C" {

int fptq_version(void) { return 200; }

int fptq_init(void)
{
    const DeviceInfo *info;
    hipError_t e = device_info(&info);
    return e == hipSuccess ? FPTQ_OK : hip_fail("fptq_init", e);
}

const char *fptq_last_error(void) { return g_err; }

int64_t fptq_packed_bytes(int64_t rows, int64_t K)
{
    if (check_dims("fptq_packed_bytes", rows, K, "rows", "K")) return FPTQ_ERR_SHAPE;
    return packed_bytes(rows, K);
}

int fptq_pack_weights(const int8_t *w_int, int64_t N, int64_t K, void *w_packed, int64_t w_packed_bytes, void *stream)
{
    if (!w_int || !w_packed) {
        set_error("fptq_pack_weights: NULL pointer");
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims("fptq_pack_weights", N, K, "N", "K");
    if (rc) return rc;
    if (w_packed_bytes < packed_bytes(N, K)) {
        set_error("fptq_pack_weights: buffer of %lld bytes, need %lld", (long long)w_packed_bytes,
                  (long long)packed_bytes(N, K));
        return FPTQ_ERR_SIZE;
    }
    if ((rc = check_align("fptq_pack_weights", w_packed, 16, "w_packed"))) return rc;
    hipError_t e = launch_pack_weights(w_int, N, K, (uint8_t *)w_packed, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail("fptq_pack_weights", e);
}

static int quantize_common(const char *fn, int hadamard_block, int zero_point, const void *x_bf16, int64_t M, int64_t K, int scale_mode,
                           float eps, const float *row_scale_in, float s_a, void *xq_packed, int64_t xq_bytes,
                           float *row_scale_out, void *stream)
{
    if (!x_bf16 || !xq_packed) {
        set_error("%s: NULL pointer", fn);
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims(fn, M, K, "M", "K");
    if (rc) return rc;
    const bool block_ok = hadamard_block == 256 || hadamard_block == 512 || hadamard_block == 1024 || hadamard_block == 2048 ||
                          hadamard_block == 4096;
    if (hadamard_block != 0 && (!block_ok || K % hadamard_block != 0)) {
        set_error("%s: hadamard_block must be 256, 512, 1024, 2048 or 4096 and divide K (got block %d, K %lld)", fn, hadamard_block,
                  (long long)K);
        return FPTQ_ERR_SHAPE;
    }
    if (scale_mode != FPTQ_SCALE_NONE && scale_mode != FPTQ_SCALE_RMS && scale_mode != FPTQ_SCALE_GIVEN) {
        set_error("%s: unknown scale_mode %d", fn, scale_mode);
        return FPTQ_ERR_MODE;
    }
    if (scale_mode == FPTQ_SCALE_GIVEN && !row_scale_in) {
        set_error("%s: FPTQ_SCALE_GIVEN needs row_scale_in", fn);
        return FPTQ_ERR_MODE;
    }
    if (!(s_a > 0.0f) || !std::isfinite(s_a) || !(eps >= 0.0f) || zero_point < -8 || zero_point > 7) {
        set_error("%s: s_a must be finite and > 0, eps >= 0, zero_point in [-8, 7]", fn);
        return FPTQ_ERR_VALUE;
    }
    if (xq_bytes < packed_bytes(M, K)) {
        set_error("%s: buffer of %lld bytes, need %lld", fn, (long long)xq_bytes, (long long)packed_bytes(M, K));
        return FPTQ_ERR_SIZE;
    }
    if ((rc = check_align(fn, xq_packed, 16, "xq_packed")) || (rc = check_align(fn, x_bf16, hadamard_block ? 16 : 2, "x_bf16")) ||
        (rc = check_align(fn, row_scale_in, 4, "row_scale_in")) || (rc = check_align(fn, row_scale_out, 4, "row_scale_out")))
        return rc;
    // the one fp32 division of the quantizer happens here, on the host
    volatile float inv = 1.0f / s_a;
    hipError_t e = hadamard_block
                       ? launch_quantize_act_hadamard((const uint16_t *)x_bf16, M, K, hadamard_block, scale_mode, eps, row_scale_in, inv,
                                                      (uint8_t *)xq_packed, row_scale_out, (hipStream_t)stream)
                       : launch_quantize_act((const uint16_t *)x_bf16, M, K, scale_mode, eps, row_scale_in, inv, zero_point,
                                             (uint8_t *)xq_packed, row_scale_out, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail(fn, e);
}

int fptq_quantize_act(const void *x_bf16, int64_t M, int64_t K, int scale_mode, float eps, const float *row_scale_in,
                      float s_a, void *xq_packed, int64_t xq_bytes, float *row_scale_out, void *stream)
{
    return quantize_common("fptq_quantize_act", 0, 0, x_bf16, M, K, scale_mode, eps, row_scale_in, s_a, xq_packed, xq_bytes,
                           row_scale_out, stream);
}

int fptq_quantize_act_asym(const void *x_bf16, int64_t M, int64_t K, int scale_mode, float eps, const float *row_scale_in,
                           float s_a, int zero_point, void *xq_packed, int64_t xq_bytes, float *row_scale_out, void *stream)
{
    return quantize_common("fptq_quantize_act_asym", 0, zero_point, x_bf16, M, K, scale_mode, eps, row_scale_in, s_a, xq_packed,
                           xq_bytes, row_scale_out, stream);
}

int fptq_residual_norm_quantize(const void *x_res_bf16, const void *y_bf16, int64_t M, int64_t K, const float *s_prev,
                                float eps, float s_a, void *x_next_bf16, float *s_next, void *xq_packed, int64_t xq_bytes,
                                void *stream)
{
    const char *fn = "fptq_residual_norm_quantize";
    if (!x_res_bf16 || !y_bf16 || !x_next_bf16 || !s_next || !xq_packed) {
        set_error("%s: NULL pointer", fn);
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims(fn, M, K, "M", "K");
    if (rc) return rc;
    if (!(s_a > 0.0f) || !std::isfinite(s_a) || !(eps >= 0.0f)) {
        set_error("%s: s_a must be finite and > 0, eps >= 0", fn);
        return FPTQ_ERR_VALUE;
    }
    if (xq_bytes < packed_bytes(M, K)) {
        set_error("%s: buffer of %lld bytes, need %lld", fn, (long long)xq_bytes, (long long)packed_bytes(M, K));
        return FPTQ_ERR_SIZE;
    }
    if ((rc = check_align(fn, xq_packed, 16, "xq_packed")) || (rc = check_align(fn, x_res_bf16, 2, "x_res_bf16")) ||
        (rc = check_align(fn, y_bf16, 2, "y_bf16")) || (rc = check_align(fn, x_next_bf16, 2, "x_next_bf16")) ||
        (rc = check_align(fn, s_prev, 4, "s_prev")) || (rc = check_align(fn, s_next, 4, "s_next")))
        return rc;
    volatile float inv = 1.0f / s_a;
    hipError_t e = launch_residual_norm_quantize((const uint16_t *)x_res_bf16, (const uint16_t *)y_bf16, M, K, s_prev, eps, inv,
                                                 (uint16_t *)x_next_bf16, s_next, (uint8_t *)xq_packed, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail(fn, e);
}

int fptq_quantize_act_dynamic(const void *x_bf16, int64_t M, int64_t K, void *xq_packed, int64_t xq_bytes,
                              float *token_scale_out, void *stream)
{
    const char *fn = "fptq_quantize_act_dynamic";
    if (!x_bf16 || !xq_packed || !token_scale_out) {
        set_error("%s: NULL pointer", fn);
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims(fn, M, K, "M", "K");
    if (rc) return rc;
    if (xq_bytes < packed_bytes(M, K)) {
        set_error("%s: buffer of %lld bytes, need %lld", fn, (long long)xq_bytes, (long long)packed_bytes(M, K));
        return FPTQ_ERR_SIZE;
    }
    if ((rc = check_align(fn, xq_packed, 16, "xq_packed")) || (rc = check_align(fn, x_bf16, 2, "x_bf16")) ||
        (rc = check_align(fn, token_scale_out, 4, "token_scale_out")))
        return rc;
    hipError_t e = launch_quantize_act_dynamic((const uint16_t *)x_bf16, M, K, (uint8_t *)xq_packed, token_scale_out,
                                               (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail(fn, e);
}

int fptq_quantize_act_hadamard(const void *x_bf16, int64_t M, int64_t K, int hadamard_block, int scale_mode, float eps,
                               const float *row_scale_in, float s_a, void *xq_packed, int64_t xq_bytes,
                               float *row_scale_out, void *stream)
{
    if (hadamard_block == 0) {
        set_error("fptq_quantize_act_hadamard: hadamard_block must be 256, 512, 1024, 2048 or 4096");
        return FPTQ_ERR_SHAPE;
    }
    return quantize_common("fptq_quantize_act_hadamard", hadamard_block, 0, x_bf16, M, K, scale_mode, eps, row_scale_in, s_a,
                           xq_packed, xq_bytes, row_scale_out, stream);
}

int fptq_w4a4_linear(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                     const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream)
{
    return linear_common("fptq_w4a4_linear", nullptr, xq_packed, w_packed, M, N, K, s_a, s_w, row_out_scale, 0, nullptr,
                         y_bf16, acc_dbg, stream);
}

int fptq_w4a4_linear_zp(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                        const float *s_w, const float *row_out_scale, int zero_point, const int32_t *w_row_sum,
                        void *y_bf16, int32_t *acc_dbg, void *stream)
{
    return linear_common("fptq_w4a4_linear_zp", nullptr, xq_packed, w_packed, M, N, K, s_a, s_w, row_out_scale, zero_point,
                         w_row_sum, y_bf16, acc_dbg, stream);
}

int fptq_weight_row_sums(const int8_t *w_int, int64_t N, int64_t K, int32_t *sums, void *stream)
{
    if (!w_int || !sums) {
        set_error("fptq_weight_row_sums: NULL pointer");
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims("fptq_weight_row_sums", N, K, "N", "K");
    if (rc) return rc;
    if ((rc = check_align("fptq_weight_row_sums", sums, 4, "sums"))) return rc;
    hipError_t e = launch_weight_row_sums(w_int, N, K, sums, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail("fptq_weight_row_sums", e);
}

int fptq_w4a4_linear_ref(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                         const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream)
{
    return linear_common("fptq_w4a4_linear_ref", launch_linear_ref, xq_packed, w_packed, M, N, K, s_a, s_w,
                         row_out_scale, 0, nullptr, y_bf16, acc_dbg, stream);
}

int64_t fptq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const char *fn = "fptq_linear_workspace_bytes";
    int rc;
    if ((rc = check_dims(fn, M, K, "M", "K")) || (rc = check_dims(fn, N, K, "N", "K")) || (rc = check_dims(fn, M, N, "M", "N")))
        return rc;
    if (K > MAX_K) {
        set_error("%s: K=%lld exceeds %lld, the longest sum INT32 holds exactly", fn, (long long)K, (long long)MAX_K);
        return FPTQ_ERR_SHAPE;
    }
    return few_token_shape(M, N) ? 0 : linear_workspace_bytes(M, N, K);
}

int fptq_w4a4_linear_ws(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                        const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *workspace,
                        int64_t workspace_bytes, void *stream)
{
    return linear_common("fptq_w4a4_linear_ws", nullptr, xq_packed, w_packed, M, N, K, s_a, s_w, row_out_scale, 0, nullptr, y_bf16,
                         acc_dbg, stream, workspace, workspace_bytes);
}

int fptq_w4a4_linear_noalloc(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream)
{
    const char *fn = "fptq_w4a4_linear_noalloc";
    // shapes that would not split K anyway need no scratch: the plain layer (which allocates nothing either)
    const int64_t need = (M >= 1 && N >= 1 && K >= 1 && K <= MAX_K && M <= MAX_ELEMS / K && N <= MAX_ELEMS / K && M <= MAX_ELEMS / N &&
                          !few_token_shape(M, N))
                             ? linear_workspace_bytes(M, N, K)
                             : 0;
    if (need == 0)
        return linear_common(fn, nullptr, xq_packed, w_packed, M, N, K, s_a, s_w, row_out_scale, 0, nullptr, y_bf16, acc_dbg, stream);
    const DeviceInfo *info;
    hipError_t e = device_info(&info);
    if (e != hipSuccess) return hip_fail(fn, e);
    if (need > info->scratch_bytes) {
        set_error("%s: M=%lld N=%lld K=%lld needs %lld bytes of scratch, the built-in area holds %lld; use fptq_w4a4_linear_ws "
                  "with a caller workspace or fptq_w4a4_linear", fn, (long long)M, (long long)N, (long long)K, (long long)need,
                  (long long)info->scratch_bytes);
        return FPTQ_ERR_SIZE;
    }
    return linear_common(fn, nullptr, xq_packed, w_packed, M, N, K, s_a, s_w, row_out_scale, 0, nullptr, y_bf16, acc_dbg, stream,
                         info->scratch, info->scratch_bytes);
}

int fptq_linear_launch_plan(int64_t M, int64_t N, int64_t K, int with_workspace, char *kernel, int kernel_len,
                            int64_t *workgroups, int *threads)
{
    const char *fn = "fptq_linear_launch_plan";
    if (!kernel || kernel_len < 1 || !workgroups || !threads) {
        set_error("%s: NULL pointer", fn);
        return FPTQ_ERR_NULL;
    }
    int rc;
    if ((rc = check_dims(fn, M, K, "M", "K")) || (rc = check_dims(fn, N, K, "N", "K")) || (rc = check_dims(fn, M, N, "M", "N")))
        return rc;
    LinearPlan plan = {};
    if (few_token_shape(M, N) && forced_gemm_tile() == 0) {
        snprintf(plan.kernel, sizeof plan.kernel, "linear_decode_kernel");
        plan.workgroups = 0;
        plan.threads = 0;
    } else {
        linear_mfma_plan(M, N, K, with_workspace != 0, &plan);
    }
    snprintf(kernel, (size_t)kernel_len, "%s", plan.kernel);
    *workgroups = plan.workgroups;
    *threads = plan.threads;
    return FPTQ_OK;
}

int fptq_set_gemm_map(int mode)
{
    if (mode != 0 && mode != 1) {
        set_error("fptq_set_gemm_map: mode must be 0 or 1");
        return FPTQ_ERR_VALUE;
    }
    set_gemm_map(mode);
    return FPTQ_OK;
}

int fptq_set_decode_shape(int code)
{
    if (!set_decode_shape(code)) {
        set_error("fptq_set_decode_shape: code must be 0 or waves (8, 16) * 100 + tiles per batch (1, 2, 4) * 10 + channel groups (1, 2, 4)");
        return FPTQ_ERR_VALUE;
    }
    return FPTQ_OK;
}

int fptq_set_gemm_tile(int tile)
{
    if (tile < 0 || tile > 8) {
        set_error("fptq_set_gemm_tile: tile must be 0..8");
        return FPTQ_ERR_VALUE;
    }
    set_gemm_tile(tile);
    return FPTQ_OK;
}

int fptq_unpack(const void *packed, int64_t rows, int64_t K, int8_t *out_int8, void *stream)
{
    if (!packed || !out_int8) {
        set_error("fptq_unpack: NULL pointer");
        return FPTQ_ERR_NULL;
    }
    int rc = check_dims("fptq_unpack", rows, K, "rows", "K");
    if (rc) return rc;
    if ((rc = check_align("fptq_unpack", packed, 16, "packed"))) return rc;
    hipError_t e = launch_unpack((const uint8_t *)packed, rows, K, out_int8, (hipStream_t)stream);
    return e == hipSuccess ? FPTQ_OK : hip_fail("fptq_unpack", e);
}

}  // extern "C"
