// Shared declarations of the fptq HIP library (gfx950 only): packed layout arithmetic, error
// reporting, and the launcher prototypes that tie the translation units together.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "fptq.h"

namespace fptq {

// Packed INT4 layout: K is cut into tiles of KT values; each (tile, row) pair owns one
// 64-byte segment, tiles outermost.  Within a segment value k sits in byte (k % KT) / 2,
// low nibble first.
constexpr int KT = 128;          // values per K tile
constexpr int SEG = KT / 2;      // bytes per (row, tile) segment

__host__ __device__ inline int64_t k_tiles(int64_t K) { return (K + KT - 1) / KT; }
__host__ __device__ inline int64_t packed_bytes(int64_t rows, int64_t K) { return k_tiles(K) * rows * SEG; }

// error text of the calling thread (set by the API layer)
void set_error(const char *fmt, ...);

// kernel launchers (each returns a hipError_t from hipGetLastError after the launch)
hipError_t launch_pack_weights(const int8_t *w, int64_t N, int64_t K, uint8_t *out, hipStream_t s);
hipError_t launch_unpack(const uint8_t *packed, int64_t rows, int64_t K, int8_t *out, hipStream_t s);
hipError_t launch_quantize_act(const uint16_t *x, int64_t M, int64_t K, int mode, float eps, const float *row_in,
                               float inv_s_a, int zero_point, uint8_t *out, float *row_out, hipStream_t s);
hipError_t launch_residual_norm_quantize(const uint16_t *xr, const uint16_t *yb, int64_t M, int64_t K, const float *s_prev,
                                         float eps, float inv_s_a, uint16_t *x_next, float *s_next, uint8_t *out, hipStream_t s);
hipError_t launch_weight_row_sums(const int8_t *w, int64_t N, int64_t K, int32_t *sums, hipStream_t s);
hipError_t launch_quantize_act_dynamic(const uint16_t *x, int64_t M, int64_t K, uint8_t *out, float *s_out, hipStream_t s);
hipError_t launch_quantize_act_hadamard(const uint16_t *x, int64_t M, int64_t K, int hadamard_block, int mode, float eps,
                                        const float *row_in, float inv_s_a, uint8_t *out, float *row_out, hipStream_t s);
hipError_t launch_linear_ref(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                             hipStream_t s);
hipError_t launch_linear_mfma(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                              const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                              hipStream_t s);
hipError_t launch_linear_mfma_ws(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                 const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                                 int32_t *ws, int64_t ws_bytes, hipStream_t s);
int64_t linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
hipError_t launch_linear_decode(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                                hipStream_t s);

void set_gemm_tile(int tile);
void set_gemm_map(int mode);
int forced_gemm_tile();
bool set_decode_shape(int code);

// What a linear call would launch: kernel (template instance or name), workgroups, threads per workgroup.
struct LinearPlan {
    char kernel[96];
    int64_t workgroups;
    int threads;
};
void linear_mfma_plan(int64_t M, int64_t N, int64_t K, bool with_workspace, LinearPlan *plan);

// Per-device state, set up once per device (by fptq_init or by the first call that needs it; thread-safe):
// the number of compute units, which the launchers size their grids and pick their tile shapes by, and the
// device address of the library's built-in scratch area (fptq_w4a4_linear_noalloc).
constexpr int MAX_DEVICES = 64;
constexpr int DEFAULT_CUS = 256;                 // MI355X; used by the host-only size queries when no device answers
struct DeviceInfo {
    int device;
    int cus;
    int32_t *scratch;
    int64_t scratch_bytes;
};
hipError_t device_info(const DeviceInfo **out);  // state of the current device
int device_cus_or_default();                     // compute units of the current device, DEFAULT_CUS without one
// what each translation unit contributes to that set-up (called with the device current, under the set-up lock)
hipError_t gemm_device_init(DeviceInfo *info);
hipError_t hadamard_device_init(int device);

// fp32 -> bf16 bit pattern, round to nearest even (NaN stays a quiet NaN)
__device__ inline uint16_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// ss + v * v in fp64 for an fp32 v: the square of a value with at most 24 significant bits is exact in fp64, so the
// fused form rounds once, exactly like the separate multiply and add of the definition.
__device__ inline double add_square(double ss, float v)
{
    const double a = (double)v;
    return __builtin_fma(a, a, ss);
}

// Core of every activation quantizer: the code q + 8 in [0, 15] of q = clamp(rne(x * c) + z, -8, 7), NaN -> z,
// with zoff = z + 8.  v_cvt_i32_f32 saturates and turns NaN into 0, the add saturates too, so infinities and
// huge products end at the clamp like everything else: the same integers as rounding, adding and clamping in
// float.  XOR with 8 turns the code into the two's complement nibble (eight at a time: CODE_TO_NIBBLES).
__device__ inline uint32_t quant_code(float x, float c, int zoff)
{
    const float r = __builtin_rintf(x * c);
    int i, j;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(i) : "v"(r));
    asm("v_add_i32 %0, %1, %2 clamp" : "=v"(j) : "v"(i), "v"(zoff));
    return (uint32_t)min(max(j, 0), 15);
}
constexpr uint32_t CODE_TO_NIBBLES = 0x88888888u;

// Zero-point correction of an accumulator: sum_k (v - z) w = acc - z * sum_k w (wsum == NULL: symmetric grid).
__device__ inline int32_t remove_zero_point(int32_t acc, int zp, const int32_t *wsum, int64_t o)
{
    return wsum ? acc - zp * wsum[o] : acc;
}

// The dequantizing epilogue of the layer for one output: fp32 throughout, no fused operations.
__device__ inline uint16_t dequant_bf16(int32_t acc, float cw, const float *d, int64_t t)
{
    float yf = (float)acc * cw;
    if (d) yf = yf * d[t];
    return bf16_rne(yf);
}

}  // namespace fptq
