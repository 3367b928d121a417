// One step of the scaled residual stream of Sec. 3.1.3 (Eq. 5-7 of the paper), fused with the
// quantizer of the next block's input: Z~ = X~ + Y~, nrm = RMS(Z~), S_n = S_{n-1} / nrm,
// X~_n = Z~ / nrm (new residual = gain-free RMSNorm output), q = clamp(rne(X~_n / s_a), -8, 7),
// packed.  One pass: both inputs are read once, the sum stays in registers as fp32 between the
// fp64 reduction and the two outputs.  Bound: HBM, 4 bytes read and 2.5 bytes written per value.
//
// fp32 recipe: z = (float)x + (float)y; inv = (float)(1 / sqrt(sum z^2 / K + eps)) with the sum in
// fp64; S_n = S_{n-1} * inv; X~_n = bf16(z * inv); c = inv * (1.0f / s_a); q = clamp(rne(z * c)).
#include "fptq_common.h"

namespace fptq {

__device__ inline float r_bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

typedef unsigned int r_v4u __attribute__((ext_vector_type(4)));
typedef __bf16 r_bf16x2 __attribute__((ext_vector_type(2)));
typedef float r_float2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t r_pack_bf16(float lo, float hi)
{
    r_float2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, r_bf16x2));
}

// WPR waves per row: 1 (four rows per workgroup; no LDS, no barrier: for many short rows) or 4 (a workgroup per
// row).  CH > 0: K % 8 == 0, K <= 512 * WPR * CH, rows 16-byte aligned, z kept in registers.
// CH == 0 (WPR = 1): any K, the inputs are read twice (the second time from cache).
// x_next may be the same buffer as xr or yb (the update in place), so none of the three is declared restrict: every
// thread reads an element of its row before it stores that element, and no thread touches another's elements.
template <int CH, int WPR>
__global__ __launch_bounds__(256) void residual_norm_quantize_kernel(const uint16_t *xr, const uint16_t *yb,
                                                                     int64_t M, int64_t K, const float *__restrict__ s_prev,
                                                                     float eps, float inv_s_a, uint16_t *x_next,
                                                                     float *__restrict__ s_next, uint8_t *__restrict__ out)
{
    static_assert(WPR == 1 || (WPR == 4 && CH > 0), "a wave or a workgroup per row");
    __shared__ double red[4];
    constexpr int S = 64 * WPR;                          // threads per row
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = WPR == 1 ? lane : (int)threadIdx.x;    // this thread's place in its row
    const int64_t t = WPR == 1 ? (int64_t)blockIdx.x * 4 + wave : (int64_t)blockIdx.x;
    if (t >= M) return;                                  // WPR = 1: whole waves leave and nothing below synchronises
    const uint16_t *xrow = xr + t * K, *yrow = yb + t * K;
    uint16_t *orow = x_next + t * K;
    const int64_t Kpad = k_tiles(K) * KT;

    float z[CH > 0 ? CH : 1][8];
    double ss = 0.0;
    if (CH > 0) {      // both rows through row-sized buffer descriptors: chunks past the end read as zero, no branches
        const __amdgpu_buffer_rsrc_t xs = __builtin_amdgcn_make_buffer_rsrc((void *)xrow, 0, (int)K * 2, 0x00020000);
        const __amdgpu_buffer_rsrc_t ys = __builtin_amdgcn_make_buffer_rsrc((void *)yrow, 0, (int)K * 2, 0x00020000);
        r_v4u a[CH > 0 ? CH : 1], b[CH > 0 ? CH : 1];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            a[i] = __builtin_amdgcn_raw_buffer_load_b128(xs, (i * S + h) * 16, 0, 0);
            b[i] = __builtin_amdgcn_raw_buffer_load_b128(ys, (i * S + h) * 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t aw[4] = {a[i].x, a[i].y, a[i].z, a[i].w}, bw[4] = {b[i].x, b[i].y, b[i].z, b[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                z[i][2 * j] = r_bf16_to_f32(aw[j] & 0xffffu) + r_bf16_to_f32(bw[j] & 0xffffu);
                z[i][2 * j + 1] = r_bf16_to_f32(aw[j] >> 16) + r_bf16_to_f32(bw[j] >> 16);
                ss = add_square(ss, z[i][2 * j]);
                ss = add_square(ss, z[i][2 * j + 1]);
            }
        }
    } else {
        for (int64_t k = lane; k < K; k += 64) {
            const float v = r_bf16_to_f32(xrow[k]) + r_bf16_to_f32(yrow[k]);
            ss = add_square(ss, v);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (WPR > 1) {
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        ss = (red[0] + red[1]) + (red[2] + red[3]);      // the same order in every thread
    }
    const float inv = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    if (h == 0) s_next[t] = (s_prev ? s_prev[t] : 1.0f) * inv;
    const float c = inv * inv_s_a;

    if (CH > 0) {
        uint8_t *prow = out + (((int64_t)(h >> 4) * M + t) * SEG + (h & 15) * 4);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int k0 = (i * S + h) * 8;
            uint32_t word = 0, o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o[j] = r_pack_bf16(z[i][2 * j] * inv, z[i][2 * j + 1] * inv);
                word |= quant_code(z[i][2 * j], c, 8) << (8 * j);
                word |= quant_code(z[i][2 * j + 1], c, 8) << (8 * j + 4);
            }
            word ^= CODE_TO_NIBBLES;
            if (k0 < (int)K) *reinterpret_cast<uint4 *>(orow + k0) = make_uint4(o[0], o[1], o[2], o[3]);
            else word = 0u;                                      // K padding stays zero
            if (k0 < (int)Kpad) *reinterpret_cast<uint32_t *>(prow + (int64_t)((S / 16) * i) * M * SEG) = word;
        }
    } else {
        for (int64_t k0 = (int64_t)lane * 8; k0 < Kpad; k0 += 512) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int64_t k = k0 + e;
                if (k < K) {
                    const float v = r_bf16_to_f32(xrow[k]) + r_bf16_to_f32(yrow[k]);
                    orow[k] = (uint16_t)(r_pack_bf16(v * inv, 0.0f) & 0xffffu);
                    word |= (quant_code(v, c, 8) ^ 8u) << (4 * e);
                }
            }
            *reinterpret_cast<uint32_t *>(out + ((k0 / KT) * M + t) * SEG + (k0 % KT) / 2) = word;
        }
    }
}

hipError_t launch_residual_norm_quantize(const uint16_t *xr, const uint16_t *yb, int64_t M, int64_t K, const float *s_prev,
                                         float eps, float inv_s_a, uint16_t *x_next, float *s_next, uint8_t *out, hipStream_t s)
{
    const int64_t blocks = (M + 3) / 4;
    if (M > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), rows((unsigned)M), block(256);
    const bool vec = K % 8 == 0 && ((reinterpret_cast<uintptr_t>(xr) | reinterpret_cast<uintptr_t>(yb) |
                                     reinterpret_cast<uintptr_t>(x_next)) & 15) == 0;
    // As for the plain quantizer: a wave per row for many short rows (2048 x 4096: 10.2 us), otherwise a workgroup per
    // row, which spreads a row over four waves (32 x 4096: 4.3 us with a wave per row).
    if (vec && K <= 4096 && M > 768) {
        if (K <= 2048)
            residual_norm_quantize_kernel<4, 1><<<grid, block, 0, s>>>(xr, yb, M, K, s_prev, eps, inv_s_a, x_next, s_next, out);
        else
            residual_norm_quantize_kernel<8, 1><<<grid, block, 0, s>>>(xr, yb, M, K, s_prev, eps, inv_s_a, x_next, s_next, out);
        return hipGetLastError();
    }
#define FPTQ_RES_CASE(CH)                                                                                                       \
    if (vec && K <= 2048 * CH) {                                                                                                \
        residual_norm_quantize_kernel<CH, 4><<<rows, block, 0, s>>>(xr, yb, M, K, s_prev, eps, inv_s_a, x_next, s_next, out);   \
        return hipGetLastError();                                                                                               \
    }
    FPTQ_RES_CASE(1)
    FPTQ_RES_CASE(2)
    FPTQ_RES_CASE(3)
    FPTQ_RES_CASE(4)
    FPTQ_RES_CASE(6)
    FPTQ_RES_CASE(8)
#undef FPTQ_RES_CASE
    residual_norm_quantize_kernel<0, 1><<<grid, block, 0, s>>>(xr, yb, M, K, s_prev, eps, inv_s_a, x_next, s_next, out);
    return hipGetLastError();
}

}  // namespace fptq
