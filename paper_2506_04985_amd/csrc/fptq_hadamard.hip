// Online Hadamard transform in front of the down projection (Sec. 3.1.4 and App. D, "Hadamard
// non-powers of 2" of the paper), fused with the per-token scale, the static INT4 quantizer and
// the packer: x -> clamp(rne((x H_256 / 16) * S_t / s_a), -8, 7), block-wise over consecutive
// groups of 256 channels, one pass over X.
//
// The transform is evaluated by the in-place butterfly network in fp32 with strides
// 128, 64, ..., 1, each pair (a, b) -> (a + b, a - b): every output is a fixed tree of fp32
// additions, so the result does not depend on how the work is spread over lanes.
//
// One wave per token row; a wave walks the row in super-chunks of 1024 values = 4 blocks, a
// block per 16 lanes, 16 values per lane.  The four high strides need the lane to hold
// x[16 j + g] (j = 0..15), the four low strides x[16 g + e]: the raw bf16 values go through LDS
// once to get the strided view, the fp32 intermediates once more to get the contiguous view
// (padded so that both directions are bank-conflict free).  Everything is wave-private: no
// barriers.  Roofline: HBM (2 bytes read, half a byte written per value), with about 16 VALU
// operations per value close behind.
#include "fptq_common.h"

namespace fptq {

constexpr int HB = 256;                 // Hadamard block
constexpr int H_RAW_BLK = 544;          // bytes per block of raw bf16 in LDS (512 + 32: blocks land on different banks)
constexpr int H_F32_ROW = 20;           // words per 16-value row of the fp32 transpose patch (16 + 4)
constexpr int H_F32_BLK = 336;          // words per block of the patch (16 * 20 + 16)
constexpr int H_WAVE_LDS = 4 * H_RAW_BLK + 4 * H_F32_BLK * 4;   // 7552 bytes

__device__ inline float h_bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

__device__ inline uint32_t h_quant_nibble(float x, float c)
{
    float u = x * c;
    float r = __builtin_rintf(u);
    r = fminf(fmaxf(r, -8.0f), 7.0f);
    int q = (u != u) ? 0 : (int)r;
    return (uint32_t)q & 15u;
}

__device__ inline void butterflies16(float (&v)[16])
{
#pragma unroll
    for (int s = 8; s >= 1; s >>= 1)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if ((j & s) == 0) {
                float a = v[j], b = v[j + s];
                v[j] = a + b;
                v[j + s] = a - b;
            }
}

template <int MODE>
__global__ __launch_bounds__(256) void quantize_act_hadamard_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                                                    float eps, const float *__restrict__ row_in,
                                                                    float inv_s_a, float hnorm, uint8_t *__restrict__ out,
                                                                    float *__restrict__ row_out)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * H_WAVE_LDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 4 + wave;
    if (t >= M) return;                                  // whole waves leave; nothing below synchronises
    const uint16_t *row = x + t * K;

    float r = 1.0f;
    if (MODE == FPTQ_SCALE_RMS) {                        // S_t from the row as the norm layer sees it
        double ss = 0.0;
        for (int64_t k0 = (int64_t)lane * 8; k0 < K; k0 += 512) {
            const uint4 u = *reinterpret_cast<const uint4 *>(row + k0);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                double a = (double)h_bf16_to_f32(w[j] & 0xffffu), b = (double)h_bf16_to_f32(w[j] >> 16);
                ss += a * a;
                ss += b * b;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        r = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    } else if (MODE == FPTQ_SCALE_GIVEN) {
        r = row_in[t];
    }
    const float c = ((MODE == FPTQ_SCALE_NONE) ? inv_s_a : r * inv_s_a) * hnorm;
    if (lane == 0 && row_out) row_out[t] = r;

    const int b = lane >> 4, g = lane & 15;
    uint8_t *raw = lds + wave * H_WAVE_LDS + b * H_RAW_BLK;
    float *patch = reinterpret_cast<float *>(lds + wave * H_WAVE_LDS + 4 * H_RAW_BLK) + b * H_F32_BLK;

    for (int64_t sc = 0; sc < K; sc += 4 * HB) {
        const int64_t k0 = sc + b * HB + 16 * g;          // first of this lane's 16 contiguous values
        const bool live = sc + b * HB < K;
        if (live) {
            const uint4 lo = *reinterpret_cast<const uint4 *>(row + k0), hi = *reinterpret_cast<const uint4 *>(row + k0 + 8);
            *reinterpret_cast<uint4 *>(raw + g * 32) = lo;
            *reinterpret_cast<uint4 *>(raw + g * 32 + 16) = hi;
        }
        // strided view x[16 j + g]: strides 128, 64, 32, 16 of the block are strides 8, 4, 2, 1 in j
        float v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = h_bf16_to_f32(*reinterpret_cast<const uint16_t *>(raw + (16 * j + g) * 2));
        butterflies16(v);
        // transpose inside the block: value (j, g) to row j, column g; read back row g
#pragma unroll
        for (int j = 0; j < 16; ++j) patch[H_F32_ROW * j + g] = v[j];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 f = *reinterpret_cast<const float4 *>(patch + H_F32_ROW * g + 4 * i);
            v[4 * i] = f.x, v[4 * i + 1] = f.y, v[4 * i + 2] = f.z, v[4 * i + 3] = f.w;
        }
        butterflies16(v);                                 // contiguous view: strides 8, 4, 2, 1
        if (live) {
            uint32_t w0 = 0, w1 = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                w0 |= h_quant_nibble(v[e], c) << (4 * e);
                w1 |= h_quant_nibble(v[8 + e], c) << (4 * e);
            }
            *reinterpret_cast<uint2 *>(out + ((k0 / KT) * M + t) * SEG + (k0 % KT) / 2) = make_uint2(w0, w1);
        }
    }
}

hipError_t launch_quantize_act_hadamard(const uint16_t *x, int64_t M, int64_t K, int mode, float eps, const float *row_in,
                                        float inv_s_a, uint8_t *out, float *row_out, hipStream_t s)
{
    const int64_t blocks = (M + 3) / 4;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const float hnorm = 1.0f / 16.0f;       // 1 / sqrt(256)
    dim3 grid((unsigned)blocks), block(256);
    switch (mode) {
    case FPTQ_SCALE_NONE:
        quantize_act_hadamard_kernel<FPTQ_SCALE_NONE><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out);
        break;
    case FPTQ_SCALE_RMS:
        quantize_act_hadamard_kernel<FPTQ_SCALE_RMS><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out);
        break;
    default:
        quantize_act_hadamard_kernel<FPTQ_SCALE_GIVEN><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out);
    }
    return hipGetLastError();
}

}  // namespace fptq
