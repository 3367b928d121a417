// Online Hadamard transform in front of the down projection (Sec. 3.1.4 and App. D, "Hadamard
// non-powers of 2" of the paper), fused with the per-token scale, the static INT4 quantizer and
// the packer: x -> clamp(rne((x H_B / sqrt(B)) * S_t / s_a), -8, 7), block-wise over consecutive
// groups of B channels (B = 256, 512, 1024, 2048 or 4096: the largest power of two dividing the
// down projection's width is 256 for 11008, 2048 for 14336, 4096 for 28672), one pass over X.
//
// The transform is evaluated by the in-place butterfly network in fp32 with strides
// 128, 64, ..., 1, each pair (a, b) -> (a + b, a - b): every output is a fixed tree of fp32
// additions, so the result does not depend on how the work is spread over lanes.
//
// B = 256.  One wave per token row; a wave walks the row in super-chunks of 1024 values = 4 blocks, a
// block per 16 lanes, 16 values per lane.  The four high strides need the lane to hold
// x[16 j + g] (j = 0..15), the four low strides x[16 g + e]: the raw bf16 values go through LDS
// once to get the strided view, the fp32 intermediates once more to get the contiguous view
// (padded so that both directions are bank-conflict free).  Everything is wave-private: no
// barriers.  Roofline: HBM (2 bytes read, half a byte written per value), with about 16 VALU
// operations per value close behind.
//
// B = 64 V with V = 8, 16, 32, 64.  One block per wave iteration, V values per lane.  View 1: the lane
// holds x[64 j + lane] and runs strides B/2 .. 64 in registers; view 2: the lane holds
// x[V lane + e] and runs strides V/2 .. 1 in registers; the strides in between (32 .. V) pair lane l with
// lane l ^ (stride / V) and are done with DPP lane exchanges, in descending order between the two
// register passes, so the stage order is that of the definition.  The raw block and the fp32
// transposition patch share the wave's LDS region (a wave's LDS operations complete in order).
#include "fptq_common.h"

namespace fptq {

constexpr int HB = 256;                 // Hadamard block
constexpr int H_RAW_BLK = 544;          // bytes per block of raw bf16 in LDS (512 + 32: blocks land on different banks)
constexpr int H_F32_ROW = 20;           // words per 16-value row of the fp32 transpose patch (16 + 4)
constexpr int H_F32_BLK = 336;          // words per block of the patch (16 * 20 + 16)
constexpr int H_WAVE_LDS = 4 * H_RAW_BLK + 4 * H_F32_BLK * 4;   // 7552 bytes

__device__ inline float h_bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

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
                                                                    float *__restrict__ row_out, int ksplit)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * H_WAVE_LDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // ksplit waves share a row: wave `part` of them takes every ksplit-th group of four blocks
    const int64_t wid = (int64_t)blockIdx.x * 4 + wave, t = wid / ksplit;
    const int part = (int)(wid % ksplit);
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
                ss = __builtin_fma(a, a, ss);
                ss = __builtin_fma(b, b, ss);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        r = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    } else if (MODE == FPTQ_SCALE_GIVEN) {
        r = row_in[t];
    }
    const float c = ((MODE == FPTQ_SCALE_NONE) ? inv_s_a : r * inv_s_a) * hnorm;
    if (lane == 0 && part == 0 && row_out) row_out[t] = r;

    const int b = lane >> 4, g = lane & 15;
    uint8_t *raw = lds + wave * H_WAVE_LDS + b * H_RAW_BLK;
    float *patch = reinterpret_cast<float *>(lds + wave * H_WAVE_LDS + 4 * H_RAW_BLK) + b * H_F32_BLK;

    for (int64_t sc = (int64_t)part * (4 * HB); sc < K; sc += (int64_t)ksplit * (4 * HB)) {
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
                w0 |= quant_code(v[e], c, 8) << (4 * e);
                w1 |= quant_code(v[8 + e], c, 8) << (4 * e);
            }
            w0 ^= CODE_TO_NIBBLES, w1 ^= CODE_TO_NIBBLES;
            *reinterpret_cast<uint2 *>(out + ((k0 / KT) * M + t) * SEG + (k0 % KT) / 2) = make_uint2(w0, w1);
        }
    }
}


// ---------------------------------------------------------------------------------- B = 512 .. 4096
template <int V>
__device__ inline void butterflies(float (&v)[V])
{
#pragma unroll
    for (int s = V / 2; s >= 1; s >>= 1)
#pragma unroll
        for (int j = 0; j < V; ++j)
            if ((j & s) == 0) {
                float a = v[j], b = v[j + s];
                v[j] = a + b;
                v[j + s] = a - b;
            }
}

// value of lane (l ^ MASK), MASK = 1, 2 (DPP quad permutation) or 4 (swizzle within 32 lanes)
template <int MASK>
__device__ inline float lane_xor(float x)
{
    const int i = __float_as_int(x);
    if (MASK == 1) return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    if (MASK == 2) return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    return __int_as_float(__builtin_amdgcn_ds_swizzle(i, 0x101F));                                   // and 0x1f, xor 4
}

// one butterfly stage across lanes: the lower lane of a pair gets a + b, the upper one a - b, where a
// is the lower lane's value: both are other + (upper ? -own : own), and negation is exact
template <int MASK, int V>
__device__ inline void cross_stage(float (&v)[V], int lane)
{
    const uint32_t flip = (lane & MASK) ? 0x80000000u : 0u;
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = lane_xor<MASK>(v[e]) + __uint_as_float(__float_as_uint(v[e]) ^ flip);
}

template <int MODE, int V>
__global__ __launch_bounds__(256) void quantize_act_hadamard_wide_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                                                         float eps, const float *__restrict__ row_in,
                                                                         float inv_s_a, float hnorm, uint8_t *__restrict__ out,
                                                                         float *__restrict__ row_out, int ksplit)
{
    constexpr int B = 64 * V;
    constexpr int WAVE_WORDS = B + 256;          // fp32 patch: 4 pad words after every V elements (64 groups)
    extern __shared__ __attribute__((aligned(16))) uint8_t wide_lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t wid = (int64_t)blockIdx.x * 4 + wave, t = wid / ksplit;     // ksplit waves share a row, block by block
    const int part = (int)(wid % ksplit);
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
                ss = __builtin_fma(a, a, ss);
                ss = __builtin_fma(b, b, ss);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        r = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    } else if (MODE == FPTQ_SCALE_GIVEN) {
        r = row_in[t];
    }
    const float c = ((MODE == FPTQ_SCALE_NONE) ? inv_s_a : r * inv_s_a) * hnorm;
    if (lane == 0 && part == 0 && row_out) row_out[t] = r;

    uint8_t *raw = wide_lds + wave * (WAVE_WORDS * 4);
    float *patch = reinterpret_cast<float *>(raw);

    for (int64_t sc = (int64_t)part * B; sc < K; sc += (int64_t)ksplit * B) {
        // linear copy of the block into LDS, 1 KB per wave-level load
#pragma unroll
        for (int i = 0; i < V / 8; ++i)
            *reinterpret_cast<uint4 *>(raw + (i * 64 + lane) * 16) = *reinterpret_cast<const uint4 *>(row + sc + (i * 64 + lane) * 8);
        float v[V];
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = h_bf16_to_f32(*reinterpret_cast<const uint16_t *>(raw + (64 * j + lane) * 2));
        butterflies<V>(v);                                // strides B/2 .. 64
        // element e = 64 j + lane goes to word e + 4 (e / V); the lane then reads its V contiguous elements
#pragma unroll
        for (int j = 0; j < V; ++j) patch[j * (64 + 256 / V) + lane + 4 * (lane / V)] = v[j];
#pragma unroll
        for (int i = 0; i < V / 4; ++i) {
            const float4 f = *reinterpret_cast<const float4 *>(patch + lane * (V + 4) + 4 * i);
            v[4 * i] = f.x, v[4 * i + 1] = f.y, v[4 * i + 2] = f.z, v[4 * i + 3] = f.w;
        }
        if (V <= 8) cross_stage<4, V>(v, lane);           // stride 32 at V = 8
        if (V <= 16) cross_stage<2, V>(v, lane);          // stride 32 at V = 16, stride 16 at V = 8
        if (V <= 32) cross_stage<1, V>(v, lane);          // stride V
        butterflies<V>(v);                                // strides V/2 .. 1
        uint32_t w[V / 8];
#pragma unroll
        for (int i = 0; i < V / 8; ++i) {
            w[i] = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) w[i] |= quant_code(v[8 * i + e], c, 8) << (4 * e);
            w[i] ^= CODE_TO_NIBBLES;
        }
        const int64_t k0 = sc + (int64_t)V * lane;        // V <= 128 values never straddle a K tile
        uint8_t *dst = out + ((k0 / KT) * M + t) * SEG + (k0 % KT) / 2;
        if (V == 8) *reinterpret_cast<uint32_t *>(dst) = w[0];
        if (V == 16) *reinterpret_cast<uint2 *>(dst) = make_uint2(w[0], w[1]);
        if (V >= 32) {
#pragma unroll
            for (int i = 0; i < V / 32; ++i)
                *reinterpret_cast<uint4 *>(dst + 16 * i) = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
        }
    }
}

// Waves per row: with few rows a wave per row leaves the device idle (one token of 11008 values took 9.5 us, as
// long as 512 tokens), so the blocks of a row are dealt to as many waves as it takes to have about 4096 in all
// (16384 was slower again: 2048 x 11008 17.1 us against 13.9).
// In RMS mode every wave of a row sums the whole row again, which only pays while there are few rows.
static int waves_per_row(int64_t M, int64_t chunks, int mode)
{
    if (M >= 4096 || (mode == FPTQ_SCALE_RMS && M > 256)) return 1;
    const int64_t want = (4096 + M - 1) / M;
    return (int)(want < chunks ? want : chunks);
}

constexpr int wide_lds_bytes(int v) { return 4 * (64 * v + 256) * 4; }

template <int MODE, int V>
static hipError_t set_wide_attribute()
{
    if (wide_lds_bytes(V) <= 65536) return hipSuccess;
    return hipFuncSetAttribute((const void *)quantize_act_hadamard_wide_kernel<MODE, V>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               wide_lds_bytes(V));
}

// Once per device: more than 64 KB of dynamic LDS has to be asked for before the first launch.
hipError_t hadamard_device_init(int)
{
    hipError_t e = hipSuccess;
    auto one = [&](hipError_t r) { if (e == hipSuccess) e = r; };
#define FPTQ_WIDE_ATTR(V) one(set_wide_attribute<FPTQ_SCALE_NONE, V>()), one(set_wide_attribute<FPTQ_SCALE_RMS, V>()), one(set_wide_attribute<FPTQ_SCALE_GIVEN, V>())
    FPTQ_WIDE_ATTR(8);
    FPTQ_WIDE_ATTR(16);
    FPTQ_WIDE_ATTR(32);
    FPTQ_WIDE_ATTR(64);
#undef FPTQ_WIDE_ATTR
    return e;
}

template <int V>
static hipError_t launch_wide(const uint16_t *x, int64_t M, int64_t K, int mode, float eps, const float *row_in, float inv_s_a,
                              uint8_t *out, float *row_out, hipStream_t s)
{
    const int ksplit = waves_per_row(M, (K + 64 * V - 1) / (64 * V), mode);
    const int64_t blocks = (M * ksplit + 3) / 4;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    constexpr int LDS_BYTES = wide_lds_bytes(V);
    const DeviceInfo *info;
    hipError_t e0 = device_info(&info);       // the kernels that need more than 64 KB of dynamic LDS got their limit there
    if (e0 != hipSuccess) return e0;
    const float hnorm = (float)(1.0 / sqrt((double)(64 * V)));
    dim3 grid((unsigned)blocks), block(256);
#define FPTQ_LAUNCH_WIDE(MODE)                                                                                             \
    do {                                                                                                                   \
        auto kern = quantize_act_hadamard_wide_kernel<MODE, V>;                                                            \
        kern<<<grid, block, LDS_BYTES, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out, ksplit);                   \
    } while (0)
    switch (mode) {
    case FPTQ_SCALE_NONE: FPTQ_LAUNCH_WIDE(FPTQ_SCALE_NONE); break;
    case FPTQ_SCALE_RMS: FPTQ_LAUNCH_WIDE(FPTQ_SCALE_RMS); break;
    default: FPTQ_LAUNCH_WIDE(FPTQ_SCALE_GIVEN);
    }
#undef FPTQ_LAUNCH_WIDE
    return hipGetLastError();
}

hipError_t launch_quantize_act_hadamard(const uint16_t *x, int64_t M, int64_t K, int hadamard_block, int mode, float eps,
                                        const float *row_in, float inv_s_a, uint8_t *out, float *row_out, hipStream_t s)
{
    switch (hadamard_block) {
    case 512: return launch_wide<8>(x, M, K, mode, eps, row_in, inv_s_a, out, row_out, s);
    case 1024: return launch_wide<16>(x, M, K, mode, eps, row_in, inv_s_a, out, row_out, s);
    case 2048: return launch_wide<32>(x, M, K, mode, eps, row_in, inv_s_a, out, row_out, s);
    case 4096: return launch_wide<64>(x, M, K, mode, eps, row_in, inv_s_a, out, row_out, s);
    case 256: break;
    default: return hipErrorInvalidValue;
    }
    const int ksplit = waves_per_row(M, (K + 4 * HB - 1) / (4 * HB), mode);
    const int64_t blocks = (M * ksplit + 3) / 4;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    const float hnorm = 1.0f / 16.0f;       // 1 / sqrt(256)
    dim3 grid((unsigned)blocks), block(256);
    switch (mode) {
    case FPTQ_SCALE_NONE:
        quantize_act_hadamard_kernel<FPTQ_SCALE_NONE><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out, ksplit);
        break;
    case FPTQ_SCALE_RMS:
        quantize_act_hadamard_kernel<FPTQ_SCALE_RMS><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out, ksplit);
        break;
    default:
        quantize_act_hadamard_kernel<FPTQ_SCALE_GIVEN><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, hnorm, out, row_out, ksplit);
    }
    return hipGetLastError();
}

}  // namespace fptq
