// Activation path of the quantized linear layer: per-token scale (Sec. 3.1.3 Step 1), static
// per-tensor INT4 quantization (App. B) and nibble packing (App. J) in one pass over X.
//
// The row is read once from HBM and kept in registers while the sum of squares is reduced, then
// quantized from the registers.  Bandwidth-bound: 2 bytes read and half a byte written per
// element.  Rows up to 12288 values are handled by one wave each (no LDS, no barrier, the scale is
// computed once per row, and many rows are in flight per CU); longer rows by one workgroup each.
#include "fptq_common.h"

namespace fptq {

constexpr int QT = 256;        // threads per row
constexpr int QCHUNK = 8;      // bf16 values per 16-byte load

__device__ inline float bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

// Eight quantized values of one 16-byte chunk of bf16 as a packed word (value e in nibble e).
__device__ inline uint32_t quant_chunk(const uint32_t (&w)[4], float c, int zoff)
{
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        word |= quant_code(bf16_to_f32(w[j] & 0xffffu), c, zoff) << (8 * j);
        word |= quant_code(bf16_to_f32(w[j] >> 16), c, zoff) << (8 * j + 4);
    }
    return word ^ CODE_TO_NIBBLES;
}

__device__ inline double block_sum(double v, double *lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    double tot = lds[0];
#pragma unroll
    for (int w = 1; w < QT / 64; ++w) tot += lds[w];
    return tot;
}

__device__ inline void store_word(uint8_t *out, int64_t M, int64_t t, int64_t k0, uint32_t word)
{
    *reinterpret_cast<uint32_t *>(out + ((k0 / KT) * M + t) * SEG + (k0 % KT) / 2) = word;
}

typedef unsigned int q_v4u __attribute__((ext_vector_type(4)));
constexpr int Q_STREAM = 2;      // buffer-load cache policy: non-temporal
constexpr int Q_RSRC_FLAGS = 0x00020000;     // raw buffer, bounds-checked: reads past num_records return zero

// One workgroup per row.  CH > 0: K % 8 == 0, 16-byte aligned rows of at most 2048 * CH values, kept in
// registers (CH 16-byte chunks per thread) between the reduction and the quantizer and read through a row-sized
// buffer descriptor, so chunks past the end read as zero and nothing branches but the store of a chunk past
// the padded width.  CH == 0: any K and alignment, two passes over the row.
template <int MODE, int CH>
__global__ __launch_bounds__(QT) void quantize_act_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K, float eps,
                                                          const float *__restrict__ row_in, float inv_s_a, int zoff,
                                                          uint8_t *__restrict__ out, float *__restrict__ row_out, int stream_in)
{
    __shared__ double red[QT / 64];
    const int64_t t = blockIdx.x;
    const uint16_t *row = x + t * K;
    const int64_t Kpad = k_tiles(K) * KT;
    const int tid = threadIdx.x;

    q_v4u regs[CH > 0 ? CH : 1];
    if (CH > 0) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)row, 0, (int)K * 2, Q_RSRC_FLAGS);
        if (stream_in) {         // an input larger than the last-level cache: streaming loads, which do not displace what is there
#pragma unroll
            for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * QT + tid) * 16, 0, Q_STREAM);
        } else {
#pragma unroll
            for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * QT + tid) * 16, 0, 0);
        }
    }

    float r = 1.0f;
    if (MODE == FPTQ_SCALE_RMS) {
        double ss = 0.0;
        if (CH > 0) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // a * a is exact in fp64 (8 significant bits squared), so the fused form rounds like multiply, then add
                    double a = (double)bf16_to_f32(w[j] & 0xffffu), b = (double)bf16_to_f32(w[j] >> 16);
                    ss = __builtin_fma(a, a, ss);
                    ss = __builtin_fma(b, b, ss);
                }
            }
        } else {
            for (int64_t k = tid; k < K; k += QT) {
                double a = (double)bf16_to_f32(row[k]);
                ss = __builtin_fma(a, a, ss);
            }
        }
        ss = block_sum(ss, red);
        r = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
    } else if (MODE == FPTQ_SCALE_GIVEN) {
        r = row_in[t];
    }
    const float c = (MODE == FPTQ_SCALE_NONE) ? inv_s_a : r * inv_s_a;
    if (tid == 0 && row_out) row_out[t] = r;

    if (CH > 0) {
        // chunk i of thread h is values 8 (256 i + h) ..: K tile 16 i + h / 16, byte 4 (h % 16) of the row's segment
        uint8_t *orow = out + (((int64_t)(tid >> 4) * M + t) * SEG + (tid & 15) * 4);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int k0 = (i * QT + tid) * QCHUNK;
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
            uint32_t word = quant_chunk(w, c, zoff);
            if (k0 >= (int)K) word = 0u;                          // K padding stays zero
            if (k0 < (int)Kpad) *reinterpret_cast<uint32_t *>(orow + (int64_t)(16 * i) * M * SEG) = word;
        }
    } else {
        for (int64_t k0 = (int64_t)tid * QCHUNK; k0 < Kpad; k0 += (int64_t)QT * QCHUNK) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < QCHUNK; ++i) {
                int64_t k = k0 + i;
                if (k < K) word |= (quant_code(bf16_to_f32(row[k]), c, zoff) ^ 8u) << (4 * i);   // K padding stays zero
            }
            store_word(out, M, t, k0, word);
        }
    }
}

// One wave per row, for rows of at most 512 * CH values (K % 8 == 0).  The row is read through a
// row-sized buffer descriptor, so chunks past its end read as zero and neither the loads nor the
// quantizer need a branch; only the store of a chunk past the padded width is masked off.
template <int MODE, int CH>
__global__ __launch_bounds__(QT) void quantize_act_wave_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K, float eps,
                                                               const float *__restrict__ row_in, float inv_s_a, int zoff,
                                                               uint8_t *__restrict__ out, float *__restrict__ row_out, int stream_in)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t = (int64_t)blockIdx.x * (QT / 64) + wave;
    if (t >= M) return;
    const int Ki = (int)K, Kpad = (int)(k_tiles(K) * KT);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)(x + t * K), 0, Ki * 2, Q_RSRC_FLAGS);

    q_v4u regs[CH];
    if (stream_in) {
#pragma unroll
        for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * 64 + lane) * 16, 0, Q_STREAM);
    } else {
#pragma unroll
        for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * 64 + lane) * 16, 0, 0);
    }
    float r = 1.0f;
    if (MODE == FPTQ_SCALE_RMS) {
        double ss = 0.0;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                double a = (double)bf16_to_f32(w[j] & 0xffffu), b = (double)bf16_to_f32(w[j] >> 16);
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
    const float c = (MODE == FPTQ_SCALE_NONE) ? inv_s_a : r * inv_s_a;
    if (lane == 0 && row_out) row_out[t] = r;
    // chunk i of lane l is values 8 (64 i + l) ..: K tile 4 i + l / 16, byte 4 (l % 16) of the row's segment
    uint8_t *orow = out + (((int64_t)(lane >> 4) * M + t) * SEG + (lane & 15) * 4);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int k0 = (i * 64 + lane) * QCHUNK;
        const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
        uint32_t word = quant_chunk(w, c, zoff);
        if (k0 >= Ki) word = 0u;                              // K padding stays zero
        if (k0 < Kpad) *reinterpret_cast<uint32_t *>(orow + (int64_t)(4 * i) * M * SEG) = word;
    }
}

// Dynamic quantization (App. B of the paper): the scale is computed at run time per token,
// s_t = max_k |x_t,k| / 7 (NaNs ignored; a zero or infinite maximum gives s_t = 1), then
// q = clamp(rne(x * (1 / s_t)), -8, 7).  One wave per row.  CH > 0: the row (K <= 512 * CH, K % 8 == 0)
// stays in registers between the max reduction and the quantizer; CH == 0: any K, two passes.
__device__ inline uint32_t abs_bits_no_nan(uint32_t h)
{
    uint32_t m = h & 0x7fffu;
    return m > 0x7f80u ? 0u : m;       // bf16 magnitudes order like their bit patterns; NaN does not enter the max
}

template <int CH>
__global__ __launch_bounds__(QT) void quantize_act_dynamic_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                                                  uint8_t *__restrict__ out, float *__restrict__ s_out)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t t = (int64_t)blockIdx.x * (QT / 64) + wave;
    if (t >= M) return;
    const uint16_t *row = x + t * K;
    const int64_t Kpad = k_tiles(K) * KT;

    q_v4u regs[CH > 0 ? CH : 1];
    uint32_t mx = 0;
    if (CH > 0) {      // the row through a row-sized buffer descriptor: chunks past its end read as zero
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)row, 0, (int)K * 2, Q_RSRC_FLAGS);
#pragma unroll
        for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * 64 + lane) * 16, 0, 0);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) mx = max(mx, max(abs_bits_no_nan(w[j] & 0xffffu), abs_bits_no_nan(w[j] >> 16)));
        }
    } else {
        for (int64_t k = lane; k < K; k += 64) mx = max(mx, abs_bits_no_nan(row[k]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, off, 64));
    const float amax = bf16_to_f32(mx);
    const float s = (amax > 0.0f && mx < 0x7f80u) ? amax / 7.0f : 1.0f;
    const float c = 1.0f / s;
    if (lane == 0) s_out[t] = s;

    if (CH > 0) {
        uint8_t *orow = out + (((int64_t)(lane >> 4) * M + t) * SEG + (lane & 15) * 4);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int k0 = (i * 64 + lane) * QCHUNK;
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
            uint32_t word = quant_chunk(w, c, 8);
            if (k0 >= (int)K) word = 0u;                          // K padding stays zero
            if (k0 < (int)Kpad) *reinterpret_cast<uint32_t *>(orow + (int64_t)(4 * i) * M * SEG) = word;
        }
    } else {
        for (int64_t k0 = (int64_t)lane * QCHUNK; k0 < Kpad; k0 += 64 * QCHUNK) {
            uint32_t word = 0;
#pragma unroll
            for (int i = 0; i < QCHUNK; ++i) {
                int64_t k = k0 + i;
                if (k < K) word |= (quant_code(bf16_to_f32(row[k]), c, 8) ^ 8u) << (4 * i);
            }
            store_word(out, M, t, k0, word);
        }
    }
}

// The same with one workgroup per row (rows of at most 2048 * CH values, K % 8 == 0, 16-byte aligned): a row is
// spread over four waves, which is faster whenever rows are long or few.
template <int CH>
__global__ __launch_bounds__(QT) void quantize_act_dynamic_row_kernel(const uint16_t *__restrict__ x, int64_t M, int64_t K,
                                                                      uint8_t *__restrict__ out, float *__restrict__ s_out)
{
    __shared__ uint32_t red[QT / 64];
    const int64_t t = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t Kpad = k_tiles(K) * KT;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)(x + t * K), 0, (int)K * 2, Q_RSRC_FLAGS);
    q_v4u regs[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (i * QT + tid) * 16, 0, 0);
    uint32_t mx = 0;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) mx = max(mx, max(abs_bits_no_nan(w[j] & 0xffffu), abs_bits_no_nan(w[j] >> 16)));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < QT / 64; ++w) mx = max(mx, red[w]);
    const float amax = bf16_to_f32(mx);
    const float s = (amax > 0.0f && mx < 0x7f80u) ? amax / 7.0f : 1.0f;
    const float c = 1.0f / s;
    if (tid == 0) s_out[t] = s;
    uint8_t *orow = out + (((int64_t)(tid >> 4) * M + t) * SEG + (tid & 15) * 4);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int k0 = (i * QT + tid) * QCHUNK;
        const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
        uint32_t word = quant_chunk(w, c, 8);
        if (k0 >= (int)K) word = 0u;                          // K padding stays zero
        if (k0 < (int)Kpad) *reinterpret_cast<uint32_t *>(orow + (int64_t)(16 * i) * M * SEG) = word;
    }
}

hipError_t launch_quantize_act_dynamic(const uint16_t *x, int64_t M, int64_t K, uint8_t *out, float *s_out, hipStream_t s)
{
    const int64_t blocks = (M + QT / 64 - 1) / (QT / 64);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(QT);
    const bool vec = K % QCHUNK == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
    const int64_t Kpad = k_tiles(K) * KT;
    // as for the static quantizer: a wave per row only for many short rows, otherwise a workgroup per row
    if (vec && Kpad <= 512 * 8 && M > 768) {
        if (Kpad <= 512 * 4)
            quantize_act_dynamic_kernel<4><<<grid, block, 0, s>>>(x, M, K, out, s_out);
        else
            quantize_act_dynamic_kernel<8><<<grid, block, 0, s>>>(x, M, K, out, s_out);
        return hipGetLastError();
    }
    if (M > 0x7fffffff) return hipErrorInvalidValue;
#define FPTQ_DYN_CASE(CH)                                                                          \
    if (vec && Kpad <= 2048 * CH) {                                                                \
        quantize_act_dynamic_row_kernel<CH><<<dim3((unsigned)M), block, 0, s>>>(x, M, K, out, s_out); \
        return hipGetLastError();                                                                  \
    }
    FPTQ_DYN_CASE(1)
    FPTQ_DYN_CASE(2)
    FPTQ_DYN_CASE(4)
    FPTQ_DYN_CASE(6)
    FPTQ_DYN_CASE(7)
    FPTQ_DYN_CASE(8)
    FPTQ_DYN_CASE(12)
    FPTQ_DYN_CASE(14)
    FPTQ_DYN_CASE(16)
#undef FPTQ_DYN_CASE
    quantize_act_dynamic_kernel<0><<<grid, block, 0, s>>>(x, M, K, out, s_out);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_mode(const uint16_t *x, int64_t M, int64_t K, float eps, const float *row_in, float inv_s_a,
                              int zoff, uint8_t *out, float *row_out, hipStream_t s)
{
    dim3 grid((unsigned)M), block(QT);
    const bool vec = K % QCHUNK == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
    const int64_t Kpad = k_tiles(K) * KT;
    // An input that the 256 MB last-level cache cannot hold is read with streaming loads (8192 x 28672: 119 us
    // against 142); a smaller one is usually still there from its producer, and ordinary loads are faster on it.
    const int stream_in = M * K * 2 > ((int64_t)256 << 20) ? 1 : 0;
    // A wave per row pays only for short rows in large numbers (measured crossover at 4096 values: about 1000
    // rows); otherwise a workgroup per row, which spreads a row over four waves (32 x 11008: 2.9 us against 5.6;
    // 2048 x 11008: 10.8 against 12.9; 2048 x 4096 the other way, 6.0 against 5.3).
    if (vec && Kpad <= 512 * 8 && M > 768) {
        dim3 wgrid((unsigned)((M + QT / 64 - 1) / (QT / 64)));
        if (Kpad <= 512 * 4)
            quantize_act_wave_kernel<MODE, 4><<<wgrid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, zoff, out, row_out, stream_in);
        else
            quantize_act_wave_kernel<MODE, 8><<<wgrid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, zoff, out, row_out, stream_in);
        return hipGetLastError();
    }
#define FPTQ_ROW_CASE(CH)                                                                                                   \
    if (vec && Kpad <= 2048 * CH) {                                                                                         \
        quantize_act_kernel<MODE, CH><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, zoff, out, row_out, stream_in);            \
        return hipGetLastError();                                                                                           \
    }
    // chunks per thread: 6 covers the Llama-2 FFN width 11008, 7 and 14 are the Llama-3 FFN widths 14336 and 28672
    FPTQ_ROW_CASE(1)
    FPTQ_ROW_CASE(2)
    FPTQ_ROW_CASE(4)
    FPTQ_ROW_CASE(6)
    FPTQ_ROW_CASE(7)
    FPTQ_ROW_CASE(8)
    FPTQ_ROW_CASE(12)
    FPTQ_ROW_CASE(14)
    FPTQ_ROW_CASE(16)
#undef FPTQ_ROW_CASE
    quantize_act_kernel<MODE, 0><<<grid, block, 0, s>>>(x, M, K, eps, row_in, inv_s_a, zoff, out, row_out, stream_in);
    return hipGetLastError();
}

hipError_t launch_quantize_act(const uint16_t *x, int64_t M, int64_t K, int mode, float eps, const float *row_in,
                               float inv_s_a, int zero_point, uint8_t *out, float *row_out, hipStream_t s)
{
    if (M > 0x7fffffff) return hipErrorInvalidValue;
    switch (mode) {
    case FPTQ_SCALE_NONE: return launch_mode<FPTQ_SCALE_NONE>(x, M, K, eps, row_in, inv_s_a, zero_point + 8, out, row_out, s);
    case FPTQ_SCALE_RMS: return launch_mode<FPTQ_SCALE_RMS>(x, M, K, eps, row_in, inv_s_a, zero_point + 8, out, row_out, s);
    default: return launch_mode<FPTQ_SCALE_GIVEN>(x, M, K, eps, row_in, inv_s_a, zero_point + 8, out, row_out, s);
    }
}

}  // namespace fptq
