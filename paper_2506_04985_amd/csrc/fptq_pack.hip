// Offline packing of INT4 weights into the library layout (two values per byte, App. J of the
// paper), the inverse used by parity checks, and the simple one-thread-per-output linear kernel.
#include "fptq_common.h"

namespace fptq {

// One thread writes one 16-byte granule (32 values) of one (tile, row) segment.
__global__ __launch_bounds__(256) void pack_weights_kernel(const int8_t *__restrict__ w, int64_t N, int64_t K,
                                                           int64_t n_granules, uint8_t *__restrict__ out)
{
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_granules) return;
    int64_t c = g & 3;                 // granule inside the 64-byte segment
    int64_t seg = g >> 2;              // (tile, row) segment index = tile * N + row
    int64_t row = seg % N, tile = seg / N;
    int64_t k0 = tile * KT + c * 32;
    const int8_t *src = w + row * K;
    uint32_t words[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int64_t k = k0 + j * 8 + i;
            uint32_t v = k < K ? ((uint32_t)(uint8_t)src[k] & 15u) : 0u;   // K padding is zero
            word |= v << (4 * i);
        }
        words[j] = word;
    }
    *reinterpret_cast<uint4 *>(out + g * 16) = make_uint4(words[0], words[1], words[2], words[3]);
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ packed, int64_t rows, int64_t K,
                                                     int8_t *__restrict__ out)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * K) return;
    int64_t row = idx / K, k = idx % K;
    uint8_t b = packed[((k / KT) * rows + row) * SEG + (k % KT) / 2];
    int v = (k & 1) ? (b >> 4) : (b & 15);
    out[idx] = (int8_t)(v >= 8 ? v - 16 : v);
}

// acc[t][o] = sum_k q[t][k] * w[o][k], straight from the packed buffers with the 8-way INT4 dot
// instruction; one thread per output.  Also the library's answer for shapes nothing else covers.
__global__ __launch_bounds__(256) void linear_ref_kernel(const uint8_t *__restrict__ xq, const uint8_t *__restrict__ wq,
                                                         int64_t M, int64_t N, int64_t ktiles, float s_a,
                                                         const float *__restrict__ s_w, const float *__restrict__ d, int zp,
                                                         const int32_t *__restrict__ wsum, uint16_t *__restrict__ y,
                                                         int32_t *__restrict__ acc_out)
{
    const int64_t blocks_n = (N + 15) / 16;
    int64_t o = ((int64_t)blockIdx.x % blocks_n) * 16 + (threadIdx.x & 15);
    int64_t t = ((int64_t)blockIdx.x / blocks_n) * 16 + (threadIdx.x >> 4);
    if (o >= N || t >= M) return;
    int acc = 0;
    for (int64_t kt = 0; kt < ktiles; ++kt) {
        const uint4 *a = reinterpret_cast<const uint4 *>(xq + (kt * M + t) * SEG);
        const uint4 *b = reinterpret_cast<const uint4 *>(wq + (kt * N + o) * SEG);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint4 av = a[c], bv = b[c];
            acc = __builtin_amdgcn_sdot8((int)av.x, (int)bv.x, acc, false);
            acc = __builtin_amdgcn_sdot8((int)av.y, (int)bv.y, acc, false);
            acc = __builtin_amdgcn_sdot8((int)av.z, (int)bv.z, acc, false);
            acc = __builtin_amdgcn_sdot8((int)av.w, (int)bv.w, acc, false);
        }
    }
    float cw = s_a * s_w[o];
    y[t * N + o] = dequant_bf16(remove_zero_point(acc, zp, wsum, o), cw, d, t);
    if (acc_out) acc_out[t * N + o] = acc;          // the raw accumulator sum_k v w
}

hipError_t launch_pack_weights(const int8_t *w, int64_t N, int64_t K, uint8_t *out, hipStream_t s)
{
    int64_t n_granules = k_tiles(K) * N * 4;
    int64_t blocks = (n_granules + 255) / 256;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    pack_weights_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(w, N, K, n_granules, out);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint8_t *packed, int64_t rows, int64_t K, int8_t *out, hipStream_t s)
{
    int64_t blocks = (rows * K + 255) / 256;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    unpack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(packed, rows, K, out);
    return hipGetLastError();
}

// sum_k w[o][k] per output channel (what an activation zero point multiplies); one wave per row
__global__ __launch_bounds__(256) void weight_row_sums_kernel(const int8_t *__restrict__ w, int64_t N, int64_t K,
                                                              int32_t *__restrict__ sums)
{
    const int lane = threadIdx.x & 63;
    const int64_t o = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (o >= N) return;
    int s = 0;
    for (int64_t k = lane; k < K; k += 64) s += w[o * K + k];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) sums[o] = s;
}

hipError_t launch_weight_row_sums(const int8_t *w, int64_t N, int64_t K, int32_t *sums, hipStream_t s)
{
    int64_t blocks = (N + 3) / 4;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    weight_row_sums_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(w, N, K, sums);
    return hipGetLastError();
}

hipError_t launch_linear_ref(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                             hipStream_t s)
{
    int64_t blocks = ((N + 15) / 16) * ((M + 15) / 16);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    linear_ref_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(xq, wq, M, N, k_tiles(K), s_a, s_w, d, zp, wsum, y, acc);
    return hipGetLastError();
}

}  // namespace fptq
