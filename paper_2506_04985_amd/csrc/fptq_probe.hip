// Measurement aids: what the matrix pipe and the memory system of the device sustain for loops with
// nothing else in them, so that a benchmark can put the kernels' rates next to the attainable ones
// measured on the same device in the same run.  Nothing here is part of the quantized linear layer:
// this file is built into a shared object of its own (libfptq_probe.so, include/fptq_probe.h) that
// only the benchmark and its test load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>

#include "fptq_probe.h"

namespace fptq_probe {

constexpr int PROBE_MFMA_WORKGROUPS = 256;       // one workgroup of four waves per CU of an MI355X
static thread_local char g_err[160] = "";

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__device__ inline uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// 64 v_mfma_i32_32x32x32_i8 per iteration and wave on 16 independent accumulators, operands held in
// registers: all zero (dense = 0), random nibbles in the high half of every byte (the prefill kernel's 16 * v) that
// stay the same for the whole run (1), or the same form redrawn every iteration by an xorshift step per operand word
// (2: 3.5 VALU instructions per MFMA, about what the prefill kernel's nibble widening costs, and matrix-pipe inputs
// that change as they do on real data, which is what the board's power limit responds to).
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int dense, int32_t *__restrict__ out)
{
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t s = threadIdx.x * 64 + i * 4 + c + blockIdx.x * 77777u;
            a[i][c] = dense ? (int)(probe_hash(s) & 0xF0F0F0F0u) : 0;
            b[i][c] = dense ? (int)(probe_hash(s + 1234567u) & 0xF0F0F0F0u) : 0;
        }
    v16i acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][q] = 0;
    uint32_t ra[4][4], rb[4][4];      // raw xorshift states behind the operands (dense >= 2)
    const uint32_t mask = dense == 3 ? 0u : 0xF0F0F0F0u;      // 3: the same instruction stream on operands that stay zero
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            ra[i][c] = probe_hash(threadIdx.x * 131u + i * 4 + c + blockIdx.x * 7919u) | 1u;
            rb[i][c] = probe_hash(threadIdx.x * 137u + i * 4 + c + blockIdx.x * 104729u) | 1u;
        }
    if (dense < 2) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int rep = 0; rep < 4; ++rep)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i >> 2], b[i & 3], acc[i], 0, 0, 0);
        }
    } else {
        // Fresh operands: while the 64 MFMAs of an iteration consume one operand set, the next set is drawn into a
        // second one (one xorshift step and a mask per word: 7 VALU), pinned four VALU instructions behind every MFMA
        // (the prefill kernel's widening is 3 to 4.5 per MFMA), and the sets swap.
        v4i a2[4], b2[4];
        auto draw = [&](v4i (&na)[4], v4i (&nb)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    uint32_t x = ra[i][c], y = rb[i][c];
                    x ^= x << 13, x ^= x >> 17, x ^= x << 5;
                    y ^= y << 13, y ^= y >> 17, y ^= y << 5;
                    ra[i][c] = x, rb[i][c] = y;
                    na[i][c] = (int)(x & mask);
                    nb[i][c] = (int)(y & mask);
                }
        };
        auto block = [&](const v4i (&ca)[4], const v4i (&cb)[4], v4i (&na)[4], v4i (&nb)[4]) {
            draw(na, nb);
#pragma unroll
            for (int rep = 0; rep < 4; ++rep)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ca[i >> 2], cb[i & 3], acc[i], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 64; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        draw(a, b);
        for (int it = 0; it < iters; it += 2) {
            block(a, b, a2, b2);
            block(a2, b2, a, b);
        }
    }
    int32_t r = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) r ^= acc[i][q];
    out[blockIdx.x * 256 + threadIdx.x] = r;
}

// Streaming read: at most PROBE_READ_WORKGROUPS workgroups walk the buffer in steps of the whole grid, every
// thread XORing 8 16-byte words per step; one atomic per workgroup and component folds the result into
// xor4 (few enough not to show in the time), which makes the read observable and checkable.
constexpr int PROBE_READ_WORKGROUPS = 1024;
constexpr int PROBE_XOR_SLOTS = 256;      // the burst read folds into 256 x 4 words, which the caller XORs together

__global__ __launch_bounds__(256) void probe_read_kernel(const v4i *__restrict__ p, int64_t n16, int32_t *__restrict__ xor4)
{
    __shared__ int32_t part[4][4];
    v4i r = {0, 0, 0, 0};
    for (int64_t base = (int64_t)blockIdx.x * (256 * 8) + threadIdx.x; base < n16; base += (int64_t)gridDim.x * (256 * 8)) {
        v4i v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (base + u * 256 < n16) ? p[base + u * 256] : v4i{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < 8; ++u) r ^= v[u];
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        int x = r[c];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][c] = x;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        const int x = part[0][threadIdx.x] ^ part[1][threadIdx.x] ^ part[2][threadIdx.x] ^ part[3][threadIdx.x];
        if (x != 0) atomicXor(xor4 + threadIdx.x, x);
    }
}

// Burst read: the launch pattern of a kernel that is one memory round trip long.  Every thread issues LOADS
// streaming 16-byte loads at once (a wave's load covers 1 KB), the grid covers the buffer exactly once, and one
// atomic per workgroup and component folds the XOR into xor4.  THREADS and LOADS set how many bytes a CU has in flight.
template <int THREADS, int LOADS>
__global__ __launch_bounds__(THREADS) void probe_read_burst_kernel(const v4i *__restrict__ p, int64_t n16, int32_t *__restrict__ xor4)
{
    __shared__ int32_t part[THREADS / 64][4];
    const int64_t base = (int64_t)blockIdx.x * (THREADS * LOADS) + threadIdx.x;
    v4i v[LOADS];
#pragma unroll
    for (int u = 0; u < LOADS; ++u) v[u] = (base + u * THREADS < n16) ? __builtin_nontemporal_load(p + base + u * THREADS) : v4i{0, 0, 0, 0};
    v4i r = {0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < LOADS; ++u) r ^= v[u];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        int x = r[c];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off, 64);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][c] = x;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        int x = 0;
#pragma unroll
        for (int w = 0; w < THREADS / 64; ++w) x ^= part[w][threadIdx.x];
        // one of PROBE_XOR_SLOTS places per workgroup: atomics on one address would serialise and show in the time
        if (x != 0) atomicXor(xor4 + (blockIdx.x % PROBE_XOR_SLOTS) * 4 + threadIdx.x, x);
    }
}

template <int THREADS, int LOADS>
static void launch_burst(const void *src, int64_t n16, int32_t *xor4, hipStream_t s)
{
    const int64_t per = (int64_t)THREADS * LOADS;
    probe_read_burst_kernel<THREADS, LOADS><<<dim3((unsigned)((n16 + per - 1) / per)), dim3(THREADS), 0, s>>>((const v4i *)src, n16, xor4);
}

}  // namespace fptq_probe

using namespace fptq_probe;

extern "C" {

const char *fptq_probe_last_error(void) { return g_err; }

int64_t fptq_probe_mfma_rate(int iters, int dense, int32_t *out, void *stream)
{
    if (!out) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate: NULL pointer");
        return FPTQ_PROBE_ERR_NULL;
    }
    if (iters < 1 || iters > (1 << 20)) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate: iters must be in [1, 2^20]");
        return FPTQ_PROBE_ERR_VALUE;
    }
    dense = dense < 0 ? 0 : dense > 3 ? 3 : dense;
    if (dense >= 2) iters = (iters + 1) & ~1;            // the fresh-operand loop runs iterations in pairs
    probe_mfma_kernel<<<dim3(PROBE_MFMA_WORKGROUPS), dim3(256), 0, (hipStream_t)stream>>>(iters, dense, out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate: %s", hipGetErrorString(e));
        return FPTQ_PROBE_ERR_HIP;
    }
    // workgroups x waves x iterations x MFMAs per iteration x operations of one 32x32x32 MFMA
    return (int64_t)PROBE_MFMA_WORKGROUPS * 4 * iters * 64 * (2 * 32 * 32 * 32);
}

int64_t fptq_probe_mfma_rate_ex(int iters, int operands, int workgroups_per_cu, int32_t *out, void *stream)
{
    if (!out) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate_ex: NULL pointer");
        return FPTQ_PROBE_ERR_NULL;
    }
    if (iters < 1 || iters > (1 << 20) || operands < 0 || operands > 3 || workgroups_per_cu < 1 || workgroups_per_cu > 2) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate_ex: iters in [1, 2^20], operands in 0..3, workgroups_per_cu 1 or 2");
        return FPTQ_PROBE_ERR_VALUE;
    }
    const int wgs = PROBE_MFMA_WORKGROUPS * workgroups_per_cu;
    if (operands >= 2) iters = (iters + 1) & ~1;         // the fresh-operand loop runs iterations in pairs
    probe_mfma_kernel<<<dim3(wgs), dim3(256), 0, (hipStream_t)stream>>>(iters, operands, out);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof g_err, "fptq_probe_mfma_rate_ex: %s", hipGetErrorString(e));
        return FPTQ_PROBE_ERR_HIP;
    }
    return (int64_t)wgs * 4 * iters * 64 * (2 * 32 * 32 * 32);
}

int fptq_probe_read(const void *src, int64_t bytes, int32_t *xor4, void *stream)
{
    if (!src || !xor4) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read: NULL pointer");
        return FPTQ_PROBE_ERR_NULL;
    }
    if (bytes < 16 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(xor4) & 3)) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read: bytes must be a positive multiple of 16 (got %lld), src 16-byte aligned",
                 (long long)bytes);
        return FPTQ_PROBE_ERR_SHAPE;
    }
    const int64_t n16 = bytes / 16, blocks = (n16 + 256 * 8 - 1) / (256 * 8);
    const unsigned grid = (unsigned)(blocks < PROBE_READ_WORKGROUPS ? blocks : PROBE_READ_WORKGROUPS);
    probe_read_kernel<<<dim3(grid), dim3(256), 0, (hipStream_t)stream>>>((const v4i *)src, n16, xor4);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read: %s", hipGetErrorString(e));
        return FPTQ_PROBE_ERR_HIP;
    }
    return 0;
}

int fptq_probe_read_burst(const void *src, int64_t bytes, int32_t *xor4, int threads, int loads, void *stream)
{
    if (!src || !xor4) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read_burst: NULL pointer");
        return FPTQ_PROBE_ERR_NULL;
    }
    if (bytes < 16 || bytes % 16 != 0 || bytes > ((int64_t)1 << 40) || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(xor4) & 3)) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read_burst: bytes must be a positive multiple of 16 (got %lld), src 16-byte aligned",
                 (long long)bytes);
        return FPTQ_PROBE_ERR_SHAPE;
    }
    const int64_t n16 = bytes / 16;
    hipStream_t s = (hipStream_t)stream;
    const int key = threads * 10 + loads;
    switch (key) {
    case 2561: launch_burst<256, 1>(src, n16, xor4, s); break;
    case 2562: launch_burst<256, 2>(src, n16, xor4, s); break;
    case 2564: launch_burst<256, 4>(src, n16, xor4, s); break;
    case 2568: launch_burst<256, 8>(src, n16, xor4, s); break;
    case 10241: launch_burst<1024, 1>(src, n16, xor4, s); break;
    case 10242: launch_burst<1024, 2>(src, n16, xor4, s); break;
    case 10244: launch_burst<1024, 4>(src, n16, xor4, s); break;
    case 10248: launch_burst<1024, 8>(src, n16, xor4, s); break;
    default:
        snprintf(g_err, sizeof g_err, "fptq_probe_read_burst: threads must be 256 or 1024 and loads 1, 2, 4 or 8");
        return FPTQ_PROBE_ERR_VALUE;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof g_err, "fptq_probe_read_burst: %s", hipGetErrorString(e));
        return FPTQ_PROBE_ERR_HIP;
    }
    return 0;
}

}  // extern "C"
