// Few-token (decode) kernel of the quantized linear layer: M <= 64 tokens against packed INT4
// weights, INT32 accumulation, float-scale epilogue to bf16 (App. J and App. B of the paper).
//
// The job is bound by reading the packed weights once from HBM, so the kernel is built around
// keeping many weight loads in flight per CU and doing as little else as possible:
//   - a workgroup owns 16 (or 32) output channels; its WAVES waves split K (wave w takes K tiles
//     w, w + WAVES, ...), so even the smallest matrices give every CU a workgroup, and several
//     workgroups fit a CU (no LDS ring, few registers), which overlaps their ramp-up and tails;
//   - weights go HBM -> registers directly in MFMA operand order: lane (i = l % 16, g = l / 16)
//     loads granule g (16 bytes, 32 values) of row i, so a wave-level load covers one contiguous
//     1 KB chunk (16 rows x 64 bytes) and U such loads are in flight per wave; they are streaming
//     (non-temporal) loads: every weight byte is used once, and keeping it out of the caches' way
//     is worth 8 % of the layer time;
//   - the activations of the same K tile (M x 64 bytes, L2 resident) are loaded the same way,
//     token rows clamped to M - 1 (duplicate columns are computed and dropped);
//   - v_mfma_i32_16x16x64_i8 does the arithmetic: A = 16 weight rows, B = 16 tokens (MT B
//     operands for up to 16 MT tokens).  Nibbles are widened to bytes exactly as in the prefill kernel
//     (16 * value on both sides, accumulator = 256 * acc, shifted back in the epilogue);
//   - the WAVES partial accumulators are added into one LDS tile with LDS atomics (integers:
//     exact, order-free).
// Every workgroup streams all of X, so the activation traffic from L2 grows with M: beyond 32 tokens
// the kernel is no longer bound by the weights alone; up to 64 tokens (32 on wide matrices) it still beats the
// prefill kernel's smallest tiles.
#include "fptq_common.h"

namespace fptq {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ inline v4i dec_widen(int p0, int p1)
{
    v4i o;
    o.x = (p0 << 4) & (int)0xF0F0F0F0;
    o.y = p0 & (int)0xF0F0F0F0;
    o.z = (p1 << 4) & (int)0xF0F0F0F0;
    o.w = p1 & (int)0xF0F0F0F0;
    return o;
}

// MT = number of 16-token groups (M <= 16 MT); RT = number of 16-channel groups per workgroup (more of
// them cut the activation re-reads per weight byte); U = K tiles in flight per wave
template <int WAVES, int U, int MT, int RT>
__global__ __launch_bounds__(64 * WAVES) void linear_decode_kernel(
    const uint8_t *__restrict__ xq, const uint8_t *__restrict__ wq, int M, int N, int ktiles, float s_a,
    const float *__restrict__ s_w, const float *__restrict__ d, int zp, const int32_t *__restrict__ wsum,
    uint16_t *__restrict__ y, int32_t *__restrict__ acc_out)
{
    __shared__ int32_t red[RT * MT * 256];             // per (rt, mt) group a 16 x 16 tile in accumulator-register order
    for (int o = threadIdx.x; o < RT * MT * 256; o += 64 * WAVES) red[o] = 0;
    __syncthreads();
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = blockIdx.x * (16 * RT);
    const int fi = lane & 15, fg = lane >> 4;

    // lane (i, g): granule g of weight row n0 + i, and of token row i (clamped: rows past the end
    // repeat the last one; what they produce is never stored).  The low 8 bytes of a granule feed
    // the first MFMA of the K tile (k = 32 g + 0..15), the high 8 bytes the second.
    const int64_t w_slab = (int64_t)N * SEG, x_slab = (int64_t)M * SEG;
    const uint8_t *wp[RT], *xp[MT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) wp[rt] = wq + (int64_t)min(n0 + rt * 16 + fi, N - 1) * SEG + fg * 16;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xp[mt] = xq + (int64_t)min(mt * 16 + fi, M - 1) * SEG + fg * 16;

    // Scales of the first output this thread will write (for up to 16 tokens: its only one), fetched now so
    // that the epilogue of this short kernel does not end on a memory round trip.
    float cw0 = 0.0f, d0 = 1.0f;
    int32_t zw0 = 0;
    if (tid < RT * MT * 256) {
        const int g = tid >> 8, n = n0 + (g / MT) * 16 + (tid & 15), t = (g % MT) * 16 + ((tid >> 4) & 15);
        if (n < N) {
            cw0 = s_a * s_w[n];
            if (wsum) zw0 = zp * wsum[n];
        }
        if (d && t < M) d0 = d[t];
    }

    const int T = wave < ktiles ? (ktiles - wave + WAVES - 1) / WAVES : 0;   // K tiles of this wave
    v4i acc[RT][MT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = v4i{0, 0, 0, 0};

    for (int base = 0; base < T; base += U) {
        v4i wv[RT][U], xv[MT][U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u < T) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    wv[rt][u] = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(wp[rt] + (int64_t)(wave + (base + u) * WAVES) * w_slab));
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u < T) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    xv[mt][u] = *reinterpret_cast<const v4i *>(xp[mt] + (int64_t)(wave + (base + u) * WAVES) * x_slab);
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u < T) {
                v4i x0[MT], x1[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    x0[mt] = dec_widen(xv[mt][u][0], xv[mt][u][1]);
                    x1[mt] = dec_widen(xv[mt][u][2], xv[mt][u][3]);
                }
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const v4i w0 = dec_widen(wv[rt][u][0], wv[rt][u][1]), w1 = dec_widen(wv[rt][u][2], wv[rt][u][3]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        acc[rt][mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, x0[mt], acc[rt][mt], 0, 0, 0);
                        acc[rt][mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, x1[mt], acc[rt][mt], 0, 0, 0);
                    }
                }
            }
    }

    // ---- add the WAVES partial tiles in LDS.  D layout of the 16x16 MFMA: lane l, register r holds
    // D[row = 4 (l / 16) + r][col = l % 16]; rows are output channels, columns tokens.
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r)      // word 64 r + lane of the group's tile: the 64 lanes of an add hit 64 different banks
                atomicAdd(&red[(rt * MT + mt) * 256 + r * 64 + 4 * fi + fg], acc[rt][mt][r]);
    __syncthreads();
    for (int o = tid; o < RT * MT * 256; o += 64 * WAVES) {
        const int g = o >> 8, rt = g / MT, mt = g % MT, j = (o >> 4) & 15, i = o & 15;   // groups, token, channel
        const int32_t sum = red[g * 256 + (i & 3) * 64 + 4 * j + (i >> 2)];
        const int t = mt * 16 + j, n = n0 + rt * 16 + i;
        if (t < M && n < N) {
            const bool first = o == tid;
            const int32_t a = sum >> 8;                // exact: the sum is 256 * acc
            // y = bf16((float)(acc - z * wsum[n]) * (s_a * s_w[n]) [* d_t]): fp32 throughout, no fused operations
            const float cw = first ? cw0 : s_a * s_w[n];
            const int32_t zw = wsum ? (first ? zw0 : zp * wsum[n]) : 0;
            float yf = (float)(a - zw) * cw;
            if (d) yf = yf * (first ? d0 : d[t]);
            y[(int64_t)t * N + n] = bf16_rne(yf);
            if (acc_out) acc_out[(int64_t)t * N + n] = a;
        }
    }
}

template <int WAVES, int U, int MT, int RT>
static hipError_t launch_decode_cfg(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                    const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                                    hipStream_t s)
{
    linear_decode_kernel<WAVES, U, MT, RT><<<dim3((unsigned)((N + 16 * RT - 1) / (16 * RT))), dim3(64 * WAVES), 0, s>>>(
        xq, wq, (int)M, (int)N, (int)k_tiles(K), s_a, s_w, d, zp, wsum, y, acc);
    return hipGetLastError();
}

// 0 = launch shape chosen per problem; otherwise WAVES * 100 + U * 10 + RT forces one (testing and tuning)
static std::atomic<int> g_forced_decode{0};
bool set_decode_shape(int code)
{
    const int w = code / 100, u = (code / 10) % 10, rt = code % 10;
    if (code != 0 && !((w == 8 || w == 16) && (u == 1 || u == 2 || u == 4) && (rt == 1 || rt == 2 || rt == 4))) return false;
    g_forced_decode.store(code, std::memory_order_relaxed);
    return true;
}

hipError_t launch_linear_decode(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                                hipStream_t s)
{
    // Limits: M <= 64; 256 * acc must stay in int32; the grid is one workgroup per 16 RT channels.
    if (M > 64 || K > 131071 || N > (1 << 30)) return launch_linear_ref(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    const int64_t kt = k_tiles(K);
#define FPTQ_DEC(W, U, MT, RT) return launch_decode_cfg<W, U, MT, RT>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s)
    if (const int code = g_forced_decode.load(std::memory_order_relaxed)) {
        const int mt = M <= 16 ? 1 : M <= 32 ? 2 : 4;
#define FPTQ_DEC_RT(W, U, MT)                                   \
    switch (code % 10) {                                        \
    case 1: FPTQ_DEC(W, U, MT, 1);                              \
    case 2: FPTQ_DEC(W, U, MT, 2);                              \
    default:                                                    \
        if (W * MT <= 32) FPTQ_DEC(W, U, (W * MT <= 32 ? MT : 1), 4); \
        FPTQ_DEC(W, U, MT, 2);                                  \
    }
#define FPTQ_DEC_U(W, MT)                                       \
    switch ((code / 10) % 10) {                                 \
    case 1: FPTQ_DEC_RT(W, 1, MT)                               \
    case 2: FPTQ_DEC_RT(W, 2, MT)                               \
    default: FPTQ_DEC_RT(W, 4, MT)                              \
    }
#define FPTQ_DEC_W(MT)                                          \
    if (code / 100 == 8) { FPTQ_DEC_U(8, MT) } else { FPTQ_DEC_U(16, MT) }
        if (mt == 1) { FPTQ_DEC_W(1) }
        if (mt == 2) { FPTQ_DEC_W(2) }
        FPTQ_DEC_W(4)
#undef FPTQ_DEC_W
#undef FPTQ_DEC_U
#undef FPTQ_DEC_RT
    }
    // Shapes chosen by measurement (graph replay over cold weights) on the linear layers of Llama-2-7B/13B,
    // Llama-3-8B/70B and Qwen2-7B: 45 matrices times 1, 16 and 32 tokens, 14 shapes each.  16 waves split K
    // whenever there is at least one K tile per wave: small-N matrices then still put enough loads in flight
    // on every CU, and with the weights on streaming loads one K tile in flight per wave and more resident
    // workgroups beat deeper unrolling (except for very long K against few channels).  Up to 4096 channels a
    // workgroup takes 16 of them, beyond that 32, which halves the activation re-reads, and 64 from 16384 channels
    // on (fewer, longer-lived workgroups: the matrix is several rounds of workgroups long either way); with more
    // than 16 tokens, 64 from 10240 channels on.  Each choice is within about 10 % of the best shape of its case.
    const bool deep = kt >= 16;          // at least one K tile for each of 16 waves
    if (M <= 16) {
        if (!deep) FPTQ_DEC(8, 4, 1, 1);
        if (N <= 4096 && kt >= 80) FPTQ_DEC(16, 2, 1, 1);
        if (N <= 4096) FPTQ_DEC(16, 1, 1, 1);
        if (N >= 16384) FPTQ_DEC(16, 1, 1, 4);     // 28672 x 4096: 11.7 us against 12.2 with 32 channels per workgroup
        FPTQ_DEC(16, 1, 1, 2);
    }
    if (M <= 32) {
        if (!deep) FPTQ_DEC(8, 4, 2, 1);
        if (N <= 4096) FPTQ_DEC(16, 1, 2, 1);
        if (N < 10240) FPTQ_DEC(16, 1, 2, 2);
        FPTQ_DEC(8, 1, 2, 4);
    }
    if (!deep) FPTQ_DEC(8, 2, 4, 1);
    if (N <= 4096) FPTQ_DEC(16, 2, 4, 1);
    if (M <= 48) FPTQ_DEC(16, 1, 4, 2);
    FPTQ_DEC(8, 1, 4, 2);
#undef FPTQ_DEC
}

}  // namespace fptq
