// Prefill kernel of the quantized linear layer: INT4 x INT4 matmul on the INT8 matrix cores with
// INT32 accumulation, and the float-scale epilogue to bf16 (App. J and App. B of the paper).
//
// CDNA4 has no 4-bit integer MFMA, so nibbles are widened to bytes in registers just before
// v_mfma_i32_32x32x32_i8.  A packed dword p holds 8 nibbles; (p << 4) & 0xF0F0F0F0 and
// p & 0xF0F0F0F0 are 2 x 4 signed bytes equal to 16 * value (the nibble's sign bit lands on the
// byte's sign bit).  Both operands are widened the same way, so the accumulator holds exactly
// 256 * acc: |acc| <= 64 K keeps 256 * acc inside int32 for K up to 131071, and the epilogue
// shifts it back.  Which k lands in which byte of an operand does not matter as long as both
// operands agree, and they do: the same code widens the same byte offsets of X and W.
//
// Data flow: packed tiles (rows x 64 bytes per K tile, contiguous in HBM) -> LDS by direct
// global->LDS loads (no VGPR staging), STAGES-deep ring, one barrier per K tile -> ds_read_b128
// fragments -> widen -> MFMA.  The 16-byte granules of a row are XOR-swizzled in LDS so that the
// fragment reads spread over the banks.
#include "fptq_common.h"

namespace fptq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// s_waitcnt immediates for gfx9: vmcnt in bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
constexpr int WAIT_LGKM0 = 15 | (3 << 14) | (7 << 4) | (0 << 8);

__device__ inline int swz(int row) { return (row >> 1) & 3; }

template <int WAVES_N_, int WAVES_M_, int TN_, int TM_, int STAGES_>
struct GemmCfg {
    static constexpr int WAVES_N = WAVES_N_, WAVES_M = WAVES_M_, TN = TN_, TM = TM_, STAGES = STAGES_;
    static constexpr int BN = WAVES_N * TN * 32, BM = WAVES_M * TM * 32;
    static constexpr int WAVES = WAVES_N * WAVES_M, THREADS = 64 * WAVES;
    static constexpr int W_BYTES = BN * SEG, X_BYTES = BM * SEG, STAGE_BYTES = W_BYTES + X_BYTES;
    static constexpr int W_LOADS = W_BYTES / (THREADS * 16), X_LOADS = X_BYTES / (THREADS * 16);
    static constexpr int LOADS = W_LOADS + X_LOADS;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(W_BYTES % (THREADS * 16) == 0 && X_BYTES % (THREADS * 16) == 0, "tile must split over threads");
};

// widen two packed dwords (16 nibbles) into one MFMA operand of 16 bytes, each 16 * value
__device__ inline v4i widen(int p0, int p1)
{
    v4i o;
    o.x = (p0 << 4) & (int)0xF0F0F0F0;
    o.y = p0 & (int)0xF0F0F0F0;
    o.z = (p1 << 4) & (int)0xF0F0F0F0;
    o.w = p1 & (int)0xF0F0F0F0;
    return o;
}

template <class C>
__global__ __launch_bounds__(C::THREADS) void linear_mfma_kernel(
    const uint8_t *__restrict__ xq, const uint8_t *__restrict__ wq, int M, int N, int ktiles, int tiles_m,
    int tiles_n, float s_a, const float *__restrict__ s_w, const float *__restrict__ d, uint16_t *__restrict__ y,
    int32_t *__restrict__ acc_out)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_n = wave % C::WAVES_N, wave_m = wave / C::WAVES_N;

    // ---- tile of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous run of logical tiles so that its L2 sees neighbouring tiles, then walk the tile grid
    // in bands of 8 N-tiles with M fastest, so that concurrent tiles share X and W panels.
    const int total = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = (total + 7) / 8, tall = total % 8 == 0 ? 8 : total % 8;
        const int xcd = pid % 8, local = pid / 8;
        pid = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
    }
    constexpr int GN = 8;
    const int band = pid / (GN * tiles_m), in_band = pid % (GN * tiles_m);
    const int band_w = min(GN, tiles_n - band * GN);
    const int bn = band * GN + in_band % band_w, bm = in_band / band_w;
    const int n0 = bn * C::BN, m0 = bm * C::BM;

    // ---- global -> LDS copy plan.  A wave-level direct load fills 1 KB of LDS: lane l lands at
    // byte 16 l.  LDS slot s (16 bytes) of a tile holds granule (s % 4) ^ swz(row) of row s / 4.
    int64_t w_src[C::W_LOADS], x_src[C::X_LOADS];
#pragma unroll
    for (int j = 0; j < C::W_LOADS; ++j) {
        int slot = (j * C::WAVES + wave) * 64 + lane, row = slot >> 2, g = (slot & 3) ^ swz(row);
        w_src[j] = (int64_t)min(n0 + row, N - 1) * SEG + g * 16;
    }
#pragma unroll
    for (int j = 0; j < C::X_LOADS; ++j) {
        int slot = (j * C::WAVES + wave) * 64 + lane, row = slot >> 2, g = (slot & 3) ^ swz(row);
        x_src[j] = (int64_t)min(m0 + row, M - 1) * SEG + g * 16;
    }
    const int64_t w_tile_stride = (int64_t)N * SEG, x_tile_stride = (int64_t)M * SEG;

    auto issue_loads = [&](int kt, int stage) {
        uint8_t *wl = lds + stage * C::STAGE_BYTES, *xl = wl + C::W_BYTES;
        const uint8_t *wg = wq + kt * w_tile_stride, *xg = xq + kt * x_tile_stride;
#pragma unroll
        for (int j = 0; j < C::W_LOADS; ++j)
            __builtin_amdgcn_global_load_lds(GLB_PTR(wg + w_src[j]), LDS_PTR(wl + (j * C::WAVES + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < C::X_LOADS; ++j)
            __builtin_amdgcn_global_load_lds(GLB_PTR(xg + x_src[j]), LDS_PTR(xl + (j * C::WAVES + wave) * 1024), 16, 0, 0);
    };

    // ---- fragment read plan: lane (i = lane % 32, g = lane / 32) of a 32-row sub-tile reads, for
    // K half kk, the 16-byte granule 2 kk + g of row i: its low 8 bytes feed the first MFMA of the
    // half, the high 8 bytes the second.
    const int fi = lane & 31, fg = lane >> 5;
    int w_frag[C::TN], x_frag[C::TM], w_sw[C::TN], x_sw[C::TM];
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn) {
        int row = (wave_n * C::TN + tn) * 32 + fi;
        w_frag[tn] = row * SEG;
        w_sw[tn] = swz(row);
    }
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm) {
        int row = (wave_m * C::TM + tm) * 32 + fi;
        x_frag[tm] = C::W_BYTES + row * SEG;
        x_sw[tm] = swz(row);
    }

    v16i acc[C::TN][C::TM];
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0;

    // ---- pipeline prologue: STAGES - 1 tiles in flight (tiles past the end repeat the last one,
    // which keeps the outstanding-load count uniform)
#pragma unroll
    for (int s = 0; s < C::STAGES - 1; ++s) issue_loads(min(s, ktiles - 1), s);

    for (int kt = 0; kt < ktiles; ++kt) {
        const int stage = kt % C::STAGES;
        // own loads of tile kt have landed; the barrier extends that to every wave's loads and also
        // says everyone is done reading the buffer that is refilled next
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(C::LOADS * (C::STAGES - 2)));
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_s_barrier();
        issue_loads(min(kt + C::STAGES - 1, ktiles - 1), (kt + C::STAGES - 1) % C::STAGES);

        const uint8_t *base = lds + stage * C::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            v4i wraw[C::TN], xraw[C::TM];
#pragma unroll
            for (int tn = 0; tn < C::TN; ++tn)
                wraw[tn] = *reinterpret_cast<const v4i *>(base + w_frag[tn] + (((2 * kk + fg) ^ w_sw[tn]) << 4));
#pragma unroll
            for (int tm = 0; tm < C::TM; ++tm)
                xraw[tm] = *reinterpret_cast<const v4i *>(base + x_frag[tm] + (((2 * kk + fg) ^ x_sw[tm]) << 4));
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4i wop[C::TN], xop[C::TM];
#pragma unroll
                for (int tn = 0; tn < C::TN; ++tn) wop[tn] = widen(wraw[tn][2 * h], wraw[tn][2 * h + 1]);
#pragma unroll
                for (int tm = 0; tm < C::TM; ++tm) xop[tm] = widen(xraw[tm][2 * h], xraw[tm][2 * h + 1]);
#pragma unroll
                for (int tn = 0; tn < C::TN; ++tn)
#pragma unroll
                    for (int tm = 0; tm < C::TM; ++tm)
                        acc[tn][tm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop[tn], xop[tm], acc[tn][tm], 0, 0, 0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the repeated tail loads before the LDS dies

    // ---- epilogue.  W was the A operand, so the accumulator tile is [n][m]: a lane owns token
    // m = lane % 32 and, per register quad, four consecutive output channels
    // n = 8 * (r / 4) + 4 * (lane / 32) + (r % 4).
    const bool vec_ok = (N % 4) == 0;
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm) {
        const int m = m0 + (wave_m * C::TM + tm) * 32 + fi;
        if (m >= M) continue;
        const float dm = d ? d[m] : 1.0f;
#pragma unroll
        for (int tn = 0; tn < C::TN; ++tn) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + (wave_n * C::TN + tn) * 32 + 8 * q + 4 * fg;
                if (n >= N) continue;
                uint16_t o[4];
                int32_t a[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a[e] = acc[tn][tm][4 * q + e] >> 8;      // exact: the register holds 256 * acc
                    if (n + e < N) {
                        float yf = (float)a[e] * (s_a * s_w[n + e]);
                        if (d) yf = yf * dm;
                        o[e] = bf16_rne(yf);
                    }
                }
                const int64_t off = (int64_t)m * N + n;
                if (vec_ok) {   // N % 4 == 0 and n % 4 == 0: the quad is whole and 8-byte aligned
                    *reinterpret_cast<uint2 *>(y + off) = make_uint2(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16));
                    if (acc_out) *reinterpret_cast<int4 *>(acc_out + off) = make_int4(a[0], a[1], a[2], a[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) {
                            y[off + e] = o[e];
                            if (acc_out) acc_out[off + e] = a[e];
                        }
                }
            }
        }
    }
}

template <class C>
static hipError_t launch_cfg(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *d, uint16_t *y, int32_t *acc, hipStream_t s)
{
    static bool attr_set = false;
    auto kern = linear_mfma_kernel<C>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int64_t tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    if (tiles_m * tiles_n > 0x7fffffff) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(C::THREADS), C::LDS_BYTES, s>>>(
        xq, wq, (int)M, (int)N, (int)k_tiles(K), (int)tiles_m, (int)tiles_n, s_a, s_w, d, y, acc);
    return hipGetLastError();
}

hipError_t launch_linear_mfma(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                              const float *s_w, const float *d, uint16_t *y, int32_t *acc, hipStream_t s)
{
    // the widened accumulator is 256 * acc and |acc| <= 64 K: beyond this K it could leave int32
    if (K > 131071 || M > 0x7fffffff || N > 0x7fffffff || M * N > ((int64_t)1 << 40))
        return launch_linear_ref(xq, wq, M, N, K, s_a, s_w, d, y, acc, s);
    typedef GemmCfg<2, 2, 4, 4, 4> Big;     // 256 x 256 tile, 4 waves of 128 x 128, 128 KB LDS
    return launch_cfg<Big>(xq, wq, M, N, K, s_a, s_w, d, y, acc, s);
}

}  // namespace fptq
