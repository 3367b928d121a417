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
// Data flow: packed tiles (rows x 64 bytes per K tile, contiguous in HBM) -> LDS by buffer loads
// that write LDS directly (no VGPR staging; rows past the end read as zero through the buffer
// descriptor's bounds check), STAGES-deep ring, one barrier per K tile -> ds_read_b128 fragments
// -> widen -> MFMA.  The 16-byte granules of a row are XOR-swizzled in LDS so that the fragment
// reads are bank-conflict free.
#include <cmath>
#include <cstdio>

#include "fptq_common.h"

namespace fptq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// s_waitcnt immediates for gfx9: vmcnt in bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
constexpr int WAIT_LGKM0 = 15 | (3 << 14) | (7 << 4) | (0 << 8);

// raw buffer descriptor, dword 3: 32-bit data format, no swizzle (gfx9 family encoding)
constexpr int RSRC_FLAGS = 0x00020000;

constexpr int MAX_SPLITS = 4;     // K ranges per output tile in the split-K variant
constexpr int SPLIT_COUNTERS = 1024;   // arrival counters at the start of a split-K workspace (one per output tile)

// OCC_ = workgroups meant to share a CU (caps the register budget: 512 / OCC_ per lane).  KS_ = K groups:
// KS_ sets of WAVES waves work on the same output tile, set g on K tiles g, g + KS_, ..., each with its own
// LDS ring; their accumulators are added through LDS and every group runs its share of the epilogue.  A
// problem with at most one workgroup per CU runs one wave per SIMD, which cannot hide its own LDS and VALU
// latencies; more K groups give every SIMD more waves without needing more output tiles.
// SPLIT_: several workgroups share an output tile, each on a contiguous range of K tiles; they leave their
// partial accumulators in a caller-provided workspace and the last one to arrive adds them and runs the epilogue.
template <int WAVES_N_, int WAVES_M_, int TN_, int TM_, int STAGES_, int OCC_ = 1, int KS_ = 1, bool SPLIT_ = false>
struct GemmCfg {
    static constexpr int WAVES_N = WAVES_N_, WAVES_M = WAVES_M_, TN = TN_, TM = TM_, STAGES = STAGES_, OCC = OCC_, KS = KS_;
    static constexpr bool SPLIT = SPLIT_;
    static constexpr int ACC_REGS = TN_ * TM_ * 16;             // accumulator registers of a lane
    static constexpr int BN = WAVES_N * TN * 32, BM = WAVES_M * TM * 32;
    static constexpr int WAVES = WAVES_N * WAVES_M, THREADS = 64 * WAVES * KS;
    static constexpr int W_BYTES = BN * SEG, X_BYTES = BM * SEG, STAGE_BYTES = W_BYTES + X_BYTES;
    // every wave copies a contiguous run of rows of each operand tile, 1 KB (16 rows) per load
    static constexpr int W_LOADS = W_BYTES / (WAVES * 1024), X_LOADS = X_BYTES / (WAVES * 1024);
    static constexpr int LOADS = W_LOADS + X_LOADS;
    static constexpr int RING_BYTES = STAGES * STAGE_BYTES, LDS_BYTES = KS * RING_BYTES;
    static_assert(W_BYTES % (WAVES * 1024) == 0 && X_BYTES % (WAVES * 1024) == 0, "tile must split over waves");
    static_assert(W_LOADS >= 1 && W_LOADS <= 4 && X_LOADS >= 1 && X_LOADS <= 4, "the fill schedule issues at most one W and one X chunk per quarter");
    // loads issued by fill quarters 0 and 1 (a quarter q carries W chunk q and X chunk q if they exist)
    static constexpr int HALF_LOADS = (W_LOADS < 2 ? W_LOADS : 2) + (X_LOADS < 2 ? X_LOADS : 2);
    static_assert(STAGES >= 3, "pipeline needs three stages");
    static_assert(TN <= 4, "a wave's channel run must fit 16 lanes of 8 channels in the epilogue");
    // After the K loop the K groups exchange accumulators so that each ends up with the sum of SUBS of the wave's
    // TN x TM sub-tiles (counted along n first): TNE along n, TME along m.
    static constexpr int SUBS = TN * TM / KS;
    static constexpr int TNE = SUBS >= TN ? TN : SUBS, TME = SUBS >= TN ? SUBS / TN : 1;
    static constexpr int NSC = (TNE * 32 + 63) / 64;           // channel scales a lane fetches for the epilogue
    static_assert(TN * TM % KS == 0 && TNE * TME == SUBS && TN % TNE == 0, "the K groups share the sub-tiles evenly, in runs along n");
    static_assert((KS - 1) * TN * TM * WAVES * 4096 <= LDS_BYTES, "the K groups' accumulators are added through LDS");
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

// two fp32 -> packed bf16 pair (round to nearest even, hardware conversion)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16(float lo, float hi)
{
    float2_t f = {lo, hi};
    bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

// One 1 KB chunk (16 rows) of an operand tile, HBM -> LDS.  J is the chunk number inside the run of
// chunks this wave copies: the immediate offset (a compile-time constant of the instruction)
// advances the HBM and the LDS address together, so all chunks share one VGPR offset and one LDS base.
template <int J>
__device__ inline void load_chunk(__amdgpu_buffer_rsrc_t r, uint8_t *lds_base, int voff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, LDS_PTR(lds_base), 16, voff, 0, J * 1024, 0);
}

// Channel scales (and, with a zero point, the weight row sums) of a run of TNE * 32 channels, one or two per lane.
template <int TNE, bool ZP>
__device__ inline void load_scales(float (&scv)[(TNE * 32 + 63) / 64], int32_t (&zwv)[(TNE * 32 + 63) / 64],
                                   const float *__restrict__ s_w, const int32_t *__restrict__ wsum, int nw0, int N, int lane)
{
#pragma unroll
    for (int i = 0; i < (TNE * 32 + 63) / 64; ++i) {
        const int n = min(nw0 + min(lane + 64 * i, TNE * 32 - 1), N - 1);
        scv[i] = s_w[n];
        zwv[i] = ZP ? wsum[n] : 0;
    }
}

// What a wave does with its finished sub-tiles a[t][i] (t < TNE along n from channel nw0, i < TME along m from
// token mw0; sub-tile numbers sub0 .. of the wave's TN x TM, counted along n first): the split-K exchange, then
// the epilogue.
template <class C, int TNE, int TME, bool ALIGNED, bool DUMP, bool ZP>
__device__ inline void finish(v16i (&a)[TNE][TME], const float (&scv)[(TNE * 32 + 63) / 64],
                              const int32_t (&zwv)[(TNE * 32 + 63) / 64], uint8_t *lds, int wave_all, int wave, int lane,
                              int sub0, int nw0, int mw0, int M, int N, float s_a, const float *__restrict__ d, int zp,
                              const int32_t *__restrict__ wsum, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out,
                              int32_t *ws, int splits, int split, int pid, int total)
{
    const int fi = lane & 31, fg = lane >> 5;
    // ---- split K: leave the partial tile in the workspace, count the arrival, and let the last workgroup of
    // the tile add the others' partials and go on to the epilogue.  Nobody waits for anybody, so there is nothing
    // to hang on.  The workgroups of a tile run on different XCDs, whose L2s are not coherent with each other, and
    // a device-wide fence would write back and invalidate a whole L2 per workgroup; instead the partials are
    // stored and loaded with the device-coherent cache policy (sc0 sc1: written through to, and read from, the
    // memory side), the stores are complete (vmcnt) before the arrival is counted, and the count is an atomic
    // at the same scope.  Workspace: SPLIT_COUNTERS arrival counters (zero between calls; the first `total` are used:
    // a region of fixed size, so that calls of different shapes that share a workspace agree on where it ends), then
    // [splits][total][sub-tile][quad][threads of a K group] partials as 16-byte quads, lane-contiguous.
    if (C::SPLIT) {
        constexpr int TPG = C::WAVES * 64, COHERENT = 1 | 16;     // aux bits: sc0, sc1
        const int64_t slice = (int64_t)C::ACC_REGS * TPG;
        int32_t *counters = ws, *parts = ws + SPLIT_COUNTERS;
        int *flag = reinterpret_cast<int *>(lds + C::LDS_BYTES - 16);     // clear of the epilogue's patches
        const int qoff = (wave * 64 + lane) * 16 + sub0 * (4 * TPG * 16);
        const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(parts + ((int64_t)split * total + pid) * slice), 0, (int)slice * 4, RSRC_FLAGS);
#pragma unroll
        for (int i = 0; i < TME; ++i)
#pragma unroll
            for (int t = 0; t < TNE; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4i v = {a[t][i][4 * q], a[t][i][4 * q + 1], a[t][i][4 * q + 2], a[t][i][4 * q + 3]};
                    __builtin_amdgcn_raw_buffer_store_b128(v, mine, qoff + ((i * TNE + t) * 4 + q) * (TPG * 16), 0, COHERENT);
                }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // this wave's partials have reached the memory side
        __syncthreads();
        if (threadIdx.x == 0) *flag = __hip_atomic_fetch_add(counters + pid, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*flag != splits - 1) return;             // the whole workgroup: not the last one of this tile
        // the other (at most MAX_SPLITS - 1) partial tiles, read side by side so that their latencies overlap
        __amdgpu_buffer_rsrc_t other[MAX_SPLITS - 1];
#pragma unroll
        for (int j = 0; j < MAX_SPLITS - 1; ++j) {
            const int s2 = (split + 1 + j) % splits;            // j < splits - 1: every other split once
            other[j] = __builtin_amdgcn_make_buffer_rsrc((void *)(parts + ((int64_t)s2 * total + pid) * slice), 0,
                                                         j < splits - 1 ? (int)slice * 4 : 0, RSRC_FLAGS);
        }
#pragma unroll
        for (int i = 0; i < TME; ++i)
#pragma unroll
            for (int t = 0; t < TNE; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v4i v[MAX_SPLITS - 1];
#pragma unroll
                    for (int j = 0; j < MAX_SPLITS - 1; ++j)      // an empty descriptor (j >= splits - 1) reads zeros
                        v[j] = __builtin_amdgcn_raw_buffer_load_b128(other[j], qoff + ((i * TNE + t) * 4 + q) * (TPG * 16), 0, COHERENT);
#pragma unroll
                    for (int j = 0; j < MAX_SPLITS - 1; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) a[t][i][4 * q + e] += v[j][e];
                }
        if (threadIdx.x == 0) counters[pid] = 0;     // as it was found, for the next call
    }

    // ---- epilogue.  W was the A operand, so an accumulator tile is [n][m]: a lane owns token
    // m = lane % 32 and, per register quad q, four consecutive output channels
    // n = 8 q + 4 (lane / 32) + (r % 4).  The register holds 256 * acc; (float)(256 * acc) equals
    // 256 * (float)acc exactly (acc has fewer than 24 significant bits), and the 2^-8 is folded into
    // the channel scale, which is exact as well, so y = bf16((float)acc * (s_a * s_w[n]) [* d_t]) to
    // the bit.  The bf16 results go through a wave-private LDS patch ([32 tokens][TNE * 32 channels],
    // padded rows) so that HBM sees whole 16-byte-per-lane row segments instead of scattered quads.
    constexpr int WN = TNE * 32;                      // channels of this wave's run
    constexpr int PATCH_STRIDE = WN * 2 + 16;         // bytes per token row in the patch
    // With an activation zero point z the sum wanted is sum_k (v - z) w = acc - z * wsum[n]; the
    // correction is staged as 256 * z * wsum[n] next to the scales (|.| < 2^31 for K <= 65535).
    constexpr int WAVE_LDS = 32 * PATCH_STRIDE + WN * 8;
    uint8_t *patch = lds + wave_all * WAVE_LDS;
    float *cwbuf = reinterpret_cast<float *>(patch + 32 * PATCH_STRIDE);
    int32_t *zwbuf = reinterpret_cast<int32_t *>(cwbuf + WN);
#pragma unroll
    for (int i = 0; i < (WN + 63) / 64; ++i) {
        const int c = lane + 64 * i;
        if (c < WN) {
            cwbuf[c] = (s_a * scv[i]) * 0.00390625f;
            if (ZP) zwbuf[c] = (zp * zwv[i]) * 256;
        }
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int tm = 0; tm < TME; ++tm) {
        const int mt0 = mw0 + tm * 32;
        const int m = mt0 + fi;
        const float dm = (d && m < M) ? d[m] : 1.0f;
#pragma unroll
        for (int tn = 0; tn < TNE; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 c4 = *reinterpret_cast<const float4 *>(cwbuf + tn * 32 + 8 * q + 4 * fg);
                int32_t a4[4] = {a[tn][tm][4 * q + 0], a[tn][tm][4 * q + 1], a[tn][tm][4 * q + 2], a[tn][tm][4 * q + 3]};
                if (ZP) {
                    const int4 z4 = *reinterpret_cast<const int4 *>(zwbuf + tn * 32 + 8 * q + 4 * fg);
                    a4[0] -= z4.x, a4[1] -= z4.y, a4[2] -= z4.z, a4[3] -= z4.w;
                }
                float yf[4] = {(float)a4[0] * c4.x, (float)a4[1] * c4.y, (float)a4[2] * c4.z, (float)a4[3] * c4.w};
                if (d) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) yf[e] = yf[e] * dm;
                }
                *reinterpret_cast<uint2 *>(patch + fi * PATCH_STRIDE + (tn * 32 + 8 * q + 4 * fg) * 2) =
                    make_uint2(pack_bf16(yf[0], yf[1]), pack_bf16(yf[2], yf[3]));
            }
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_wave_barrier();
        // read back row segments: 16 bytes (8 channels) per lane, WN / 8 lanes per token row
        // (lanes per row rounded up to a power of two; the surplus lanes idle)
        constexpr int LANES_PER_ROW = WN / 8 <= 4 ? 4 : WN / 8 <= 8 ? 8 : 16, ROWS_PER_PASS = 64 / LANES_PER_ROW;
#pragma unroll
        for (int pass = 0; pass < 32 / ROWS_PER_PASS; ++pass) {
            const int row = pass * ROWS_PER_PASS + lane / LANES_PER_ROW, col = (lane % LANES_PER_ROW) * 8;
            const bool live = col < WN;
            const uint4 v = live ? *reinterpret_cast<const uint4 *>(patch + row * PATCH_STRIDE + col * 2) : make_uint4(0, 0, 0, 0);
            const int mm = mt0 + row, nn = nw0 + col;
            if (live && mm < M && nn < N) {
                uint16_t *dst = y + (int64_t)mm * N + nn;
                if (ALIGNED) {       // N % 8 == 0: the segment is whole and 16-byte aligned
                    __builtin_nontemporal_store(v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w}, reinterpret_cast<v4i *>(dst));
                } else {
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (nn + e < N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_wave_barrier();
        if (DUMP) {      // parity dump of the integer accumulators (never a timed path)
#pragma unroll
            for (int tn = 0; tn < TNE; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int n = nw0 + tn * 32 + 8 * q + 4 * fg + e;
                        if (m < M && n < N) acc_out[(int64_t)m * N + n] = a[tn][tm][4 * q + e] >> 8;
                    }
        }
    }
}

// ZP: the epilogue removes an activation zero point (wsum is then non-null); a separate instance, so that the symmetric
// grid's epilogue carries neither its code nor its registers (the 256 x 256 instance spilled 13 registers with both in one).
template <class C, bool ALIGNED, bool DUMP, bool ZP>
__global__ __launch_bounds__(C::THREADS, C::OCC) void linear_mfma_kernel(
    const uint8_t *__restrict__ xq, const uint8_t *__restrict__ wq, int M, int N, int ktiles, int tiles_m,
    int tiles_n, float s_a, const float *__restrict__ s_w, const float *__restrict__ d, int zp,
    const int32_t *__restrict__ wsum, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out, int32_t *ws, int splits, int map_mode)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = C::KS > 1 ? wave_all / C::WAVES : 0, wave = C::KS > 1 ? wave_all % C::WAVES : wave_all;   // K group, wave in it
    const int wave_n = wave % C::WAVES_N, wave_m = wave / C::WAVES_N;
    uint8_t *const ring = lds + kg * C::RING_BYTES;                      // this K group's LDS ring

    // ---- tile of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous run of logical tiles so that its L2 sees neighbouring tiles, then walk the tile grid
    // in bands of 8 N-tiles with M fastest, so that concurrent tiles share X and W panels.
    const int total = tiles_m * tiles_n;
    int pid = blockIdx.x, split = 0;
    if (C::SPLIT) {                                  // workgroup = (split, tile), tiles fastest
        split = pid / total;
        pid -= split * total;
    }
    if (map_mode == 0) {                             // (map_mode 1, a measurement aid: tiles dealt round-robin to the XCDs as they come)
        const int per = (total + 7) / 8, tall = total % 8 == 0 ? 8 : total % 8;
        const int xcd = pid % 8, local = pid / 8;
        pid = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
    }
    constexpr int GN = 8;
    const int band = pid / (GN * tiles_m), in_band = pid % (GN * tiles_m);
    const int band_w = min(GN, tiles_n - band * GN);
    const int bn = band * GN + in_band % band_w, bm = in_band / band_w;
    const int n0 = bn * C::BN, m0 = bm * C::BM;

    // ---- global -> LDS copy plan.  One K tile of an operand is rows x 64 bytes, contiguous in HBM,
    // and its LDS image has the same linear layout except that the four 16-byte granules of a row
    // are permuted: LDS slot s of a row holds granule s ^ swz(row), swz(row) = (row >> 2) & 3.
    // (A ds_read_b128 is served 16 lanes at a time; the 16 rows they read then fall into 16
    // different 16-byte bank groups: address bits 7:4 = (row % 4) * 4 + slot.)
    // A wave-level load fills 1 KB: lane l lands at byte 16 l, i.e. row l / 4, slot l % 4, and the
    // row's swizzle is (l / 16) & 3 for every 16-row chunk.  Each wave copies W_LOADS (X_LOADS)
    // consecutive chunks, addressed by one VGPR offset plus 1 KB immediates, which move the HBM
    // and the LDS address together.
    const int lane_src = (lane >> 2) * SEG + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);
    const int w_voff = (n0 + wave * (C::W_LOADS * 16)) * SEG + lane_src;
    const int x_voff = (m0 + wave * (C::X_LOADS * 16)) * SEG + lane_src;
    const int w_lds0 = wave * (C::W_LOADS * 1024), x_lds0 = C::W_BYTES + wave * (C::X_LOADS * 1024);
    const int64_t w_slab = (int64_t)N * SEG, x_slab = (int64_t)M * SEG;   // bytes per K tile of all rows

    // per-slab descriptors: rows past N (M) fail the bounds check and read as zero.  Step j of this K group
    // is K tile kt_begin + j * KS + kg; a step past the last tile gets an empty descriptor, so its loads are still
    // issued (the outstanding-load count stays uniform) but read nothing and land as zeros.
    int kt_begin = 0, kt_end = ktiles;               // K tiles of this workgroup
    if (C::SPLIT) {
        const int per = (ktiles + splits - 1) / splits;
        kt_begin = split * per;
        kt_end = min(ktiles, kt_begin + per);
    }
    auto w_desc = [&](int j) {
        const int kt = kt_begin + j * C::KS + kg;
        const bool in = kt < kt_end;
        return __builtin_amdgcn_make_buffer_rsrc((void *)(wq + (in ? kt : 0) * w_slab), 0, in ? (int)w_slab : 0, RSRC_FLAGS);
    };
    auto x_desc = [&](int j) {
        const int kt = kt_begin + j * C::KS + kg;
        const bool in = kt < kt_end;
        return __builtin_amdgcn_make_buffer_rsrc((void *)(xq + (in ? kt : 0) * x_slab), 0, in ? (int)x_slab : 0, RSRC_FLAGS);
    };
    // quarter q (0..3) of the fill of one K tile: W chunk q and X chunk q, where they exist
    auto fill_quarter = [&](__amdgpu_buffer_rsrc_t wr, __amdgpu_buffer_rsrc_t xr, int stage, int q) {
        uint8_t *sb = ring + stage * C::STAGE_BYTES;
        if (q == 0) { load_chunk<0>(wr, sb + w_lds0, w_voff); load_chunk<0>(xr, sb + x_lds0, x_voff); }
        if (q == 1) {
            if (C::W_LOADS > 1) load_chunk<1>(wr, sb + w_lds0, w_voff);
            if (C::X_LOADS > 1) load_chunk<1>(xr, sb + x_lds0, x_voff);
        }
        if (q == 2) {
            if (C::W_LOADS > 2) load_chunk<2>(wr, sb + w_lds0, w_voff);
            if (C::X_LOADS > 2) load_chunk<2>(xr, sb + x_lds0, x_voff);
        }
        if (q == 3) {
            if (C::W_LOADS > 3) load_chunk<3>(wr, sb + w_lds0, w_voff);
            if (C::X_LOADS > 3) load_chunk<3>(xr, sb + x_lds0, x_voff);
        }
    };

    // ---- fragment read plan: lane (i = lane % 32, g = lane / 32) of a 32-row sub-tile reads, for
    // K half kk, granule 2 kk + g of row i (one ds_read_b128): its low 8 bytes feed the first MFMA
    // step of the half, the high 8 bytes the second.  Sub-tile bases are multiples of 32 rows, so
    // the swizzle depends on the lane only.
    const int fi = lane & 31, fg = lane >> 5;
    int frag_off[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) frag_off[kk] = fi * SEG + (((2 * kk + fg) ^ ((fi >> 2) & 3)) << 4);
    const int w_wave = wave_n * (C::TN * 32 * SEG), x_wave = C::W_BYTES + wave_m * (C::TM * 32 * SEG);

    v16i acc[C::TN][C::TM];
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0;

    // ---- software pipeline.
    // A K tile is four MFMA steps of 32 values, i.e. four groups G0..G3 of TN*TM MFMAs.  One
    // ds_read_b128 per operand row brings two steps (R0: steps 0-1, R1: steps 2-3).  While the
    // MFMAs of step s run, the operands of step s+1 are widened (3 VALU per MFMA), the next batch of
    // fragment reads is issued one read every other MFMA, and the HBM->LDS fill of a later tile is
    // issued a quarter per group.  Spreading the LDS reads and the fill matters: the four waves run
    // in lock step, and a burst of either backs up the LDS / address queues and stalls MFMA issue.
    //   G0(kt): MFMA step 0 | widen step 1 (R0 high)  | read R1(kt)     | fill(kt+S-1) quarter 2
    //   G1(kt): MFMA step 1 | widen step 2 (R1 low)   |                 | fill(kt+S-1) quarter 3
    //   -- tile kt+1 has landed; barrier; every wave is done reading tile kt --
    //   G2(kt): MFMA step 2 | widen step 3 (R1 high)  | read R0(kt+1)   | fill(kt+S) quarter 0, into tile kt's buffer
    //   G3(kt): MFMA step 3 | widen step 0' (R0' low) |                 | fill(kt+S) quarter 1
    v4i opW[2][C::TN], opX[2][C::TM], rawW[2][C::TN], rawX[2][C::TM];
    auto read_frags = [&](int stage, int kk, v4i (&wraw)[C::TN], v4i (&xraw)[C::TM]) {
        const uint8_t *wb = ring + stage * C::STAGE_BYTES + w_wave + frag_off[kk];
        const uint8_t *xb = ring + stage * C::STAGE_BYTES + x_wave + frag_off[kk];
#pragma unroll
        for (int tn = 0; tn < C::TN; ++tn) wraw[tn] = *reinterpret_cast<const v4i *>(wb + tn * (32 * SEG));
#pragma unroll
        for (int tm = 0; tm < C::TM; ++tm) xraw[tm] = *reinterpret_cast<const v4i *>(xb + tm * (32 * SEG));
    };
    // MFMAs on the current operands, widening half h of the raw fragments into the next operands
    auto group = [&](const v4i (&cw)[C::TN], const v4i (&cx)[C::TM], v4i (&nw)[C::TN], v4i (&nx)[C::TM],
                     const v4i (&rw)[C::TN], const v4i (&rx)[C::TM], int h) {
        constexpr int NM = C::TN * C::TM, NOP = C::TN + C::TM;
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            const int tn = i / C::TM, tm = i % C::TM;
            acc[tn][tm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cw[tn], cx[tm], acc[tn][tm], 0, 0, 0);
#pragma unroll
            for (int o = (i * NOP) / NM; o < ((i + 1) * NOP) / NM; ++o) {   // spread the NOP widenings over the NM MFMAs
                if (o == 0) nw[0] = widen(rw[0][2 * h], rw[0][2 * h + 1]);    // order: W0, X0..X(TM-1), W1..W(TN-1)
                else if (o <= C::TM) nx[o - 1] = widen(rx[o - 1][2 * h], rx[o - 1][2 * h + 1]);
                else nw[o - C::TM] = widen(rw[o - C::TM][2 * h], rw[o - C::TM][2 * h + 1]);
            }
        }
    };
    // pin the interleave of one group: one MFMA, then its share of VALU work; an LDS read after
    // the MFMAs that are followed by a widening when the group issues reads; the fill loads of
    // quarter q in the middle
    auto pin = [&](bool reads, int q) {
        constexpr int NM = C::TN * C::TM, NOP = C::TN + C::TM, VPM = (6 * NOP + NM - 1) / NM;
        const int n_vmem = (q < C::W_LOADS ? 1 : 0) + (q < C::X_LOADS ? 1 : 0);
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (reads) {
#pragma unroll
                for (int o = (i * NOP) / NM; o < ((i + 1) * NOP) / NM; ++o) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            if ((i == NM / 4 && n_vmem > 0) || (i == (3 * NM) / 4 && n_vmem > 1)) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // K-group shapes serve problems whose whole time is one workgroup's walk through K, and have registers to
    // spare: the epilogue's channel scales are fetched here, so that their latency hides under the first tile's.
    const int sub0 = C::KS > 1 ? kg * C::SUBS : 0;                          // first sub-tile of this wave's share of the epilogue
    const int fin_nw0 = n0 + (wave_n * C::TN + sub0 % C::TN) * 32, fin_mw0 = m0 + (wave_m * C::TM + sub0 / C::TN) * 32;
    float scv[C::NSC];
    int32_t zwv[C::NSC];
    if (C::KS > 1) load_scales<C::TNE, ZP>(scv, zwv, s_w, wsum, fin_nw0, N, lane);

    const int steps = (max(kt_end - kt_begin, 0) + C::KS - 1) / C::KS;      // the same for every K group: they share the barriers
#pragma unroll
    for (int s = 0; s < C::STAGES - 1; ++s) {
        __amdgpu_buffer_rsrc_t wr = w_desc(s), xr = x_desc(s);
#pragma unroll
        for (int q = 0; q < 4; ++q) fill_quarter(wr, xr, s, q);
    }
    // descriptors of the fill that is half way (step kt+S-1) and of the one that starts in G2 (step kt+S)
    __amdgpu_buffer_rsrc_t wr_a = w_desc(C::STAGES - 1), xr_a = x_desc(C::STAGES - 1);
    __amdgpu_buffer_rsrc_t wr_b = w_desc(C::STAGES), xr_b = x_desc(C::STAGES);
    fill_quarter(wr_a, xr_a, C::STAGES - 1, 0);
    fill_quarter(wr_a, xr_a, C::STAGES - 1, 1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(C::LOADS * (C::STAGES - 2) + C::HALF_LOADS));   // tile 0 is in
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, rawW[0], rawX[0]);
#pragma unroll
    for (int tn = 0; tn < C::TN; ++tn) opW[0][tn] = widen(rawW[0][tn][0], rawW[0][tn][1]);
#pragma unroll
    for (int tm = 0; tm < C::TM; ++tm) opX[0][tm] = widen(rawX[0][tm][0], rawX[0][tm][1]);
    __builtin_amdgcn_sched_barrier(0);

    int stage = 0;      // ring position of tile kt
    __builtin_amdgcn_s_setprio(2);     // MFMA loop: ahead of other workgroups' prologues and epilogues on this SIMD
    for (int kt = 0; kt < steps; ++kt) {
        const int stage_next = stage + 1 == C::STAGES ? 0 : stage + 1;
        const int stage_prev = stage == 0 ? C::STAGES - 1 : stage - 1;   // holds tile kt+S-1 (being filled)
        // G0
        read_frags(stage, 1, rawW[1], rawX[1]);
        fill_quarter(wr_a, xr_a, stage_prev, 2);
        group(opW[0], opX[0], opW[1], opX[1], rawW[0], rawX[0], 1);
        pin(true, 2);
        // G1
        fill_quarter(wr_a, xr_a, stage_prev, 3);
        group(opW[1], opX[1], opW[0], opX[0], rawW[1], rawX[1], 0);
        pin(false, 3);
        // own loads of tile kt+1 have landed (younger: all of tiles kt+2 .. kt+S-1); the barrier
        // extends that to every wave's loads and says every wave is done reading tile kt
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(C::LOADS * (C::STAGES - 2)));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // G2 (after the last tile the fragment reads hit a repeated copy; its results are unused)
        read_frags(stage_next, 0, rawW[0], rawX[0]);
        fill_quarter(wr_b, xr_b, stage, 0);
        group(opW[0], opX[0], opW[1], opX[1], rawW[1], rawX[1], 1);
        pin(true, 0);
        // G3
        fill_quarter(wr_b, xr_b, stage, 1);
        wr_a = wr_b;
        xr_a = xr_b;
        wr_b = w_desc(kt + C::STAGES + 1);
        xr_b = x_desc(kt + C::STAGES + 1);
        group(opW[1], opX[1], opW[0], opX[0], rawW[0], rawX[0], 0);
        pin(false, 1);
        stage = stage_next;
    }
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));   // drain the tail loads before LDS is reused
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
    __builtin_amdgcn_s_barrier();

    // ---- K groups: the accumulators of the KS groups are added through LDS (integers: exact, order-free) and the
    // sum stays distributed: group g ends up with sub-tiles g * P .. g * P + P - 1 of the wave's TN x TM (counted
    // along n first), so every wave of the workgroup adds 1 / KS of the registers and runs 1 / KS of the epilogue.
    // Every wave first stores the sub-tiles that belong to other groups (16-byte quads, lane-contiguous), then,
    // after one barrier, adds what the others stored for it.
    if (C::KS > 1) {
        constexpr int P = C::SUBS, TPG = C::WAVES * 64, QUAD_BYTES = TPG * 16;
        uint8_t *const xlane = lds + (wave * 64 + lane) * 16;
#pragma unroll
        for (int f = 0; f < C::TN * C::TM; ++f) {
            constexpr int KS1 = C::KS - 1;
            const int h = f / P, p = f % P;                          // receiving group, position in its share
            if (kg != h) {
                const int sender = kg - (kg > h ? 1 : 0);
                uint8_t *dst = xlane + ((h * KS1 + sender) * P + p) * (4 * QUAD_BYTES);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v16i &a = acc[f % C::TN][f / C::TN];
                    *reinterpret_cast<v4i *>(dst + q * QUAD_BYTES) = v4i{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_s_barrier();
        v16i mine[C::TNE][C::TME];
#pragma unroll
        for (int h = 0; h < C::KS; ++h) {
            if (kg == h) {
#pragma unroll
                for (int p = 0; p < P; ++p) mine[p % C::TNE][p / C::TNE] = acc[(h * P + p) % C::TN][(h * P + p) / C::TN];
#pragma unroll
                for (int sender = 0; sender < C::KS - 1; ++sender)
#pragma unroll
                    for (int p = 0; p < P; ++p)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v4i v = *reinterpret_cast<const v4i *>(xlane + (((h * (C::KS - 1) + sender) * P + p) * 4 + q) * QUAD_BYTES);
#pragma unroll
                            for (int e = 0; e < 4; ++e) mine[p % C::TNE][p / C::TNE][4 * q + e] += v[e];
                        }
            }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);
        __builtin_amdgcn_s_barrier();                                // the exchange area is free for the epilogue
        finish<C, C::TNE, C::TME, ALIGNED, DUMP, ZP>(mine, scv, zwv, lds, wave_all, wave, lane, sub0, fin_nw0, fin_mw0, M, N, s_a, d,
                                                 zp, wsum, y, acc_out, ws, splits, split, pid, total);
    } else {
        load_scales<C::TN, ZP>(scv, zwv, s_w, wsum, fin_nw0, N, lane);
        finish<C, C::TN, C::TM, ALIGNED, DUMP, ZP>(acc, scv, zwv, lds, wave_all, wave, lane, 0, fin_nw0, fin_mw0, M, N, s_a, d, zp,
                                               wsum, y, acc_out, ws, splits, split, pid, total);
    }
}

// 0 = choose the tile shape per problem; 1..8 = force one (testing and tuning)
static std::atomic<int> g_forced_tile{0};
static std::atomic<int> g_tile_map{0};
void set_gemm_tile(int tile) { g_forced_tile.store(tile, std::memory_order_relaxed); }
void set_gemm_map(int mode) { g_tile_map.store(mode, std::memory_order_relaxed); }
int forced_gemm_tile() { return g_forced_tile.load(std::memory_order_relaxed); }

template <class C, bool ALIGNED, bool DUMP, bool ZP>
static hipError_t launch_inst(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                              const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                              hipStream_t s, int32_t *ws = nullptr, int splits = 1)
{
    auto kern = linear_mfma_kernel<C, ALIGNED, DUMP, ZP>;
    const DeviceInfo *info;
    hipError_t e0 = device_info(&info);          // sets every instantiation's LDS attribute on the device's first use
    if (e0 != hipSuccess) return e0;
    int64_t tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    if (tiles_m * tiles_n * splits > 0x7fffffff) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)(tiles_m * tiles_n * splits)), dim3(C::THREADS), C::LDS_BYTES, s>>>(
        xq, wq, (int)M, (int)N, (int)k_tiles(K), (int)tiles_m, (int)tiles_n, s_a, s_w, d, zp, wsum, y, acc, ws, splits, g_tile_map.load(std::memory_order_relaxed));
    return hipGetLastError();
}

template <class C>
static hipError_t launch_cfg(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                             hipStream_t s, int32_t *ws = nullptr, int splits = 1)
{
    const bool aligned = N % 8 == 0;
#define FPTQ_GEMM_INST(A, D, Z) return launch_inst<C, A, D, Z>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s, ws, splits)
    if (wsum) {
        if (acc) { if (aligned) FPTQ_GEMM_INST(true, true, true); FPTQ_GEMM_INST(false, true, true); }
        if (aligned) FPTQ_GEMM_INST(true, false, true);
        FPTQ_GEMM_INST(false, false, true);
    }
    if (acc) { if (aligned) FPTQ_GEMM_INST(true, true, false); FPTQ_GEMM_INST(false, true, false); }
    if (aligned) FPTQ_GEMM_INST(true, false, false);
    FPTQ_GEMM_INST(false, false, false);
#undef FPTQ_GEMM_INST
}

// ---- tile shapes (all with 4 waves per K group).  The 256 x 256 tile has the best operand reuse and wins for long
// K; 256 x 128 with two workgroups per CU hides prologue and epilogue and fills partial rounds, and wins elsewhere;
// the 192- and one-workgroup 128-row shapes are kept for shapes neither fits; the K-group shapes serve problems with
// at most one workgroup per CU.
typedef GemmCfg<2, 2, 4, 4, 4> T256x256;           // waves of 128 x 128
typedef GemmCfg<2, 2, 3, 4, 4> T192x256;           // BN = 192: waves of 96 (n) x 128 (m)
typedef GemmCfg<2, 2, 4, 2, 4> T256x128;           // BM = 128: waves of 128 (n) x 64 (m)
typedef GemmCfg<2, 2, 4, 2, 3, 2> T256x128o2;      // the same tile, two workgroups per CU
typedef GemmCfg<2, 2, 2, 2, 3, 1, 2> T128x128k2;   // 128 x 128 alone on a CU, two K groups
typedef GemmCfg<2, 2, 4, 2, 3, 1, 2> T256x128k2;   // 256 x 128 alone on a CU, two K groups
typedef GemmCfg<1, 1, 2, 2, 4, 1, 4> T64x64k4;     // small tiles for problems with few of the larger ones, four K groups:
typedef GemmCfg<2, 1, 2, 2, 3, 1, 4> T128x64k4;    // 64 x 64 with one wave per group, 128 (N) x 64 (M) with two
// split K over workgroups, for problems whose 64 x 64 tiles cover at most half of the CUs
typedef GemmCfg<1, 1, 2, 2, 4, 1, 4, true> T64x64k4split;

// ---- the library's own scratch area, for callers that cannot allocate a workspace: device memory that lives as
// long as the process, one copy per GPU.  Its name is a host-side handle only; the device address is looked up once
// per device (gemm_device_init) and that pointer is what kernels and every other host-side use get.  Sized for the
// split-K exchange on a device of up to 256 CUs: one 64 x 64 INT32 partial tile per workgroup, at most one workgroup
// per CU, plus the counters.  The arrival counters at its start are zero when the code object is loaded and every
// launch leaves them zero (the last workgroup of a tile clears its counter); the partial tiles behind them are
// always written before they are read, so calls in sequence need nothing cleared in between.
constexpr int64_t SCRATCH_BYTES = (int64_t)256 * T64x64k4split::ACC_REGS * 64 * 4 + 4096;
static __device__ __align__(256) int32_t scratch[SCRATCH_BYTES / 4];

template <class C, bool ALIGNED, bool DUMP, bool ZP>
static hipError_t set_lds_attribute()
{
    return hipFuncSetAttribute((const void *)linear_mfma_kernel<C, ALIGNED, DUMP, ZP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               C::LDS_BYTES);
}

template <class... Cs>
static hipError_t set_lds_attributes()
{
    hipError_t e = hipSuccess;
    auto one = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    (void)one;
    ((one(set_lds_attribute<Cs, true, true, false>()), one(set_lds_attribute<Cs, true, false, false>()),
      one(set_lds_attribute<Cs, false, true, false>()), one(set_lds_attribute<Cs, false, false, false>()),
      one(set_lds_attribute<Cs, true, true, true>()), one(set_lds_attribute<Cs, true, false, true>()),
      one(set_lds_attribute<Cs, false, true, true>()), one(set_lds_attribute<Cs, false, false, true>())),
     ...);
    return e;
}

// Once per device, with that device current: every kernel instantiation gets its dynamic-LDS limit (so no launch
// has to set it later, e.g. under graph capture), and the scratch area's address on this device is looked up.
hipError_t gemm_device_init(DeviceInfo *info)
{
    hipError_t e = set_lds_attributes<T256x256, T192x256, T256x128, T256x128o2, T128x128k2, T256x128k2, T64x64k4, T128x64k4,
                                      T64x64k4split>();
    if (e != hipSuccess) return e;
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    info->scratch = static_cast<int32_t *>(ptr);
    info->scratch_bytes = SCRATCH_BYTES;
    return hipSuccess;
}

// Number of K ranges: as many as keep the workgroup count within the CUs, at most MAX_SPLITS, at least 16 K tiles
// (four per K group) each, none empty.  The exchange of partials pays from K = 6144 on (measured on N = 1024,
// M = 256: K = 4096 takes 8.0 us unsplit and 8.6 split, K = 6144 9.8 and 9.0, K = 14336 16.6 and 11.4, K = 28672
// 28.3 and 16.7).
static int64_t split_tiles(int64_t M, int64_t N) { return ((N + T64x64k4split::BN - 1) / T64x64k4split::BN) * ((M + T64x64k4split::BM - 1) / T64x64k4split::BM); }
static int split_count(int64_t M, int64_t N, int64_t K, int cus)
{
    const int64_t tiles = split_tiles(M, N), kt = k_tiles(K);
    if (tiles > cus / 2 || tiles > SPLIT_COUNTERS || K > 131071 || kt < 48) return 1;
    int64_t sp = cus / tiles;
    if (sp > kt / 16) sp = kt / 16;
    if (sp > MAX_SPLITS) sp = MAX_SPLITS;
    if (sp < 2) return 1;
    const int64_t per = (kt + sp - 1) / sp;
    return (int)((kt + per - 1) / per);
}

int64_t linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const int sp = split_count(M, N, K, device_cus_or_default());
    if (sp < 2) return 0;
    const int64_t tiles = split_tiles(M, N);
    return (SPLIT_COUNTERS + sp * tiles * T64x64k4split::ACC_REGS * (T64x64k4split::WAVES * 64)) * 4;
}

hipError_t launch_linear_mfma_ws(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                 const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                                 int32_t *ws, int64_t ws_bytes, hipStream_t s)
{
    const int sp = split_count(M, N, K, device_cus_or_default());
    if (sp < 2 || !ws || ws_bytes < linear_workspace_bytes(M, N, K) || (wsum && K > 65535) || forced_gemm_tile() != 0)
        return launch_linear_mfma(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    return launch_cfg<T64x64k4split>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s, ws, sp);
}

// Tile shape for a problem: index into the launch table (0 = 256 x 256, 1 = 192 x 256, 2 = 256 x 128, 3 = 256 x 128 with
// two workgroups per CU, 4 = 128 x 128 and 5 = 256 x 128 with two K groups, 6 = 64 x 64 and 7 = 128 x 64 with four).
static int choose_tile(int64_t M, int64_t N, int64_t K, int cus)
{
    const int forced = forced_gemm_tile();
    if (forced > 0) return forced - 1;
    // Estimated time in microseconds, fitted to measurements on uniform random operands on MI355X (the clock is
    // power-limited there, so a K tile costs about the same time whatever the MFMA utilisation):
    // one-workgroup-per-CU shapes run ceil(tiles / CUs) rounds of (fixed + per-K-tile) each.  With two
    // workgroups per CU the older one is served first, so epilogues overlap the other's main loop and
    // a partial last round of r * 2 CUs tiles costs about 0.5 + 0.15 r of a full one instead of 1; a partial
    // only round with more tiles than CUs runs at the pace of the CUs that hold two (0.88 of a full round
    // measured at r = 0.6).  At most one 256 x 128 tile per CU: the two-K-group variant, whose K tiles go
    // faster the fewer CUs are busy (0.67 us at 256 tiles, 0.55 at 160: the power limit again).
    auto tiles = [&](int64_t bn, int64_t bm) { return (double)(((N + bn - 1) / bn) * ((M + bm - 1) / bm)); };
    const double kt = (double)k_tiles(K), CUS = (double)cus;
    const double t21 = tiles(256, 128), x = t21 / (2 * CUS), frac = x - floor(x);
    const double rounds_o2 = x < 1.0 ? 0.7 + 0.3 * x : floor(x) + (frac > 0 ? fmax(frac, 0.5 + 0.15 * frac) : 0.0);
    const double never = 1e30;
    const double cost[5] = {
        ceil(tiles(256, 256) / CUS) * (12.9 + 1.235 * kt),
        ceil(tiles(192, 256) / CUS) * (11.0 + 0.900 * kt),
        t21 > CUS ? ceil(t21 / CUS) * (9.4 + 0.667 * kt) : never,
        // From 64 K tiles on the two large shapes tie in isolated launches, and the tie goes to the 256 x 256 tile: it
        // moves half the operand bytes through L2 and LDS per operation, and in a sustained sequence of launches (the
        // Llama-3-70B layer step, where the clock follows the board's power history) every launch runs 1 to 12 %
        // faster when all of them use it.
        t21 > CUS ? rounds_o2 * (7.8 + 1.304 * kt) * (kt >= 64 ? 1.03 : 1.0) : never,
        t21 <= CUS ? 8.5 + (0.35 + 0.32 * t21 / CUS) * kt : never,
    };
    int pick = 0;
    for (int i = 1; i < 5; ++i)
        if (cost[i] < cost[pick]) pick = i;
    if (pick == 4) pick = 5;       // the launch table: 4 = 128 x 128, 5 = 256 x 128, both with two K groups
    // Problems so small that even 128 x 128 tiles give every CU at most one workgroup take that tile: the
    // kernel time is then one workgroup's walk through K and the small tile walks fastest (17 against 25 us at
    // K = 4096).  A deeper ring does not help there.
    if (tiles(128, 128) <= CUS) pick = 4;
    // Fewer tiles still: the smallest tile shape that still gives every CU at most one workgroup, as four K
    // groups whose waves each hold a whole 64 x 64 block of outputs (half the LDS reads per MFMA of a 32 x 32
    // block).  Measured at K = 4096, N = 4096: 256 tokens 9 us on 64 x 64 tiles against 17 on 128 x 128; 512
    // tokens 12.5 us on 128 x 64 against 18.
    if (tiles(128, 64) <= CUS) pick = 7;
    if (tiles(64, 64) <= CUS) pick = 6;
    return pick;
}

// Limits of the MFMA kernel: the widened accumulator is 256 * acc with |acc| <= 64 K, and one K tile of all rows
// (rows * 64 bytes) must fit a 32-bit buffer descriptor.  Beyond them the simple kernel answers.
static bool mfma_serves(int64_t M, int64_t N, int64_t K, bool zero_point)
{
    return !(K > 131071 || (zero_point && K > 65535) || M > (1 << 24) || N > (1 << 24));
}

template <class C>
static void describe(int64_t M, int64_t N, int splits, LinearPlan *plan)
{
    snprintf(plan->kernel, sizeof plan->kernel, "GemmCfg<%d, %d, %d, %d, %d, %d, %d, %s>", C::WAVES_N, C::WAVES_M, C::TN, C::TM,
             C::STAGES, C::OCC, C::KS, C::SPLIT ? "true" : "false");
    plan->workgroups = ((M + C::BM - 1) / C::BM) * ((N + C::BN - 1) / C::BN) * splits;
    plan->threads = C::THREADS;
}

// What launch_linear_mfma / launch_linear_mfma_ws would launch for a shape on the current device (host arithmetic only).
void linear_mfma_plan(int64_t M, int64_t N, int64_t K, bool with_workspace, LinearPlan *plan)
{
    const int cus = device_cus_or_default();
    if (!mfma_serves(M, N, K, false)) {
        snprintf(plan->kernel, sizeof plan->kernel, "linear_ref_kernel");
        plan->workgroups = 0;
        plan->threads = 0;
        return;
    }
    const int sp = with_workspace && forced_gemm_tile() == 0 ? split_count(M, N, K, cus) : 1;
    if (sp >= 2) return describe<T64x64k4split>(M, N, sp, plan);
    switch (choose_tile(M, N, K, cus)) {
    case 1: return describe<T192x256>(M, N, 1, plan);
    case 2: return describe<T256x128>(M, N, 1, plan);
    case 3: return describe<T256x128o2>(M, N, 1, plan);
    case 4: return describe<T128x128k2>(M, N, 1, plan);
    case 5: return describe<T256x128k2>(M, N, 1, plan);
    case 6: return describe<T64x64k4>(M, N, 1, plan);
    case 7: return describe<T128x64k4>(M, N, 1, plan);
    default: return describe<T256x256>(M, N, 1, plan);
    }
}

hipError_t launch_linear_mfma(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                              const float *s_w, const float *d, int zp, const int32_t *wsum, uint16_t *y, int32_t *acc,
                              hipStream_t s)
{
    if (!mfma_serves(M, N, K, wsum != nullptr)) return launch_linear_ref(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    switch (choose_tile(M, N, K, device_cus_or_default())) {
    case 1: return launch_cfg<T192x256>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 2: return launch_cfg<T256x128>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 3: return launch_cfg<T256x128o2>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 4: return launch_cfg<T128x128k2>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 5: return launch_cfg<T256x128k2>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 6: return launch_cfg<T64x64k4>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    case 7: return launch_cfg<T128x64k4>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    default: return launch_cfg<T256x256>(xq, wq, M, N, K, s_a, s_w, d, zp, wsum, y, acc, s);
    }
}

}  // namespace fptq
