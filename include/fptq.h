/*
 * fptq -- statically quantized INT4-weight x INT4-activation linear layer for AMD MI355X (gfx950).
 *
 * The library implements the run-time side of FPTQuant's quantized linear map:
 *
 *     x~_t   = S_t * x_t                         per-token scale,            Sec. 3.1.3 (Step 1)
 *     q_t,k  = clamp(rne(x~_t,k / s_a), -8, 7)   static per-tensor INT4,     App. B "Static quantization"
 *     acc_t,o = sum_k q_t,k * w_o,k              INT32 accumulation,         App. J "Setup"
 *     y_t,o  = bf16(acc_t,o * s_a * s_w[o])      float scales after the
 *                                                integer matmul,             App. B "Static quantization"
 *
 * with 4-bit operands stored two per byte (App. J).  The mergeable transforms of Sec. 3.1.1 and
 * 3.1.2 are folded into the weights offline and never appear here.
 *
 * Conventions
 *   - Plain C ABI.  Every tensor pointer is a DEVICE pointer; scalars are passed by value.
 *   - The caller owns all memory.  Entry points allocate nothing, never synchronise, and enqueue their
 *     kernels on `stream` (a hipStream_t; NULL = the null stream).  They can be captured into a HIP graph
 *     (kernel launches only, no memset or copy nodes).  The first call on a device sets that device up (kernel
 *     attributes, device properties); call fptq_init() on the device, or any entry point, before capturing.
 *     Entry points may be called from several threads and on several devices (the current device is used).
 *   - Every function returns 0 (FPTQ_OK) or a negative FPTQ_ERR_* code; arguments are validated
 *     before anything is launched, so a failed call writes nothing.  fptq_last_error() returns a
 *     thread-local description of the last failure.
 *   - X is [M x K] bf16 row-major (tokens x in-features).  W is [N x K] (out x in).  Y is [M x N]
 *     bf16 row-major.  Any M, N, K >= 1 is accepted (M*K, N*K, M*N < 2^40); the linear entry points also need
 *     K <= 2^25 - 1 (K <= 2^24 - 1 with a zero point), the longest sums for which INT32 accumulation is exact,
 *     and return FPTQ_ERR_SHAPE beyond that.
 *
 * Packed INT4 layout (the same for activations and weights, produced only by this library):
 *   K is cut into tiles of 128 values (64 bytes); the buffer holds, tile after tile, one 64-byte
 *   segment per row:   byte(row, k) = ((k / 128) * rows + row) * 64 + (k % 128) / 2,
 *   value k in the low nibble when k is even, the high nibble when odd, two's complement.
 *   K is padded to a multiple of 128 with zeros.  fptq_packed_bytes() gives the buffer size.
 *   fptq_unpack() converts back to one int8 per value, so callers never depend on this layout.
 */
#ifndef FPTQ_H
#define FPTQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FPTQ_OK 0
#define FPTQ_ERR_NULL (-1)  /* a required pointer is NULL                          */
#define FPTQ_ERR_SHAPE (-2) /* M, N or K is < 1 or too large                       */
#define FPTQ_ERR_SIZE (-3)  /* a buffer size passed by the caller is too small     */
#define FPTQ_ERR_MODE (-4)  /* unknown scale mode, or its arguments are missing    */
#define FPTQ_ERR_HIP (-5)   /* the HIP runtime refused a launch (see last_error)   */
#define FPTQ_ERR_VALUE (-6) /* a scalar is not usable (s_a not finite or <= 0)     */
#define FPTQ_ERR_ALIGN (-7) /* a pointer is misaligned: packed buffers, y_bf16 and
                               acc_dbg need 16 bytes, fp32 vectors 4, x_bf16 2     */

/* How fptq_quantize_act obtains the per-token scale S_t (Sec. 3.1.3). */
#define FPTQ_SCALE_NONE 0  /* S_t = 1                                                          */
#define FPTQ_SCALE_RMS 1   /* S_t = 1 / sqrt(mean_k x_t,k^2 + eps): what the block's RMSNorm computes */
#define FPTQ_SCALE_GIVEN 2 /* S_t = row_scale_in[t]: the S_n carried by the recursion of Eq. (6)-(7)  */

int fptq_version(void);
const char *fptq_last_error(void);

/* Optional: set the current device up now (otherwise the first call that launches on it does).  Idempotent,
 * thread-safe; call it once per device before capturing entry points into a HIP graph. */
int fptq_init(void);

/* Bytes of a packed [rows x K] INT4 buffer in the library layout; negative FPTQ_ERR_SHAPE if
 * rows < 1 or K < 1. */
int64_t fptq_packed_bytes(int64_t rows, int64_t K);

/*
 * Offline: pack INT4 weights (App. J double-packed storage).
 *   w_int          device, int8 [N x K] row-major, one value per byte; only the low nibble is kept,
 *                  so values outside [-8, 7] are a caller error.
 *   w_packed       device, at least fptq_packed_bytes(N, K) bytes (w_packed_bytes is checked).
 * The packed blob serves both the prefill and the decode kernels.
 */
int fptq_pack_weights(const int8_t *w_int, int64_t N, int64_t K, void *w_packed, int64_t w_packed_bytes,
                      void *stream);

/*
 * Per-token scale + static quantization + packing of the activations, one pass over X
 * (Sec. 3.1.3 Step 1; App. B static quantization; App. J storage).
 *   x_bf16         device, bf16 [M x K] row-major (leading dimension K)
 *   scale_mode     FPTQ_SCALE_*; eps is used by RMS only; row_scale_in [M] fp32 is required by GIVEN
 *   s_a            static activation scale (> 0, finite), fixed by calibration ahead of time
 *   xq_packed      device, at least fptq_packed_bytes(M, K) bytes (xq_bytes is checked)
 *   row_scale_out  device, fp32 [M] or NULL: receives S_t (1 for NONE), e.g. to continue the
 *                  recursion or to undo the scale later
 * Arithmetic: sum of squares in fp64; S_t = (float)(1 / sqrt(ss / K + eps)); c_t = S_t * (1.0f / s_a)
 * in fp32; q = clamp(rne((float)x * c_t), -8, 7); NaN quantizes to 0, +-Inf to 7 / -8.
 */
int fptq_quantize_act(const void *x_bf16, int64_t M, int64_t K, int scale_mode, float eps,
                      const float *row_scale_in, float s_a, void *xq_packed, int64_t xq_bytes,
                      float *row_scale_out, void *stream);

/*
 * The same with the online Hadamard transform T_d in front of the quantizer (Sec. 3.1.4; App. D,
 * "Hadamard non-powers of 2"): every row is transformed block-wise, x' = x blockdiag(H_B / sqrt(B)),
 * then scaled, quantized and packed as above.  The inverse is merged into the weights offline.
 *   hadamard_block  B, a power of two dividing K: 256, 512, 1024, 2048 or 4096 (the paper takes the largest
 *                   power of two dividing the width: 256 for 11008 = 43 * 256, 2048 for 14336, 4096 for
 *                   28672); anything else, or a K that B does not divide, returns FPTQ_ERR_SHAPE.
 *                   x_bf16 must be 16-byte aligned.
 *   FPTQ_SCALE_RMS takes S_t from the untransformed row (what the norm layer computes).
 * Arithmetic: in-place butterflies in fp32 with strides B/2, ..., 1, each pair (a, b) -> (a + b, a - b);
 * c_t = (S_t * (1.0f / s_a)) * (float)(1 / sqrt(B)); q = clamp(rne(h * c_t), -8, 7).
 */
int fptq_quantize_act_hadamard(const void *x_bf16, int64_t M, int64_t K, int hadamard_block, int scale_mode, float eps,
                               const float *row_scale_in, float s_a, void *xq_packed, int64_t xq_bytes,
                               float *row_scale_out, void *stream);

/*
 * One step of the scaled residual stream (Sec. 3.1.3, Eq. 5-7) fused with the quantizer of the next
 * block's input, in one pass over the two inputs:
 *     Z~ = X~_{n-1} + Y~_{n-1};  nrm = sqrt(mean_k Z~^2 + eps);  S_n = S_{n-1} / nrm;
 *     X~_n = Z~ / nrm  (new residual and, at once, the gain-free RMSNorm output);
 *     q = clamp(rne(X~_n / s_a), -8, 7), packed.
 *   x_res_bf16, y_bf16  device, bf16 [M x K]: the scaled residual and the scaled block output
 *   s_prev              device, fp32 [M] or NULL (= all ones, the first block)
 *   x_next_bf16         device, bf16 [M x K]: receives X~_n (may alias x_res_bf16 or y_bf16)
 *   s_next              device, fp32 [M]: receives S_n
 *   xq_packed           device, packed INT4 of X~_n / s_a for fptq_w4a4_linear
 * Arithmetic (fp32 unless noted): z = (float)x + (float)y; sum of z^2 in fp64;
 * inv = (float)(1 / sqrt(ss / K + eps)); S_n = S_{n-1} * inv; X~_n = bf16(z * inv);
 * c = inv * (1.0f / s_a); q = clamp(rne(z * c), -8, 7).
 */
int fptq_residual_norm_quantize(const void *x_res_bf16, const void *y_bf16, int64_t M, int64_t K, const float *s_prev,
                                float eps, float s_a, void *x_next_bf16, float *s_next, void *xq_packed, int64_t xq_bytes,
                                void *stream);

/*
 * Dynamic activation quantization (App. B "Dynamic quantization"; the paper's second run-time
 * setting, App. J "Dynamic INT4 runtime"): the scale is computed per token at run time,
 *     s_t = max_k |x_t,k| / 7,   q = clamp(rne(x * (1 / s_t)), -8, 7)    (fp32; NaNs ignored in the
 * maximum; a zero or infinite maximum gives s_t = 1).
 *   token_scale_out  device, fp32 [M], required: receives s_t.  Feed the packed result to
 *                    fptq_w4a4_linear with s_a = 1.0f and row_out_scale = token_scale_out, which makes
 *                    the epilogue y = bf16(acc * s_w[o] * s_t).
 */
int fptq_quantize_act_dynamic(const void *x_bf16, int64_t M, int64_t K, void *xq_packed, int64_t xq_bytes,
                              float *token_scale_out, void *stream);

/*
 * The quantized linear layer proper: INT4 x INT4 matmul with INT32 accumulation and the
 * float-scale epilogue (App. J; App. B).  Picks a few-token kernel (bound by the weight read) for
 * M <= 32, and for M <= 64 against fewer than 10240 channels, and the INT8-MFMA GEMM otherwise.
 *   xq_packed      device, packed activations [M x K] from fptq_quantize_act
 *   w_packed       device, packed weights [N x K] from fptq_pack_weights
 *   s_a            the same static activation scale given to fptq_quantize_act
 *   s_w            device, fp32 [N]: per-output-channel weight scales
 *   row_out_scale  device, fp32 [M] or NULL: optional extra per-token factor d_t on the output
 *                  (NULL leaves the output in the scaled representation Y~ = S * Y of Eq. (5))
 *   y_bf16         device, bf16 [M x N] row-major
 *   acc_dbg        device, int32 [M x N] or NULL: when given, also receives the exact integer
 *                  accumulators (for parity checks; leave NULL in timed runs)
 * Epilogue arithmetic (fp32): y = bf16_rne((float)acc * (s_a * s_w[o]) [* d_t]).
 */
int fptq_w4a4_linear(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                     const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream);

/*
 * Asymmetric static activation grid (App. D: the scale and the offset of every quantizer are
 * parameters): the integer code is shifted by a zero point z in [-8, 7] before clamping,
 *     v = clamp(rne(x * S_t / s_a) + z, -8, 7),   representing s_a * (v - z)   (NaN -> z),
 * and the linear layer removes it after the integer matmul:
 *     y = bf16((acc - z * w_row_sum[o]) * (s_a * s_w[o]) [* d_t]),   w_row_sum[o] = sum_k w[o, k].
 * fptq_weight_row_sums computes w_row_sum (device int32 [N]) offline from the unpacked int8 weights.
 * Everything else is as in fptq_quantize_act / fptq_w4a4_linear; acc_dbg receives the raw sum_k v w.
 */
int fptq_quantize_act_asym(const void *x_bf16, int64_t M, int64_t K, int scale_mode, float eps, const float *row_scale_in,
                           float s_a, int zero_point, void *xq_packed, int64_t xq_bytes, float *row_scale_out, void *stream);
int fptq_weight_row_sums(const int8_t *w_int, int64_t N, int64_t K, int32_t *sums, void *stream);
int fptq_w4a4_linear_zp(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                        const float *s_w, const float *row_out_scale, int zero_point, const int32_t *w_row_sum,
                        void *y_bf16, int32_t *acc_dbg, void *stream);

/*
 * fptq_w4a4_linear with a workspace.  A problem with at most 128 output tiles of 64 x 64 (M * N up to about
 * half a million outputs) and K >= 6144 leaves half of the CUs or more idle; with a workspace the kernel splits
 * K over up to four workgroups per tile, which leave their partial INT32 accumulators in the workspace, and the
 * last one to arrive adds them (integers: the result does not depend on the order) and writes y.
 *   workspace        device, 256-byte aligned, at least fptq_linear_workspace_bytes(M, N, K) bytes, or NULL.
 *                    It must be zero-filled once before its first use; every call leaves the part that has
 *                    to be zero as it found it, so one workspace (sized for the largest problem) can serve calls
 *                    of any shapes in turn.  Calls that share a workspace must not overlap in time.
 *   workspace_bytes  its size.  Too small, NULL, or a shape that does not profit (fptq_linear_workspace_bytes
 *                    returns 0): the call behaves exactly like fptq_w4a4_linear.
 * Results are identical to fptq_w4a4_linear's.
 */
int64_t fptq_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);
int fptq_w4a4_linear_ws(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                        const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *workspace,
                        int64_t workspace_bytes, void *stream);

/*
 * fptq_w4a4_linear_ws without the workspace argument, for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid it): the split-K exchange goes through a scratch
 * area built into the library, 4 MiB + 4 KiB of device memory per GPU that the library's code object holds from
 * load until the process ends.  Nothing is allocated or freed by this call, ever; the per-device set-up (fptq_init,
 * or the first call on the device) only looks the area's address up.
 *   - Same arguments, results and errors as fptq_w4a4_linear.  A shape whose split would need more scratch than the
 *     area holds (possible only on a device with more than 256 compute units) returns FPTQ_ERR_SIZE and launches
 *     nothing; shapes that would not split K run exactly as in fptq_w4a4_linear.
 *   - All calls on one GPU share that GPU's area.  Every call leaves the part that must be zero (the arrival
 *     counters) zero, and writes every partial sum before reading it, so calls in sequence, of any mix of shapes,
 *     need no clearing in between.  Calls that overlap in time on one GPU (two streams, two threads) race on it
 *     and must not be made; use fptq_w4a4_linear_ws with one workspace per stream for that.
 */
int fptq_w4a4_linear_noalloc(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                             const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream);

/* Same contract as fptq_w4a4_linear but always runs the simple one-thread-per-output kernel
 * (no MFMA, no LDS).  A second, independent GPU implementation used by the tests to cross-check
 * the tuned kernels at full size. */
int fptq_w4a4_linear_ref(const void *xq_packed, const void *w_packed, int64_t M, int64_t N, int64_t K, float s_a,
                         const float *s_w, const float *row_out_scale, void *y_bf16, int32_t *acc_dbg, void *stream);

/* Library layout -> one int8 per value, [rows x K] row-major (for parity checks and debugging). */
int fptq_unpack(const void *packed, int64_t rows, int64_t K, int8_t *out_int8, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FPTQ_H */
