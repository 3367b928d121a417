/*
 * fptq_probe -- measurement aids for benchmarks of the fptq library on AMD MI355X (gfx950).  Not part of the
 * quantized linear layer and not linked into libfptq.so: loops with nothing but the resource being measured, so a
 * benchmark can report the rate the device sustains next to the kernels' own, from the same run.
 *
 * Plain C ABI, device pointers, kernels enqueued on `stream` (a hipStream_t; NULL = the null stream), nothing
 * allocated, nothing synchronised.  Errors are negative; fptq_probe_last_error() describes the last one of the thread.
 */
#ifndef FPTQ_PROBE_H
#define FPTQ_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FPTQ_PROBE_ERR_NULL (-1)
#define FPTQ_PROBE_ERR_SHAPE (-2)
#define FPTQ_PROBE_ERR_HIP (-5)
#define FPTQ_PROBE_ERR_VALUE (-6)

const char *fptq_probe_last_error(void);

/*
 * 256 workgroups of 4 waves, each wave issuing iters x 64 v_mfma_i32_32x32x32_i8 on register operands: dense = 0 all
 * zero; 1 random nibbles in the high half of every byte (the operand form of the prefill kernel), the same for the whole
 * run; 2 the same form redrawn every iteration (3.5 VALU instructions per MFMA beside the matrix pipe, about the prefill
 * kernel's widening load, and inputs that change like real data: the rate the power limit allows a kernel that feeds
 * the matrix pipe fresh dense operands, before any memory traffic).
 *   out  device, 65536 int32: receives a checksum per thread.
 * Returns the number of integer operations launched (> 0) or a negative error.  The caller times the launch.
 */
int64_t fptq_probe_mfma_rate(int iters, int dense, int32_t *out, void *stream);

/*
 * The same loop with the choices spelled out: operands 0 zero, 1 fixed random, 2 redrawn every iteration, 3 the
 * instruction stream of 2 on operands that stay zero (what the extra VALU instructions cost by themselves);
 * workgroups_per_cu 1 or 2 (one or two waves per SIMD).  out: device, 65536 x workgroups_per_cu int32.
 */
int64_t fptq_probe_mfma_rate_ex(int iters, int operands, int workgroups_per_cu, int32_t *out, void *stream);

/*
 * Streams `bytes` (a multiple of 16; src 16-byte aligned) once and XORs all 16-byte words into xor4 (device,
 * 4 int32, which the caller zeroes first), component by component.
 */
int fptq_probe_read(const void *src, int64_t bytes, int32_t *xor4, void *stream);

/*
 * The same read as one burst, the launch pattern of a kernel that is one memory round trip long: `threads` threads per
 * workgroup (256 or 1024), each issuing `loads` (1, 2, 4 or 8) streaming 16-byte loads at once; the grid covers the
 * buffer exactly once.  For buffers of a few megabytes this is the read a few-token linear layer cannot beat.
 *   xor1024  device, 1024 int32 (256 slots of 4), zeroed by the caller: workgroup b XORs into slot b % 256, so that the
 *            atomics do not serialise on one address; the XOR of all slots is the XOR of the buffer's 16-byte words.
 */
int fptq_probe_read_burst(const void *src, int64_t bytes, int32_t *xor1024, int threads, int loads, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FPTQ_PROBE_H */
