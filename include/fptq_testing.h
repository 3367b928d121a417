/*
 * fptq_testing -- a knob and a query of libfptq.so for its own tests, profiles and tuning runs; applications have
 * no use for them.
 */
#ifndef FPTQ_TESTING_H
#define FPTQ_TESTING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Forces the prefill kernel's tile shape for every later fptq_w4a4_linear call of the process (an atomic, so it may
 * be set while other threads launch; those calls see the old or the new value): 0 = chosen per problem (default),
 * 1 = 256x256, 2 = 192 (N) x 256 (M), 3 = 256 (N) x 128 (M), 4 = 256 x 128 with two workgroups per CU, 5 = 128 x 128
 * and 6 = 256 x 128 with two K groups per workgroup, 7 = 64 x 64 and 8 = 128 (N) x 64 (M) with four K groups.
 * A forced shape also sends calls with few tokens to the prefill kernel.  Results do not depend on it.
 * Returns 0, or FPTQ_ERR_VALUE (-6) for a value outside 0..8. */
int fptq_set_gemm_tile(int tile);

/* How the prefill kernel's workgroups map to output tiles: 0 (default) = every XCD (the hardware deals consecutive
 * workgroups to the 8 XCDs in turn) works through a contiguous run of tiles, in bands of 8 N-tiles, so that the tiles
 * in flight on an XCD share operand panels in its L2; 1 = tiles in launch order, i.e. dealt round-robin to the XCDs
 * (for measuring what the mapping is worth).  Results do not depend on it.  Returns 0 or FPTQ_ERR_VALUE (-6). */
int fptq_set_gemm_map(int mode);

/* The same for the few-token kernel's launch shape: 0 = chosen per problem (default), otherwise
 * waves per workgroup (8 or 16) * 100 + K tiles per batch of loads (1, 2 or 4) * 10 + 16-channel groups per workgroup
 * (1, 2 or 4), e.g. 1612.  Results do not depend on it.  Returns 0, or FPTQ_ERR_VALUE (-6) for any other value. */
int fptq_set_decode_shape(int code);

/* Host arithmetic only: which kernel fptq_w4a4_linear (with_workspace = 0) or fptq_w4a4_linear_ws with a large enough
 * workspace (1) would launch for this shape on the current device (an MI355X's 256 compute units are assumed when no
 * device answers).  kernel receives the tile configuration as it appears in a profiler's kernel name, e.g.
 * "GemmCfg<2, 2, 4, 4, 4, 1, 1, false>", or "linear_decode_kernel" / "linear_ref_kernel" (workgroups and threads are
 * 0 for those two); workgroups x threads is the grid a kernel trace shows.  Returns 0 or a negative FPTQ_ERR_* code. */
int fptq_linear_launch_plan(int64_t M, int64_t N, int64_t K, int with_workspace, char *kernel, int kernel_len,
                            int64_t *workgroups, int *threads);

#ifdef __cplusplus
}
#endif
#endif /* FPTQ_TESTING_H */
