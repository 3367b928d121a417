/*
 * fptq_testing -- a knob of libfptq.so for its own tests and for tuning runs; applications have no use for it.
 */
#ifndef FPTQ_TESTING_H
#define FPTQ_TESTING_H

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

#ifdef __cplusplus
}
#endif
#endif /* FPTQ_TESTING_H */
