// Few-token (decode) kernel of the quantized linear layer.
#include "fptq_common.h"

namespace fptq {

hipError_t launch_linear_decode(const uint8_t *xq, const uint8_t *wq, int64_t M, int64_t N, int64_t K, float s_a,
                                const float *s_w, const float *d, uint16_t *y, int32_t *acc, hipStream_t s)
{
    return launch_linear_ref(xq, wq, M, N, K, s_a, s_w, d, y, acc, s);
}

}  // namespace fptq
