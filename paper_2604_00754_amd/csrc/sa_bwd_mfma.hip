// bf16 backward of Stochastic Attention on gfx950 matrix cores (placeholder until the kernels land).
#include "sa_common.h"

namespace sa {

hipError_t launch_bwd_mfma_bf16(const Pass&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace sa
