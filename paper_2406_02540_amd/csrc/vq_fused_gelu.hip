// The GELU producers (exact and tanh form) of the quantizers fused behind their producers
// (vq_fused_kernel.h), a translation unit of their own to share the compile time.
#include "vq_fused_kernel.h"

namespace vq {

hipError_t launch_producer_gelu(int producer, const FusedArgs& a, hipStream_t stream) {
    return producer == kGeluErf ? launch_producer<kGeluErf>(a, stream) : launch_producer<kGeluTanh>(a, stream);
}

}  // namespace vq
