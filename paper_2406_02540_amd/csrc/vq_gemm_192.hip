// The 256 x 192 workgroup tile of the GEMM kernel template (vq_gemm_kernel.h): 4 x 3
// wavefronts of 64 tokens x 64 channels, three per SIMD.  For channel counts that tiles of
// 256 channels cover badly: a DiT hidden size of 1152 is 6 x 192 but 4.5 x 256.
#include "vq_gemm_kernel.h"

namespace vq {

namespace {
typedef TileShape<4, 3, 2> Tile192;
}

hipError_t launch_gemm_192(const GemmArgs& a, int w_bits, int num_cus, hipStream_t stream) {
    return launch_gemm_shape<Tile192>(a, w_bits, num_cus, stream);
}

}  // namespace vq
