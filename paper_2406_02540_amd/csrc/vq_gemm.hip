// The int8 (and packed 4-bit, and fp16 comparison) GEMM with the dequantization epilogue:
// the 256 x 256 workgroup tile of the kernel template in vq_gemm_kernel.h, and the choice
// between it, the 256 x 192 tile (vq_gemm_192.hip) and the small-tile kernel
// (vq_gemm_small.hip) for a given problem.
#include "vq_gemm_kernel.h"

namespace vq {

namespace {
typedef TileShape<2, 4, 4> Tile256;  // 2 x 4 wavefronts of 128 tokens x 64 channels

// How long a launch takes in units of one 256 x 256 tile on one CU: every XCD walks its
// share of the tiles in rounds of one tile per CU, and a tile costs what it holds.
double rounds_cost(int M, int N, int tile_c, int num_cus) {
    const long tiles = (long)((M + 255) / 256) * ((N + tile_c - 1) / tile_c);
    const long per_xcd = (tiles + kXcds - 1) / kXcds;
    const int cus_per_xcd = num_cus >= kXcds ? num_cus / kXcds : 1;
    const long rounds = (per_xcd + cus_per_xcd - 1) / cus_per_xcd;
    return (double)rounds * tile_c / 256.0;
}
}  // namespace

hipError_t launch_gemm(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
                       const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out,
                       int M, int N, int K, int num_cus, hipStream_t stream) {
    // A problem whose large tiles would leave more than half of the CUs idle is latency
    // bound: the small-tile kernel puts many more loads in flight.
    const long tiles256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (tiles256 * 2 <= num_cus && w_bits != 16)
        return launch_gemm_small(xq, x_scale, w, w_bits, w_scale, bias_f16, y_f16, acc_out, M, N, K, stream);
    GemmArgs a;
    a.xq = xq;
    a.x_scale = x_scale;
    a.w = w;
    a.w_scale = w_scale;
    a.bias = (const _Float16*)bias_f16;
    a.y = (_Float16*)y_f16;
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.K = K;
    a.tiles_t = a.tiles_c = a.tiles = a.tiles_per_xcd = a.slots = 0;  // (set for the chosen tile)
    // The narrower tile moves a sixth more operand bytes per multiply-add and is chosen only
    // where it saves rounds of tiles.
    const bool narrow = rounds_cost(M, N, 192, num_cus) * 1.05 < rounds_cost(M, N, 256, num_cus);
    if (narrow) return launch_gemm_192(a, w_bits, num_cus, stream);
    return launch_gemm_shape<Tile256>(a, w_bits, num_cus, stream);
}

}  // namespace vq
