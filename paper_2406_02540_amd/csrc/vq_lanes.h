// Host-side choice of how many lanes of a wavefront share a token (plain C++, no device code:
// the CPU tests compile this header on its own).
#pragma once

namespace vq {

// Lanes per token for a row of k8 chunks held as fp32 (8 registers per chunk and lane): the
// widest group that still keeps 85 % of its lanes busy, so that the row takes few registers
// and many wavefronts are resident; failing that, the group with the fewest idle lanes.
// Returns 16, 32 or 64 (at most 16 chunks per lane of a group of 64 are supported).
inline int lanes_for_row(int k8) {
    int best = 64, best_idle = 1 << 30;
    for (int lanes = 64; lanes >= 16; lanes >>= 1) {
        const int nch = (k8 + lanes - 1) / lanes;
        if (nch > 16) break;
        const int idle = nch * lanes - k8;
        if (idle * 100 <= 15 * nch * lanes) return lanes;
        if (idle < best_idle) {
            best_idle = idle;
            best = lanes;
        }
    }
    return best;
}

}  // namespace vq
