// The register-resident token row of the quantizers: how a wavefront holds a token,
// and the steps from the fp32 row to int8 codes and the token's scale (ViDiT-Q Sec. 4.1,
// Sec. 3.1 Eq. 2 in symmetric form, activation side of Sec. 4.2 Eq. 3).  Shared by the
// stand-alone quantizer and by the kernels that fuse it behind a producer.
//
// LANES (64, 32 or 16) lanes of a wavefront share a token, so a wavefront holds
// 64 / LANES tokens.  Lane s of a token owns its 16-byte chunks s, s + LANES, ...
// (8 fp16 each): every load instruction of the wave covers contiguous pieces of
// 16 * LANES bytes and every store half of that.  NCH = chunks per lane.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vq_lanes.h"

namespace vq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int int2v __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kQuantThreads = 256;
constexpr int kRowsPerBlock = kQuantThreads / kWave;

// Rounds to the nearest integer (halves to even), clamps to [-qmax, qmax].
__device__ __forceinline__ int quantize_one(float t, float inv, float qmax) {
    float q = __builtin_rintf(t * inv);
    q = fminf(fmaxf(q, -qmax), qmax);
    return (int)q;
}

__device__ __forceinline__ int pack4(int a, int b, int c, int d) {
    return (a & 0xFF) | ((b & 0xFF) << 8) | ((c & 0xFF) << 16) | (d << 24);
}

// Which token and which lane of it this thread is.
template <int LANES>
struct RowLane {
    long m;       // token
    int sub;      // lane within the token's group
    bool row_ok;  // lanes of a missing token idle but take part in the shuffles
    __device__ __forceinline__ RowLane(int M) {
        const int lane = threadIdx.x & (kWave - 1);
        sub = lane & (LANES - 1);
        m = ((long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6)) * (kWave / LANES) + lane / LANES;
        row_ok = m < M;
    }
};

// Sum (or maximum) over the LANES lanes of a token; every lane gets the result.
// Data moves between lanes without LDS round trips where the hardware allows it: DPP quad
// permutes (lane ^ 1, lane ^ 2), then the mirrored lane of the other half of 8 and of 16
// lanes (by then both halves are uniform, so any lane of the other half will do), a
// ds_swizzle for lane ^ 16 and a permute through LDS only for lane ^ 32.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int LANES, class Op>
__device__ __forceinline__ float group_reduce(float v, Op op) {
    static_assert(LANES == 16 || LANES == 32 || LANES == 64, "lane groups are 16, 32 or 64 wide");
    v = op(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    v = op(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    v = op(v, dpp_move<0x141>(v));  // row_half_mirror
    v = op(v, dpp_move<0x140>(v));  // row_mirror
    if (LANES >= 32)
        v = op(v, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (16 << 10) | 0x1F)));
    if (LANES >= 64) v = op(v, __shfl_xor(v, 32, kWave));
    return v;
}
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
    return group_reduce<LANES>(v, [](float a, float b) { return a + b; });
}
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
    return group_reduce<LANES>(v, [](float a, float b) { return fmaxf(a, b); });
}

// The token's fp16 row -> fp32 registers (chunks past the row, or of a missing token: zeros).
// MUL_AT_LOAD: the balancing factor is multiplied in here, chunk by chunk as the data
// arrives (the plain quantizer; a producer in between needs it after itself instead).
template <int NCH, int LANES, bool MUL_AT_LOAD = false>
__device__ __forceinline__ void load_row(const half8* __restrict__ row, bool row_ok, int sub, int K8,
                                         float (&t)[NCH][8], const float4v* __restrict__ chan_mul = nullptr) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + sub;
        if (row_ok && c < K8) {
            const half8 v = __builtin_nontemporal_load(row + c);
#pragma unroll
            for (int j = 0; j < 8; ++j) t[i][j] = (float)v[j];
            if (MUL_AT_LOAD) {
                const float4v m0 = chan_mul[2 * c], m1 = chan_mul[2 * c + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t[i][j] = t[i][j] * m0[j];
                    t[i][4 + j] = t[i][4 + j] * m1[j];
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) t[i][j] = 0.0f;
        }
    }
}

// fp32 row -> balancing factor folded in, absmax of the token, its scale, int8 codes.
// Two IEEE divisions per token, none per element.  HAS_MUL = false: chan_mul is not looked
// at (there is none, or load_row has applied it).
template <int NCH, int LANES, bool HAS_MUL>
__device__ __forceinline__ void fold_quantize_store(float (&t)[NCH][8], const float4v* __restrict__ chan_mul,
                                                    bool row_ok, int sub, int K8, long m,
                                                    int2v* __restrict__ xq, float* __restrict__ x_scale) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + sub;
        if (row_ok && c < K8) {
            if (HAS_MUL) {
                const float4v m0 = chan_mul[2 * c], m1 = chan_mul[2 * c + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t[i][j] = t[i][j] * m0[j];
                    t[i][4 + j] = t[i][4 + j] * m1[j];
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(t[i][j]));
        }
    }
    amax = group_max<LANES>(amax);

    float scale = 0.0f, inv = 0.0f;
    if (amax != 0.0f) {
        scale = amax / 127.0f;
        inv = 127.0f / amax;
    }
    if (row_ok && sub == 0) x_scale[m] = scale;

    int2v* qrow = xq + (row_ok ? m : 0) * K8;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + sub;
        if (row_ok && c < K8) {
            int q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = quantize_one(t[i][j], inv, 127.0f);
            int2v o;
            o.x = pack4(q[0], q[1], q[2], q[3]);
            o.y = pack4(q[4], q[5], q[6], q[7]);
            qrow[c] = o;
        }
    }
}

}  // namespace vq
