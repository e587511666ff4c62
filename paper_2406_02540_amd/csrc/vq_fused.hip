// The per-token quantizer fused behind the operation that produces its input
// (ViDiT-Q Sec. 5.1 "Hardware Implementation Settings": the quantization is integrated
// into the preceding LayerNorm, GELU and residual operations; Sec. 4.1 notes that the
// dynamic parameters only need the extrema of the token and can be fused with the
// previous operation).  The producer's output never goes to memory as fp16: a token is
// read once, transformed in registers as fp32, and its int8 codes and scale are written
// (the residual variant also writes the new fp16 residual stream, which the model needs).
//
// HBM-bound like the plain quantizer: 3 bytes per element (residual: 7), against the
// 7 (11) bytes of running the producer and the quantizer as two kernels.
//
// The textbook producers, the paper giving no formulas for them:
//   LayerNorm over the channels of a token (biased variance, eps inside the root, no
//   learned affine) followed by the DiT feature modulation (1 + scale[b]) y + shift[b]
//   of the token's sample b; GELU x Phi(x) exactly (erf) or in its tanh form;
//   r = x + gate[b] y.
// Compiled with -ffp-contract=off: every fp32 operation rounds on its own.
#include "vq_internal.h"
#include "vq_quantize_row.h"

namespace vq {
namespace {

enum Producer { kGeluErf = 0, kGeluTanh = 1, kLayerNorm = 2, kResidual = 3, kHadamard = 4 };

struct FusedArgs {
    const half8* x;          // [M,K8] the producer's input
    const half8* y;          // residual: the branch output added to x
    half8* r_out;            // residual: the sum, fp16
    const float4v* mod_a;    // LayerNorm: scale [B,K]; residual: gate [B,K]; or null
    const float4v* mod_b;    // LayerNorm: shift [B,K]; or null
    const float4v* chan_mul; // [K] or null
    int2v* xq;
    float* x_scale;
    int M, K8;
    int tokens_per_sample;
    float eps;
};

__device__ __forceinline__ float gelu_erf(float x) {
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f));
}

// x Phi(x) with Phi(x) ~ (1 + tanh(u)) / 2 = 1 / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3).
// exp(-2u) = exp2(x (c1 + c2 x^2)) with log2(e) folded into c1 = -2 sqrt(2/pi) log2(e) and
// c2 = 0.044715 c1: one fma, two multiplies, v_exp_f32, v_rcp_f32 (1 ulp each).  exp2
// overflows to +inf for very negative x, where the product with the reciprocal 0 is the
// correct -0.
__device__ __forceinline__ float gelu_tanh(float x) {
    constexpr float c1 = -2.302208198f;   // -2 * 0.7978845608 * 1.4426950409
    constexpr float c2 = -0.1029432397f;  // 0.044715 * c1
    const float e = __builtin_amdgcn_exp2f(x * __builtin_fmaf(x * x, c2, c1));
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// The value of the lane whose index differs in one bit (1, 2, 4 or 8), as data movement
// inside a row of 16 lanes: DPP quad permutes for 1 and 2, ds_swizzle (bit mode) for 4 and 8.
template <int MASK>
__device__ __forceinline__ float from_lane_xor(float v) {
    const int iv = __builtin_bit_cast(int, v);
    int r;
    if (MASK == 1) r = __builtin_amdgcn_mov_dpp(iv, 0xB1, 0xF, 0xF, true);       // quad_perm [1,0,3,2]
    else if (MASK == 2) r = __builtin_amdgcn_mov_dpp(iv, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    else r = __builtin_amdgcn_ds_swizzle(iv, (MASK << 10) | 0x1F);               // and 0x1F, or 0, xor MASK
    return __builtin_bit_cast(float, r);
}

// One stage of the Walsh-Hadamard transform across lanes: index bit MASK of the lane.
// The lane with the bit clear gets a + b, the one with it set a - b (a = the clear lane's value).
template <int MASK, int NCH>
__device__ __forceinline__ void hadamard_lane_stage(float (&t)[NCH][8], int sub) {
    const int sign = (sub & MASK) ? (int)0x80000000 : 0;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float other = from_lane_xor<MASK>(t[i][j]);
            t[i][j] = other + __builtin_bit_cast(float, __builtin_bit_cast(int, t[i][j]) ^ sign);
        }
}

template <int PRODUCER, int NCH, int LANES>
__global__ __launch_bounds__(kQuantThreads) void produce_quantize_tokens(const FusedArgs a) {
    const RowLane<LANES> rl(a.M);
    const int K8 = a.K8;
    const long row_off = (rl.row_ok ? rl.m : 0) * K8;
    const long mod_off = (rl.row_ok ? rl.m / a.tokens_per_sample : 0) * (2 * K8);  // in float4v units

    float t[NCH][8];
    load_row<NCH, LANES>(a.x + row_off, rl.row_ok, rl.sub, K8, t);

    if (PRODUCER == kHadamard) {
        // Rotation-based balancing (Sec. 4.2): t = (x * chan_mul) Q with Q block diagonal,
        // blocks H_128 / sqrt(128).  A block is 16 consecutive chunks = the 16 lanes sub%16 of a
        // token with one chunk index i, so element 8 (sub%16) + j of the block sits in lane
        // sub, register t[i][j]: three butterfly stages inside the registers, four across lanes.
        if (a.chan_mul) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int c = i * LANES + rl.sub;
                if (rl.row_ok && c < K8) {
                    const float4v m0 = a.chan_mul[2 * c], m1 = a.chan_mul[2 * c + 1];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        t[i][j] = t[i][j] * m0[j];
                        t[i][4 + j] = t[i][4 + j] * m1[j];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
#pragma unroll
            for (int bit = 1; bit < 8; bit <<= 1)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (!(j & bit)) {
                        const float lo = t[i][j], hi = t[i][j | bit];
                        t[i][j] = lo + hi;
                        t[i][j | bit] = lo - hi;
                    }
        }
        hadamard_lane_stage<1>(t, rl.sub);
        hadamard_lane_stage<2>(t, rl.sub);
        hadamard_lane_stage<4>(t, rl.sub);
        hadamard_lane_stage<8>(t, rl.sub);
#pragma unroll
        for (int i = 0; i < NCH; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) t[i][j] = t[i][j] * 0.08838834764831845f;  // 1 / sqrt(128)
    }

    if (PRODUCER == kGeluErf || PRODUCER == kGeluTanh) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
#pragma unroll
            for (int j = 0; j < 8; ++j) t[i][j] = (PRODUCER == kGeluErf) ? gelu_erf(t[i][j]) : gelu_tanh(t[i][j]);
            // one chunk at a time: interleaving all of them would need a register per
            // temporary of every element
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    if (PRODUCER == kLayerNorm) {
        // two passes over the registers: the mean, then the variance about it
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) s = s + t[i][j];  // (chunks past the row hold zeros)
        const float mean = group_sum<LANES>(s) / (float)(8 * K8);
        float ss = 0.0f;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const bool in_row = i * LANES + rl.sub < K8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                t[i][j] = in_row ? t[i][j] - mean : 0.0f;
                ss = __builtin_fmaf(t[i][j], t[i][j], ss);
            }
        }
        const float var = group_sum<LANES>(ss) / (float)(8 * K8);
        const float rstd = 1.0f / __builtin_sqrtf(var + a.eps);
        // t = (x - mean) rstd (1 + scale) + shift as one multiply and one fma per element
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = i * LANES + rl.sub;
            if (rl.row_ok && c < K8) {
                float mul[8], add[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    mul[j] = rstd;
                    add[j] = 0.0f;
                }
                if (a.mod_a) {
                    const float4v s0 = a.mod_a[mod_off + 2 * c], s1 = a.mod_a[mod_off + 2 * c + 1];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        mul[j] = rstd * (1.0f + s0[j]);
                        mul[4 + j] = rstd * (1.0f + s1[j]);
                    }
                }
                if (a.mod_b) {
                    const float4v h0 = a.mod_b[mod_off + 2 * c], h1 = a.mod_b[mod_off + 2 * c + 1];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        add[j] = h0[j];
                        add[4 + j] = h1[j];
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) t[i][j] = __builtin_fmaf(t[i][j], mul[j], add[j]);
            }
        }
    }

    if (PRODUCER == kResidual) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int c = i * LANES + rl.sub;
            if (rl.row_ok && c < K8) {
                const half8 yv = __builtin_nontemporal_load(a.y + row_off + c);
                float p[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) p[j] = (float)yv[j];
                if (a.mod_a) {
                    const float4v g0 = a.mod_a[mod_off + 2 * c], g1 = a.mod_a[mod_off + 2 * c + 1];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        p[j] = g0[j] * p[j];
                        p[4 + j] = g1[j] * p[4 + j];
                    }
                }
                half8 r;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float s = t[i][j] + p[j];
                    asm("" : "+v"(s));       // (the fp32 sum is rounded before it is narrowed)
                    r[j] = (_Float16)s;      // the new residual stream is fp16 ...
                    t[i][j] = (float)r[j];   // ... and that is what the next layer quantizes
                }
                a.r_out[row_off + c] = r;
            }
        }
    }

    if (PRODUCER != kHadamard && a.chan_mul)  // (the rotation has the scaling before itself)
        fold_quantize_store<NCH, LANES, true>(t, a.chan_mul, rl.row_ok, rl.sub, K8, rl.m, a.xq, a.x_scale);
    else
        fold_quantize_store<NCH, LANES, false>(t, a.chan_mul, rl.row_ok, rl.sub, K8, rl.m, a.xq, a.x_scale);
}

// Weight side of the rotation, offline: one workgroup per output channel, the row in LDS,
// seven butterfly stages per block of 128 with a barrier after each.
__global__ __launch_bounds__(kQuantThreads) void rotate_weight_rows(const float* __restrict__ w,
                                                                    const float* __restrict__ chan_s,
                                                                    float* __restrict__ out, int K) {
    __shared__ float row[8192];
    const long n = blockIdx.x;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) {
        float v = w[n * K + k];
        if (chan_s) v = v * chan_s[k];
        row[k] = v;
    }
    __syncthreads();
    for (int bit = 1; bit < 128; bit <<= 1) {
        for (int p = threadIdx.x; p < K / 2; p += kQuantThreads) {
            // pair p: insert a zero at position `bit` of the index
            const int lo = ((p & ~(bit - 1)) << 1) | (p & (bit - 1));
            const float a0 = row[lo], a1 = row[lo | bit];
            row[lo] = a0 + a1;
            row[lo | bit] = a0 - a1;
        }
        __syncthreads();
    }
    for (int k = threadIdx.x; k < K; k += kQuantThreads) out[n * K + k] = row[k] * 0.08838834764831845f;
}

template <int PRODUCER, int NCH, int LANES>
hipError_t launch_fused(const FusedArgs& a, hipStream_t stream) {
    constexpr int rows_per_block = kRowsPerBlock * (kWave / LANES);
    const dim3 grid((unsigned)((a.M + rows_per_block - 1) / rows_per_block)), block(kQuantThreads);
    hipLaunchKernelGGL((produce_quantize_tokens<PRODUCER, NCH, LANES>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// NCH is a template parameter: pick the instantiation for the run-time chunk count.
template <int PRODUCER, int LANES, int NCH = 1>
hipError_t launch_fused_nch(int nch, const FusedArgs& a, hipStream_t stream) {
    if constexpr (NCH > 16) {
        return hipErrorInvalidValue;
    } else {
        if (nch == NCH) return launch_fused<PRODUCER, NCH, LANES>(a, stream);
        return launch_fused_nch<PRODUCER, LANES, NCH + 1>(nch, a, stream);
    }
}

template <int PRODUCER>
hipError_t launch_producer(const FusedArgs& a, hipStream_t stream) {
    const int k8 = a.K8;
    switch (lanes_for_row(k8)) {
        case 16: return launch_fused_nch<PRODUCER, 16>((k8 + 15) / 16, a, stream);
        case 32: return launch_fused_nch<PRODUCER, 32>((k8 + 31) / 32, a, stream);
        default: return launch_fused_nch<PRODUCER, 64>((k8 + 63) / 64, a, stream);
    }
}

}  // namespace

hipError_t launch_gelu_quantize(const void* h_f16, int approximate, const float* chan_mul, int8_t* xq,
                                float* x_scale, int M, int K, hipStream_t stream) {
    FusedArgs a{};
    a.x = (const half8*)h_f16;
    a.chan_mul = (const float4v*)chan_mul;
    a.xq = (int2v*)xq;
    a.x_scale = x_scale;
    a.M = M;
    a.K8 = K / 8;
    a.tokens_per_sample = 1;
    return approximate ? launch_producer<kGeluTanh>(a, stream) : launch_producer<kGeluErf>(a, stream);
}

hipError_t launch_hadamard_quantize(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale,
                                    int M, int K, hipStream_t stream) {
    FusedArgs a{};
    a.x = (const half8*)x_f16;
    a.chan_mul = (const float4v*)chan_mul;
    a.xq = (int2v*)xq;
    a.x_scale = x_scale;
    a.M = M;
    a.K8 = K / 8;
    a.tokens_per_sample = 1;
    return launch_producer<kHadamard>(a, stream);
}

hipError_t launch_rotate_weight(const float* w, const float* chan_s, float* w_rot, int N, int K,
                                hipStream_t stream) {
    hipLaunchKernelGGL(rotate_weight_rows, dim3((unsigned)N), dim3(kQuantThreads), 0, stream, w, chan_s, w_rot, K);
    return hipGetLastError();
}

hipError_t launch_layernorm_quantize(const void* x_f16, const float* mod_scale, const float* mod_shift,
                                     int tokens_per_sample, float eps, const float* chan_mul, int8_t* xq,
                                     float* x_scale, int M, int K, hipStream_t stream) {
    FusedArgs a{};
    a.x = (const half8*)x_f16;
    a.mod_a = (const float4v*)mod_scale;
    a.mod_b = (const float4v*)mod_shift;
    a.chan_mul = (const float4v*)chan_mul;
    a.xq = (int2v*)xq;
    a.x_scale = x_scale;
    a.M = M;
    a.K8 = K / 8;
    a.tokens_per_sample = tokens_per_sample;
    a.eps = eps;
    return launch_producer<kLayerNorm>(a, stream);
}

hipError_t launch_residual_quantize(const void* x_f16, const void* y_f16, const float* gate,
                                    int tokens_per_sample, void* r_f16, const float* chan_mul, int8_t* xq,
                                    float* x_scale, int M, int K, hipStream_t stream) {
    FusedArgs a{};
    a.x = (const half8*)x_f16;
    a.y = (const half8*)y_f16;
    a.r_out = (half8*)r_f16;
    a.mod_a = (const float4v*)gate;
    a.chan_mul = (const float4v*)chan_mul;
    a.xq = (int2v*)xq;
    a.x_scale = x_scale;
    a.M = M;
    a.K8 = K / 8;
    a.tokens_per_sample = tokens_per_sample;
    return launch_producer<kResidual>(a, stream);
}

}  // namespace vq
