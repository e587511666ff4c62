// The quantizers fused behind their producers (kernel template and its description:
// vq_fused_kernel.h): the entry points, the LayerNorm, residual and Hadamard kernels (the GELU
// ones are compiled in vq_fused_gelu.hip), and the offline weight rotation.
#include "vq_fused_kernel.h"

namespace vq {
namespace {

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

}  // namespace

hipError_t launch_producer_other(int producer, const FusedArgs& a, hipStream_t stream) {
    switch (producer) {
        case kLayerNorm: return launch_producer<kLayerNorm>(a, stream);
        case kResidual: return launch_producer<kResidual>(a, stream);
        default: return launch_producer<kHadamard>(a, stream);
    }
}

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
    return launch_producer_gelu(approximate ? kGeluTanh : kGeluErf, a, stream);
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
    return launch_producer_other(kHadamard, a, stream);
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
    return launch_producer_other(kLayerNorm, a, stream);
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
    return launch_producer_other(kResidual, a, stream);
}

}  // namespace vq
