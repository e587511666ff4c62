// Internal launch interface between the C-ABI front end (vq_api.hip) and the
// gfx950 kernels.  Every launcher enqueues on `stream` and returns the HIP
// error of the launch; arguments were validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vq {

hipError_t launch_quantize_per_token(const void* x_f16, const float* chan_mul, int8_t* xq,
                                     float* x_scale, int M, int K, hipStream_t stream);

// The quantizer fused behind its producer (vq_fused.hip): K % 8 == 0, K <= 8192.
hipError_t launch_gelu_quantize(const void* h_f16, int approximate, const float* chan_mul, int8_t* xq,
                                float* x_scale, int M, int K, hipStream_t stream);
hipError_t launch_hadamard_quantize(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale,
                                    int M, int K, hipStream_t stream);  // K % 128 == 0
hipError_t launch_rotate_weight(const float* w, const float* chan_s, float* w_rot, int N, int K,
                                hipStream_t stream);                  // K % 128 == 0, K <= 8192
hipError_t launch_layernorm_quantize(const void* x_f16, const float* mod_scale, const float* mod_shift,
                                     int tokens_per_sample, float eps, const float* chan_mul, int8_t* xq,
                                     float* x_scale, int M, int K, hipStream_t stream);
hipError_t launch_residual_quantize(const void* x_f16, const void* y_f16, const float* gate,
                                    int tokens_per_sample, void* r_f16, const float* chan_mul, int8_t* xq,
                                    float* x_scale, int M, int K, hipStream_t stream);

// Calibration of Eq. 3's mask: column absmax of fp16 (is_f32 = 0) or fp32 rows, and the mask itself.
hipError_t launch_channel_absmax(const void* a, int is_f32, float* amax, int R, int K, int accumulate,
                                 hipStream_t stream);
hipError_t launch_balance_mask(const float* amax_x, const float* amax_w, float alpha, float* s, float* chan_mul,
                               int K, hipStream_t stream);

hipError_t launch_quantize_static(const void* x_f16, const float* chan_mul, float inv_scale, int8_t* xq,
                                  int M, int K, hipStream_t stream);

hipError_t launch_quantize_weight(const float* w, const float* chan_s, int w_bits, void* wq_out,
                                  float* w_scale, int N, int K, hipStream_t stream);

// w_bits 8: w is int8 [N,K]; 4: w is packed nibbles [N,K/2]; 16: the fp16 comparison layer, xq and w
// are fp16 [M,K] and [N,K], x_scale and w_scale are not read, acc_out must be null.  num_cus: compute units of
// the device the stream belongs to (the kernel is persistent, one workgroup per CU).
hipError_t launch_gemm(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
                       const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out,
                       int M, int N, int K, int num_cus, hipStream_t stream);

// The small-tile kernel (64 x 64 tiles, deep load ring) that launch_gemm switches to when
// the large tiles would occupy less than half of the CUs.
hipError_t launch_gemm_small(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
                             const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out,
                             int M, int N, int K, hipStream_t stream);

}  // namespace vq
