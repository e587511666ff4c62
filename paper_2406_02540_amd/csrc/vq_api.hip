// C-ABI front end: argument validation, device check, kernel enqueue.
// Declarations and the contract of every entry point are in include/vq.h.
#include <atomic>

#include "vq.h"
#include "vq_internal.h"

namespace {

constexpr size_t kAlign = 16;
constexpr int kMaxDevices = 64;

inline bool misaligned(const void* p) { return ((uintptr_t)p % kAlign) != 0; }

// Scratch of vq_linear_static: the int8 activations and the token scales between its two
// kernels.  One copy per device that loads the library, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; the address kernels are given is the
// one that call returns (static_scratch() below).
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[VQ_LINEAR_STATIC_SCRATCH_BYTES];
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// The current device's copy of `scratch`, looked up once per device; nullptr on failure.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

// 0 = not looked at yet, 1 = gfx950, 2 = something else.  A benign cache: the
// answer for a device ordinal never changes during the life of the process.
std::atomic<int> g_arch_state[kMaxDevices];
std::atomic<int> g_num_cus[kMaxDevices];

// VQ_OK if the current device is gfx950; *num_cus (if asked for) gets its CU count.
int check_arch(int* num_cus = nullptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();
        return VQ_ERR_ARCH;
    }
    if (dev < kMaxDevices) {
        const int s = g_arch_state[dev].load(std::memory_order_acquire);
        if (s == 1) {
            if (num_cus) *num_cus = g_num_cus[dev].load(std::memory_order_relaxed);
            return VQ_OK;
        }
        if (s == 2) return VQ_ERR_ARCH;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return VQ_ERR_ARCH;
    }
    const char* name = prop.gcnArchName;  // e.g. "gfx950:sramecc+:xnack-"
    const bool ok = name[0] == 'g' && name[1] == 'f' && name[2] == 'x' && name[3] == '9' &&
                    name[4] == '5' && name[5] == '0' && (name[6] == '\0' || name[6] == ':');
    if (num_cus) *num_cus = prop.multiProcessorCount;
    if (dev < kMaxDevices) {
        g_num_cus[dev].store(prop.multiProcessorCount, std::memory_order_relaxed);
        g_arch_state[dev].store(ok ? 1 : 2, std::memory_order_release);
    }
    return ok ? VQ_OK : VQ_ERR_ARCH;
}

int launch_status(hipError_t e) { return e == hipSuccess ? VQ_OK : VQ_ERR_LAUNCH; }

int validate_gemm(const void* xq, const void* x_scale, const void* w, const void* w_scale,
                  const void* bias, const void* y, const void* acc_out, int w_bits, int M, int N,
                  int K) {
    if (w_bits != 8 && w_bits != 4) return VQ_ERR_BITS;
    if (M < 0 || N < 0 || K <= 0 || K > VQ_MAX_K) return VQ_ERR_SHAPE;
    if (K % (w_bits == 8 ? 16 : 32) != 0) return VQ_ERR_SHAPE;
    if (M == 0 || N == 0) return VQ_OK;
    if (!xq || !x_scale || !w || !w_scale || !y) return VQ_ERR_NULL;
    if (misaligned(xq) || misaligned(x_scale) || misaligned(w) || misaligned(w_scale) ||
        misaligned(y) || (bias && misaligned(bias)) || (acc_out && misaligned(acc_out)))
        return VQ_ERR_ALIGN;
    return VQ_OK;
}

int gemm_entry(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
               const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out, int M,
               int N, int K, void* hip_stream) {
    const int v = validate_gemm(xq, x_scale, w, w_scale, bias_f16, y_f16, acc_out, w_bits, M, N, K);
    if (v != VQ_OK) return v;
    if (M == 0 || N == 0) return VQ_OK;
    int num_cus = 0;
    const int arch = check_arch(&num_cus);
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_gemm(xq, x_scale, w, w_bits, w_scale, bias_f16, y_f16, acc_out,
                                         M, N, K, num_cus, (hipStream_t)hip_stream));
}

int validate_quantize(const void* x, const void* chan_mul, const void* xq, const void* x_scale,
                      int M, int K) {
    if (M < 0 || K <= 0 || K > VQ_MAX_K) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    if (!x || !xq || !x_scale) return VQ_ERR_NULL;
    if (misaligned(x) || misaligned(xq) || misaligned(x_scale) || (chan_mul && misaligned(chan_mul)))
        return VQ_ERR_ALIGN;
    return VQ_OK;
}

// The fused variants keep the token in registers: whole 16-byte chunks, at most 16 per lane.
int validate_fused(const void* x, const void* chan_mul, const void* xq, const void* x_scale, int M, int K) {
    const int v = validate_quantize(x, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (K % 8 != 0 || K > VQ_MAX_FUSED_K) return VQ_ERR_SHAPE;
    return VQ_OK;
}

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Shared by the layer entry points that take a workspace: validates the layer, splits the
// workspace into xq and x_scale, lets `quantize` enqueue the (plain or fused) quantizer into
// them and enqueues the GEMM behind it.  `fused`: the quantizer is one of the fused ones, which
// hold a token in registers (K % 8 == 0, K <= VQ_MAX_FUSED_K).
template <class Quantize>
int linear_through_workspace(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
                             const float* w_scale, const void* bias_f16, void* y_f16, void* workspace,
                             size_t workspace_bytes, int M, int N, int K, void* hip_stream, bool fused,
                             Quantize quantize) {
    if (w_bits != 8 && w_bits != 4) return VQ_ERR_BITS;
    if (M < 0 || N < 0 || K <= 0 || K > VQ_MAX_K) return VQ_ERR_SHAPE;
    if (K % (w_bits == 8 ? 16 : 32) != 0) return VQ_ERR_SHAPE;
    if (fused && K > VQ_MAX_FUSED_K) return VQ_ERR_SHAPE;
    if (M == 0 || N == 0) return VQ_OK;
    if (!workspace) return VQ_ERR_NULL;
    if (misaligned(workspace)) return VQ_ERR_ALIGN;
    if (workspace_bytes < vq_linear_workspace_bytes(M, N, K, w_bits)) return VQ_ERR_WORKSPACE;
    int8_t* xq = (int8_t*)workspace;
    float* x_scale = (float*)((char*)workspace + round_up((size_t)M * (size_t)K, kAlign));
    // validate both halves before anything is enqueued
    int v = validate_quantize(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    v = validate_gemm(xq, x_scale, w, w_scale, bias_f16, y_f16, nullptr, w_bits, M, N, K);
    if (v != VQ_OK) return v;
    int num_cus = 0;
    const int arch = check_arch(&num_cus);
    if (arch != VQ_OK) return arch;
    hipStream_t stream = (hipStream_t)hip_stream;
    v = launch_status(quantize(xq, x_scale, stream));
    if (v != VQ_OK) return v;
    return launch_status(vq::launch_gemm(xq, x_scale, w, w_bits, w_scale, bias_f16, y_f16, nullptr,
                                         M, N, K, num_cus, stream));
}

}  // namespace

extern "C" {

int vq_quantize_per_token(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale,
                          int M, int K, void* hip_stream) {
    const int v = validate_quantize(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (M == 0) return VQ_OK;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_quantize_per_token(x_f16, chan_mul, xq, x_scale, M, K,
                                                       (hipStream_t)hip_stream));
}

int vq_gelu_quantize(const void* h_f16, int approximate, const float* chan_mul, int8_t* xq,
                     float* x_scale, int M, int K, void* hip_stream) {
    const int v = validate_fused(h_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (approximate != 0 && approximate != 1) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_gelu_quantize(h_f16, approximate, chan_mul, xq, x_scale, M, K,
                                                  (hipStream_t)hip_stream));
}

int vq_hadamard_quantize(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale, int M, int K,
                         void* hip_stream) {
    const int v = validate_fused(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (K % VQ_HADAMARD_BLOCK != 0) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_hadamard_quantize(x_f16, chan_mul, xq, x_scale, M, K,
                                                      (hipStream_t)hip_stream));
}

int vq_rotate_weight(const float* w_f32, const float* chan_s, float* w_rot_f32, int N, int K, void* hip_stream) {
    if (N < 0 || K <= 0 || K > VQ_MAX_FUSED_K || K % VQ_HADAMARD_BLOCK != 0) return VQ_ERR_SHAPE;
    if (N == 0) return VQ_OK;
    if (!w_f32 || !w_rot_f32) return VQ_ERR_NULL;
    if (misaligned(w_f32) || misaligned(w_rot_f32) || (chan_s && misaligned(chan_s))) return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_rotate_weight(w_f32, chan_s, w_rot_f32, N, K, (hipStream_t)hip_stream));
}

int vq_layernorm_quantize(const void* x_f16, const float* mod_scale, const float* mod_shift,
                          int tokens_per_sample, float eps, const float* chan_mul, int8_t* xq,
                          float* x_scale, int M, int K, void* hip_stream) {
    const int v = validate_fused(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (tokens_per_sample <= 0 || !(eps >= 0.0f)) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    if ((mod_scale && misaligned(mod_scale)) || (mod_shift && misaligned(mod_shift))) return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_layernorm_quantize(x_f16, mod_scale, mod_shift, tokens_per_sample, eps,
                                                       chan_mul, xq, x_scale, M, K,
                                                       (hipStream_t)hip_stream));
}

int vq_residual_quantize(const void* x_f16, const void* y_f16, const float* gate, int tokens_per_sample,
                         void* r_f16, const float* chan_mul, int8_t* xq, float* x_scale, int M, int K,
                         void* hip_stream) {
    const int v = validate_fused(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    if (tokens_per_sample <= 0) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    if (!y_f16 || !r_f16) return VQ_ERR_NULL;
    if (misaligned(y_f16) || misaligned(r_f16) || (gate && misaligned(gate))) return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_residual_quantize(x_f16, y_f16, gate, tokens_per_sample, r_f16, chan_mul,
                                                      xq, x_scale, M, K, (hipStream_t)hip_stream));
}

int vq_channel_absmax(const void* a, int is_f32, float* amax, int R, int K, int accumulate, void* hip_stream) {
    if (R < 0 || K <= 0 || K > VQ_MAX_K || (is_f32 != 0 && is_f32 != 1)) return VQ_ERR_SHAPE;
    if (!amax || (R > 0 && !a)) return VQ_ERR_NULL;
    if (misaligned(amax) || (a && misaligned(a))) return VQ_ERR_ALIGN;
    if (R == 0 && accumulate) return VQ_OK;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_channel_absmax(a, is_f32, amax, R, K, accumulate, (hipStream_t)hip_stream));
}

int vq_balance_mask(const float* amax_x, const float* amax_w, float alpha, float* s, float* chan_mul, int K,
                    void* hip_stream) {
    if (K <= 0 || K > VQ_MAX_K || !(alpha >= 0.0f && alpha <= 1.0f)) return VQ_ERR_SHAPE;
    if (!amax_x || !amax_w || !s || !chan_mul) return VQ_ERR_NULL;
    if (misaligned(amax_x) || misaligned(amax_w) || misaligned(s) || misaligned(chan_mul)) return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_balance_mask(amax_x, amax_w, alpha, s, chan_mul, K, (hipStream_t)hip_stream));
}

int vq_gemm_f16(const void* x_f16, const void* w_f16, const void* bias_f16, void* y_f16, int M, int N, int K,
                void* hip_stream) {
    if (M < 0 || N < 0 || K <= 0 || K > VQ_MAX_K || K % 8 != 0) return VQ_ERR_SHAPE;
    if (M == 0 || N == 0) return VQ_OK;
    if (!x_f16 || !w_f16 || !y_f16) return VQ_ERR_NULL;
    if (misaligned(x_f16) || misaligned(w_f16) || misaligned(y_f16) || (bias_f16 && misaligned(bias_f16)))
        return VQ_ERR_ALIGN;
    int num_cus = 0;
    const int arch = check_arch(&num_cus);
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_gemm((const int8_t*)x_f16, nullptr, w_f16, 16, nullptr, bias_f16, y_f16,
                                         nullptr, M, N, K, num_cus, (hipStream_t)hip_stream));
}

int vq_quantize_static(const void* x_f16, const float* chan_mul, float scale, int8_t* xq, int M, int K,
                       void* hip_stream) {
    if (M < 0 || K <= 0 || K > VQ_MAX_K || !(scale > 0.0f)) return VQ_ERR_SHAPE;
    if (M == 0) return VQ_OK;
    if (!x_f16 || !xq) return VQ_ERR_NULL;
    if (misaligned(x_f16) || misaligned(xq) || (chan_mul && misaligned(chan_mul))) return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_quantize_static(x_f16, chan_mul, 1.0f / scale, xq, M, K,
                                                    (hipStream_t)hip_stream));
}

int vq_gemm_w8a8(const int8_t* xq, const float* x_scale, const int8_t* wq, const float* w_scale,
                 const void* bias_f16, void* y_f16, int32_t* acc_out, int M, int N, int K,
                 void* hip_stream) {
    return gemm_entry(xq, x_scale, wq, 8, w_scale, bias_f16, y_f16, acc_out, M, N, K, hip_stream);
}

int vq_gemm_w4a8(const int8_t* xq, const float* x_scale, const uint8_t* wq4, const float* w_scale,
                 const void* bias_f16, void* y_f16, int32_t* acc_out, int M, int N, int K,
                 void* hip_stream) {
    return gemm_entry(xq, x_scale, wq4, 4, w_scale, bias_f16, y_f16, acc_out, M, N, K, hip_stream);
}

size_t vq_linear_workspace_bytes(int M, int N, int K, int w_bits) {
    if (M < 0 || N < 0 || K <= 0 || K > VQ_MAX_K || (w_bits != 8 && w_bits != 4)) return 0;
    // xq [M,K] int8, then x_scale [M] fp32, each rounded up to the alignment
    return round_up((size_t)M * (size_t)K, kAlign) + round_up((size_t)M * sizeof(float), kAlign);
}

int vq_linear(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
              const float* w_scale, const void* bias_f16, void* y_f16, void* workspace,
              size_t workspace_bytes, int M, int N, int K, void* hip_stream) {
    return linear_through_workspace(x_f16, chan_mul, w, w_bits, w_scale, bias_f16, y_f16, workspace, workspace_bytes,
                                    M, N, K, hip_stream, false, [&](int8_t* xq, float* x_scale, hipStream_t stream) {
                                        return vq::launch_quantize_per_token(x_f16, chan_mul, xq, x_scale, M, K, stream);
                                    });
}

int vq_layernorm_linear(const void* x_f16, const float* mod_scale, const float* mod_shift,
                        int tokens_per_sample, float eps, const float* chan_mul, const void* w, int w_bits,
                        const float* w_scale, const void* bias_f16, void* y_f16, void* workspace,
                        size_t workspace_bytes, int M, int N, int K, void* hip_stream) {
    if (tokens_per_sample <= 0 || !(eps >= 0.0f)) return VQ_ERR_SHAPE;
    if ((mod_scale && misaligned(mod_scale)) || (mod_shift && misaligned(mod_shift))) return VQ_ERR_ALIGN;
    return linear_through_workspace(x_f16, chan_mul, w, w_bits, w_scale, bias_f16, y_f16, workspace, workspace_bytes,
                                    M, N, K, hip_stream, true, [&](int8_t* xq, float* x_scale, hipStream_t stream) {
                                        return vq::launch_layernorm_quantize(x_f16, mod_scale, mod_shift, tokens_per_sample,
                                                                             eps, chan_mul, xq, x_scale, M, K, stream);
                                    });
}

int vq_gelu_linear(const void* h_f16, int approximate, const float* chan_mul, const void* w, int w_bits,
                   const float* w_scale, const void* bias_f16, void* y_f16, void* workspace,
                   size_t workspace_bytes, int M, int N, int K, void* hip_stream) {
    if (approximate != 0 && approximate != 1) return VQ_ERR_SHAPE;
    return linear_through_workspace(h_f16, chan_mul, w, w_bits, w_scale, bias_f16, y_f16, workspace, workspace_bytes,
                                    M, N, K, hip_stream, true, [&](int8_t* xq, float* x_scale, hipStream_t stream) {
                                        return vq::launch_gelu_quantize(h_f16, approximate, chan_mul, xq, x_scale, M, K,
                                                                        stream);
                                    });
}

int vq_residual_linear(const void* x_f16, const void* y_in_f16, const float* gate, int tokens_per_sample,
                       void* r_f16, const float* chan_mul, const void* w, int w_bits, const float* w_scale,
                       const void* bias_f16, void* y_f16, void* workspace, size_t workspace_bytes, int M, int N,
                       int K, void* hip_stream) {
    if (tokens_per_sample <= 0) return VQ_ERR_SHAPE;
    if (M > 0 && N > 0) {
        if (!y_in_f16 || !r_f16) return VQ_ERR_NULL;
        if (misaligned(y_in_f16) || misaligned(r_f16) || (gate && misaligned(gate))) return VQ_ERR_ALIGN;
    }
    return linear_through_workspace(x_f16, chan_mul, w, w_bits, w_scale, bias_f16, y_f16, workspace, workspace_bytes,
                                    M, N, K, hip_stream, true, [&](int8_t* xq, float* x_scale, hipStream_t stream) {
                                        return vq::launch_residual_quantize(x_f16, y_in_f16, gate, tokens_per_sample,
                                                                            r_f16, chan_mul, xq, x_scale, M, K, stream);
                                    });
}

int vq_hadamard_linear(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
                       const float* w_scale, const void* bias_f16, void* y_f16, void* workspace,
                       size_t workspace_bytes, int M, int N, int K, void* hip_stream) {
    if (K > 0 && K % VQ_HADAMARD_BLOCK != 0) return VQ_ERR_SHAPE;
    return linear_through_workspace(x_f16, chan_mul, w, w_bits, w_scale, bias_f16, y_f16, workspace, workspace_bytes,
                                    M, N, K, hip_stream, true, [&](int8_t* xq, float* x_scale, hipStream_t stream) {
                                        return vq::launch_hadamard_quantize(x_f16, chan_mul, xq, x_scale, M, K, stream);
                                    });
}

int vq_linear_static(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
                     const float* w_scale, const void* bias_f16, void* y_f16, int M, int N, int K,
                     void* hip_stream) {
    if (w_bits != 8 && w_bits != 4) return VQ_ERR_BITS;
    if (M < 0 || N < 0 || K <= 0 || K > VQ_MAX_K) return VQ_ERR_SHAPE;
    if (K % (w_bits == 8 ? 16 : 32) != 0) return VQ_ERR_SHAPE;
    if (M == 0 || N == 0) return VQ_OK;
    if (vq_linear_workspace_bytes(M, N, K, w_bits) > (size_t)VQ_LINEAR_STATIC_SCRATCH_BYTES)
        return VQ_ERR_WORKSPACE;
    int num_cus = 0;
    const int arch = check_arch(&num_cus);
    if (arch != VQ_OK) return arch;
    void* const ws = static_scratch();
    if (!ws) return VQ_ERR_LAUNCH;
    int8_t* xq = (int8_t*)ws;
    float* x_scale = (float*)((char*)ws + round_up((size_t)M * (size_t)K, kAlign));
    int v = validate_quantize(x_f16, chan_mul, xq, x_scale, M, K);
    if (v != VQ_OK) return v;
    v = validate_gemm(xq, x_scale, w, w_scale, bias_f16, y_f16, nullptr, w_bits, M, N, K);
    if (v != VQ_OK) return v;
    hipStream_t stream = (hipStream_t)hip_stream;
    v = launch_status(vq::launch_quantize_per_token(x_f16, chan_mul, xq, x_scale, M, K, stream));
    if (v != VQ_OK) return v;
    return launch_status(vq::launch_gemm(xq, x_scale, w, w_bits, w_scale, bias_f16, y_f16, nullptr,
                                         M, N, K, num_cus, stream));
}

int vq_quantize_weight(const float* w_f32, const float* chan_s, int w_bits, void* wq_out,
                       float* w_scale, int N, int K, void* hip_stream) {
    if (w_bits != 8 && w_bits != 4) return VQ_ERR_BITS;
    if (N < 0 || K <= 0 || K > VQ_MAX_K) return VQ_ERR_SHAPE;
    if (w_bits == 4 && (K % 2) != 0) return VQ_ERR_SHAPE;
    if (N == 0) return VQ_OK;
    if (!w_f32 || !wq_out || !w_scale) return VQ_ERR_NULL;
    if (misaligned(w_f32) || misaligned(wq_out) || misaligned(w_scale) ||
        (chan_s && misaligned(chan_s)))
        return VQ_ERR_ALIGN;
    const int arch = check_arch();
    if (arch != VQ_OK) return arch;
    return launch_status(vq::launch_quantize_weight(w_f32, chan_s, w_bits, wq_out, w_scale, N, K,
                                                    (hipStream_t)hip_stream));
}

const char* vq_status_string(int status) {
    switch (status) {
        case VQ_OK: return "ok";
        case VQ_ERR_NULL: return "a required pointer is NULL";
        case VQ_ERR_SHAPE: return "invalid or unsupported M, N or K";
        case VQ_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case VQ_ERR_WORKSPACE: return "workspace too small (or the layer exceeds the built-in scratch)";
        case VQ_ERR_LAUNCH: return "kernel launch failed";
        case VQ_ERR_ARCH: return "current device is not gfx950";
        case VQ_ERR_BITS: return "w_bits must be 8 or 4";
        default: return "unknown status";
    }
}

}  // extern "C"
