// Measured ceilings of the device the library runs on, printed as one JSON object:
//   - register-only v_mfma_i32_32x32x32_i8 loop (no memory traffic at all) for several operand
//     distributions: the sustained matrix-core rate depends on the operand data on this part,
//     so the nominal int8 peak is not what a GEMM on realistic data can be measured against
//     (and, for one distribution, the same loop of v_mfma_i32_16x16x64_i8);
//   - a plain device-to-device copy kernel (HBM bandwidth ceiling for the quantizer).
// Stand-alone program (hipcc --offload-arch=gfx950); bench.py runs it before its own work unless --no-ceilings is given.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

constexpr int kSets = 4;      // operand pairs per lane, cycled through
constexpr int kThreads = 512; // 8 wavefronts per CU, two per SIMD

// Every lane loads kSets operand pairs once; the loop then only issues MFMAs (8 independent
// accumulators per wave, so the pipe never waits on a result).
__global__ __launch_bounds__(kThreads) void mfma_only(const v4i* data, int* out, int iters) {
    v4i a[kSets], b[kSets];
    for (int s = 0; s < kSets; ++s) {
        a[s] = data[(2 * s) * kThreads + threadIdx.x];
        b[s] = data[(2 * s + 1) * kThreads + threadIdx.x];
    }
    v16i acc[8];
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < kSets; ++s)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[s], b[(s + i) % kSets], acc[i], 0, 0, 0);
    }
    int sum = 0;
    for (int i = 0; i < 8; ++i)
        for (int r = 0; r < 16; ++r) sum += acc[i][r];
    if (sum == 0x12345678) out[0] = sum;  // keeps the loop alive
}

// The same loop with the other int8 shape (16 x 16 x 64: as many operations per second of
// matrix pipe, half the accumulator registers moved per operation).
__global__ __launch_bounds__(kThreads) void mfma_only_16x16x64(const v4i* data, int* out, int iters) {
    v4i a[kSets], b[kSets];
    for (int s = 0; s < kSets; ++s) {
        a[s] = data[(2 * s) * kThreads + threadIdx.x];
        b[s] = data[(2 * s + 1) * kThreads + threadIdx.x];
    }
    v4i acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 4; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < kSets; ++s)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[(s + (i >> 2)) % kSets], b[(s + i) % kSets], acc[i], 0,
                                                               0, 0);
    }
    int sum = 0;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 4; ++r) sum += acc[i][r];
    if (sum == 0x12345678) out[0] = sum;  // keeps the loop alive
}

__global__ void copy16(const v4i* __restrict__ in, v4i* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in[i];
}

static float gauss() {
    const double span = (double)RAND_MAX + 2.0;
    const float u = (float)((rand() + 1.0) / span), v = (float)((rand() + 1.0) / span);
    return sqrtf(-2.0f * logf(u)) * cosf(6.2831853f * v);
}
static int8_t clamp8(float g) { return (int8_t)fmaxf(-127.0f, fminf(127.0f, roundf(g))); }

int main() {
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    printf("{\"device\": \"%s\", \"cus\": %d", prop.gcnArchName, cus);

    // ---- MFMA-only loop ---------------------------------------------------------------
    const size_t n = (size_t)kSets * 2 * kThreads * 16;
    int8_t* h = (int8_t*)malloc(n);
    int8_t* d;
    int* out;
    CK(hipMalloc((void**)&d, n));
    CK(hipMalloc((void**)&out, 64));
    const char* names[] = {"zeros", "uniform_int8", "activation_like_x_weight_like", "activation_like_x_w4_widened"};
    const int iters = 3000;  // ~4 ms per launch
    for (int mode = 0; mode < 4; ++mode) {
        srand(1);
        for (size_t i = 0; i < n; ++i) {
            const bool is_b = ((i / (kThreads * 16)) & 1) != 0;  // odd blocks are the second operand
            switch (mode) {
                case 0: h[i] = 0; break;
                case 1: h[i] = (int8_t)(rand() % 255 - 127); break;
                // per-token absmax quantization of a Gaussian row of ~1000 channels puts the
                // extreme near 3.3 sigma; weights of a 1152-wide channel likewise
                case 2: h[i] = clamp8(gauss() * 127.0f / 3.3f); break;
                default: h[i] = is_b ? (int8_t)(16 * (int)fmaxf(-7.0f, fminf(7.0f, roundf(gauss() * 7.0f / 3.3f))))
                                     : clamp8(gauss() * 127.0f / 3.3f);
            }
        }
        CK(hipMemcpy(d, h, n, hipMemcpyHostToDevice));
        for (int rep = 0; rep < 10; ++rep)
            hipLaunchKernelGGL(mfma_only, dim3(cus), dim3(kThreads), 0, 0, (const v4i*)d, out, iters);
        CK(hipDeviceSynchronize());
        const int reps = 20;
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < reps; ++rep)
            hipLaunchKernelGGL(mfma_only, dim3(cus), dim3(kThreads), 0, 0, (const v4i*)d, out, iters);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        ms /= reps;
        const double ops = (double)cus * (kThreads / 64) * iters * kSets * 8 * 2.0 * 32 * 32 * 32;
        printf(", \"mfma_only_tops_%s\": %.0f", names[mode], ops / ms / 1e9);
        if (mode == 2) {  // the other shape on the same operands (16 MFMAs of half the size per set)
            for (int rep = 0; rep < 10; ++rep)
                hipLaunchKernelGGL(mfma_only_16x16x64, dim3(cus), dim3(kThreads), 0, 0, (const v4i*)d, out, iters);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            for (int rep = 0; rep < reps; ++rep)
                hipLaunchKernelGGL(mfma_only_16x16x64, dim3(cus), dim3(kThreads), 0, 0, (const v4i*)d, out, iters);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
            ms /= reps;
            const double ops16 = (double)cus * (kThreads / 64) * iters * kSets * 16 * 2.0 * 16 * 16 * 64;
            printf(", \"mfma_only_tops_16x16x64_%s\": %.0f", names[mode], ops16 / ms / 1e9);
        }
    }

    // ---- copy --------------------------------------------------------------------------
    const size_t bytes = (size_t)1 << 30;
    v4i *src, *dst;
    CK(hipMalloc((void**)&src, bytes));
    CK(hipMalloc((void**)&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    double best = 0;
    for (int blocks_per_cu : {4, 8, 16}) {
        for (int rep = 0; rep < 3; ++rep)
            hipLaunchKernelGGL(copy16, dim3(cus * blocks_per_cu), dim3(256), 0, 0, src, dst, bytes / 16);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < 10; ++rep)
            hipLaunchKernelGGL(copy16, dim3(cus * blocks_per_cu), dim3(256), 0, 0, src, dst, bytes / 16);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        const double gbs = 2.0 * bytes / (ms / 10) / 1e6;
        if (gbs > best) best = gbs;
    }
    printf(", \"copy_1gib_read_plus_write_gbs\": %.0f}\n", best);
    return 0;
}
