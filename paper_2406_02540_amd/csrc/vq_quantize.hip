// Quantizers for gfx950.
//
// 1. Dynamic per-token activation quantizer (ViDiT-Q Sec. 4.1; Eq. 2 of Sec. 3.1
//    in symmetric form; activation side of the channel balancing, Eq. 3 of
//    Sec. 4.2).  HBM-bound: a token is read once (2 B/element), kept in
//    registers as fp32 across the absmax reduction, and written once
//    (1 B/element + one fp32 scale).
// 2. Offline per-output-channel weight quantizer (same recipe, qmax 127 or 7,
//    weight side of Eq. 3), with the 4-bit packer fused.
//
// This file is compiled with -ffp-contract=off: every fp32 operation rounds on
// its own, the two divisions per row are the correctly rounded IEEE ones, and
// rounding to integer is v_rndne_f32 (halves to even).
#include "vq_internal.h"
#include "vq_quantize_row.h"

namespace vq {
namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// The token row held in registers (layout and steps: vq_quantize_row.h).  LANES is chosen
// so that K / 8 = NCH * LANES exactly where possible (K = 1152: 16 lanes x 9 chunks),
// which keeps every lane busy on every instruction.
template <int NCH, int LANES, bool HAS_MUL>
__global__ __launch_bounds__(kQuantThreads) void quantize_tokens_wave(
    const half8* __restrict__ x, const float4v* __restrict__ chan_mul, int2v* __restrict__ xq,
    float* __restrict__ x_scale, int M, int K8) {
    const RowLane<LANES> rl(M);
    float t[NCH][8];
    load_row<NCH, LANES, HAS_MUL>(x + (rl.row_ok ? rl.m : 0) * K8, rl.row_ok, rl.sub, K8, t, chan_mul);
    fold_quantize_store<NCH, LANES, false>(t, nullptr, rl.row_ok, rl.sub, K8, rl.m, xq, x_scale);
}

__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < kRowsPerBlock; ++i) r = fmaxf(r, red[i]);
    __syncthreads();
    return r;
}

// Any K, any alignment: one workgroup per token, two passes over the row
// (the second one hits in cache).  Used when K is not a multiple of 8 or the
// row does not fit the register-resident kernel.
template <bool HAS_MUL>
__global__ __launch_bounds__(kQuantThreads) void quantize_tokens_generic(
    const _Float16* __restrict__ x, const float* __restrict__ chan_mul, int8_t* __restrict__ xq,
    float* __restrict__ x_scale, int K) {
    __shared__ float red[kRowsPerBlock];
    const long m = blockIdx.x;
    const _Float16* row = x + m * (long)K;
    float amax = 0.0f;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) {
        float t = (float)row[k];
        if (HAS_MUL) t = t * chan_mul[k];
        amax = fmaxf(amax, fabsf(t));
    }
    amax = block_max(amax, red);
    float scale = 0.0f, inv = 0.0f;
    if (amax != 0.0f) {
        scale = amax / 127.0f;
        inv = 127.0f / amax;
    }
    if (threadIdx.x == 0) x_scale[m] = scale;
    int8_t* qrow = xq + m * (long)K;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) {
        float t = (float)row[k];
        if (HAS_MUL) t = t * chan_mul[k];
        qrow[k] = (int8_t)quantize_one(t, inv, 127.0f);
    }
}

// Static quantizer (the comparison point: one scale for the whole tensor, fixed beforehand):
// element-wise, 8 values per thread where the rows are whole 16-byte chunks.
template <bool VEC>
__global__ __launch_bounds__(kQuantThreads) void quantize_static_elems(
    const _Float16* __restrict__ x, const float* __restrict__ chan_mul, float inv, int8_t* __restrict__ xq,
    long total, int K) {
    const long step = (long)gridDim.x * kQuantThreads;
    if (VEC) {
        const int K8 = K / 8;
        for (long c = (long)blockIdx.x * kQuantThreads + threadIdx.x; c < total / 8; c += step) {
            const half8 v = __builtin_nontemporal_load((const half8*)x + c);
            const int k = (int)(c % K8) * 8;
            int q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float t = (float)v[j];
                if (chan_mul) t = t * chan_mul[k + j];
                q[j] = quantize_one(t, inv, 127.0f);
            }
            int2v o;
            o.x = pack4(q[0], q[1], q[2], q[3]);
            o.y = pack4(q[4], q[5], q[6], q[7]);
            ((int2v*)xq)[c] = o;
        }
    } else {
        for (long e = (long)blockIdx.x * kQuantThreads + threadIdx.x; e < total; e += step) {
            float t = (float)x[e];
            if (chan_mul) t = t * chan_mul[e % K];
            xq[e] = (int8_t)quantize_one(t, inv, 127.0f);
        }
    }
}

// Calibration side of Eq. 3 (Sec. 4.2): per-input-channel absmax over the rows of a matrix
// (tokens of a calibration batch, or output channels of a weight).  Thread t of a block owns
// column 256 b_x + t for a slab of rows; slabs are combined with an integer atomic max on
// the bit pattern (non-negative floats order like their bits).  amax must hold valid
// non-negative values on entry (zeros, or the running maximum of earlier batches).
template <typename T>
__global__ __launch_bounds__(kQuantThreads) void channel_absmax_cols(const T* __restrict__ a,
                                                                     float* __restrict__ amax, int R, int K,
                                                                     int rows_per_block) {
    const int k = blockIdx.x * kQuantThreads + threadIdx.x;
    if (k >= K) return;
    const long r0 = (long)blockIdx.y * rows_per_block;
    const long r1 = r0 + rows_per_block < R ? r0 + rows_per_block : R;
    float m = 0.0f;
    for (long r = r0; r < r1; ++r) m = fmaxf(m, fabsf((float)a[r * K + k]));
    atomicMax((int*)amax + k, __builtin_bit_cast(int, m));
}

__global__ __launch_bounds__(kQuantThreads) void fill_zero_f32(float* __restrict__ p, int n) {
    const int i = blockIdx.x * kQuantThreads + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// s = max|X|^alpha / max|W|^(1 - alpha) per channel, statistics raised to 1e-5, s kept in
// [1e-5, 1e5]; chan_mul = 1 / s (IEEE division).
__global__ __launch_bounds__(kQuantThreads) void balance_mask_elems(const float* __restrict__ ax,
                                                                    const float* __restrict__ aw, float alpha,
                                                                    float* __restrict__ s_out,
                                                                    float* __restrict__ chan_mul, int K) {
    const int k = blockIdx.x * kQuantThreads + threadIdx.x;
    if (k >= K) return;
    const float x = fmaxf(ax[k], 1e-5f), w = fmaxf(aw[k], 1e-5f);
    float s = powf(x, alpha) / powf(w, 1.0f - alpha);
    s = fminf(fmaxf(s, 1e-5f), 1e5f);
    s_out[k] = s;
    chan_mul[k] = 1.0f / s;
}

// Offline weight quantizer: one workgroup per output channel, fp32 input.
// BITS == 4 writes two nibbles per byte (k even in bits 0..3, k odd in 4..7).
template <int BITS, bool HAS_S>
__global__ __launch_bounds__(kQuantThreads) void quantize_weight_rows(
    const float* __restrict__ w, const float* __restrict__ chan_s, void* __restrict__ wq_out,
    float* __restrict__ w_scale, int K) {
    __shared__ float red[kRowsPerBlock];
    constexpr float qmax = (BITS == 8) ? 127.0f : 7.0f;
    const long n = blockIdx.x;
    const float* row = w + n * (long)K;
    float amax = 0.0f;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) {
        float t = row[k];
        if (HAS_S) t = t * chan_s[k];
        amax = fmaxf(amax, fabsf(t));
    }
    amax = block_max(amax, red);
    float scale = 0.0f, inv = 0.0f;
    if (amax != 0.0f) {
        scale = amax / qmax;
        inv = qmax / amax;
    }
    if (threadIdx.x == 0) w_scale[n] = scale;
    if (BITS == 8) {
        int8_t* qrow = (int8_t*)wq_out + n * (long)K;
        for (int k = threadIdx.x; k < K; k += kQuantThreads) {
            float t = row[k];
            if (HAS_S) t = t * chan_s[k];
            qrow[k] = (int8_t)quantize_one(t, inv, qmax);
        }
    } else {
        uint8_t* qrow = (uint8_t*)wq_out + n * (long)(K / 2);
        for (int j = threadIdx.x; j < K / 2; j += kQuantThreads) {
            float t0 = row[2 * j], t1 = row[2 * j + 1];
            if (HAS_S) {
                t0 = t0 * chan_s[2 * j];
                t1 = t1 * chan_s[2 * j + 1];
            }
            const int q0 = quantize_one(t0, inv, qmax), q1 = quantize_one(t1, inv, qmax);
            qrow[j] = (uint8_t)((q0 & 0xF) | ((q1 & 0xF) << 4));
        }
    }
}

template <int NCH, int LANES>
hipError_t launch_wave(const void* x, const float* chan_mul, int8_t* xq, float* x_scale, int M,
                       int K, hipStream_t stream) {
    constexpr int rows_per_block = kRowsPerBlock * (kWave / LANES);
    const dim3 grid((unsigned)((M + rows_per_block - 1) / rows_per_block)), block(kQuantThreads);
    if (chan_mul)
        hipLaunchKernelGGL((quantize_tokens_wave<NCH, LANES, true>), grid, block, 0, stream,
                           (const half8*)x, (const float4v*)chan_mul, (int2v*)xq, x_scale, M, K / 8);
    else
        hipLaunchKernelGGL((quantize_tokens_wave<NCH, LANES, false>), grid, block, 0, stream,
                           (const half8*)x, (const float4v*)nullptr, (int2v*)xq, x_scale, M, K / 8);
    return hipGetLastError();
}

// NCH is a template parameter: pick the instantiation for the run-time chunk count.
template <int LANES, int NCH = 1>
hipError_t launch_wave_nch(int nch, const void* x, const float* chan_mul, int8_t* xq, float* x_scale,
                           int M, int K, hipStream_t stream) {
    if constexpr (NCH > 16) {
        return hipErrorInvalidValue;
    } else {
        if (nch == NCH) return launch_wave<NCH, LANES>(x, chan_mul, xq, x_scale, M, K, stream);
        return launch_wave_nch<LANES, NCH + 1>(nch, x, chan_mul, xq, x_scale, M, K, stream);
    }
}

}  // namespace

hipError_t launch_quantize_per_token(const void* x_f16, const float* chan_mul, int8_t* xq,
                                     float* x_scale, int M, int K, hipStream_t stream) {
    // Register-resident path: rows of 16-byte chunks, at most 16 chunks per lane.
    const bool vec = (K % 8 == 0) && (K <= 8 * kWave * 16) &&
                     (((uintptr_t)x_f16 | (uintptr_t)xq) % 16 == 0) &&
                     (chan_mul == nullptr || (uintptr_t)chan_mul % 16 == 0);
    if (vec) {
        const int k8 = K / 8;
        // the widest lane group that divides the row exactly; a whole wavefront otherwise
        if (k8 % 64 == 0) return launch_wave_nch<64>(k8 / 64, x_f16, chan_mul, xq, x_scale, M, K, stream);
        if (k8 % 32 == 0 && k8 / 32 <= 16)
            return launch_wave_nch<32>(k8 / 32, x_f16, chan_mul, xq, x_scale, M, K, stream);
        if (k8 % 16 == 0 && k8 / 16 <= 16)
            return launch_wave_nch<16>(k8 / 16, x_f16, chan_mul, xq, x_scale, M, K, stream);
        return launch_wave_nch<64>((k8 + 63) / 64, x_f16, chan_mul, xq, x_scale, M, K, stream);
    }
    const dim3 grid((unsigned)M), block(kQuantThreads);
    if (chan_mul)
        hipLaunchKernelGGL((quantize_tokens_generic<true>), grid, block, 0, stream,
                           (const _Float16*)x_f16, chan_mul, xq, x_scale, K);
    else
        hipLaunchKernelGGL((quantize_tokens_generic<false>), grid, block, 0, stream,
                           (const _Float16*)x_f16, (const float*)nullptr, xq, x_scale, K);
    return hipGetLastError();
}

hipError_t launch_channel_absmax(const void* a, int is_f32, float* amax, int R, int K, int accumulate,
                                 hipStream_t stream) {
    const dim3 block(kQuantThreads);
    if (!accumulate) {
        hipLaunchKernelGGL(fill_zero_f32, dim3((unsigned)((K + kQuantThreads - 1) / kQuantThreads)), block, 0,
                           stream, amax, K);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    if (R == 0) return hipSuccess;
    const int col_blocks = (K + kQuantThreads - 1) / kQuantThreads;
    // enough row slabs to fill the chip, at least 64 rows each
    int slabs = (2048 + col_blocks - 1) / col_blocks;
    if (slabs > (R + 63) / 64) slabs = (R + 63) / 64;
    if (slabs < 1) slabs = 1;
    const int rows_per_block = (R + slabs - 1) / slabs;
    const dim3 grid((unsigned)col_blocks, (unsigned)((R + rows_per_block - 1) / rows_per_block));
    if (is_f32)
        hipLaunchKernelGGL((channel_absmax_cols<float>), grid, block, 0, stream, (const float*)a, amax, R, K,
                           rows_per_block);
    else
        hipLaunchKernelGGL((channel_absmax_cols<_Float16>), grid, block, 0, stream, (const _Float16*)a, amax, R,
                           K, rows_per_block);
    return hipGetLastError();
}

hipError_t launch_balance_mask(const float* amax_x, const float* amax_w, float alpha, float* s, float* chan_mul,
                               int K, hipStream_t stream) {
    hipLaunchKernelGGL(balance_mask_elems, dim3((unsigned)((K + kQuantThreads - 1) / kQuantThreads)),
                       dim3(kQuantThreads), 0, stream, amax_x, amax_w, alpha, s, chan_mul, K);
    return hipGetLastError();
}

hipError_t launch_quantize_static(const void* x_f16, const float* chan_mul, float inv_scale, int8_t* xq,
                                  int M, int K, hipStream_t stream) {
    const long total = (long)M * K;
    const bool vec = (K % 8 == 0);
    const long work = vec ? total / 8 : total;
    const long blocks = (work + kQuantThreads - 1) / kQuantThreads;
    const dim3 grid((unsigned)(blocks < 16384 ? (blocks < 1 ? 1 : blocks) : 16384)), block(kQuantThreads);
    if (vec)
        hipLaunchKernelGGL((quantize_static_elems<true>), grid, block, 0, stream, (const _Float16*)x_f16,
                           chan_mul, inv_scale, xq, total, K);
    else
        hipLaunchKernelGGL((quantize_static_elems<false>), grid, block, 0, stream, (const _Float16*)x_f16,
                           chan_mul, inv_scale, xq, total, K);
    return hipGetLastError();
}

hipError_t launch_quantize_weight(const float* w, const float* chan_s, int w_bits, void* wq_out,
                                  float* w_scale, int N, int K, hipStream_t stream) {
    const dim3 grid((unsigned)N), block(kQuantThreads);
#define VQ_LAUNCH_W(BITS, HAS)                                                                  \
    hipLaunchKernelGGL((quantize_weight_rows<BITS, HAS>), grid, block, 0, stream, w, chan_s, \
                       wq_out, w_scale, K)
    if (w_bits == 8) {
        if (chan_s) VQ_LAUNCH_W(8, true); else VQ_LAUNCH_W(8, false);
    } else {
        if (chan_s) VQ_LAUNCH_W(4, true); else VQ_LAUNCH_W(4, false);
    }
#undef VQ_LAUNCH_W
    return hipGetLastError();
}

}  // namespace vq
