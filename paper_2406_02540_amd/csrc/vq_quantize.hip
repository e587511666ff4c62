// Quantizers for gfx950.
//
// 1. Dynamic per-token activation quantizer (ViDiT-Q Sec. 4.1; Eq. 2 of Sec. 3.1
//    in symmetric form; activation side of the channel balancing, Eq. 3 of
//    Sec. 4.2).  HBM-bound: a token is read once (2 B/element), kept in
//    registers across the absmax reduction (as the fp16 it arrived as, or as
//    fp32 products where a balancing factor is folded in), and written once
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

// The token row held in registers (layout and steps: vq_quantize_row.h).  This kernel folds
// the balancing factor in as the row arrives and keeps the products in fp32: 8 registers per
// chunk, so the launcher prefers few chunks per lane (K = 1152: 32 lanes x 5 chunks).
template <int NCH, int LANES>
__global__ __launch_bounds__(kQuantThreads) void quantize_tokens_wave_mul(
    const half8* __restrict__ x, const float4v* __restrict__ chan_mul, int2v* __restrict__ xq,
    float* __restrict__ x_scale, int M, int K8) {
    const RowLane<LANES> rl(M);
    float t[NCH][8];
    load_row<NCH, LANES, true>(x + (rl.row_ok ? rl.m : 0) * K8, rl.row_ok, rl.sub, K8, t, chan_mul);
    fold_quantize_store<NCH, LANES, false>(t, nullptr, rl.row_ok, rl.sub, K8, rl.m, xq, x_scale);
}

// Wavefronts per SIMD the register allocation below is held to (4 registers per chunk of the row,
// 512 registers per SIMD lane).
constexpr int quant_waves(int nch) { return nch <= 10 ? 8 : nch == 11 ? 7 : nch == 12 ? 6 : nch <= 15 ? 5 : 4; }

// No balancing factor: LANES is chosen so that K / 8 = NCH * LANES exactly where possible
// (K = 1152: 16 lanes x 9 chunks), which keeps every lane busy on every instruction, and
// the row stays in registers as the fp16 it arrived as (half the
// registers of an fp32 copy, so that twice as many wavefronts are resident and every
// workgroup of the video-sized problem is in flight at once).  The absolute maximum is
// taken on the fp16 values (exact: fp16 -> fp32 is monotonic and exact), each value is
// widened once more where it is scaled and rounded.
template <int NCH, int LANES>
__global__ __launch_bounds__(kQuantThreads, quant_waves(NCH)) void quantize_tokens_wave(
    const half8* __restrict__ x, int2v* __restrict__ xq, float* __restrict__ x_scale, int M, int K8) {
    const RowLane<LANES> rl(M);
    const half8* row = x + (rl.row_ok ? rl.m : 0) * K8;
    half8 raw[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + rl.sub;
        if (rl.row_ok && c < K8) raw[i] = __builtin_nontemporal_load(row + c);
        else raw[i] = (half8){0, 0, 0, 0, 0, 0, 0, 0};
    }
    half8 hmax = __builtin_elementwise_abs(raw[0]);
#pragma unroll
    for (int i = 1; i < NCH; ++i) hmax = __builtin_elementwise_max(hmax, __builtin_elementwise_abs(raw[i]));
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) amax = fmaxf(amax, (float)hmax[j]);
    amax = group_max<LANES>(amax);

    float scale = 0.0f, inv = 0.0f;
    if (amax != 0.0f) {
        scale = amax / 127.0f;
        inv = 127.0f / amax;
    }
    if (rl.row_ok && rl.sub == 0) x_scale[rl.m] = scale;

    int2v* qrow = xq + (rl.row_ok ? rl.m : 0) * K8;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + rl.sub;
        if (rl.row_ok && c < K8) {
            // (opaque to the optimizer: the widening happens here, chunk by chunk, and no
            // fp32 copy of the row is carried over from above)
            asm volatile("" : "+v"(raw[i]));
            int q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = quantize_one((float)raw[i][j], inv, 127.0f);
            int2v o;
            o.x = pack4(q[0], q[1], q[2], q[3]);
            o.y = pack4(q[4], q[5], q[6], q[7]);
            qrow[c] = o;
        }
    }
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

// Static quantizer (the comparison point: one scale for the whole tensor, fixed beforehand).
// Rows of whole 16-byte chunks: a wavefront takes CHUNKS KiB of contiguous input, a thread
// its chunks one wavefront width apart (every load and store instruction of a wavefront is
// contiguous), all loads first.
template <bool HAS_MUL, int CHUNKS>
__global__ __launch_bounds__(kQuantThreads, 8) void quantize_static_chunks(
    const half8* __restrict__ x, const float4v* __restrict__ chan_mul, float inv, int2v* __restrict__ xq,
    unsigned chunks, unsigned K8) {
    const unsigned base = blockIdx.x * (kQuantThreads * CHUNKS) + (threadIdx.x >> 6) * (kWave * CHUNKS) +
                          (threadIdx.x & (kWave - 1));
    half8 v[CHUNKS];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const unsigned c = base + i * kWave;
        if (c < chunks) v[i] = __builtin_nontemporal_load(x + c);
    }
    int2v o[CHUNKS];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const unsigned c = base + i * kWave;
        if (c < chunks) {
            float t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (float)v[i][j];
            if (HAS_MUL) {
                const unsigned k8 = c % K8;
                const float4v m0 = chan_mul[2 * k8], m1 = chan_mul[2 * k8 + 1];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t[j] = t[j] * m0[j];
                    t[4 + j] = t[4 + j] * m1[j];
                }
            }
            int q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = quantize_one(t[j], inv, 127.0f);
            o[i].x = pack4(q[0], q[1], q[2], q[3]);
            o[i].y = pack4(q[4], q[5], q[6], q[7]);
        }
    }
    // the stores leave together, behind the last load (reads and writes in bursts, not mixed)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const unsigned c = base + i * kWave;
        if (c < chunks) xq[c] = o[i];
    }
}

// Any K: element by element.
__global__ __launch_bounds__(kQuantThreads) void quantize_static_elems(
    const _Float16* __restrict__ x, const float* __restrict__ chan_mul, float inv, int8_t* __restrict__ xq,
    long total, int K) {
    const long step = (long)gridDim.x * kQuantThreads;
    for (long e = (long)blockIdx.x * kQuantThreads + threadIdx.x; e < total; e += step) {
        float t = (float)x[e];
        if (chan_mul) t = t * chan_mul[e % K];
        xq[e] = (int8_t)quantize_one(t, inv, 127.0f);
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
        hipLaunchKernelGGL((quantize_tokens_wave_mul<NCH, LANES>), grid, block, 0, stream,
                           (const half8*)x, (const float4v*)chan_mul, (int2v*)xq, x_scale, M, K / 8);
    else
        hipLaunchKernelGGL((quantize_tokens_wave<NCH, LANES>), grid, block, 0, stream,
                           (const half8*)x, (int2v*)xq, x_scale, M, K / 8);
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
        if (chan_mul) {  // the row is held as fp32 products: few chunks per lane first
            switch (lanes_for_row(k8)) {
                case 16: return launch_wave_nch<16>((k8 + 15) / 16, x_f16, chan_mul, xq, x_scale, M, K, stream);
                case 32: return launch_wave_nch<32>((k8 + 31) / 32, x_f16, chan_mul, xq, x_scale, M, K, stream);
                default: return launch_wave_nch<64>((k8 + 63) / 64, x_f16, chan_mul, xq, x_scale, M, K, stream);
            }
        }
        // held as fp16: the widest lane group that divides the row exactly; a whole wavefront otherwise
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

template <int CHUNKS>
hipError_t launch_static_chunks(const void* x_f16, const float* chan_mul, float inv_scale, int8_t* xq,
                                unsigned chunks, unsigned K8, hipStream_t stream) {
    constexpr unsigned per_block = kQuantThreads * CHUNKS;
    const dim3 grid((chunks + per_block - 1) / per_block), block(kQuantThreads);
    if (chan_mul)
        hipLaunchKernelGGL((quantize_static_chunks<true, CHUNKS>), grid, block, 0, stream, (const half8*)x_f16,
                           (const float4v*)chan_mul, inv_scale, (int2v*)xq, chunks, K8);
    else
        hipLaunchKernelGGL((quantize_static_chunks<false, CHUNKS>), grid, block, 0, stream, (const half8*)x_f16,
                           (const float4v*)nullptr, inv_scale, (int2v*)xq, chunks, K8);
    return hipGetLastError();
}

hipError_t launch_quantize_static(const void* x_f16, const float* chan_mul, float inv_scale, int8_t* xq,
                                  int M, int K, hipStream_t stream) {
    const long total = (long)M * K;
    if (K % 8 == 0 && total / 8 < (1L << 31)) {
        // Chunks per thread: the count whose grid wastes least of its last round of resident
        // workgroups (8 per compute unit, 256 units).
        const long chunks = total / 8, slots = 8 * 256;
        int best = 8;
        long best_cost = 1L << 62;
        for (int u : {8, 9, 10}) {
            const long blocks = (chunks + kQuantThreads * u - 1) / (kQuantThreads * u);
            const long cost = (blocks + slots - 1) / slots * u;
            if (cost < best_cost) {
                best_cost = cost;
                best = u;
            }
        }
        switch (best) {
            case 9: return launch_static_chunks<9>(x_f16, chan_mul, inv_scale, xq, (unsigned)chunks, (unsigned)(K / 8), stream);
            case 10: return launch_static_chunks<10>(x_f16, chan_mul, inv_scale, xq, (unsigned)chunks, (unsigned)(K / 8), stream);
            default: return launch_static_chunks<8>(x_f16, chan_mul, inv_scale, xq, (unsigned)chunks, (unsigned)(K / 8), stream);
        }
    }
    const long blocks = (total + kQuantThreads - 1) / kQuantThreads;
    const dim3 grid((unsigned)(blocks < 16384 ? (blocks < 1 ? 1 : blocks) : 16384)), block(kQuantThreads);
    hipLaunchKernelGGL(quantize_static_elems, grid, block, 0, stream, (const _Float16*)x_f16, chan_mul, inv_scale,
                       xq, total, K);
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
