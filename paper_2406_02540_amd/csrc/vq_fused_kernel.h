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
//
// Compiled with -ffp-contract=off: every fp32 operation rounds on its own.
#pragma once
#include "vq_internal.h"
#include "vq_quantize_row.h"

namespace vq {

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

// The producers are compiled in two translation units (each (producer, chunks, lanes) combination
// is a kernel of its own, 48 per producer).
hipError_t launch_producer_gelu(int producer, const FusedArgs& a, hipStream_t stream);   // vq_fused_gelu.hip: both GELU forms
hipError_t launch_producer_other(int producer, const FusedArgs& a, hipStream_t stream);  // vq_fused.hip

namespace {


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

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
constexpr int kBufFlags = 0x00020000;          // raw buffer, 32-bit data format
constexpr int kPastEnd = 0x7FFFFFF0;           // a buffer offset behind every buffer: loads give zero, stores are dropped

// A wavefront takes 64 / LANES tokens.  Everything it reads or writes goes through range-checked
// buffers: the rows through buffers that start at the wavefront's first token and end behind its
// last one, so that tokens past M and chunks past K (whose offset is pushed behind the buffer) read
// as zero and are never written, without a branch; the per-channel vectors (balancing factor,
// modulation scale and shift or gate) through buffers over the whole arrays, addressed by 32-bit
// offsets from a scalar base (a pointer per chunk and vector would cost two registers each).  A
// kernel without branches and with few registers keeps many wavefronts per SIMD resident, and that,
// not a loop over tokens with a prefetch, is what overlaps the producers' arithmetic with the memory
// time of other wavefronts' rows (the loop was built and measured: slower for every producer but one).
template <int PRODUCER, int NCH, int LANES>
__global__ __launch_bounds__(kQuantThreads) void produce_quantize_tokens(const FusedArgs a) {
    constexpr int kTokensPerWave = kWave / LANES;
    const int lane = threadIdx.x & (kWave - 1);
    const int sub = lane & (LANES - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // (uniform: the buffer descriptors below are scalar)
    const int K8 = a.K8;
    const long w_first = ((long)blockIdx.x * kRowsPerBlock + wave) * kTokensPerWave;  // first token of this wavefront
    if (w_first >= a.M) return;  // (uniform per wavefront)
    const long m = w_first + lane / LANES;
    const bool row_ok = m < a.M;

    const int ntok = (int)(a.M - w_first < kTokensPerWave ? a.M - w_first : kTokensPerWave);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.x + w_first * K8), 0, ntok * K8 * 16, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_q =
        __builtin_amdgcn_make_buffer_rsrc((void*)(a.xq + w_first * K8), 0, ntok * K8 * 8, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(PRODUCER == kResidual ? a.y + w_first * K8 : a.x), 0, PRODUCER == kResidual ? ntok * K8 * 16 : 0, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_r = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(PRODUCER == kResidual ? a.r_out + w_first * K8 : (half8*)a.x), 0, PRODUCER == kResidual ? ntok * K8 * 16 : 0,
        kBufFlags);
    const int n_samples = (int)((a.M + (long)a.tokens_per_sample - 1) / a.tokens_per_sample);
    const __amdgpu_buffer_rsrc_t rs_cm =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.chan_mul, 0, a.chan_mul ? K8 * 32 : 0, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_a =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.mod_a, 0, a.mod_a ? n_samples * K8 * 32 : 0, kBufFlags);
    const __amdgpu_buffer_rsrc_t rs_b =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.mod_b, 0, a.mod_b ? n_samples * K8 * 32 : 0, kBufFlags);

    int voff[NCH];  // byte offset of this lane's chunk i in the fp16 rows (half of it in the int8 rows)
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = i * LANES + sub;
        voff[i] = (c < K8) ? ((lane / LANES) * K8 + c) * 16 : kPastEnd;
    }
    // The 8 floats of a per-channel vector that belong to chunk i of this lane, row `row` of a
    // [rows][K] array (chunks past K take the last chunk's: finite values that meet only zeros).
    struct Vec8 { float4v lo, hi; };
    auto vec_chunk = [&](const __amdgpu_buffer_rsrc_t& rs, int row, int i) {
        const int off = (row * K8 + min(i * LANES + sub, K8 - 1)) * 32;
        Vec8 v;
        v.lo = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
        v.hi = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16, 0, 0));
        return v;
    };
    // The vectors are asked for one chunk ahead of their use.  After every chunk a barrier for
    // memory accesses that also pins the chunk's results keeps the compiler from asking for the
    // vectors of all chunks first and doing the arithmetic afterwards (16 to 32 registers per chunk).
    auto chunk_done = [](float(&c)[8]) {
        asm volatile("" : "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]), "+v"(c[4]), "+v"(c[5]), "+v"(c[6]), "+v"(c[7])
                     :
                     : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // which sample's modulation this token takes
    const int b = (int)((unsigned)(row_ok ? m : a.M - 1) / (unsigned)a.tokens_per_sample);

    float t[NCH][8];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const half8 raw = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(rs_x, voff[i], 0, 2 /* nontemporal */));
#pragma unroll
        for (int j = 0; j < 8; ++j) t[i][j] = (float)raw[j];
    }

    if (PRODUCER == kHadamard) {
        // Rotation-based balancing (Sec. 4.2): t = (x * chan_mul) Q with Q block diagonal,
        // blocks H_128 / sqrt(128).  A block is 16 consecutive chunks = the 16 lanes sub%16 of a
        // token with one chunk index i, so element 8 (sub%16) + j of the block sits in lane
        // sub, register t[i][j]: three butterfly stages inside the registers, four across lanes.
        if (a.chan_mul) {
            Vec8 nxt = vec_chunk(rs_cm, 0, 0);
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const Vec8 cm = nxt;
                if (i + 1 < NCH) nxt = vec_chunk(rs_cm, 0, i + 1);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    t[i][j] = t[i][j] * cm.lo[j];
                    t[i][4 + j] = t[i][4 + j] * cm.hi[j];
                }
                chunk_done(t[i]);
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
        hadamard_lane_stage<1>(t, sub);
        hadamard_lane_stage<2>(t, sub);
        hadamard_lane_stage<4>(t, sub);
        hadamard_lane_stage<8>(t, sub);
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
            const bool in_row = i * LANES + sub < K8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                t[i][j] = in_row ? t[i][j] - mean : 0.0f;
                ss = __builtin_fmaf(t[i][j], t[i][j], ss);
            }
        }
        const float var = group_sum<LANES>(ss) / (float)(8 * K8);
        const float rstd = 1.0f / __builtin_sqrtf(var + a.eps);
        // t = (x - mean) rstd (1 + scale) + shift as one multiply and one fma per element
        Vec8 nxt_a{}, nxt_b{};
        if (a.mod_a) nxt_a = vec_chunk(rs_a, b, 0);
        if (a.mod_b) nxt_b = vec_chunk(rs_b, b, 0);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const Vec8 sc = nxt_a, sh = nxt_b;
            if (i + 1 < NCH) {
                if (a.mod_a) nxt_a = vec_chunk(rs_a, b, i + 1);
                if (a.mod_b) nxt_b = vec_chunk(rs_b, b, i + 1);
            }
            float mul[8], add[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mul[j] = a.mod_a ? rstd * (1.0f + sc.lo[j]) : rstd;
                mul[4 + j] = a.mod_a ? rstd * (1.0f + sc.hi[j]) : rstd;
                add[j] = a.mod_b ? sh.lo[j] : 0.0f;
                add[4 + j] = a.mod_b ? sh.hi[j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) t[i][j] = __builtin_fmaf(t[i][j], mul[j], add[j]);
            chunk_done(t[i]);
        }
    }

    if constexpr (PRODUCER == kResidual) {
        Vec8 nxt{};
        if (a.mod_a) nxt = vec_chunk(rs_a, b, 0);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const Vec8 gate = nxt;
            if (a.mod_a && i + 1 < NCH) nxt = vec_chunk(rs_a, b, i + 1);
            const half8 yv = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(rs_y, voff[i], 0, 2 /* nontemporal */));
            float p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) p[j] = (float)yv[j];
            if (a.mod_a) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    p[j] = gate.lo[j] * p[j];
                    p[4 + j] = gate.hi[j] * p[4 + j];
                }
            }
            half8 r;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float sum = t[i][j] + p[j];
                asm("" : "+v"(sum));     // (the fp32 sum is rounded before it is narrowed)
                r[j] = (_Float16)sum;    // the new residual stream is fp16 ...
                t[i][j] = (float)r[j];   // ... and that is what the next layer quantizes
            }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, r), rs_r, voff[i], 0, 0);
        }
    }

    // ---- the quantizer: balancing factor, absmax of the token, its scale, int8 codes ----
    // (two IEEE divisions per token, none per element)
    float amax = 0.0f;
    const bool fold = PRODUCER != kHadamard && a.chan_mul;  // (the rotation has the scaling before itself)
    Vec8 nxt_cm{};
    if (fold) nxt_cm = vec_chunk(rs_cm, 0, 0);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        if (fold) {
            const Vec8 cm = nxt_cm;
            if (i + 1 < NCH) nxt_cm = vec_chunk(rs_cm, 0, i + 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                t[i][j] = t[i][j] * cm.lo[j];
                t[i][4 + j] = t[i][4 + j] * cm.hi[j];
            }
        }
        const bool in_row = i * LANES + sub < K8;
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, in_row ? fabsf(t[i][j]) : 0.0f);
        if (fold) {
            asm volatile("" : : : "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    amax = group_max<LANES>(amax);
    float scale = 0.0f, inv = 0.0f;
    if (amax != 0.0f) {
        scale = amax / 127.0f;
        inv = 127.0f / amax;
    }
    if (row_ok && sub == 0) a.x_scale[m] = scale;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        int q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = quantize_one(t[i][j], inv, 127.0f);
        int2v o;
        o.x = pack4(q[0], q[1], q[2], q[3]);
        o.y = pack4(q[4], q[5], q[6], q[7]);
        __builtin_amdgcn_raw_buffer_store_b64(o, rs_q, voff[i] == kPastEnd ? kPastEnd : voff[i] / 2, 0, 0);
    }
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
}  // namespace vq
