// Small-tile variant of the int8 GEMM + dequantization (same arithmetic as
// vq_gemm.hip; ViDiT-Q appendix "Hardware implementation of quantized linear
// layers") for problems that the 256 x 256 tiles of the persistent kernel would
// spread over only a few CUs: few tokens (the cross-attention projections of a
// text prompt, a single small linear) times a long K.
//
// Such a launch is bound by memory latency, not by the matrix cores: what counts
// is how many bytes of weights are in flight.  So: 64 token x 64 channel tiles
// (many workgroups), 4 wavefronts each owning one 32x32 MFMA block, and a ring of
// 8 LDS stages of 128 bytes of K with 7 stages of direct-to-LDS loads in flight
// per workgroup.  Stores go straight from registers (32 bytes per lane and row).
#include "vq_gemm_common.h"
#include "vq_internal.h"

namespace vq {
namespace {

constexpr int kT = 64;            // tokens per workgroup
constexpr int kC = 64;            // output channels per workgroup
constexpr int kK = 128;           // K bytes per stage
constexpr int kThreadsS = 256;    // 4 wavefronts
constexpr int kRing = 8;          // LDS stages
constexpr int kXS = kT * kK;      // 8 KiB
constexpr int kWS = kC * kK;      // 8 KiB (4 KiB used by packed 4-bit weights)

struct SmallArgs {
    const int8_t* xq;
    const float* x_scale;
    const void* w;
    const float* w_scale;
    const _Float16* bias;
    _Float16* y;
    int32_t* acc_out;
    int M, N, K;
    int tiles_c;
};

template <int PENDING>
__device__ __forceinline__ void wait_pending_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(PENDING) : "memory");
}

template <int W_BITS, bool K_TAIL>
__global__ __launch_bounds__(kThreadsS) void gemm_i8_dequant_small(const SmallArgs a) {
    __shared__ __attribute__((aligned(1024))) int8_t lds[kRing * (kXS + kWS)];
    int8_t* const lds_x = lds;
    int8_t* const lds_w = lds + kRing * kXS;
    const unsigned lds_x_addr = (unsigned)(uintptr_t)(lds_ptr)lds_x;
    const unsigned lds_w_addr = (unsigned)(uintptr_t)(lds_ptr)lds_w;

    const int tile_t = blockIdx.x / a.tiles_c, tile_c = blockIdx.x % a.tiles_c;
    const long tok0 = (long)tile_t * kT, ch0 = (long)tile_c * kC;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_t = wave & 1;   // which 32 tokens
    const int wave_c = wave >> 1;  // which MFMA block of the 64 channels
    const int K = a.K;
    const int rows_x = (int)min((long)kT, a.M - tok0);
    const int rows_w = (int)min((long)kC, a.N - ch0);
    constexpr int kWDiv = (W_BITS == 8) ? 1 : 2;
    const v4i rsrc_x = make_rsrc(a.xq + tok0 * K, clamp_u32((a.M - tok0) * (long)K));
    const v4i rsrc_w = make_rsrc((const int8_t*)a.w + ch0 * (K / kWDiv),
                                 clamp_u32((a.N - ch0) * (long)(K / kWDiv)));

    // global -> LDS: one direct load = 8 rows x 128 B, lane l = row l/8, physical chunk
    // l%8 holding logical chunk (l%8) ^ ((row/2)%8); wave w loads row groups w and w+4 of
    // both tiles.  Packed 4-bit tile [64 rows][64 B]: 16 rows x 64 B per load, lane l = row
    // l/4, logical chunk (l%4) ^ (l/16); wave w loads row group w.
    const int ld_chunk16 = ((lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7)) << 4;
    int voff_x[2], voff_w[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = (wave + 4 * j) * 8 + (lane >> 3);
        voff_x[j] = min(r, rows_x - 1) * K + ld_chunk16;
        voff_w[j] = min(w_row_to_channel(r), rows_w - 1) * K + ld_chunk16;
    }
    if (W_BITS == 4) {
        const int r4 = wave * 16 + (lane >> 2);
        voff_w[0] = min(w_row_to_channel(r4), rows_w - 1) * (K / 2) + (((lane & 3) ^ (lane >> 4)) << 4);
    }
    constexpr int kLoadsPerStage = (W_BITS == 8) ? 4 : 3;  // per wave
    auto issue_stage = [&](int slot, int k0) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
            load_stage_to_lds_16<K_TAIL>(rsrc_x, lds_x_addr + slot * kXS + (wave + 4 * j) * 1024, voff_x[j], k0);
        if (W_BITS == 8) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
                load_stage_to_lds_16<K_TAIL>(rsrc_w, lds_w_addr + slot * kWS + (wave + 4 * j) * 1024, voff_w[j], k0);
        } else {
            load_stage_to_lds_16<K_TAIL>(rsrc_w, lds_w_addr + slot * kWS + wave * 1024, voff_w[0], k0 / 2);
        }
    };

    // LDS -> MFMA operands: lane l supplies row l%32 and the 16 bytes of K chosen by l/32
    const int fr_row = lane & 31;
    const int x_off0 = (wave_t * 32 + fr_row) * kK + (((lane >> 5) ^ ((fr_row >> 1) & 7)) << 4);
    const int w_off0 = (W_BITS == 8)
                           ? (wave_c * 32 + fr_row) * kK + (((lane >> 5) ^ ((fr_row >> 1) & 7)) << 4)
                           : (wave_c * 32 + fr_row) * (kK / 2) + (((fr_row >> 2) & 3) << 4) + (lane >> 5) * 8;

    // Scales and bias of this lane's outputs, requested before the mainloop.  Lane
    // (h = lane/32, t = lane%32) ends up with token t of the wave's 32 and the 16
    // channels 32 h + 16 wave_c .. + 15 of the tile (accumulator register r <-> + r).
    const int h = lane >> 5;
    const long tok = tok0 + wave_t * 32 + (lane & 31);
    const long chl = ch0 + 32 * h + 16 * wave_c;
    const bool tok_ok = tok < a.M;
    // (unconditional loads at clamped indices, converted only in the epilogue: nothing
    // here waits for memory; what belongs to a channel or token past the matrix is never stored)
    const float xsc = a.x_scale[min(tok, (long)a.M - 1)];
    const float wmul = (W_BITS == 4) ? 0.0625f : 1.0f;  // the 4-bit path accumulates 16 * w
    const _Float16* bias_src = a.bias ? a.bias : (const _Float16*)a.w_scale;  // any readable N halves
    float wraw[16];
    _Float16 braw[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const long c = min(chl + r, (long)a.N - 1);
        wraw[r] = a.w_scale[c];
        braw[r] = bias_src[c];
    }

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;

    const int nk = (K + kK - 1) / kK;
    // prologue: up to kRing - 1 stages in flight
#pragma unroll 1
    for (int s = 0; s < kRing - 1 && s < nk; ++s) issue_stage(s, s * kK);

    int slot = 0;
#pragma unroll 1
    for (int it = 0; it < nk; ++it) {
        // Stage `it` must have landed.  While new stages are still being issued exactly
        // kRing - 2 younger stages may stay in flight; afterwards simply drain.
        if (it + kRing - 1 <= nk)
            wait_pending_and_barrier<kLoadsPerStage*(kRing - 2)>();
        else
            wait_pending_and_barrier<0>();
        // every wave is past stage it-1: its slot takes stage it + kRing - 1
        if (it + kRing - 1 < nk) issue_stage(slot == 0 ? kRing - 1 : slot - 1, (it + kRing - 1) * kK);

        const int8_t* xs = lds_x + slot * kXS;
        const int8_t* ws = lds_w + slot * kWS;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            v4i wf;
            if (W_BITS == 8)
                wf = *(const v4i*)(ws + (w_off0 ^ (ks << 5)));
            else
                wf = widen_nibbles(*(const v2i*)(ws + (w_off0 ^ (ks << 4))));
            const v4i xf = *(const v4i*)(xs + (x_off0 ^ (ks << 5)));
            if (K_TAIL && it == nk - 1 && it * kK + (2 * ks + (lane >> 5)) * 16 >= K) wf = v4i{0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xf, acc, 0, 0, 0);
        }
        slot = (slot == kRing - 1) ? 0 : slot + 1;
    }

    // epilogue, straight from registers
    if (!tok_ok) return;
    _Float16* yrow = a.y + tok * a.N + chl;
    int32_t* arow = a.acc_out ? a.acc_out + tok * a.N + chl : nullptr;
    const bool vec = (a.N % 8) == 0;
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        int iv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) iv[e] = (W_BITS == 4) ? (acc[8 * g + e] >> 4) : acc[8 * g + e];
        // y = fp16(float(acc) * (x_scale * w_scale) + bias), as in the large-tile kernel: the
        // product of the scales in fp32 (the exact 1/16 of the 4-bit path on the token scale),
        // the rest exact and rounded once
        v4i outv;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float s0 = (xsc * wmul) * wraw[8 * g + e], s1 = (xsc * wmul) * wraw[8 * g + e + 1];
            unsigned b2 = 0;
            if (a.bias) {
                const _Float16 pair[2] = {braw[8 * g + e], braw[8 * g + e + 1]};
                __builtin_memcpy(&b2, pair, 4);
            }
            outv[e / 2] = (int)dequant_pair((float)acc[8 * g + e], s0, (float)acc[8 * g + e + 1], s1, b2);
        }
        const half8 out = (half8)outv;  // (reinterprets the bits)
        if (vec) {
            if (chl + 8 * g < a.N) {
                *(half8*)(yrow + 8 * g) = out;
                if (arow) {
                    *(v4i*)(arow + 8 * g) = v4i{iv[0], iv[1], iv[2], iv[3]};
                    *(v4i*)(arow + 8 * g + 4) = v4i{iv[4], iv[5], iv[6], iv[7]};
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (chl + 8 * g + e < a.N) {
                    yrow[8 * g + e] = out[e];
                    if (arow) arow[8 * g + e] = iv[e];
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm_small(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
                             const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out,
                             int M, int N, int K, hipStream_t stream) {
    SmallArgs a;
    a.xq = xq;
    a.x_scale = x_scale;
    a.w = w;
    a.w_scale = w_scale;
    a.bias = (const _Float16*)bias_f16;
    a.y = (_Float16*)y_f16;
    a.acc_out = acc_out;
    a.M = M;
    a.N = N;
    a.K = K;
    a.tiles_c = (N + kC - 1) / kC;
    const long tiles = (long)((M + kT - 1) / kT) * a.tiles_c;
    if (tiles > 0x7FFFFFF0l) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles), block(kThreadsS);
    const bool tail = (K % kK) != 0;
    if (w_bits == 8) {
        if (tail) hipLaunchKernelGGL((gemm_i8_dequant_small<8, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemm_i8_dequant_small<8, false>), grid, block, 0, stream, a);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_i8_dequant_small<4, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemm_i8_dequant_small<4, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace vq
