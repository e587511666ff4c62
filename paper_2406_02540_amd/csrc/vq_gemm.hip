// int8 x int8 -> int32 MFMA GEMM with the dequantization epilogue, for gfx950.
//
// Computes, for tokens m and output channels n (ViDiT-Q appendix "Hardware
// implementation of quantized linear layers"; Sec. 4.1 for the grouping):
//     acc[m,n] = sum_k xq[m,k] * wq[n,k]
//     y[m,n]   = fp16(float(acc) * x_scale[m] * w_scale[n] + bias[n])
// W4A8 (appendix "Performance under lower bitwidth"): 4-bit weights are widened
// to int8 on their way into LDS and then take the same mainloop.
//
// Shape of the kernel
//   - workgroup tile: 256 tokens x 128 output channels, 4 wavefronts (2 x 2),
//     each wavefront 128 tokens x 64 channels = 2 x 4 MFMA 32x32x32 blocks,
//     128 int32 accumulators per lane; two workgroups per CU so that one
//     group's epilogue and LDS traffic overlap the other's MFMAs.
//   - K is walked in stages of 64 bytes, double buffered in LDS.  Activations
//     (and int8 weights) go global -> LDS directly (buffer_load ... lds, 16 B
//     per lane); 4-bit weights go through registers, are widened there and
//     written to LDS as int8.
//   - LDS tiles are [row][64 B] with the four 16-byte chunks of a row XOR-ed
//     by (row/4)%4, which makes the 16-lane groups of a ds_read_b128 hit 16
//     different bank groups.
//   - The weights are the MFMA row operand and the tokens the column operand,
//     so a lane owns one token and, by permuting which weight row sits in
//     which MFMA row, 32 consecutive output channels of it: the epilogue
//     writes 16-byte pieces of a row of Y without a transpose.
//   - Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the
//     id is remapped so that each XCD works on a contiguous run of tiles,
//     ordered in bands of 8 token tiles, and its L2 sees each panel once.
//
// Integer accumulation is exact and order independent, so the result is the
// same whatever the tiling; the 4-bit path multiplies by 16 * w (nibble left in
// the high half of the byte) and divides the sum by 16 exactly afterwards.
//
// Compiled with -ffp-contract=off: the epilogue is two fp32 multiplies and one
// add, each rounded on its own, then a round-to-nearest-even narrowing.
#include "vq_internal.h"

namespace vq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kTileT = 256;                 // tokens per workgroup
constexpr int kTileC = 128;                 // output channels per workgroup
constexpr int kTileK = 64;                  // K bytes per stage
constexpr int kThreads = 256;
constexpr int kXStage = kTileT * kTileK;    // 16 KiB
constexpr int kWStage = kTileC * kTileK;    // 8 KiB
constexpr int kLdsBytes = 2 * (kXStage + kWStage);
constexpr int kBand = 8;                    // token tiles per band in the tile order
constexpr int kXcds = 8;
constexpr unsigned kRsrcFlags = 0x00020000; // raw buffer, 32-bit data format

struct GemmArgs {
    const int8_t* xq;
    const float* x_scale;
    const void* w;
    const float* w_scale;
    const _Float16* bias;
    _Float16* y;
    int32_t* acc_out;
    int M, N, K;
    int tiles_t, tiles_c, tiles, tiles_per_xcd;
};

// Byte offset of 16-byte chunk `chunk` of `row` in a swizzled [rows][64] tile.
__device__ __forceinline__ int swz(int row, int chunk) {
    return row * kTileK + ((chunk ^ ((row >> 2) & 3)) << 4);
}

// LDS row r of the weight tile holds which output channel of the tile.
// Rows are kept in MFMA order: r = slab*64 + b*32 + rho with rho = 8j + 4h + i
// the row index inside MFMA block b; the accumulator register 4j + i of lanes
// with lane/32 == h holds that row.  Sending channel slab*64 + 32h + 16b + 4j + i
// there gives lane half h the 32 consecutive channels slab*64 + 32h .. +31.
__device__ __forceinline__ int w_row_to_channel(int r) {
    const int slab = r >> 6, b = (r >> 5) & 1, rho = r & 31;
    const int j = rho >> 3, h = (rho >> 2) & 1, i = rho & 3;
    return slab * 64 + 32 * h + 16 * b + 4 * j + i;
}

__device__ __forceinline__ unsigned clamp_u32(long v) {
    return v > 0xFFFFFFFFl ? 0xFFFFFFFFu : (unsigned)v;
}

template <int W_BITS>
__global__ __launch_bounds__(kThreads, 2) void gemm_i8_dequant(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) int8_t lds[kLdsBytes];
    // layout: [X stage 0][X stage 1][W stage 0][W stage 1]
    int8_t* const lds_x = lds;
    int8_t* const lds_w = lds + 2 * kXStage;

    // ---- which tile ------------------------------------------------------
    const int pid = blockIdx.x;
    const int logical = (pid % kXcds) * a.tiles_per_xcd + pid / kXcds;
    if (pid / kXcds >= a.tiles_per_xcd || logical >= a.tiles) return;  // uniform per workgroup
    const int band_tiles = kBand * a.tiles_c;
    const int band = logical / band_tiles;
    const int band_first = band * kBand;
    const int band_rows = min(a.tiles_t - band_first, kBand);
    const int in_band = logical - band * band_tiles;
    const int tile_t = band_first + in_band % band_rows;
    const int tile_c = in_band / band_rows;
    const long tok0 = (long)tile_t * kTileT;
    const long ch0 = (long)tile_c * kTileC;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_t = wave & 1;   // which 128 tokens
    const int wave_c = wave >> 1;  // which 64 channels

    const int K = a.K;
    const int rows_x = (int)min((long)kTileT, a.M - tok0);
    const int rows_w = (int)min((long)kTileC, a.N - ch0);

    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.xq + tok0 * K), 0, clamp_u32((a.M - tok0) * (long)K), kRsrcFlags);
    constexpr int kWDiv = (W_BITS == 8) ? 1 : 2;  // bytes of K per stored byte
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const int8_t*)a.w + ch0 * (K / kWDiv)), 0,
        clamp_u32((a.N - ch0) * (long)(K / kWDiv)), kRsrcFlags);

    // ---- global -> LDS mapping ---------------------------------------------
    // One direct load fills 1 KiB = 16 rows x 64 B; lane l writes bytes
    // [16 l, 16 l + 16), i.e. row l/4, physical chunk l%4, which under the
    // swizzle is logical chunk (l%4) ^ (l/16).
    const int ld_row = lane >> 2;
    const int ld_chunk = (lane & 3) ^ (lane >> 4);
    int voff_x[4];  // wave w loads X row groups w, w+4, w+8, w+12 (16 groups)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = min((wave + 4 * j) * 16 + ld_row, rows_x - 1);
        voff_x[j] = r * K + ld_chunk * 16;
    }
    int voff_w[2];  // W8: wave w loads W row groups w, w+4 (8 groups)
    if (W_BITS == 8) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = (wave + 4 * j) * 16 + ld_row;
            const int c = min(w_row_to_channel(r), rows_w - 1);
            voff_w[j] = c * K + ld_chunk * 16;
        }
    }
    // W4: thread t brings 32 nibbles (16 B) of LDS row t/2, K-half t%2.
    const int w4_row = tid >> 1, w4_half = tid & 1;
    int voff_w4 = 0;
    if (W_BITS == 4) {
        const int c = min(w_row_to_channel(w4_row), rows_w - 1);
        voff_w4 = c * (K / 2) + w4_half * 16;
    }

    auto issue_x_and_w8 = [&](int stage, int k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rsrc_x, (lds_ptr)(lds_x + stage * kXStage + (wave + 4 * j) * 1024), 16, voff_x[j],
                k0, 0, 0);
        if (W_BITS == 8) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rsrc_w, (lds_ptr)(lds_w + stage * kWStage + (wave + 4 * j) * 1024), 16,
                    voff_w[j], k0, 0, 0);
        }
    };
    auto load_w4 = [&](int k0) -> v4i {
        return __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, voff_w4, k0 / 2, 0);
    };
    // Widen 32 nibbles to 32 bytes holding 16 * w (nibble moved to the high
    // half of its byte, sign bit included) and store them as chunks 2*half and
    // 2*half + 1 of the row.
    auto store_w4 = [&](int stage, v4i p) {
        v4i lo, hi;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned w = (unsigned)p[d];
            const unsigned even = (w << 4) & 0xF0F0F0F0u;  // k = 0,2,4,6 of this dword
            const unsigned odd = w & 0xF0F0F0F0u;          // k = 1,3,5,7
            const unsigned k0123 = __builtin_amdgcn_perm(odd, even, 0x05010400u);
            const unsigned k4567 = __builtin_amdgcn_perm(odd, even, 0x07030602u);
            if (d < 2) {
                lo[2 * d] = (int)k0123;
                lo[2 * d + 1] = (int)k4567;
            } else {
                hi[2 * (d - 2)] = (int)k0123;
                hi[2 * (d - 2) + 1] = (int)k4567;
            }
        }
        int8_t* base = lds_w + stage * kWStage;
        *(v4i*)(base + swz(w4_row, 2 * w4_half)) = lo;
        *(v4i*)(base + swz(w4_row, 2 * w4_half + 1)) = hi;
    };

    // ---- LDS -> MFMA operand mapping -----------------------------------------
    // Operand rows of a 32x32x32 block: lane l supplies row l%32, 16 bytes of K
    // chosen by l/32; a stage holds two such K steps (chunks 0,1 and 2,3).
    const int fr_row = lane & 31;
    const int fr_sw = (fr_row >> 2) & 3;
    int x_off[2], w_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int phys = ((2 * ks + (lane >> 5)) ^ fr_sw) << 4;
        x_off[ks] = (wave_t * 128 + fr_row) * kTileK + phys;
        w_off[ks] = (wave_c * 64 + fr_row) * kTileK + phys;
    }

    v16i acc[2][4];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][tb][r] = 0;

    const int nk = (K + kTileK - 1) / kTileK;
    const bool k_tail = (K % kTileK) != 0;

    // prologue: stage 0
    issue_x_and_w8(0, 0);
    if (W_BITS == 4) store_w4(0, load_w4(0));

    for (int it = 0; it < nk; ++it) {
        const int stage = it & 1;
        __syncthreads();  // stage `it` has landed for every wave; stage it-1 is no longer read

        v4i xf[2][4], wf[2][2];
        const int8_t* xs = lds_x + stage * kXStage;
        const int8_t* ws = lds_w + stage * kWStage;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
                wf[ks][cb] = *(const v4i*)(ws + w_off[ks] + cb * 32 * kTileK);
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                xf[ks][tb] = *(const v4i*)(xs + x_off[ks] + tb * 32 * kTileK);
        }
        if (k_tail && it == nk - 1) {
            // K is a multiple of 16 but not of 64: chunks past K hold bytes of
            // the next row (or nothing); a zero weight operand removes them.
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bool valid = it * kTileK + (2 * ks + (lane >> 5)) * 16 < K;
                if (!valid) {
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb) wf[ks][cb] = v4i{0, 0, 0, 0};
                }
            }
        }

        v4i w4_next;
        const bool more = it + 1 < nk;
        if (more) {
            issue_x_and_w8(stage ^ 1, (it + 1) * kTileK);
            if (W_BITS == 4) w4_next = load_w4((it + 1) * kTileK);
        }

#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    acc[cb][tb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks][cb], xf[ks][tb],
                                                                        acc[cb][tb], 0, 0, 0);

        if (W_BITS == 4 && more) store_w4(stage ^ 1, w4_next);
    }

    // ---- epilogue ------------------------------------------------------------
    // Lane (h = lane/32, t = lane%32) holds, for each of its 4 token blocks, the
    // 32 channels chl .. chl+31: accumulator block b, register r <-> chl + 16 b + r.
    const int h = lane >> 5;
    const long ch = ch0 + wave_c * 64 + 32 * h;
    const bool vec = (a.N % 8) == 0;
    // the 4-bit path accumulated 16 * w: fold the exact 1/16 into the channel scale
    const float wmul = (W_BITS == 4) ? 0.0625f : 1.0f;

    float wsc[32], bsc[32];
    if (vec) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (ch + 8 * g < a.N) {
                const v4f s0 = *(const v4f*)(a.w_scale + ch + 8 * g);
                const v4f s1 = *(const v4f*)(a.w_scale + ch + 8 * g + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wsc[8 * g + e] = s0[e] * wmul;
                    wsc[8 * g + 4 + e] = s1[e] * wmul;
                }
                if (a.bias) {
                    const half8 bv = *(const half8*)(a.bias + ch + 8 * g);
#pragma unroll
                    for (int e = 0; e < 8; ++e) bsc[8 * g + e] = (float)bv[e];
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) bsc[8 * g + e] = 0.0f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) wsc[8 * g + e] = 0.0f, bsc[8 * g + e] = 0.0f;
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            const bool ok = ch + q < a.N;
            wsc[q] = ok ? a.w_scale[ch + q] * wmul : 0.0f;
            bsc[q] = (ok && a.bias) ? (float)a.bias[ch + q] : 0.0f;
        }
    }

#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const long tok = tok0 + wave_t * 128 + tb * 32 + (lane & 31);
        if (tok >= a.M) continue;
        const float xsc = a.x_scale[tok];
        _Float16* yrow = a.y + tok * a.N + ch;
        int32_t* arow = a.acc_out ? a.acc_out + tok * a.N + ch : nullptr;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int b = g >> 1, r0 = (g & 1) * 8;
            half8 out;
            int iv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int v = acc[b][tb][r0 + e];
                iv[e] = (W_BITS == 4) ? (v >> 4) : v;
                float f = (float)v * xsc;
                f = f * wsc[8 * g + e];
                f = f + bsc[8 * g + e];
                out[e] = (_Float16)f;
            }
            if (vec) {
                if (ch + 8 * g < a.N) {
                    *(half8*)(yrow + 8 * g) = out;
                    if (arow) {
                        *(v4i*)(arow + 8 * g) = v4i{iv[0], iv[1], iv[2], iv[3]};
                        *(v4i*)(arow + 8 * g + 4) = v4i{iv[4], iv[5], iv[6], iv[7]};
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (ch + 8 * g + e < a.N) {
                        yrow[8 * g + e] = out[e];
                        if (arow) arow[8 * g + e] = iv[e];
                    }
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm(const int8_t* xq, const float* x_scale, const void* w, int w_bits,
                       const float* w_scale, const void* bias_f16, void* y_f16, int32_t* acc_out,
                       int M, int N, int K, hipStream_t stream) {
    GemmArgs a;
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
    a.tiles_t = (M + kTileT - 1) / kTileT;
    a.tiles_c = (N + kTileC - 1) / kTileC;
    const long tiles = (long)a.tiles_t * a.tiles_c;
    if (tiles > 0x7FFFFFF0l) return hipErrorInvalidValue;
    a.tiles = (int)tiles;
    a.tiles_per_xcd = (a.tiles + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)(a.tiles_per_xcd * kXcds)), block(kThreads);
    if (w_bits == 8)
        hipLaunchKernelGGL((gemm_i8_dequant<8>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((gemm_i8_dequant<4>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace vq
