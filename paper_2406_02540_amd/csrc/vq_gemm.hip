// int8 x int8 -> int32 MFMA GEMM with the dequantization epilogue, for gfx950.
//
// Computes, for tokens m and output channels n (ViDiT-Q appendix "Hardware
// implementation of quantized linear layers"; Sec. 4.1 for the grouping):
//     acc[m,n] = sum_k xq[m,k] * wq[n,k]
//     y[m,n]   = fp16(float(acc) * x_scale[m] * w_scale[n] + bias[n])
// W4A8 (appendix "Performance under lower bitwidth"): 4-bit weights are staged
// in LDS packed and widened to int8 on their way from LDS into the MFMA operand
// registers; the mainloop is otherwise the same.
//
// Shape of the kernel
//   - workgroup tile: 256 tokens x 256 output channels, 8 wavefronts (2 x 4),
//     each wavefront 128 tokens x 64 channels = 2 x 4 MFMA 32x32x32 blocks,
//     128 int32 accumulators per lane, two wavefronts per SIMD.  The tile is
//     large because the L2 -> CU path, not HBM, is what the operand traffic
//     loads: bytes per multiply-add fall with the tile edge.
//   - K is walked in stages of 128 bytes, double buffered in LDS.  A stage
//     takes one full 128-byte cache line per row, so every L2 request is a
//     whole line.  Activations and weights go global -> LDS directly
//     (buffer_load ... lds, 16 B per lane, no registers in between); the loads
//     of stage i+1 are in flight while stage i is multiplied.  4-bit weights
//     travel packed (half the bytes).
//   - The direct loads are issued from inline assembly and waited for with an
//     explicit s_waitcnt: the compiler would otherwise wait for all of them
//     before every LDS read and undo the prefetch.
//   - LDS tiles are [row][128 B] with the eight 16-byte chunks of a row XOR-ed
//     by (row/2)%8, which makes the 16-lane groups of a ds_read_b128 hit 16
//     different bank groups.
//   - The weights are the MFMA row operand and the tokens the column operand,
//     so a lane owns one token and, by permuting which weight row sits in
//     which MFMA row, 32 consecutive output channels of it.  The epilogue
//     scales and narrows in registers, turns each wavefront's 128 x 64 block
//     through LDS and writes whole 128-byte lines of Y, bypassing the caches'
//     retention (nontemporal): the operands keep the L2.
//   - Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the
//     id is remapped so that each XCD works on a contiguous run of tiles,
//     ordered in bands of 8 token tiles, and its L2 sees each panel once.
//
// Integer accumulation is exact and order independent, so the result is the
// same whatever the tiling; the 4-bit path multiplies by 16 * w (nibble left in
// the high half of the byte) and divides the sum by 16 exactly afterwards.
//
// The epilogue computes fp16(fma(float(acc) * x_scale, w_scale, bias)) in fp32: one
// rounding fewer than the three separate operations, so an output can differ from
// the separately rounded value in the last fp16 place.
#include "vq_internal.h"

namespace vq {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kTileT = 256;                 // tokens per workgroup
constexpr int kTileC = 256;                 // output channels per workgroup
constexpr int kTileK = 128;                 // K bytes per stage (one cache line per row)
constexpr int kThreads = 512;               // 8 wavefronts
constexpr int kWaves = kThreads / 64;
constexpr int kXStage = kTileT * kTileK;    // 32 KiB
constexpr int kWStage = kTileC * kTileK;    // 32 KiB (16 KiB used by packed 4-bit weights)
constexpr int kStages = 2;
constexpr int kLdsBytes = kStages * (kXStage + kWStage);  // 128 KiB
constexpr int kScaleBytes = 3 * 1024;       // w_scale[256] fp32 | bias[256] fp16 (+pad) | x_scale[256] fp32
constexpr int kEpiRow = 128 + 16;           // bytes per token row of the epilogue staging (padded)
constexpr int kEpiWave = 64 * kEpiRow;      // one wavefront stages 64 tokens x 64 channels at a time
constexpr int kBand = 8;                    // token tiles per band in the tile order
constexpr int kXcds = 8;
constexpr unsigned kRsrcFlags = 0x00020000; // raw buffer, 32-bit data format
static_assert(kWaves * kEpiWave <= kLdsBytes, "epilogue staging must fit the stage buffers");

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

// Raw buffer descriptor: base address, no stride, size in bytes (accesses past
// it read as zero and never fault), 32-bit data format.
__device__ __forceinline__ v4i make_rsrc(const void* base, unsigned bytes) {
    const unsigned long long p = (unsigned long long)base;
    v4i r;
    r[0] = (int)(unsigned)p;
    r[1] = (int)(unsigned)(p >> 32) & 0xFFFF;
    r[2] = (int)bytes;
    r[3] = (int)kRsrcFlags;
    return r;
}

// 16 bytes per lane from buffer offset voff + soff straight into LDS at
// lds_addr + 16 * lane (lds_addr is wave-uniform and goes through M0).  Counts
// in vmcnt; the compiler does not know about it, see wait_loads_and_barrier().
__device__ __forceinline__ void load_to_lds_16(v4i rsrc, unsigned lds_addr, int voff, int soff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds"
        :
        : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
        : "memory");
}

// Waits until all of this wave's direct loads have landed and all its LDS
// accesses are done, then joins the workgroup barrier.
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" : : : "memory");
}

// 16 nibbles (two dwords) -> 16 bytes holding 16 * w: the nibble is moved to
// the high half of its byte, sign bit included, in the order of K.
__device__ __forceinline__ v4i widen_nibbles(v2i p) {
    v4i o;
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const unsigned w = (unsigned)p[d];
        const unsigned even = (w << 4) & 0xF0F0F0F0u;  // k = 0,2,4,6 of this dword
        const unsigned odd = w & 0xF0F0F0F0u;          // k = 1,3,5,7
        o[2 * d] = (int)__builtin_amdgcn_perm(odd, even, 0x05010400u);      // k = 0,1,2,3
        o[2 * d + 1] = (int)__builtin_amdgcn_perm(odd, even, 0x07030602u);  // k = 4,5,6,7
    }
    return o;
}

// K_TAIL: K is a multiple of 16 but not of 128 (the last stage is partly past K).
template <int W_BITS, bool K_TAIL>
__global__ __launch_bounds__(kThreads, 2) void gemm_i8_dequant(const GemmArgs a) {
    __shared__ __attribute__((aligned(1024))) int8_t lds[kLdsBytes + kScaleBytes];
    // layout: [X stage 0][X stage 1][W stage 0][W stage 1]; a W stage is
    // [256 rows][128 B] of int8 or, for 4-bit weights, [256 rows][64 B] of nibbles.
    int8_t* const lds_x = lds;
    int8_t* const lds_w = lds + kStages * kXStage;
    const unsigned lds_x_addr = (unsigned)(uintptr_t)(lds_ptr)lds_x;
    const unsigned lds_w_addr = (unsigned)(uintptr_t)(lds_ptr)lds_w;
    int8_t* const lds_sc = lds + kLdsBytes;  // the tile's scales and bias, fetched during the mainloop
    const unsigned lds_sc_addr = (unsigned)(uintptr_t)(lds_ptr)lds_sc;

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
    // Waves w and w+4 share a SIMD: they get the same token half and channel
    // slabs two apart, so a tile that is only half full of channels still
    // leaves one working wave on every SIMD.
    const int wave_t = wave & 1;   // which 128 tokens
    const int wave_c = wave >> 1;  // which 64 channels

    const int K = a.K;
    const int rows_x = (int)min((long)kTileT, a.M - tok0);
    const int rows_w = (int)min((long)kTileC, a.N - ch0);
    // a wave whose 64 channels (or 128 tokens) lie wholly past the matrix has nothing to multiply
    const bool wave_live = (wave_c * 64 < rows_w) && (wave_t * 128 < rows_x);

    constexpr int kWDiv = (W_BITS == 8) ? 1 : 2;  // values of K per stored byte
    const v4i rsrc_x = make_rsrc(a.xq + tok0 * K, clamp_u32((a.M - tok0) * (long)K));
    const v4i rsrc_w = make_rsrc((const int8_t*)a.w + ch0 * (K / kWDiv),
                                 clamp_u32((a.N - ch0) * (long)(K / kWDiv)));

    // ---- global -> LDS mapping ---------------------------------------------
    // One direct load fills 1 KiB; lane l writes bytes [16 l, 16 l + 16).
    // int8 tiles: 8 rows x 128 B per load, lane l = row l/8, physical chunk l%8,
    // which under the swizzle holds logical chunk (l%8) ^ ((row/2)%8).  Wave w
    // loads row groups w, w+8, w+16, w+24 of each tile, so row/2 mod 8 is
    // (4 (w%2) + l/16) % 8 for all of them.
    const int ld_row = lane >> 3;
    const int ld_chunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
    int voff_x[4], voff_w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (wave + 8 * j) * 8 + ld_row;
        voff_x[j] = min(r, rows_x - 1) * K + ld_chunk * 16;
        voff_w[j] = min(w_row_to_channel(r), rows_w - 1) * K + ld_chunk * 16;
    }
    if (W_BITS == 4) {
        // packed tile [256 rows][64 B]: 16 rows x 64 B per load, lane l = row l/4,
        // physical chunk l%4 holding logical chunk (l%4) ^ ((row/4)%4) = (l%4) ^ (l/16).
        // Wave w loads row groups w and w+8.
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = (wave + 8 * j) * 16 + (lane >> 2);
            voff_w[j] = min(w_row_to_channel(r), rows_w - 1) * (K / 2) + (((lane & 3) ^ (lane >> 4)) << 4);
        }
    }

    // The loads of a stage are issued in four parts, one per K step of the stage being
    // multiplied, so that no wave sits in a queue of eight loads while the MFMA pipe idles.
    auto issue_part = [&](int st, int k0, int j) {
        load_to_lds_16(rsrc_x, lds_x_addr + st * kXStage + (wave + 8 * j) * 1024, voff_x[j], k0);
        if (W_BITS == 8)
            load_to_lds_16(rsrc_w, lds_w_addr + st * kWStage + (wave + 8 * j) * 1024, voff_w[j], k0);
        else if (j < 2)
            load_to_lds_16(rsrc_w, lds_w_addr + st * kWStage + (wave + 8 * j) * 1024, voff_w[j], k0 / 2);
    };
    auto issue_stage = [&](int st, int k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_part(st, k0, j);
    };

    // ---- LDS -> MFMA operand mapping -----------------------------------------
    // Operand rows of a 32x32x32 block: lane l supplies row l%32, 16 bytes of K
    // chosen by l/32; a stage holds four such K steps (chunks 2ks and 2ks+1).
    const int fr_row = lane & 31;
    int x_off[4], w_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int phys = ((2 * ks + (lane >> 5)) ^ ((fr_row >> 1) & 7)) << 4;
        x_off[ks] = (wave_t * 128 + fr_row) * kTileK + phys;
        if (W_BITS == 8)
            w_off[ks] = (wave_c * 64 + fr_row) * kTileK + phys;
        else  // 8 bytes of nibbles: 16-byte chunk ks (swizzled by (row/4)%4), half l/32
            w_off[ks] = (wave_c * 64 + fr_row) * (kTileK / 2) + ((ks ^ ((fr_row >> 2) & 3)) << 4) +
                        (lane >> 5) * 8;
    }

    v16i acc[2][4];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][tb][r] = 0;

    const int nk = (K + kTileK - 1) / kTileK;

    // Scales and bias of the tile: threads 0..255 fetch one channel and one token each
    // here and park them in LDS after the first stage has been multiplied, so that the
    // epilogue finds them on chip.  Entries past N or M, and a missing bias, are zero.
    float pre_ws = 0.0f, pre_xs = 0.0f;
    _Float16 pre_b = (_Float16)0.0f;
    if (tid < 256) {
        if (ch0 + tid < a.N) {
            pre_ws = a.w_scale[ch0 + tid];
            if (a.bias) pre_b = a.bias[ch0 + tid];
        }
        if (tok0 + tid < a.M) pre_xs = a.x_scale[tok0 + tid];
    }

    issue_stage(0, 0);
    for (int it = 0; it < nk; ++it) {
        const int st = it & 1;
        // Stage `it` has landed for every wave, and every wave is done reading
        // stage it-1, whose buffer the loads issued next overwrite.
        wait_loads_and_barrier();
        const bool more = it + 1 < nk;
        if (it == 1 && tid < 256) {  // (the values were requested a whole stage ago)
            *(float*)(lds_sc + tid * 4) = pre_ws;
            *(_Float16*)(lds_sc + 1024 + tid * 2) = pre_b;
            *(float*)(lds_sc + 2048 + tid * 4) = pre_xs;
        }
        if (!wave_live) {  // nothing to multiply, but this wave's share of the loads is needed
            if (more) issue_stage(st ^ 1, (it + 1) * kTileK);
            continue;
        }

        const int8_t* xs = lds_x + st * kXStage;
        const int8_t* ws = lds_w + st * kWStage;
        // Operand registers are double buffered: the LDS reads of K step ks+1 are
        // issued before the MFMAs of step ks, which cover their latency.
        v4i xf[2][4], wf[2][2];
        auto read_step = [&](int ks, v4i(&xo)[4], v4i(&wo)[2]) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                if (W_BITS == 8)
                    wo[cb] = *(const v4i*)(ws + w_off[ks] + cb * 32 * kTileK);
                else
                    wo[cb] = widen_nibbles(*(const v2i*)(ws + w_off[ks] + cb * 32 * (kTileK / 2)));
            }
#pragma unroll
            for (int tb = 0; tb < 4; ++tb) xo[tb] = *(const v4i*)(xs + x_off[ks] + tb * 32 * kTileK);
            if (K_TAIL && it == nk - 1) {
                // K is a multiple of 16 but not of 128: chunks past K hold bytes of the
                // next row (or nothing); a zero weight operand removes them.
                if (it * kTileK + (2 * ks + (lane >> 5)) * 16 >= K) {
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb) wo[cb] = v4i{0, 0, 0, 0};
                }
            }
        };
        read_step(0, xf[0], wf[0]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) read_step(ks + 1, xf[(ks + 1) & 1], wf[(ks + 1) & 1]);
            if (more) issue_part(st ^ 1, (it + 1) * kTileK, ks);
            // nothing moves across: the reads above stay ahead of the MFMAs below (the
            // scheduler would otherwise sink them next to their uses to save registers)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    acc[cb][tb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks & 1][cb], xf[ks & 1][tb],
                                                                        acc[cb][tb], 0, 0, 0);
        }
    }

    // ---- epilogue ------------------------------------------------------------
    // Lane (h = lane/32, t = lane%32) holds, for each of its 4 token blocks, the
    // 32 channels chl .. chl+31: accumulator block b, register r <-> chl + 16 b + r.
    if (nk == 1 && tid < 256) {
        *(float*)(lds_sc + tid * 4) = pre_ws;
        *(_Float16*)(lds_sc + 1024 + tid * 2) = pre_b;
        *(float*)(lds_sc + 2048 + tid * 4) = pre_xs;
    }
    wait_loads_and_barrier();  // the stage buffers are free: they become the staging area
    if (!wave_live) return;
    const int h = lane >> 5;
    const long chw = ch0 + wave_c * 64;  // first channel of this wave
    const long ch = chw + 32 * h;        // first channel of this lane
    const bool vec = (a.N % 8) == 0;
    // the 4-bit path accumulated 16 * w: fold the exact 1/16 into the channel scale
    const float wmul = (W_BITS == 4) ? 0.0625f : 1.0f;

    float wsc[32];
    half8 bh[4];
    const int8_t* sc_w = lds_sc + (wave_c * 64 + 32 * h) * 4;
    const int8_t* sc_b = lds_sc + 1024 + (wave_c * 64 + 32 * h) * 2;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const v4f sv = *(const v4f*)(sc_w + 16 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) wsc[4 * g + e] = sv[e] * wmul;
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) bh[g] = *(const half8*)(sc_b + 16 * g);

    int8_t* const stage = lds + wave * kEpiWave;  // this wave's 64 tokens x (128 + 16) bytes
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const long tok = tok0 + wave_t * 128 + tb * 32 + (lane & 31);
        const bool tok_ok = tok < a.M;
        const float xsc = *(const float*)(lds_sc + 2048 + (wave_t * 128 + tb * 32 + (lane & 31)) * 4);
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
                const float f = (float)v * xsc;
                out[e] = (_Float16)__builtin_fmaf(f, wsc[8 * g + e], (float)bh[g][e]);
            }
            if (vec) {
                // staged: token row (tb%2)*32 + t, byte column 64 h + 16 g
                *(half8*)(stage + ((tb & 1) * 32 + (lane & 31)) * kEpiRow + 64 * h + 16 * g) = out;
                if (arow && tok_ok && ch + 8 * g < a.N) {
                    *(v4i*)(arow + 8 * g) = v4i{iv[0], iv[1], iv[2], iv[3]};
                    *(v4i*)(arow + 8 * g + 4) = v4i{iv[4], iv[5], iv[6], iv[7]};
                }
            } else if (tok_ok) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (ch + 8 * g + e < a.N) {
                        yrow[8 * g + e] = out[e];
                        if (arow) arow[8 * g + e] = iv[e];
                    }
                }
            }
        }
        if (vec && (tb & 1)) {
            // 64 token rows x 128 B are staged: write them out a full line per 8 lanes.
            // Only this wave touches its staging area; LDS operations of a wave execute
            // in order, the fence only keeps the compiler from reordering them.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = i * 8 + (lane >> 3);
                const half8 v = *(const half8*)(stage + row * kEpiRow + (lane & 7) * 16);
                const long t = tok0 + wave_t * 128 + (tb - 1) * 32 + row;
                const long c = chw + (lane & 7) * 8;
                if (t < a.M && c < a.N) __builtin_nontemporal_store(v, (half8*)(a.y + t * a.N + c));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
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
    const bool tail = (K % kTileK) != 0;
    if (w_bits == 8) {
        if (tail) hipLaunchKernelGGL((gemm_i8_dequant<8, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemm_i8_dequant<8, false>), grid, block, 0, stream, a);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_i8_dequant<4, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemm_i8_dequant<4, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace vq
