// int8 x int8 -> int32 MFMA GEMM with the dequantization epilogue, for gfx950: the kernel
// template.  vq_gemm.hip and vq_gemm_192.hip instantiate it for two workgroup tiles and
// vq_gemm.hip chooses between them.
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
//   - workgroup tile: 256 tokens x (64 WC) output channels, WT x WC wavefronts, each
//     wavefront (32 TB) tokens x 64 channels = 2 x TB MFMA 32x32x32 blocks.  Two tiles:
//       256 x 256: 2 x 4 wavefronts of 128 x 64 (128 int32 accumulators per lane), two
//                  wavefronts per SIMD;
//       256 x 192: 4 x 3 wavefronts of 64 x 64 (64 accumulators), three per SIMD: for
//                  channel counts that 256 does not divide well (1152 = 6 x 192: no
//                  half-empty column of tiles, and 768 tiles of 3/4 of the work fill 256
//                  CUs in three even rounds where 640 tiles of 256 x 256 need three
//                  rounds of whole tiles for 2.25 rounds of work).
//     The tile is large because the L2 -> CU path, not HBM, is what the operand traffic
//     loads: bytes per multiply-add fall with the tile edge.
//   - K is walked in stages of 128 bytes, double buffered in LDS.  A stage
//     takes one full 128-byte cache line per row, so every L2 request is a
//     whole line (with 64-byte stages the same bytes cost twice the requests and the
//     CU's address path saturates).  Activations and weights go global -> LDS directly
//     (buffer_load ... lds, 16 B per lane, no registers in between); the loads
//     of stage i+1 are in flight while stage i is multiplied.  4-bit weights
//     travel packed (half the bytes).
//   - The direct loads are issued from inline assembly and waited for with an
//     explicit s_waitcnt: the compiler would otherwise wait for all of them
//     before every LDS read and undo the prefetch.  They are paced, one load per
//     two MFMAs from the start of a stage: the CU's load path takes 64 bytes
//     per cycle, and a wave that queues there issues no MFMA.
//   - LDS tiles are [row][128 B] with the eight 16-byte chunks of a row XOR-ed
//     by (row/2)%8, which makes the 16-lane groups of a ds_read_b128 hit 16
//     different bank groups.
//   - The weights are the MFMA row operand and the tokens the column operand,
//     so a lane owns one token and, by permuting which weight row sits in
//     which MFMA row, 32 consecutive output channels of it.  The epilogue
//     scales and narrows in registers, turns each wavefront's block
//     through LDS and writes whole 128-byte lines of Y, bypassing the caches'
//     retention (nontemporal): the operands keep the L2.
//   - The kernel is persistent: one workgroup per CU walks a list of tiles.
//     The first stage of the next tile is requested while the last stage of
//     the current one is multiplied, its second stage right behind that stage's
//     barrier, ahead of the epilogue's stores; the epilogue turns its blocks through
//     a small LDS area of its own, so the waves go from it into the next tile without
//     meeting at a barrier.
//   - Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; each
//     XCD gets a contiguous run of tiles, ordered in bands of 8 token tiles,
//     and the workgroups of an XCD take them in turn, so that its L2 sees each
//     operand panel once.
//
// Integer accumulation is exact and order independent, so the result is the
// same whatever the tiling; the 4-bit path multiplies by 16 * w (nibble left in
// the high half of the byte) and divides the sum by 16 exactly afterwards.
//
// The epilogue computes fp16_rne(float(acc) * fp32(x_scale * w_scale) + bias): the product of
// the two scales is rounded to fp32, the multiply-add is exact and rounded once, to fp16
// (two vector instructions per output instead of four).  An output can differ from the
// value of three separately rounded fp32 operations in the last fp16 place.
//
// W_BITS == 16 instantiates the same kernel for fp16 operands and fp32 sums
// (v_mfma_f32_32x32x16_f16, the same 16 bytes of K per lane and operand): the FP16 layer
// the paper's hardware evaluation compares against (Sec. 5.3), y = fp16(sum + bias).
#pragma once
#include <type_traits>

#include "vq_gemm_common.h"
#include "vq_internal.h"

namespace vq {

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
    int slots;  // workgroups per XCD; workgroup (xcd, slot) takes tiles slot, slot + slots, ... of its XCD
};

// The 256 x 192 tile (vq_gemm_192.hip); the tile fields of `a` are filled in by the callee.
hipError_t launch_gemm_192(const GemmArgs& a, int w_bits, int num_cus, hipStream_t stream);

namespace {

constexpr int kTileK = 128;                 // K bytes per stage (one cache line per row)
constexpr int kStages = 2;
constexpr int kScaleBytes = 3 * 1024;       // w_scale[256] fp32 | bias[256] fp16 (+pad) | x_scale[256] fp32
constexpr int kBand = 8;                    // token tiles per band in the tile order
constexpr int kXcds = 8;
constexpr int kTouchRounds = 4;             // weight lines asked for up front: at most 4 x 8 KiB per wave (64 MiB per 256 CUs)

// WT x WC wavefronts of (32 TB) tokens x 64 channels.
template <int WT_, int WC_, int TB_>
struct TileShape {
    static constexpr int WT = WT_, WC = WC_, TB = TB_;
    static constexpr int kWaves = WT * WC;
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kWavesPerSimd = kWaves / 4;
    static constexpr int kTileT = WT * TB * 32;       // tokens per workgroup
    static constexpr int kTileC = WC * 64;            // output channels per workgroup
    static constexpr int kXStage = kTileT * kTileK;   // 32 KiB
    static constexpr int kWStage = kTileC * kTileK;   // (half of it used by packed 4-bit weights)
    static constexpr int kLdsBytes = kStages * (kXStage + kWStage);
    // Global -> LDS loads of 1 KiB (8 rows of int8, 16 rows of nibbles).  The X tile is 32 of them,
    // four for each of the first eight waves.  With eight waves every wave also takes its share
    // of the W tile; with twelve, waves 8..11 load the W tile and nothing else.
    static constexpr bool kSplitRoles = kWaves > 8;
    static constexpr int kWLoaders = kSplitRoles ? kWaves - 8 : 8;
    static constexpr int kWPer8 = kTileC / 8 / kWLoaders;    // int8 (and fp16) W loads per loading wave
    static constexpr int kWPer4 = kTileC / 16 / kWLoaders;   // packed 4-bit W loads per loading wave
    // Epilogue: every wave has a staging area of its own behind the stage buffers, 16 token
    // rows x 128 B, through which half a block of 32 tokens x 64 channels of fp16 is turned at
    // a time.  (The stage buffers themselves are busy: the next tile's first two stages land
    // there while the epilogue runs.)
    static constexpr int kEpiRows = 16;
    static constexpr int kEpiWave = kEpiRows * 128;
    static constexpr int kEpiBytes = kWaves * kEpiWave;
    static constexpr int kStoresPerTile = TB * 4;            // 128-bit stores of a wave's epilogue
    static_assert(kTileT == 256, "scales are fetched by threads 0..255, one token each");
    static_assert(kTileC <= 256 && kWaves % 4 == 0 && kWaves >= 8, "tile shape");
    static_assert(kTileC / 8 % kWLoaders == 0 && kTileC / 16 % kWLoaders == 0, "W loads divide evenly");
    static_assert(kLdsBytes + kScaleBytes + kEpiBytes <= 160 * 1024, "LDS of one CU");
};

// Where a tile sits in the output (wave-uniform).
struct TilePos {
    long tok0, ch0;
    int rows_x, rows_w;  // rows of the tile that exist (the rest is clamped on load, masked on store)
};
// What this wave's share of a tile's loads needs: buffer descriptors and per-lane offsets.
struct TileLoads {
    v4i rsrc_x, rsrc_w;
    int voff_x[4], voff_w[6];
};

// One 32 x 32 block: int8 operands (32 values of K per lane pair) into int32 sums, or,
// for the fp16 comparison layer, fp16 operands (16 values of K) into fp32 sums.  Both take
// 16 bytes of each operand per lane and as long to issue.
typedef float v16f __attribute__((ext_vector_type(16)));
template <int W_BITS>
struct AccOf { typedef v16i type; };
template <>
struct AccOf<16> { typedef v16f type; };
__device__ __forceinline__ v16i mfma_block(v4i w, v4i x, v16i c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, c, 0, 0, 0);
}
__device__ __forceinline__ v16f mfma_block(v4i w, v4i x, v16f c) {
    // (a cast between vector types of one size reinterprets the bits)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16((half8)w, (half8)x, c, 0, 0, 0);
}

// K_TAIL:  K is a multiple of 16 but not of 128 (the last stage is partly past K).
// GENERIC: any N and an optional copy of the integer sums; stores go out element by
//          element.  The fast variant needs N % 8 == 0 and writes whole lines.
template <class S, int W_BITS, bool K_TAIL, bool GENERIC>
__global__ __launch_bounds__(S::kThreads, S::kWavesPerSimd) void gemm_i8_dequant(const GemmArgs a) {
    constexpr int TB = S::TB;
    constexpr int kXStage = S::kXStage, kWStage = S::kWStage, kLdsBytes = S::kLdsBytes;
    __shared__ __attribute__((aligned(1024))) int8_t lds[kLdsBytes + kScaleBytes + S::kEpiBytes];
    // layout: [X buffer 0][X buffer 1][W buffer 0][W buffer 1][scales][epilogue staging]; a W
    // buffer is [rows][128 B] of int8 or, for 4-bit weights, [rows][64 B] of nibbles.
    int8_t* const lds_x = lds;
    int8_t* const lds_w = lds + kStages * kXStage;
    const unsigned lds_x_addr = (unsigned)(uintptr_t)(lds_ptr)lds_x;
    const unsigned lds_w_addr = (unsigned)(uintptr_t)(lds_ptr)lds_w;
    int8_t* const lds_sc = lds + kLdsBytes;  // w_scale | bias | x_scale of the current tile

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Waves w, w+4 (and w+8) share a SIMD: they get the same token part and different
    // channel slabs, so a tile that is only partly full of channels still
    // leaves a working wave on every SIMD.
    const int wave_t = wave % S::WT;   // which 32 TB tokens
    const int wave_c = wave / S::WT;   // which 64 channels
    // (W_BITS == 16: fp16 operands, the comparison layer; rows are 2 K bytes and everything up
    // to the MFMA itself treats them like int8 rows of that many bytes)
    const int K = (W_BITS == 16) ? 2 * a.K : a.K;      // bytes per activation row
    constexpr int kWDiv = (W_BITS == 4) ? 2 : 1;        // activation bytes per weight byte
    const int nk = (K + kTileK - 1) / kTileK;

    // What this wave loads per stage.
    constexpr int kWPer = (W_BITS != 4) ? S::kWPer8 : S::kWPer4;
    const bool loads_x = !S::kSplitRoles || wave < 8;
    const bool loads_w = !S::kSplitRoles || wave >= 8;
    const int w_loader = S::kSplitRoles ? wave - 8 : wave;
    const int n_singles = S::kSplitRoles ? (wave < 8 ? 4 : kWPer) : 4 + kWPer;

    // ---- global -> LDS mapping ---------------------------------------------
    // One direct load fills 1 KiB; lane l writes bytes [16 l, 16 l + 16).
    // int8 tiles: 8 rows x 128 B per load, lane l = row l/8, physical chunk l%8,
    // which under the swizzle holds logical chunk (l%8) ^ ((row/2)%8).  A wave's row
    // groups g all have the parity of the wave's number, so row/2 mod 8 is
    // (4 (g%2) + l/16) % 8 for all of them.
    // Packed 4-bit tile [rows][64 B]: 16 rows x 64 B per load, lane l = row l/4,
    // physical chunk l%4 holding logical chunk (l%4) ^ ((row/4)%4) = (l%4) ^ (l/16).
    // The tiles of an XCD are numbered band by band (kBand token tiles), column by column
    // within a band, token tile by token tile within a column.  A workgroup's tiles lie
    // a.slots apart: the first one is located by division, the later ones by stepping.
    const int band_tiles = kBand * a.tiles_c;
    int dec_band, dec_in_band;   // where the tile decoded last sits (wave-uniform)
    bool ld_full = false;        // that tile was a full one: its per-lane offsets hold for any full tile
    auto locate_tile = [&](int idx) {
        const int logical = (blockIdx.x % kXcds) * a.tiles_per_xcd + idx;
        dec_band = logical / band_tiles;
        dec_in_band = logical - dec_band * band_tiles;
    };
    auto step_tile = [&]() {
        dec_in_band += a.slots;
        while (dec_in_band >= band_tiles) {
            dec_in_band -= band_tiles;
            ++dec_band;
        }
    };
    auto decode_tile = [&](TilePos& t, TileLoads& ld) {
        const int band_first = dec_band * kBand;
        const int band_rows = min(a.tiles_t - band_first, kBand);
        int row, col;
        if (band_rows == kBand) {
            row = dec_in_band % kBand;
            col = dec_in_band / kBand;
        } else {  // the last band of a matrix whose token tiles are not a multiple of kBand
            row = dec_in_band % band_rows;
            col = dec_in_band / band_rows;
        }
        t.tok0 = (long)(band_first + row) * S::kTileT;
        t.ch0 = (long)col * S::kTileC;
        t.rows_x = (int)min((long)S::kTileT, a.M - t.tok0);
        t.rows_w = (int)min((long)S::kTileC, a.N - t.ch0);
        ld.rsrc_x = make_rsrc(a.xq + t.tok0 * K, clamp_u32((a.M - t.tok0) * (long)K));
        ld.rsrc_w = make_rsrc((const int8_t*)a.w + t.ch0 * (K / kWDiv),
                              clamp_u32((a.N - t.ch0) * (long)(K / kWDiv)));
        // The per-lane offsets are relative to the tile and clamp rows past the matrix: between
        // two full tiles they do not change.  (Rows < 256 and row lengths < 2^24: 24-bit products.)
        const bool full = t.rows_x == S::kTileT && t.rows_w == S::kTileC;
        if (full && ld_full) return;
        ld_full = full;
        const int l = opaque(lane);
        if (loads_x) {
            const int ld_chunk16 = ((l & 7) ^ ((4 * (wave & 1) + (l >> 4)) & 7)) << 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = (wave + 8 * j) * 8 + (l >> 3);
                ld.voff_x[j] = __mul24(min(r, t.rows_x - 1), K) + ld_chunk16;
            }
        }
        if (loads_w) {
            const int ld_chunk16 = ((l & 7) ^ ((4 * (w_loader & 1) + (l >> 4)) & 7)) << 4;
            const int ld_chunk16_w4 = ((l & 3) ^ (l >> 4)) << 4;
#pragma unroll
            for (int j = 0; j < kWPer; ++j) {
                const int g = w_loader + S::kWLoaders * j;   // row group of this load
                if (W_BITS != 4)
                    ld.voff_w[j] = __mul24(min(w_row_to_channel(g * 8 + (l >> 3)), t.rows_w - 1), K) + ld_chunk16;
                else
                    ld.voff_w[j] = __mul24(min(w_row_to_channel(g * 16 + (l >> 2)), t.rows_w - 1), K / 2) + ld_chunk16_w4;
            }
        }
    };
    auto tile_exists = [&](int idx) {
        return idx < a.tiles_per_xcd && (int)(blockIdx.x % kXcds) * a.tiles_per_xcd + idx < a.tiles;
    };

    // One load of a wave's share of a stage.  A wave with both kinds alternates them (X, W, X,
    // W, ...) as long as it has W loads left.
    auto issue_x = [&](const TileLoads& ld, int buf, int k0, int j) {
        load_stage_to_lds_16<K_TAIL>(ld.rsrc_x, lds_x_addr + buf * kXStage + (wave + 8 * j) * 1024, ld.voff_x[j], k0);
    };
    auto issue_w = [&](const TileLoads& ld, int buf, int k0, int j) {
        load_stage_to_lds_16<K_TAIL>(ld.rsrc_w, lds_w_addr + buf * kWStage + (w_loader + S::kWLoaders * j) * 1024,
                                     ld.voff_w[j], W_BITS != 4 ? k0 : k0 / 2);
    };
    auto issue_single = [&](const TileLoads& ld, int buf, int k0, int s) {
        if (S::kSplitRoles) {
            // (s is a compile-time constant at every call; the role is wave-uniform)
            if (wave < 8) { if (s < 4) issue_x(ld, buf, k0, s); }
            else          { if (s < kWPer) issue_w(ld, buf, k0, s); }
        } else if (s < 2 * kWPer) {
            if (s & 1) issue_w(ld, buf, k0, s >> 1); else issue_x(ld, buf, k0, s >> 1);
        } else {
            issue_x(ld, buf, k0, s - kWPer);
        }
    };
    constexpr int kMaxSingles = S::kSplitRoles ? (kWPer > 4 ? kWPer : 4) : 4 + kWPer;
    auto issue_all = [&](const TileLoads& ld, int buf, int k0) {
#pragma unroll
        for (int s = 0; s < kMaxSingles; ++s)
            if (s < n_singles) issue_single(ld, buf, k0, s);
    };

    // ---- LDS -> MFMA operand mapping -----------------------------------------
    // Operand rows of a 32x32x32 block: lane l supplies row l%32, 16 bytes of K
    // chosen by l/32; a stage holds four such K steps (chunks 2ks and 2ks+1).
    // The chunk index of K step ks is (2 ks + l/32) ^ swizzle = ((l/32) ^ swizzle) ^ 2 ks, so the
    // byte offset of step ks is that of step 0 with 32 ks XOR-ed in.
    const int fr_row = lane & 31;
    const int x_off0 = (wave_t * 32 * TB + fr_row) * kTileK + (((lane >> 5) ^ ((fr_row >> 1) & 7)) << 4);
    const int w_off0 = (W_BITS != 4)
                           ? (wave_c * 64 + fr_row) * kTileK + (((lane >> 5) ^ ((fr_row >> 1) & 7)) << 4)
                           // 8 bytes of nibbles: 16-byte chunk ks (swizzled by (row/4)%4), half l/32
                           : (wave_c * 64 + fr_row) * (kTileK / 2) + (((fr_row >> 2) & 3) << 4) + (lane >> 5) * 8;
    auto x_off = [&](int ks) { return x_off0 ^ (ks << 5); };
    auto w_off = [&](int ks) { return w_off0 ^ (ks << (W_BITS != 4 ? 5 : 4)); };

    // ---- the tiles of this workgroup -------------------------------------------
    int idx = blockIdx.x / kXcds;
    if (!tile_exists(idx)) return;  // uniform per workgroup
    TilePos cur;   // the tile being multiplied
    TileLoads ld;  // the tile whose stages are being requested (the next one during the last stage)
    locate_tile(idx);
    decode_tile(cur, ld);
    int buf = 0;  // LDS buffer of the stage about to be multiplied
    bool requested1 = false;        // the current tile's second stage was requested before the previous epilogue
    bool stores_in_flight = false;  // this wave wrote outputs in the previous epilogue (kStoresPerTile stores)
    issue_all(ld, 0, 0);
    // Every line of the weight matrix is asked for once, here, by the whole grid (one dword per
    // 128-byte line and lane, 8 KiB per wave and round): the weights are a few MB that every XCD
    // walks through completely, and a column's panel is otherwise first asked for by the eight
    // CUs that need it at that moment, which then wait out the memory latency at every stage of
    // their tile.  Fetched up front the lines are in the memory-side cache when their column's
    // turn comes.  (Range-checked loads: lanes past the end of the matrix fetch nothing.)
    int touched[kTouchRounds];
    {
        const long w_bytes = (long)a.N * (K / kWDiv);
        const __amdgpu_buffer_rsrc_t rsrc_all = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<void*>(a.w), 0, (int)clamp_u32(w_bytes), kRsrcFlags);
        const unsigned per_round = gridDim.x * (unsigned)S::kWaves * 8192u;
        const unsigned off = (blockIdx.x * (unsigned)S::kWaves + (unsigned)wave) * 8192u + (unsigned)lane * 128u;
#pragma unroll
        for (int i = 0; i < kTouchRounds; ++i) {
            touched[i] = 0;
            if ((long)i * per_round < w_bytes)  // (uniform; all rounds are in flight together)
                touched[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_all, (int)(off + i * per_round), 0, 0);
        }
    }
    wait_loads_and_barrier();  // the first tile's first stage (later ones arrive behind an epilogue)
#pragma unroll
    for (int i = 0; i < kTouchRounds; ++i) asm volatile("" : : "v"(touched[i]));  // (not used; they have arrived by now)

    // Invariant at the top of a stage: its operands have landed in buffer `buf` for every
    // wave, and nobody reads or writes the other buffer any more.
    while (true) {
        const int next_idx = idx + a.slots;
        const bool has_next = tile_exists(next_idx);
        TilePos nxt = cur;

        // a wave whose 64 channels (or tokens) lie wholly past the matrix has nothing to multiply
        const bool wave_live = (wave_c * 64 < cur.rows_w) && (wave_t * 32 * TB < cur.rows_x);

        // Scales and bias of the tile: threads 0..255 fetch one channel and one token each
        // here and park them in LDS behind the last stage, where every lane of the epilogue
        // finds them.  Entries past N or M, and a missing bias, are zero.
        float pre_ws = 0.0f, pre_xs = 0.0f;
        _Float16 pre_b = (_Float16)0.0f;
        if (wave < 4) {
            const int i = wave * 64 + opaque(lane);
            if (i < S::kTileC && cur.ch0 + i < a.N) {
                if (W_BITS != 16) pre_ws = a.w_scale[cur.ch0 + i];
                if (a.bias) pre_b = a.bias[cur.ch0 + i];
            }
            if (W_BITS != 16 && cur.tok0 + i < a.M) pre_xs = a.x_scale[cur.tok0 + i];
        }

        auto park_scales = [&]() {
            if (wave < 4) {
                const int i = wave * 64 + opaque(lane);
                *(float*)(lds_sc + i * 4) = pre_ws;
                *(_Float16*)(lds_sc + 1024 + i * 2) = pre_b;
                *(float*)(lds_sc + 2048 + i * 4) = pre_xs;
            }
        };

        typedef typename AccOf<W_BITS>::type acc_t;
        acc_t acc[2][TB];
        v4i xf[2][TB], wf[2][2];  // operand registers, double buffered; [1] carries K step 3 across stages
        const acc_t kZero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

        // One stage = four K steps of 2 TB MFMAs per wave.  The schedule is skewed by one K step:
        // the MFMAs of a stage's last K step are issued at the start of the next stage, behind
        // the barrier, where they cover the latency of that stage's first LDS reads (otherwise
        // every wave of the CU would sit idle there).  Compile-time flags: FIRST = the tile's
        // first stage (nothing deferred to run; its first K step starts the accumulators from
        // a constant zero), LAST = its last one (nothing is deferred past the epilogue).
        // `requested`: the loads this stage would issue are already in flight.
        auto stage = [&](const int it, auto first_tag, auto last_tag, const bool requested) __attribute__((always_inline)) {
            constexpr bool FIRST = decltype(first_tag)::value;
            constexpr bool LAST = decltype(last_tag)::value;
            // what to request while this stage is multiplied: the next stage of this tile,
            // or the first stage of the next tile
            const bool more = it + 1 < nk;
            const bool fetch = (more || has_next) && !requested;
            if (!more && has_next) {
                step_tile();
                decode_tile(nxt, ld);
            }
            const int fk0 = more ? (it + 1) * kTileK : 0;

            const int8_t* xs = lds_x + buf * kXStage;
            const int8_t* ws = lds_w + buf * kWStage;
            // Operand registers are double buffered: the LDS reads of K step ks+1 are issued
            // among the MFMAs of step ks, which cover their latency.
            // A K step = 2 TB MFMAs in TB pieces of two.  A piece carries at most one global load
            // (so that a wave never sits in the load queue while the matrix pipe waits for it)
            // and its share of the LDS reads of the step after; sched_barrier(0) keeps the pieces
            // apart.  Reads of the next step in the order of their first use: w0 x0 x1 .. w1
            // (128-token waves: w0 x0 | x1 x2 | x3 w1; 64-token waves: w0 x0 x1 w1 in the first piece).
            constexpr int kReads = TB + 2;
            constexpr int kReadsPerPiece = (kReads + TB - 2) / (TB - 1);   // spread over all pieces but the last
            auto read_one = [&](int ks, int r, v4i(&xo)[TB], v4i(&wo)[2]) __attribute__((always_inline)) {
                const bool past_k = K_TAIL && it == nk - 1 && it * kTileK + (2 * ks + (lane >> 5)) * 16 >= K;
                if (r == 0 || r == kReads - 1) {
                    const int cb = (r == 0) ? 0 : 1;
                    if (W_BITS != 4)
                        wo[cb] = *(const v4i*)(ws + w_off(ks) + cb * 32 * kTileK);
                    else
                        wo[cb] = widen_nibbles(*(const v2i*)(ws + w_off(ks) + cb * 32 * (kTileK / 2)));
                    // K is a multiple of 16 but not of 128: chunks past K hold bytes of the next
                    // row (or nothing); a zero weight operand removes them.
                    if (past_k) wo[cb] = v4i{0, 0, 0, 0};
                } else {
                    const int tb = r - 1;
                    xo[tb] = *(const v4i*)(xs + x_off(ks) + tb * 32 * kTileK);
                }
            };
            auto mfma_one = [&](int i, const v4i(&xi)[TB], const v4i(&wi)[2], auto zero_tag) __attribute__((always_inline)) {
                const int cb = i / TB, tb = i % TB;
                if constexpr (decltype(zero_tag)::value)
                    acc[cb][tb] = mfma_block(wi[cb], xi[tb], kZero16);
                else
                    acc[cb][tb] = mfma_block(wi[cb], xi[tb], acc[cb][tb]);
            };
            // read_ks < 0: nothing left to read (the tile's last K step); first_load < 0: no loads
            auto k_step = [&](const v4i(&xi)[TB], const v4i(&wi)[2], auto zero_tag, int read_ks, v4i(&xo)[TB],
                              v4i(&wo)[2], int first_load) __attribute__((always_inline)) {
#pragma unroll
                for (int p = 0; p < TB; ++p) {
                    if (fetch && first_load >= 0 && first_load + p < kMaxSingles && first_load + p < n_singles)
                        issue_single(ld, buf ^ 1, fk0, first_load + p);
                    mfma_one(2 * p, xi, wi, zero_tag);
                    mfma_one(2 * p + 1, xi, wi, zero_tag);
                    if (read_ks >= 0) {
#pragma unroll
                        for (int r = p * kReadsPerPiece; r < (p + 1) * kReadsPerPiece && r < kReads; ++r)
                            read_one(read_ks, r, xo, wo);
                        if (W_BITS != 4 && p * kReadsPerPiece < kReads) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   // one MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerPiece / 2, 0);  // LDS reads
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x100, kReadsPerPiece / 2, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            constexpr std::false_type kAccumulate{};
            // K steps in the order they are issued; the e-th one of a stage carries the loads
            // e TB .. e TB + TB - 1 of this wave's share.
            if (FIRST) {
                // nothing deferred to cover them: the first K step's operands are read up front
#pragma unroll
                for (int r = 0; r < kReads; ++r) read_one(0, r, xf[0], wf[0]);
                __builtin_amdgcn_sched_barrier(0);
                k_step(xf[0], wf[0], first_tag, 1, xf[1], wf[1], 0);          // K step 0
                k_step(xf[1], wf[1], kAccumulate, 2, xf[0], wf[0], TB);      // K step 1
                k_step(xf[0], wf[0], kAccumulate, 3, xf[1], wf[1], 2 * TB);  // K step 2
            } else {
                k_step(xf[1], wf[1], kAccumulate, 0, xf[0], wf[0], 0);       // K step 3 of the previous stage
                k_step(xf[0], wf[0], kAccumulate, 1, xf[1], wf[1], TB);      // K step 0
                k_step(xf[1], wf[1], kAccumulate, 2, xf[0], wf[0], 2 * TB);  // K step 1
                k_step(xf[0], wf[0], kAccumulate, 3, xf[1], wf[1], 3 * TB);  // K step 2
            }
            // K step 3 (otherwise at the start of the next stage)
            if (LAST) k_step(xf[1], wf[1], kAccumulate, -1, xf[0], wf[0], -1);
            if (!more) park_scales();
            // The stage requested above has landed for every wave and every wave is done
            // reading this one.  After the last stage this also says: the scales are in LDS,
            // the next tile's first stage is in, and only stores can be outstanding later.
            // (A stage whose loads were requested before the previous tile's epilogue has this
            // wave's stores of that epilogue behind them, and nothing else: the stores may stay
            // in flight.  Vector memory operations complete in the order they were issued.)
            if (requested && stores_in_flight)
                wait_loads_before_and_barrier<S::kStoresPerTile>();
            else
                wait_loads_and_barrier();
            buf ^= 1;
        };
        constexpr std::true_type kYes{};
        constexpr std::false_type kNo{};
        if (!wave_live) {
            // nothing to multiply in this tile, but this wave's share of the loads is needed
#pragma unroll 1
            for (int it = 0; it < nk; ++it) {
                const bool more = it + 1 < nk;
                if (!more && has_next) {
                    step_tile();
                    decode_tile(nxt, ld);
                }
                if ((more || has_next) && !(it == 0 && requested1)) issue_all(ld, buf ^ 1, more ? (it + 1) * kTileK : 0);
                if (!more) park_scales();
                wait_loads_and_barrier();
                buf ^= 1;
            }
        } else if (nk == 1) {
            stage(0, kYes, kYes, false);
        } else {
            stage(0, kYes, kNo, requested1);
#pragma unroll 1
            for (int it = 1; it < nk - 1; ++it) stage(it, kNo, kNo, false);
            stage(nk - 1, kNo, kYes, false);
        }
        // `buf` now names the buffer that holds the next tile's first stage and the other one
        // is free: the next tile's second stage is requested into it here, ahead of the
        // epilogue's stores, so that it arrives while the epilogue computes.
        requested1 = has_next && nk >= 2;
        if (requested1) issue_all(ld, buf ^ 1, kTileK);
        stores_in_flight = false;

        // ---- epilogue ------------------------------------------------------------
        // Lane (h = lane/32, t = lane%32) holds, for each of its TB token blocks, the
        // 32 channels chl .. chl+31: accumulator block b, register r <-> chl + 16 b + r.
        if (wave_live) {
            stores_in_flight = !GENERIC;
            const int el = opaque(lane);  // (the epilogue's per-lane values are not kept across the mainloop)
            const int h = el >> 5;
            const long chw = cur.ch0 + wave_c * 64;  // first channel of this wave
            // the 4-bit path accumulated 16 * w: the exact 1/16 rides on the token scale
            const float xmul = (W_BITS == 4) ? 0.0625f : 1.0f;
            // channel scales are read from LDS where they are used (32 registers fewer across
            // the epilogue); the bias is kept as it is stored, two fp16 values to a register
            const int8_t* sc_w = lds_sc + (wave_c * 64 + 32 * h) * 4;
            const int8_t* sc_b = lds_sc + 1024 + (wave_c * 64 + 32 * h) * 2;
            v4i bias2[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) bias2[g] = *(const v4i*)(sc_b + 16 * g);

            // staging: [16 token rows][128 B] of this wave, 16-byte chunks XOR-ed by (row/2)%8
            // (byte offsets into `lds`; the area is 1 KiB aligned, so the XORs below stay inside
            // the chunk bits)
            const int stg = kLdsBytes + kScaleBytes + wave * S::kEpiWave;
            // writes: this lane's token row (el%16 of its half block), logical chunk 4h+g
            const int st_wr = stg + (el & 15) * 128 + ((4 * h ^ ((el >> 1) & 7)) << 4);
            // flush reads: row 8i + el/8, logical chunk el%8 (its XOR mask alternates with i)
            const int st_rd = stg + (el >> 3) * 128 + (((el & 7) ^ (el >> 4)) << 4);
            // Flush stores are range-checked buffer stores relative to the tile's first token
            // row: rows past M fall behind the end of the buffer, lanes whose channels lie past
            // N get an offset behind it (N < 2^21 on this path, so nothing wraps).
            const int cl = (int)chw + (el & 7) * 8;
            const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(
                a.y + cur.tok0 * a.N, 0, (int)clamp_u32((long)cur.rows_x * a.N * 2), kRsrcFlags);
            const unsigned y_off0 =
                (cl < a.N) ? (unsigned)(((wave_t * 32 * TB + (el >> 3)) * a.N + cl) * 2) : 0x80000000u;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int tl = wave_t * 32 * TB + tb * 32 + (el & 31);  // token within the tile
                const float xsc = *(const float*)(lds_sc + 2048 + tl * 4) * xmul;
                v4i out[4];  // eight fp16 outputs each
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int b = g >> 1, r0 = (g & 1) * 8;
                    // y = fp16(float(acc) * (x_scale * w_scale) + bias): the product of the two
                    // scales rounded to fp32, the rest exact and rounded once (dequant_pair)
                    float sp[8];
                    if (W_BITS != 16) {
                        const v4f s0 = *(const v4f*)(sc_w + 32 * g), s1 = *(const v4f*)(sc_w + 32 * g + 16);
#pragma unroll
                        for (int e = 0; e < 4; ++e) sp[e] = xsc * s0[e], sp[4 + e] = xsc * s1[e];
                    }
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        if (W_BITS == 16)  // the fp32 sum of the fp16 products, plus the bias
                            out[g][e / 2] = (int)add_bias_pair((float)acc[b][tb][r0 + e], (float)acc[b][tb][r0 + e + 1],
                                                               (unsigned)bias2[g][e / 2]);
                        else
                            out[g][e / 2] = (int)dequant_pair((float)acc[b][tb][r0 + e], sp[e], (float)acc[b][tb][r0 + e + 1],
                                                              sp[e + 1], (unsigned)bias2[g][e / 2]);
                    }
                    if (GENERIC && tl < cur.rows_x) {
                        const long tok = cur.tok0 + tl;
                        const long c0 = chw + 32 * h + 8 * g;
                        const half8 oh = (half8)out[g];  // (reinterprets the bits)
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            if (c0 + e < a.N) {
                                a.y[tok * a.N + c0 + e] = oh[e];
                                if (a.acc_out) {
                                    const int v = (int)acc[b][tb][r0 + e];
                                    a.acc_out[tok * a.N + c0 + e] = (W_BITS == 4) ? (v >> 4) : v;
                                }
                            }
                        }
                    }
                }
                if (!GENERIC) {
                    // The block goes out in two halves of 16 token rows: the lanes that hold them
                    // stage their 64 bytes each, then the wave writes the 16 rows x 128 B out, a
                    // full line per 8 lanes.  Only this wave touches its staging area and the LDS
                    // operations of a wave execute in order; the fences only keep the compiler
                    // from reordering them.
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        if (((el >> 4) & 1) == p) {
#pragma unroll
                            for (int g = 0; g < 4; ++g) *(v4i*)(lds + (st_wr ^ (g << 4))) = out[g];
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        v4i rows[2];
#pragma unroll
                        for (int i = 0; i < 2; ++i) rows[i] = *(const v4i*)(lds + (st_rd ^ (i << 6)) + i * 1024);
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            __builtin_amdgcn_raw_buffer_store_b128(
                                rows[i], rsrc_y, y_off0 + (unsigned)((tb * 32 + p * 16 + i * 8) * a.N * 2), 0,
                                2 /* nontemporal */);
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
                }
            }
        }
        if (!has_next) break;
        // A one-stage tile parks its scales before its only barrier: nobody may still be
        // reading this tile's.  (Otherwise the waves go on without meeting: every wave stages
        // in an area of its own, and a barrier of the next tile's first stage comes before its
        // scales are parked.)
        if (nk == 1) wait_lds_and_barrier();
        cur = nxt;
        idx = next_idx;
    }
}

// Enqueues the kernel for tile shape S; `a` holds the operands and sizes.
template <class S>
hipError_t launch_gemm_shape(GemmArgs a, int w_bits, int num_cus, hipStream_t stream) {
    a.tiles_t = (a.M + S::kTileT - 1) / S::kTileT;
    a.tiles_c = (a.N + S::kTileC - 1) / S::kTileC;
    const long tiles = (long)a.tiles_t * a.tiles_c;
    if (tiles > 0x7FFFFFF0l) return hipErrorInvalidValue;
    a.tiles = (int)tiles;
    a.tiles_per_xcd = (a.tiles + kXcds - 1) / kXcds;
    // one workgroup per CU (the kernel needs most of a CU's LDS), fewer if there are fewer tiles
    const int cus_per_xcd = num_cus >= kXcds ? num_cus / kXcds : 1;
    a.slots = a.tiles_per_xcd < cus_per_xcd ? a.tiles_per_xcd : cus_per_xcd;
    const dim3 grid((unsigned)(a.slots * kXcds)), block(S::kThreads);
    const bool tail = ((w_bits == 16 ? 2 * a.K : a.K) % kTileK) != 0;  // (in bytes of an activation row)
    const bool generic = (a.N % 8) != 0 || a.acc_out != nullptr || a.N >= (1 << 21);
#define VQ_LAUNCH_GEMM(BITS, TAIL, GEN) \
    hipLaunchKernelGGL((gemm_i8_dequant<S, BITS, TAIL, GEN>), grid, block, 0, stream, a)
    if (w_bits == 8) {
        if (tail) { if (generic) VQ_LAUNCH_GEMM(8, true, true); else VQ_LAUNCH_GEMM(8, true, false); }
        else      { if (generic) VQ_LAUNCH_GEMM(8, false, true); else VQ_LAUNCH_GEMM(8, false, false); }
    } else if (w_bits == 16) {
        if (tail) { if (generic) VQ_LAUNCH_GEMM(16, true, true); else VQ_LAUNCH_GEMM(16, true, false); }
        else      { if (generic) VQ_LAUNCH_GEMM(16, false, true); else VQ_LAUNCH_GEMM(16, false, false); }
    } else {
        if (tail) { if (generic) VQ_LAUNCH_GEMM(4, true, true); else VQ_LAUNCH_GEMM(4, true, false); }
        else      { if (generic) VQ_LAUNCH_GEMM(4, false, true); else VQ_LAUNCH_GEMM(4, false, false); }
    }
#undef VQ_LAUNCH_GEMM
    return hipGetLastError();
}

}  // namespace
}  // namespace vq
