// Device helpers shared by the GEMM kernels of this library (vq_gemm.hip: large
// persistent tiles; vq_gemm_small.hip: small tiles for problems that do not fill the
// chip).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vq {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr unsigned kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format

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
    // (base and size are the same for every lane of a wave: saying so keeps the descriptor in
    // scalar registers, where the buffer instructions want it, however it was computed)
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)p);
    r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(p >> 32) & 0xFFFF);
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = (int)kRsrcFlags;
    return r;
}

// (M0 is a reserved register: naming it as clobbered is what tells the compiler that these
// statements change it, and the compiler answers with a warning that says no more than that.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 16 bytes per lane from buffer offset voff + soff straight into LDS at
// lds_addr + 16 * lane (lds_addr is wave-uniform and goes through M0, which the
// statement declares as clobbered).  Counts in vmcnt; the compiler does not know
// about it, see wait_loads_and_barrier().
__device__ __forceinline__ void load_to_lds_16(v4i rsrc, unsigned lds_addr, int voff, int soff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds"
        :
        : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
        : "memory", "m0");
}

// 4 bytes per lane from buffer offset voff + soff into LDS at lds_addr + 4 * lane.
__device__ __forceinline__ void load_to_lds_4(v4i rsrc, unsigned lds_addr, int voff, int soff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dword %1, %2, %3 offen lds"
        :
        : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
        : "memory", "m0");
}

#pragma clang diagnostic pop

// The same for a stage at byte k0 of the rows.  K a multiple of the stage: k0 rides in the scalar
// offset.  Otherwise (the last stage reaches past K) it is added to the per-lane offset, the part
// of the address that the buffer's range check looks at: 16-byte pieces past the end of the last
// row of the buffer then read as zero instead of touching memory behind it.
template <bool K_TAIL>
__device__ __forceinline__ void load_stage_to_lds_16(v4i rsrc, unsigned lds_addr, int voff, int k0) {
    if (K_TAIL)
        load_to_lds_16(rsrc, lds_addr, voff + k0, 0);
    else
        load_to_lds_16(rsrc, lds_addr, voff, k0);
}

// Waits until all of this wave's direct loads (and stores) have completed and all
// its LDS accesses are done, then joins the workgroup barrier.
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" : : : "memory");
}

// The same, but the newest N vector memory operations of this wave may stay in flight
// (they complete in the order of issue: everything older has completed).
template <int N>
__device__ __forceinline__ void wait_loads_before_and_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}

// Barrier for LDS traffic only: loads in flight stay in flight.
__device__ __forceinline__ void wait_lds_and_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory");
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

// The dequantization of two neighbouring outputs into one register of two fp16 values:
//     y = fp16( a * s + float(bias) ),
// the multiply-add exact and rounded once, to nearest even, straight to fp16 (the mixed-precision
// multiply-add takes fp32 a and s and the fp16 bias as they are).  bias2 holds the two bias
// values as they lie in memory (low half first).  Every GEMM kernel of the library narrows
// through these, so that an output does not depend on which kernel computed it.
__device__ __forceinline__ unsigned dequant_pair(float a0, float s0, float a1, float s1, unsigned bias2) {
    unsigned d;
    asm("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,0,1]" : "=v"(d) : "v"(a0), "v"(s0), "v"(bias2));
    asm("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "+v"(d) : "v"(a1), "v"(s1), "v"(bias2));
    return d;
}
// The same without a scale (the fp16 comparison layer): y = fp16( a + float(bias) ), rounded once.
__device__ __forceinline__ unsigned add_bias_pair(float a0, float a1, unsigned bias2) {
    unsigned d;
    asm("v_fma_mixlo_f16 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[0,0,1]" : "=v"(d) : "v"(a0), "v"(bias2));
    asm("v_fma_mixhi_f16 %0, %1, 1.0, %2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "+v"(d) : "v"(a1), "v"(bias2));
    return d;
}

// Returns v unchanged but opaque to the optimiser: what is derived from the result is
// recomputed where it is used instead of being kept in registers across the mainloop.
__device__ __forceinline__ int opaque(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

}  // namespace vq
