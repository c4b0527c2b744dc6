// LDS-DMA primitives and fragment types shared by the pipelined tile kernels (gemm_v2.hip, gemm_wgrad.hip).
//
// Register layouts of the two matrix instructions used there (measured on gfx950 with one-hot operands):
//   v_smfmac_f32_32x32x32_bf16  A: lane l -> row l%32, survivors 8*(l/32)..+7 of the 16 (k in 16*(l/32)..+15),
//                                  index VGPR bits [2e+1:2e] = position of survivor e inside its group of 4
//                                  (ABID 0: bits 15:0 of the VGPR, ABID 1: bits 31:16);
//                               B: lane l -> column l%32; elements 0-7 = k 8*(l/32)..+7, elements 8-15 = k 16+8*(l/32)..+7;
//                               D: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//   v_mfma_f32_32x32x16_bf16    A, B: lane l -> row / column l%32, k 8*(l/32)..+7;  D as above.
//   v_smfmac_f32_32x32x64_fp8_fp8  A: lane l -> row l%32, the 16 survivors (one byte each) of k in 32*(l/32)..+31, index VGPR bits
//                                  [2e+1:2e] = position of survivor e inside its group of 4 (all 32 bits are used, no ABID);
//                               B: lane l -> column l%32; bytes 0-15 = k 16*(l/32)..+15, bytes 16-31 = k 32+16*(l/32)..+15;  D as above.
//                               (byte for byte the bf16 instruction's operand layout with twice the k per byte)
// The 2-bit positions are exactly the packed format's metadata nibbles, so metadata goes from HBM to the index
// VGPR without re-encoding.
#pragma once
#include "common.hpp"

namespace sffn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
union Frag8 { uint4 u; bf16x8 v; i32x4 q; };            // q: the same 16 bytes as 16 fp8 codes
union Frag16 { uint4 u[2]; bf16x16 v; i32x8 q; };

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// The LDS-DMA loads are issued through inline assembly so that their completion is tracked only by the
// explicit vmcnt waits of the main loop (the ring keeps the loads of the next tiles in flight across
// the fragment reads of the current one).  m0 carries the wave-uniform LDS destination.  The source is
// a wave-uniform 64-bit base in SGPRs plus a 32-bit per-lane byte offset: with per-lane 64-bit VGPR
// addresses the loads crawl while the matrix cores are busy (measured: smfmac + DMA 1.22 us per step
// against 0.76 us in this form, 0.67 us for the smfmacs alone).
__device__ __forceinline__ uint64_t uniform64(const void* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(v >> 32)) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int)(v & 0xFFFFFFFFu));
}
__device__ __forceinline__ void dma16(uint64_t base, uint32_t lane_off, unsigned char* lds_wave_base) {
    // every lane fetches 16 bytes at base + lane_off; the wave's 64 chunks land at lds_wave_base + 16 * lane
    const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void*)lds_wave_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(dst) : "m0", "memory");
}
__device__ __forceinline__ void dma4(uint64_t base, uint32_t lane_off, unsigned char* lds_wave_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void*)lds_wave_base);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(lane_off), "s"(base), "s"(dst) : "m0", "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    // gfx9 s_waitcnt immediate: vmcnt = bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8 (left at "no wait")
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// ordering point between LDS writes and reads of lanes of the same wavefront (its LDS operations execute in
// issue order; this only stops the compiler from moving them)
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// s_waitcnt with vmcnt = N and lgkmcnt = 0 (N: loads that may stay in flight)
template <int N>
__device__ __forceinline__ void wait_vmcnt_lgkm0() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

}  // namespace sffn
