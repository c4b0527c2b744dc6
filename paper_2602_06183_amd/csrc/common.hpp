// Shared device helpers for the gfx950 sparsified-FFN kernels (bf16 bit handling, 2:4 selection).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Tile rows per band of the workgroup -> tile map of the 256 x 256 tile kernels: the 32 workgroups that an XCD runs at a time
// cover GROUP tile rows x 32 / GROUP tile columns, and its L2 fetches the operand panels of exactly those rows and columns.
#ifndef SFFN_TILE_GROUP
#define SFFN_TILE_GROUP 4
#endif

namespace sffn {

__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16 bits, round to nearest even, through gfx950's v_cvt_pk_bf16_f32 (checked against integer
// rounding on every bf16 pattern x tie / near-tie low halves, subnormals included; only NaN payloads differ).
typedef __attribute__((ext_vector_type(2))) float sffn_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 sffn_bf16x2;
__device__ __forceinline__ uint32_t f2bf2(float lo, float hi) {      // -> bf16(lo) | bf16(hi) << 16
    const sffn_f32x2 v = {lo, hi};
    const sffn_bf16x2 b = __builtin_convertvector(v, sffn_bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint32_t f2bf(float f) { return f2bf2(f, 0.0f) & 0xFFFFu; }

// two real values -> two OCP E4M3 codes in the low 16 bits (first value in the low byte): one float32 product with inv = 1 / scale,
// saturation to +-448 (v_cvt_pk_fp8_f32 would give NaN above 464), one round-to-nearest-even
__device__ __forceinline__ uint32_t fp8_enc2(float a, float b, float inv) {
    const float ma = __builtin_fminf(__builtin_fmaxf(a * inv, -448.0f), 448.0f);
    const float mb = __builtin_fminf(__builtin_fmaxf(b * inv, -448.0f), 448.0f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(ma, mb, 0, false) & 0xFFFFu;
}

// Largest magnitude seen by a wavefront -> *amax (device float32, atomic max on the bit pattern: non-negative floats order like their bits).
// m >= 0; every lane of the wavefront must call it.  At most one atomic per wavefront, and none when the value already there is
// at least as large (tens of thousands of wavefronts hitting one address serialise in L2: 1.5 ms instead of 0.03 for a pass over
// 128 MB; a stale read only costs a redundant atomic).
__device__ __forceinline__ void note_amax(float* amax, float m) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, o, 64));
    if (amax && (threadIdx.x & 63) == 0) {
        unsigned int* p = reinterpret_cast<unsigned int*>(amax);
        if (__float_as_uint(m) > __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(p, __float_as_uint(m));
    }
}

// The same for the kernels of the fused fp8 step: 64 slots per tensor, 256 bytes apart (slot = workgroup id % 64), so that the reads and
// atomics of a launch spread over cache lines and L2 channels; amax_finish_kernel (fp8.hip) folds the slots at the end of the step.
constexpr int kAmaxSlots = 64, kAmaxSlotStride = 64;      // floats
__device__ __forceinline__ void note_amax_slots(float* slots, float m) {
    if (slots) note_amax(slots + (((blockIdx.y * gridDim.x + blockIdx.x) & (kAmaxSlots - 1)) * kAmaxSlotStride), m);
    else note_amax(nullptr, m);
}

// 2:4 selection on one group of four bf16 (a0..a3 as 16-bit patterns): rank by magnitude
// descending, index ascending; the two first survive (Section 2.2 of the paper, with the tie rule
// of the packed-format contract).  Returns v0 | v1 << 16 (survivors in ascending position) and
// the metadata nibble p0 | p1 << 2.  SOFT: survivors move towards zero by the third-largest
// magnitude, evaluated in fp32 and rounded once to bf16.
template <bool SOFT>
__device__ __forceinline__ uint32_t select24(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, uint32_t& nib) {
    const uint32_t m0 = a0 & 0x7FFFu, m1 = a1 & 0x7FFFu, m2 = a2 & 0x7FFFu, m3 = a3 & 0x7FFFu;
    const int c01 = m0 >= m1, c02 = m0 >= m2, c03 = m0 >= m3, c12 = m1 >= m2, c13 = m1 >= m3, c23 = m2 >= m3;
    const int r0 = 3 - c01 - c02 - c03;          // how many entries outrank entry 0
    const int r1 = c01 + 2 - c12 - c13;
    const int r2 = c02 + c12 + 1 - c23;
    const int r3 = c03 + c13 + c23;
    const bool k0 = r0 < 2, k1 = r1 < 2, k2 = r2 < 2, k3 = r3 < 2;
    const uint32_t p0 = k0 ? 0u : (k1 ? 1u : 2u);
    const uint32_t p1 = k3 ? 3u : (k2 ? 2u : 1u);
    uint32_t v0 = k0 ? a0 : (k1 ? a1 : a2);
    uint32_t v1 = k3 ? a3 : (k2 ? a2 : a1);
    if (SOFT) {
        const uint32_t tm = (r0 == 2) ? m0 : (r1 == 2) ? m1 : (r2 == 2) ? m2 : m3;
        const float t = bf2f(tm);
        const float f0 = bf2f(v0), f1 = bf2f(v1);
        nib = p0 | (p1 << 2);
        return f2bf2((v0 & 0x8000u) ? f0 + t : f0 - t, (v1 & 0x8000u) ? f1 + t : f1 - t);
    }
    nib = p0 | (p1 << 2);
    return v0 | (v1 << 16);
}

// "Blocked" operand layout used between the kernels of the fused step: a K-contiguous matrix of
// 2-byte elements is cut into 1 KB blocks of 16 rows x 32 elements, block (r / 16, k / 32) stored at
// ((r / 16) * KC + k / 32) * 512 elements with KC = K / 32.  One wavefront-wide 16-byte-per-lane
// LDS-DMA load then moves exactly one contiguous block, which the L2 -> LDS path serves at close to
// twice the rate of eight separate 128-byte row segments.
__host__ __device__ __forceinline__ int64_t blk_off(int64_t r, int64_t k, int64_t KC) {
    return (((r >> 4) * KC + (k >> 5)) << 9) + ((r & 15) << 5) + (k & 31);
}
// fp8 operands use the same layout with a pair of 1-byte codes in the place of a 2-byte element (a block = 16 rows x 64 codes):
// blk_off(r, kbyte / 2, row bytes / 64) indexes 16-bit pairs.
// Metadata of a 2:4 matrix, blocked for the sparse matrix instruction: one 256-byte unit per (32 rows, 64 k).
// v_smfmac_f32_32x32x32_bf16 wants, in lane (row % 32) + 32 * h, the sixteen index bits of the row's survivors
// in k 16h..16h+15 of a 32-k step; a unit stores, for each such lane, the two 32-k steps s = 0, 1 of its 64 k as
// one 32-bit word (low half: s = 0) at byte 128 h + 4 (row % 32).  A wavefront therefore fetches a unit with one
// 4-byte-per-lane LDS-DMA load, reads it back with one conflict-free ds_read_b32 and picks the step through the
// instruction's ABID field.  mblk_off = byte address of the metadata byte covering k..k+7 of row r, KS = K / 64.
__host__ __device__ __forceinline__ int64_t mblk_off(int64_t r, int64_t k, int64_t KS) {
    return (((r >> 5) * KS + (k >> 6)) << 8) + (((k >> 4) & 1) << 7) + ((r & 31) << 2) + (((k >> 5) & 1) << 1) + ((k >> 3) & 1);
}

// The same for fp8 operands (v_smfmac_f32_32x32x64_fp8_fp8 wants a 32-bit index word per lane and 64-k step, no ABID halves): one
// 512-byte unit per (32 rows, 128 k), row-major inside (16 bytes per row); a wavefront fetches its 32 rows of a stage with two
// contiguous 4-byte-per-lane loads.  m8blk_off = byte address of the metadata byte covering k..k+7 of row r, KS = K / 128.
__host__ __device__ __forceinline__ int64_t m8blk_off(int64_t r, int64_t k, int64_t KS) {
    return (((r >> 5) * KS + (k >> 7)) << 9) + ((r & 31) << 4) + ((k & 127) >> 3);
}

// Operands of the V:2:8 activation GEMM (gemm_vnm8.hip), written by the fused epilogues of eqs. (1), (4):
// survivors (element index of the pair of (token t, column block blk); F = d_ffn): 1 KB per (32 tokens, 64 hidden units)
__host__ __device__ __forceinline__ int64_t vcb_off(int64_t t, int64_t blk, int64_t F) {
    return ((((t >> 5) * (F >> 6) + (blk >> 3)) << 9) + ((t & 31) << 4) + ((blk & 7) << 1));
}
// metadata (byte address of the 4 bytes = 8 nibbles of (token t, 64 hidden units starting at column block blk8 * 8))
__host__ __device__ __forceinline__ int64_t mcb_off(int64_t t, int64_t blk8, int64_t F) {
    return (((t >> 6) * (F >> 6) + blk8) << 8) + ((t & 63) << 2);
}
// kept-column offsets, regrouped per (64 hidden units, token block) into the 8 words the transposing reads want (byte address of word 0)
__host__ __device__ __forceinline__ int64_t cixt_off(int64_t tb, int64_t blk8, int64_t n_tok_blocks) {
    return (blk8 * n_tok_blocks + tb) << 5;
}

// The same for the fp8 form of that kernel (a stage is 128 hidden units): byte address of the two codes of (token t, column block blk);
// of the 4 metadata bytes of (token t, 64 hidden units starting at column block blk8 * 8); of word 0 of the 16 offset words of
// (token block tb, 128 hidden units number s128)
__host__ __device__ __forceinline__ int64_t vcb8_off(int64_t t, int64_t blk, int64_t F) {
    return (((t >> 5) * (F >> 7) + (blk >> 4)) << 10) + ((t & 31) << 5) + ((blk & 15) << 1);
}
__host__ __device__ __forceinline__ int64_t mcb8_off(int64_t t, int64_t blk8, int64_t F) {
    return (((t >> 6) * (F >> 7) + (blk8 >> 1)) << 9) + ((t & 63) << 3) + ((blk8 & 1) << 2);
}
__host__ __device__ __forceinline__ int64_t cixt8_off(int64_t tb, int64_t s128, int64_t n_tok_blocks) {
    return (s128 * n_tok_blocks + tb) << 6;
}

// The same in two steps, for kernels whose stores would otherwise stand between the early-out read and its use (loads and stores share one
// in-order counter): amax_slot_peek reads the workgroup's slot before the stores are issued, note_amax_slots_seen compares against that value.
__device__ __forceinline__ uint32_t amax_slot_peek(const float* slots) {
    if (!slots) return 0u;
    const unsigned int* p = reinterpret_cast<const unsigned int*>(slots + (((blockIdx.y * gridDim.x + blockIdx.x) & (kAmaxSlots - 1)) * kAmaxSlotStride));
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void note_amax_slots_seen(float* slots, float m, uint32_t seen) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, o, 64));
    if (slots && (threadIdx.x & 63) == 0 && __float_as_uint(m) > seen)
        atomicMax(reinterpret_cast<unsigned int*>(slots + (((blockIdx.y * gridDim.x + blockIdx.x) & (kAmaxSlots - 1)) * kAmaxSlotStride)), __float_as_uint(m));
}

// Two survivors per 8 columns leave at most two per aligned group of four, so a V:2:8 row block is
// also two plain 2:4 groups.  Inputs: v = the two survivors (low half first), nib = their positions
// among the four kept columns, cw = the four kept column offsets (one per byte).  Outputs: the two
// packed groups (empty slots are +0 at unused positions) and their metadata byte.
__device__ __forceinline__ void vnm_block_to_24(uint32_t v, uint32_t nib, uint32_t cw, uint32_t& a, uint32_t& b, uint32_t& mbyte) {
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;   // o0 < o1
    const uint32_t v0 = v & 0xFFFFu, v1 = v >> 16;
    const bool lo0 = o0 < 4, lo1 = o1 < 4;            // survivor in columns 0-3?  (lo1 implies lo0)
    // low group: both survivors | only the first (kept next to an empty slot at position 3, or after one at 0) | none
    const uint32_t a_split = (o0 < 3) ? v0 : (v0 << 16), na_split = (o0 < 3) ? (o0 | (3u << 2)) : (3u << 2);
    a = lo1 ? v : (lo0 ? a_split : 0u);
    const uint32_t na = lo1 ? (o0 | (o1 << 2)) : (lo0 ? na_split : 0x4u);
    // high group: both | only the second | none
    const uint32_t q = o1 - 4;
    const uint32_t b_split = (q > 0) ? (v1 << 16) : v1, nb_split = (q > 0) ? (q << 2) : 0x4u;
    b = !lo0 ? v : (!lo1 ? b_split : 0u);
    const uint32_t nb = !lo0 ? ((o0 - 4) | (q << 2)) : (!lo1 ? nb_split : 0x4u);
    mbyte = na | (nb << 4);
}

// lane i <- lane i + N inside a row of 16 lanes (0 past the row's end): one DPP move instead of an LDS permute
template <int N>
__device__ __forceinline__ uint32_t row_shl(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x100 | N, 0xF, 0xF, true);
}

// y1 at y2's kept slots, as the fused epilogues write and read it: 2 KB runs of (64 tokens x 8 column blocks);
// index in 32-bit words of (token t, column block blk), F = d_ffn.
__host__ __device__ __forceinline__ int64_t ykept_off(int64_t t, int64_t blk, int64_t F) {
    return ((((t >> 6) * (F >> 6) + (blk >> 3)) << 6) + (t & 63)) * 8 + (blk & 7);
}

}  // namespace sffn
