// Shared device helpers for the gfx950 sparsified-FFN kernels (bf16 bit handling, 2:4 selection).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sffn {

__device__ __forceinline__ float bf2f(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16 bits, round to nearest even; NaN keeps its sign and becomes quiet.
__device__ __forceinline__ uint32_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (f != f) ? ((u >> 16) | 0x7FC0u) : r;
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
        v0 = f2bf((v0 & 0x8000u) ? f0 + t : f0 - t);
        v1 = f2bf((v1 & 0x8000u) ? f1 + t : f1 - t);
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
// Metadata of a 2:4 matrix in blocks of 64 rows x 8 bytes (one main-loop step of 64 k): byte address of
// the metadata byte covering k..k+7 of row r, with KS = K / 64.
__host__ __device__ __forceinline__ int64_t mblk_off(int64_t r, int64_t k, int64_t KS) {
    return (((r >> 6) * KS + (k >> 6)) << 9) + ((r & 63) << 3) + ((k & 63) >> 3);
}

// Two survivors per 8 columns leave at most two per aligned group of four, so a V:2:8 row block is
// also two plain 2:4 groups.  Inputs: v = the two survivors (low half first), nib = their positions
// among the four kept columns, cw = the four kept column offsets (one per byte).  Outputs: the two
// packed groups (empty slots are +0 at unused positions) and their metadata byte.
__device__ __forceinline__ void vnm_block_to_24(uint32_t v, uint32_t nib, uint32_t cw, uint32_t& a, uint32_t& b, uint32_t& mbyte) {
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;   // o0 < o1
    const uint32_t v0 = v & 0xFFFFu, v1 = v >> 16;
    uint32_t na, nb;
    if (o1 < 4) {
        a = v; na = o0 | (o1 << 2); b = 0; nb = 0x4;
    } else if (o0 >= 4) {
        a = 0; na = 0x4; b = v; nb = (o0 - 4) | ((o1 - 4) << 2);
    } else {
        if (o0 < 3) { a = v0; na = o0 | (3u << 2); } else { a = v0 << 16; na = 0u | (3u << 2); }
        const uint32_t q = o1 - 4;
        if (q > 0) { b = v1 << 16; nb = 0u | (q << 2); } else { b = v1; nb = 0u | (1u << 2); }
    }
    mbyte = na | (nb << 4);
}

}  // namespace sffn
