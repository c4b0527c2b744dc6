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

}  // namespace sffn
