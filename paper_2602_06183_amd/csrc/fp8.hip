// fp8 operands (paper Section 3.4, closing paragraph: quantisation fused into the sparsification scans; Section 1: the 2:4
// hardware covers bf16 and fp8).  Format: OCP E4M3, finite-only (largest finite 448), which is what gfx950's matrix cores
// and v_cvt_pk_fp8_f32 implement.  One float32 scale per tensor, given by the caller: code = E4M3_RNE(clamp(x * inv, +-448)),
// inv = 1 / scale computed once on the host in float32.  Selection always looks at the bf16 magnitudes first, so positions,
// metadata and column indices are those of the bf16 kernels; only the stored survivors become 1-byte codes.
//   quantize_fp8_kernel            dense operand of eqs. (1), (3), (4), (7): plain scan
//   prune24_rows_fp8 / cols_fp8    Section 2.2 (HARD / SOFT) + quantisation: codes [R, K/2], metadata [R, K/8]
//   sqrelu_vnm_compress_fp8        eq. (2) + Section 2.3 + quantisation: codes [T, 2F/M], metadata, column indices
//   vnm_to_24_fp8                  the V:2:M code matrix as a plain 2:4 code matrix over all columns (operand of eqs. (3), (7))
//   transpose_u8                   [R, C] bytes -> [C, R]
//   quantize_fp8_blocked / transpose_quantize_fp8_blocked / prune24_*_fp8 with codes_blk: operands of the fused fp8 step, in the blocked
//                                  layout of common.hpp with a pair of codes per 2-byte element
// Every kernel can record the largest magnitude it quantised (float32, atomic max on the bit pattern) for the caller's next scale.
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

namespace {

__device__ __forceinline__ uint32_t enc2(float a, float b, float inv) { return fp8_enc2(a, b, inv); }

// 2:4 selection as select24 (common.hpp) but returning the survivors as float32 reals: bit copies widened (HARD) or
// a -/+ t evaluated in float32 (SOFT), not rounded to bf16.
template <bool SOFT>
__device__ __forceinline__ void select24_f32(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, uint32_t& nib, float& f0, float& f1) {
    const uint32_t m0 = a0 & 0x7FFFu, m1 = a1 & 0x7FFFu, m2 = a2 & 0x7FFFu, m3 = a3 & 0x7FFFu;
    const int c01 = m0 >= m1, c02 = m0 >= m2, c03 = m0 >= m3, c12 = m1 >= m2, c13 = m1 >= m3, c23 = m2 >= m3;
    const int r0 = 3 - c01 - c02 - c03, r1 = c01 + 2 - c12 - c13, r2 = c02 + c12 + 1 - c23, r3 = c03 + c13 + c23;
    const bool k0 = r0 < 2, k1 = r1 < 2, k2 = r2 < 2, k3 = r3 < 2;
    const uint32_t p0 = k0 ? 0u : (k1 ? 1u : 2u), p1 = k3 ? 3u : (k2 ? 2u : 1u);
    const uint32_t v0 = k0 ? a0 : (k1 ? a1 : a2), v1 = k3 ? a3 : (k2 ? a2 : a1);
    nib = p0 | (p1 << 2);
    f0 = bf2f(v0); f1 = bf2f(v1);
    if (SOFT) {
        const float t = bf2f((r0 == 2) ? m0 : (r1 == 2) ? m1 : (r2 == 2) ? m2 : m3);
        f0 = (v0 & 0x8000u) ? f0 + t : f0 - t;
        f1 = (v1 & 0x8000u) ? f1 + t : f1 - t;
    }
}

}  // namespace

__global__ void __launch_bounds__(256) quantize_fp8_kernel(const uint4* __restrict__ src, int64_t n8, float inv, uint2* __restrict__ codes,
                                                          float* __restrict__ amax) {
    float m = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const uint4 w = src[i];
        const float f[8] = {bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16),
                            bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16)};
#pragma unroll
        for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(f[e]));
        codes[i] = make_uint2(enc2(f[0], f[1], inv) | (enc2(f[2], f[3], inv) << 16), enc2(f[4], f[5], inv) | (enc2(f[6], f[7], inv) << 16));
    }
    note_amax(amax, m);
}

// rows K-contiguous: one thread per 8 consecutive elements (two groups) -> 4 codes + 1 metadata byte
template <bool SOFT>
__global__ void __launch_bounds__(256) prune24_rows_fp8_kernel(const uint16_t* __restrict__ src, int64_t nchunks, int cpr, int64_t ld, float inv,
                                                              uint8_t* __restrict__ codes, uint8_t* __restrict__ meta, float* __restrict__ amax,
                                                              uint16_t* __restrict__ codes_blk, uint8_t* __restrict__ meta_blk, uint8_t* __restrict__ src_q,
                                                              float* __restrict__ amax_src) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float m = 0.0f, m_src = 0.0f;
    if (c < nchunks) {
        const int64_t r = c / cpr;
        const uint4 w = *reinterpret_cast<const uint4*>(src + r * ld + (c - r * cpr) * 8);
        if (src_q) {        // the unpruned source itself, quantised, row-major [R, K] codes (its dense use shares the scale)
            const float f[8] = {bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16),
                                bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16)};
#pragma unroll
            for (int e = 0; e < 8; ++e) m_src = __builtin_fmaxf(m_src, __builtin_fabsf(f[e]));
            *reinterpret_cast<uint2*>(src_q + c * 8) =
                make_uint2(enc2(f[0], f[1], inv) | (enc2(f[2], f[3], inv) << 16), enc2(f[4], f[5], inv) | (enc2(f[6], f[7], inv) << 16));
        }
        uint32_t n0, n1;
        float a, b, d, e;
        select24_f32<SOFT>(w.x & 0xFFFFu, w.x >> 16, w.y & 0xFFFFu, w.y >> 16, n0, a, b);
        select24_f32<SOFT>(w.z & 0xFFFFu, w.z >> 16, w.w & 0xFFFFu, w.w >> 16, n1, d, e);
        m = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(a), __builtin_fabsf(b)), __builtin_fmaxf(__builtin_fabsf(d), __builtin_fabsf(e)));
        const uint32_t q4 = enc2(a, b, inv) | (enc2(d, e, inv) << 16);
        if (codes) {
            *reinterpret_cast<uint32_t*>(codes + c * 4) = q4;
            meta[c] = (uint8_t)(n0 | (n1 << 4));
        }
        if (codes_blk) *reinterpret_cast<uint32_t*>(codes_blk + blk_off(r, (c - r * cpr) * 2, cpr / 16)) = q4;   // 4 codes = pairs 2 c', 2 c' + 1; K / 2 bytes per row
        if (meta_blk) meta_blk[m8blk_off(r, (c - r * cpr) * 8, cpr / 16)] = (uint8_t)(n0 | (n1 << 4));
    }
    note_amax(amax, m);
    if (amax_src) note_amax_slots(amax_src, m_src);
}

// groups run along the strided axis: S[r, k] = src[k * ld + r]; a workgroup takes 64 logical rows x 128 k through LDS
template <bool SOFT>
__global__ void __launch_bounds__(256) prune24_cols_fp8_kernel(const uint16_t* __restrict__ src, int64_t R, int K, int64_t ld, float inv,
                                                              uint8_t* __restrict__ codes, uint8_t* __restrict__ meta, float* __restrict__ amax,
                                                              uint16_t* __restrict__ codes_blk, float* __restrict__ amax_src,
                                                              uint8_t* __restrict__ meta_blk, uint8_t* __restrict__ s_q) {
    constexpr int TK = 128, TR = 64, PITCH = TR + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[TK * PITCH];
    const int64_t r0 = (int64_t)blockIdx.x * TR;
    const int k0 = blockIdx.y * TK;
    const int tid = threadIdx.x;
    float m_src = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int kk = tid / 8 + 32 * i, seg = tid % 8;
        uint4 w = make_uint4(0, 0, 0, 0);
        if (k0 + kk < K) w = *reinterpret_cast<const uint4*>(src + (int64_t)(k0 + kk) * ld + r0 + seg * 8);
        *reinterpret_cast<uint4*>(&tile[kk * PITCH + seg * 8]) = w;
        if (s_q && amax_src) {      // the magnitudes of the source (its dense use, written below as S itself quantised, shares the scale)
            m_src = __builtin_fmaxf(m_src, __builtin_fmaxf(__builtin_fmaxf(bf2f(w.x & 0x7FFFu), bf2f((w.x >> 16) & 0x7FFFu)), __builtin_fmaxf(bf2f(w.y & 0x7FFFu), bf2f((w.y >> 16) & 0x7FFFu))));
            m_src = __builtin_fmaxf(m_src, __builtin_fmaxf(__builtin_fmaxf(bf2f(w.z & 0x7FFFu), bf2f((w.z >> 16) & 0x7FFFu)), __builtin_fmaxf(bf2f(w.w & 0x7FFFu), bf2f((w.w >> 16) & 0x7FFFu))));
        }
    }
    __syncthreads();
    const int rr = tid % 64, q = tid / 64;
    float m = 0.0f;
    if (k0 + 32 * q < K) {
        uint32_t oc[4], mbytes = 0, sq[8];
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const uint16_t* p = &tile[(32 * q + 4 * g) * PITCH + rr];
            uint32_t nib;
            float a, b;
            select24_f32<SOFT>(p[0], p[PITCH], p[2 * PITCH], p[3 * PITCH], nib, a, b);
            if (s_q) sq[g] = enc2(bf2f(p[0]), bf2f(p[PITCH]), inv) | (enc2(bf2f(p[2 * PITCH]), bf2f(p[3 * PITCH]), inv) << 16);
            m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(a), __builtin_fabsf(b)));
            const uint32_t c2 = enc2(a, b, inv);
            if (g & 1) oc[g >> 1] |= c2 << 16; else oc[g >> 1] = c2;
            mbytes |= nib << (4 * g);
        }
        const int64_t r = r0 + rr;
        if (codes) {
            *reinterpret_cast<uint4*>(codes + r * (K / 2) + (k0 + 32 * q) / 2) = make_uint4(oc[0], oc[1], oc[2], oc[3]);
            *reinterpret_cast<uint32_t*>(meta + r * (K / 8) + (k0 + 32 * q) / 8) = mbytes;
        }
        if (codes_blk) *reinterpret_cast<uint4*>(codes_blk + blk_off(r, (k0 + 32 * q) / 4, K / 128)) = make_uint4(oc[0], oc[1], oc[2], oc[3]);   // 16 codes = 8 pairs
        if (meta_blk) *reinterpret_cast<uint32_t*>(meta_blk + m8blk_off(r, k0 + 32 * q, K / 128)) = mbytes;
        if (s_q) {          // the unpruned logical matrix S itself, quantised, row-major [R, K] codes (eq. (3) contracts its kept rows)
            uint4* d = reinterpret_cast<uint4*>(s_q + r * K + k0 + 32 * q);
            d[0] = make_uint4(sq[0], sq[1], sq[2], sq[3]);
            d[1] = make_uint4(sq[4], sq[5], sq[6], sq[7]);
        }
    }
    note_amax(amax, m);
    if (amax_src) note_amax_slots(amax_src, m_src);      // over every element of the source
}

// eq. (2) + V:N:M compression with fp8 values: the structure of sqrelu_vnm_compress_m_kernel (vnm_general.hip): one workgroup =
// one 64-token block x 256 columns, wavefront w owns 64 columns; scores, column choice and the per-row 2:4 choice on the bf16 y2.
template <int M>
__global__ void __launch_bounds__(256) sqrelu_vnm_compress_fp8_kernel(const uint16_t* __restrict__ y1, int64_t F, float inv, uint8_t* __restrict__ codes,
                                                                     uint8_t* __restrict__ meta, uint8_t* __restrict__ colidx, float* __restrict__ amax) {
    constexpr int NB = 64 / M, PITCH = 64 * 2 + 16;
    __shared__ __attribute__((aligned(16))) unsigned char tiles[4][64 * PITCH];
    __shared__ uint8_t nibs[64][256 / M];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tb = blockIdx.y;
    const int64_t c0 = (int64_t)blockIdx.x * 256 + wave * 64;
    const bool active = c0 < F;
    unsigned char* tl = tiles[wave];
    float mx = 0.0f;
    if (active) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 8 + (lane >> 3), seg = lane & 7;
            const uint4 w = *reinterpret_cast<const uint4*>(y1 + (tb * 64 + row) * F + c0 + seg * 8);
            const uint32_t in[4] = {w.x, w.y, w.z, w.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = bf2f(in[e] & 0xFFFFu), b = bf2f(in[e] >> 16);
                const float ra = a > 0.0f ? a : 0.0f, rb = b > 0.0f ? b : 0.0f;
                o[e] = f2bf2(ra * ra, rb * rb);
            }
            *reinterpret_cast<uint4*>(tl + row * PITCH + seg * 16) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
    __syncthreads();
    if (active) {
        float sc = 0.0f;                                  // strict ascending-row fp32 sum of y2
#pragma unroll 8
        for (int r = 0; r < 64; ++r) sc = sc + bf2f(*reinterpret_cast<const uint16_t*>(tl + r * PITCH + lane * 2));
        const int c = lane % M, base = lane - c;
        int rank = 0;
        for (int k = 0; k < M; ++k) {
            const float o = __shfl(sc, base + k, 64);
            rank += (k < c) ? (o >= sc) : ((k > c) ? (o > sc) : 0);
        }
        const unsigned long long kept = __ballot(rank < 4);
        unsigned long long bits = (M == 64) ? kept : ((kept >> base) & ((1ull << (M & 63)) - 1ull));
        uint32_t cw = 0;
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            cw |= (uint32_t)__builtin_ctzll(bits) << (8 * n);
            bits &= bits - 1ull;
        }
        if (c == 0) *reinterpret_cast<uint32_t*>(colidx + (tb * (F / M) + (c0 + base) / M) * 4) = cw;
#pragma unroll
        for (int sweep = 0; sweep < NB; ++sweep) {
            const int pair = sweep * 64 + lane, row = pair / NB, b = pair % NB;
            const uint32_t cb = (uint32_t)__shfl((int)cw, b * M, 64);
            const unsigned char* rp = tl + row * PITCH + b * M * 2;
            const uint32_t y0 = *reinterpret_cast<const uint16_t*>(rp + (cb & 0xFFu) * 2);
            const uint32_t y1v = *reinterpret_cast<const uint16_t*>(rp + ((cb >> 8) & 0xFFu) * 2);
            const uint32_t y2v = *reinterpret_cast<const uint16_t*>(rp + ((cb >> 16) & 0xFFu) * 2);
            const uint32_t y3v = *reinterpret_cast<const uint16_t*>(rp + (cb >> 24) * 2);
            uint32_t nib;
            float a, bb;
            select24_f32<false>(y0, y1v, y2v, y3v, nib, a, bb);
            mx = __builtin_fmaxf(mx, __builtin_fmaxf(a, bb));
            *reinterpret_cast<uint16_t*>(codes + (tb * 64 + row) * (2 * F / M) + (c0 / M + b) * 2) = (uint16_t)enc2(a, bb, inv);
            nibs[row][wave * NB + b] = (uint8_t)nib;
        }
    }
    __syncthreads();
    constexpr int BYTES = 128 / M;
    for (int e = threadIdx.x; e < 64 * BYTES; e += 256) {
        const int row = e / BYTES, j = e % BYTES;
        if ((int64_t)blockIdx.x * 256 + 2 * j * M < F)
            meta[(tb * 64 + row) * (F / (2 * M)) + (int64_t)blockIdx.x * BYTES + j] = (uint8_t)(nibs[row][2 * j] | (nibs[row][2 * j + 1] << 4));
    }
    note_amax(amax, mx);
}

// The V:2:M code matrix as a plain 2:4 code matrix over all F columns: codes24 [T, F/2], meta24 [T, F/8] (row-major); a group holds
// both survivors, one (next to an empty slot, code 0 = +0) or none.  One thread per (token, block).
__global__ void __launch_bounds__(256) vnm_to_24_fp8_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ meta,
                                                           const uint8_t* __restrict__ colidx, int64_t F, int M, int nblk,
                                                           uint8_t* __restrict__ codes24, uint8_t* __restrict__ meta24) {
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (blk >= nblk) return;
    const int64_t t = blockIdx.y;
    const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + ((t >> 6) * nblk + blk) * 4);
    const uint32_t nib = (meta[t * (nblk / 2) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
    const uint32_t v = *reinterpret_cast<const uint16_t*>(codes + t * (2 * (int64_t)nblk) + (int64_t)blk * 2);
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;    // o0 < o1
    const uint32_t v0 = v & 0xFFu, v1 = v >> 8;
    uint16_t* vo = reinterpret_cast<uint16_t*>(codes24 + t * (F / 2) + (int64_t)blk * (M / 2));
    uint8_t* mo = meta24 + t * (F / 8) + (int64_t)blk * (M / 8);
    uint32_t prev = 0;
    for (int g = 0; g < M / 4; ++g) {
        const bool in0 = (o0 >> 2) == (uint32_t)g, in1 = (o1 >> 2) == (uint32_t)g;
        const uint32_t p = o0 & 3u, q = o1 & 3u;
        uint32_t a = 0, n = 0x4u;                                   // empty group: +0 at positions 0, 1
        if (in0 && in1) { a = v; n = p | (q << 2); }
        else if (in0)   { a = (p < 3) ? v0 : (v0 << 8); n = (p < 3) ? (p | (3u << 2)) : (3u << 2); }
        else if (in1)   { a = (q > 0) ? (v1 << 8) : v1; n = (q > 0) ? (q << 2) : 0x4u; }
        vo[g] = (uint16_t)a;
        if (g & 1) mo[g >> 1] = (uint8_t)(prev | (n << 4)); else prev = n;
    }
}

__global__ void __launch_bounds__(256) transpose_u8_kernel(const uint8_t* __restrict__ in, int64_t R, int64_t C, int64_t ld, uint8_t* __restrict__ out) {
    __shared__ uint8_t tile[64][64 + 4];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = tid / 16 + 16 * i, seg = tid % 16;
        *reinterpret_cast<uint32_t*>(&tile[r][seg * 4]) = *reinterpret_cast<const uint32_t*>(in + (r0 + r) * ld + c0 + seg * 4);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid / 16 + 16 * i, seg = tid % 16;
        const uint32_t w = tile[seg * 4][c] | (tile[seg * 4 + 1][c] << 8) | (tile[seg * 4 + 2][c] << 16) | ((uint32_t)tile[seg * 4 + 3][c] << 24);
        *reinterpret_cast<uint32_t*>(out + (c0 + c) * R + r0 + seg * 4) = w;
    }
}

// [R, C] bf16 (row stride ld) -> codes in the blocked pair layout, same orientation: one thread per 8 elements
__global__ void __launch_bounds__(256) quantize_fp8_blocked_kernel(const uint16_t* __restrict__ src, int64_t R, int C8, int64_t ld, float inv,
                                                                  uint16_t* __restrict__ out, float* __restrict__ amax) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float m = 0.0f;
    if (i < R * C8) {
        const int64_t r = i / C8;
        const int c = (int)(i - r * C8) * 8;
        const uint4 w = *reinterpret_cast<const uint4*>(src + r * ld + c);
        const float f[8] = {bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16),
                            bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16)};
#pragma unroll
        for (int e = 0; e < 8; ++e) m = __builtin_fmaxf(m, __builtin_fabsf(f[e]));
        *reinterpret_cast<uint2*>(out + blk_off(r, c / 2, C8 / 8)) =
            make_uint2(enc2(f[0], f[1], inv) | (enc2(f[2], f[3], inv) << 16), enc2(f[4], f[5], inv) | (enc2(f[6], f[7], inv) << 16));
    }
    note_amax_slots(amax, m);
}

// [R, C] bf16 -> codes of the transposed matrix [C, R] in the blocked pair layout; 64 x 64 tiles through LDS.  While the tile is in
// registers the same pass can also write (EXTRA) the codes in the source's own orientation, blocked (X, dY of the fp8 step with fp8
// weight gradients).
template <bool EXTRA>
__global__ void __launch_bounds__(256) transpose_quantize_fp8_blocked_kernel(const uint16_t* __restrict__ src, int64_t R, int64_t C, int64_t ld, float inv,
                                                                            uint16_t* __restrict__ out, float* __restrict__ amax, uint16_t* __restrict__ out_same) {
    __shared__ uint16_t tile[64][64 + 2];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = tid / 8 + 32 * i, seg = tid % 8;
        const uint4 w = *reinterpret_cast<const uint4*>(src + (r0 + r) * ld + c0 + seg * 8);
        uint32_t* d = reinterpret_cast<uint32_t*>(&tile[r][seg * 8]);
        d[0] = w.x; d[1] = w.y; d[2] = w.z; d[3] = w.w;
        if (EXTRA)
            *reinterpret_cast<uint2*>(out_same + blk_off(r0 + r, (c0 + seg * 8) / 2, C / 64)) =
                make_uint2(enc2(bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), inv) | (enc2(bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16), inv) << 16),
                           enc2(bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), inv) | (enc2(bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16), inv) << 16));
    }
    __syncthreads();
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid / 8 + 32 * i, rs = (tid % 8) * 8;          // output row c0 + c, its 8 codes for source rows r0 + rs .. + 7
        uint32_t q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float lo = bf2f(tile[rs + 2 * j][c]), hi = bf2f(tile[rs + 2 * j + 1][c]);
            m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(lo), __builtin_fabsf(hi)));
            q[j] = enc2(lo, hi, inv);
        }
        *reinterpret_cast<uint2*>(out + blk_off(c0 + c, (r0 + rs) / 2, R / 64)) = make_uint2(q[0] | (q[1] << 16), q[2] | (q[3] << 16));
    }
    note_amax_slots(amax, m);
}

hipError_t launch_quantize_fp8_blocked(const uint16_t* src, int64_t R, int64_t C, int64_t ld, float inv, uint8_t* out_blk, hipStream_t s, float* amax) {
    if (C % 64 != 0 || R % 16 != 0) return hipErrorInvalidValue;
    const int64_t n = R * (C / 8);
    hipLaunchKernelGGL(quantize_fp8_blocked_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, R, (int)(C / 8), ld, inv, reinterpret_cast<uint16_t*>(out_blk), amax);
    return hipGetLastError();
}

// The amax slots of the fused fp8 step (common.hpp): n tensors x 64 slots.  clear: before the first kernel (a kernel, not a memset node:
// the step may be captured in a graph); finish: out[i] = max over tensor i's slots.
__global__ void amax_clear_kernel(float* slots) { slots[(blockIdx.x * kAmaxSlots + threadIdx.x) * kAmaxSlotStride] = 0.0f; }
__global__ void amax_finish_kernel(const float* slots, float* out) {
    float m = slots[(blockIdx.x * kAmaxSlots + threadIdx.x) * kAmaxSlotStride];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, o, 64));
    if (threadIdx.x == 0) out[blockIdx.x] = m;
}
hipError_t launch_amax_clear(float* slots, int n, hipStream_t s) {
    hipLaunchKernelGGL(amax_clear_kernel, dim3(n), dim3(kAmaxSlots), 0, s, slots);
    return hipGetLastError();
}
hipError_t launch_amax_finish(const float* slots, int n, float* out, hipStream_t s) {
    hipLaunchKernelGGL(amax_finish_kernel, dim3(n), dim3(kAmaxSlots), 0, s, slots, out);
    return hipGetLastError();
}

hipError_t launch_transpose_quantize_fp8_blocked(const uint16_t* src, int64_t R, int64_t C, int64_t ld, float inv, uint8_t* out_t_blk, hipStream_t s, float* amax,
                                                 uint8_t* out_same_blk) {
    if (C % 64 != 0 || R % 64 != 0) return hipErrorInvalidValue;
    dim3 grid((unsigned)(C / 64), (unsigned)(R / 64));
    uint16_t* o = reinterpret_cast<uint16_t*>(out_t_blk);
    if (out_same_blk) hipLaunchKernelGGL((transpose_quantize_fp8_blocked_kernel<true>), grid, dim3(256), 0, s, src, R, C, ld, inv, o, amax, reinterpret_cast<uint16_t*>(out_same_blk));
    else              hipLaunchKernelGGL((transpose_quantize_fp8_blocked_kernel<false>), grid, dim3(256), 0, s, src, R, C, ld, inv, o, amax, (uint16_t*)nullptr);
    return hipGetLastError();
}

hipError_t launch_quantize_fp8(const uint16_t* src, int64_t n, float inv, uint8_t* codes, float* amax, hipStream_t s) {
    const int64_t n8 = n / 8, blocks = (n8 + 255) / 256;
    hipLaunchKernelGGL(quantize_fp8_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, s, (const uint4*)src, n8, inv, (uint2*)codes, amax);
    return hipGetLastError();
}

static hipError_t launch_prune24_fp8_impl(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float inv, uint8_t* codes, uint8_t* meta,
                                          float* amax, uint16_t* blk, float* amax_src, uint8_t* mblk, uint8_t* s_q, hipStream_t s) {
    if (!trans) {
        const int64_t nchunks = R * (K / 8);
        const unsigned grid = (unsigned)((nchunks + 255) / 256);
        if (mode == 0) hipLaunchKernelGGL((prune24_rows_fp8_kernel<false>), dim3(grid), dim3(256), 0, s, src, nchunks, (int)(K / 8), ld, inv, codes, meta, amax, blk, mblk, s_q, amax_src);
        else           hipLaunchKernelGGL((prune24_rows_fp8_kernel<true>), dim3(grid), dim3(256), 0, s, src, nchunks, (int)(K / 8), ld, inv, codes, meta, amax, blk, mblk, s_q, amax_src);
    } else {
        dim3 grid((unsigned)(R / 64), (unsigned)((K + 127) / 128));
        if (mode == 0) hipLaunchKernelGGL((prune24_cols_fp8_kernel<false>), grid, dim3(256), 0, s, src, R, (int)K, ld, inv, codes, meta, amax, blk, amax_src, mblk, s_q);
        else           hipLaunchKernelGGL((prune24_cols_fp8_kernel<true>), grid, dim3(256), 0, s, src, R, (int)K, ld, inv, codes, meta, amax, blk, amax_src, mblk, s_q);
    }
    return hipGetLastError();
}

hipError_t launch_prune24_fp8(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float inv, uint8_t* codes, uint8_t* meta,
                              float* amax, hipStream_t s) {
    return launch_prune24_fp8_impl(src, R, K, ld, trans, mode, inv, codes, meta, amax, nullptr, nullptr, nullptr, nullptr, s);
}

hipError_t launch_prune24_fp8_step(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float inv, uint8_t* codes, uint8_t* meta,
                                   uint8_t* codes_blk, uint8_t* meta_blk, hipStream_t s, float* amax_src, uint8_t* s_q) {
    if (K % 128 != 0 || R % 64 != 0 || !codes_blk || !meta_blk || !s_q) return hipErrorInvalidValue;   // a block row holds whole 64-byte pieces of the K / 2 codes per row
    return launch_prune24_fp8_impl(src, R, K, ld, trans, mode, inv, codes, meta, nullptr, reinterpret_cast<uint16_t*>(codes_blk), amax_src, meta_blk, s_q, s);
}

hipError_t launch_sqrelu_vnm_compress_fp8(const uint16_t* y1, int64_t T, int64_t F, int M, float inv, uint8_t* codes, uint8_t* meta, uint8_t* colidx,
                                          float* amax, hipStream_t s) {
    dim3 grid((unsigned)((F + 255) / 256), (unsigned)(T / 64));
    if (M == 8)       hipLaunchKernelGGL((sqrelu_vnm_compress_fp8_kernel<8>), grid, dim3(256), 0, s, y1, F, inv, codes, meta, colidx, amax);
    else if (M == 16) hipLaunchKernelGGL((sqrelu_vnm_compress_fp8_kernel<16>), grid, dim3(256), 0, s, y1, F, inv, codes, meta, colidx, amax);
    else if (M == 32) hipLaunchKernelGGL((sqrelu_vnm_compress_fp8_kernel<32>), grid, dim3(256), 0, s, y1, F, inv, codes, meta, colidx, amax);
    else if (M == 64) hipLaunchKernelGGL((sqrelu_vnm_compress_fp8_kernel<64>), grid, dim3(256), 0, s, y1, F, inv, codes, meta, colidx, amax);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_vnm_to_24_fp8(const uint8_t* codes, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M, uint8_t* codes24,
                                uint8_t* meta24, hipStream_t s) {
    const int nblk = (int)(F / M);
    dim3 grid((unsigned)((nblk + 255) / 256), (unsigned)T);
    hipLaunchKernelGGL(vnm_to_24_fp8_kernel, grid, dim3(256), 0, s, codes, meta, colidx, F, M, nblk, codes24, meta24);
    return hipGetLastError();
}

// The canonical fp8 V:2:8 arrays (codes [T, F/4], meta [T, F/16], colidx [T/64, F/8, 4]) regrouped into the units of the fp8 form of the V:2:8
// activation GEMM (gemm_vnm8.hip; the fused epilogues of the fp8 step write them directly): one thread per (token, 128 hidden units) moves 32
// codes and 8 metadata bytes; the first 16 threads of a token block also build the 16 offset words of their (token block, 128 hidden units).
__global__ void __launch_bounds__(256) vnm8_repack_fp8_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ meta,
                                                             const uint8_t* __restrict__ colidx, int64_t T, int F, uint8_t* __restrict__ vcb,
                                                             uint8_t* __restrict__ mcb, uint8_t* __restrict__ cixt) {
    const int KS = F >> 7;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= T * KS) return;
    const int64_t t = i / KS;
    const int kt = (int)(i - t * KS);
    const uint4* src = reinterpret_cast<const uint4*>(codes + t * (F >> 2) + kt * 32);
    uint4* dst = reinterpret_cast<uint4*>(vcb + vcb8_off(t, (int64_t)kt * 16, F));
    dst[0] = src[0];
    dst[1] = src[1];
    *reinterpret_cast<uint2*>(mcb + mcb8_off(t, (int64_t)kt * 2, F)) = *reinterpret_cast<const uint2*>(meta + t * (F >> 4) + kt * 8);
    const int q = (int)(t & 63);
    if (q < 16) {       // word (h, p), byte j = kept column p % 4 of column block 8 (j / 2) + 4 h + 2 (j % 2) + p / 4
        const int h = q >> 3, p = q & 7;
        const uint8_t* c = colidx + ((t >> 6) * (F >> 3) + kt * 16) * 4;
        uint32_t dw = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) dw |= (uint32_t)c[(8 * (j >> 1) + 4 * h + 2 * (j & 1) + (p >> 2)) * 4 + (p & 3)] << (8 * j);
        *reinterpret_cast<uint32_t*>(cixt + cixt8_off(t >> 6, kt, T >> 6) + q * 4) = dw;
    }
}

hipError_t launch_vnm8_repack_fp8(const uint8_t* codes, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, uint8_t* vcb, uint8_t* mcb,
                                  uint8_t* cixt, hipStream_t s) {
    if (T % 64 != 0 || F % 128 != 0) return hipErrorInvalidValue;
    const int64_t n = T * (F / 128);
    hipLaunchKernelGGL(vnm8_repack_fp8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, codes, meta, colidx, T, (int)F, vcb, mcb, cixt);
    return hipGetLastError();
}

hipError_t launch_transpose_u8(const uint8_t* in, int64_t R, int64_t C, int64_t ld, uint8_t* out, hipStream_t s) {
    hipLaunchKernelGGL(transpose_u8_kernel, dim3((unsigned)(C / 64), (unsigned)(R / 64)), dim3(256), 0, s, in, R, C, ld, out);
    return hipGetLastError();
}

}  // namespace sffn
