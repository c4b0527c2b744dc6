// V:2:M with wider blocks, M in {16, 32, 64} (paper Section 2.3 and Table 5: 64 x M blocks keep 4 columns by L1 score,
// then 2:4 inside them; density 2 / M).  Stand-alone, HBM-bound kernels for the same operations as vnm.hip (M = 8):
// SquaredReLU + compression (eq. (2), Alg. 1 lines 5-6), eq. (6) on the kept slots, the re-expression as a plain 2:4
// matrix over all columns (two survivors per M columns still leave at most two per aligned group of four) and the dense
// transposed expansion for the weight-gradient GEMMs.  Packed layout as for M = 8: vals [T, 2F/M], meta [T, F/(2M)]
// (one nibble per block, two blocks per byte), colidx [T/64, F/M, 4] (offsets inside the block, ascending).
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

namespace {
constexpr int kPitch = 64 * 2 + 16;     // bytes per row of a wavefront's 64 x 64 tile of y2 in LDS

__device__ __forceinline__ uint32_t sqrelu_pair_g(uint32_t w) {
    const float a = bf2f(w & 0xFFFFu), b = bf2f(w >> 16);
    const float ra = a > 0.0f ? a : 0.0f, rb = b > 0.0f ? b : 0.0f;
    return f2bf2(ra * ra, rb * rb);
}
}  // namespace

// One workgroup = one 64-token block x 256 columns; wavefront w owns columns 64 w .. 64 w + 63 (64 / M whole blocks).
// Lane = column for the ordered fp32 column scores and the ranking inside the block, lane = (row, block) for the
// per-row 2:4 selection.  The nibbles of the workgroup's blocks meet in LDS so that two blocks share a metadata byte
// also when they belong to different wavefronts (M = 64).
template <int M>
__global__ void __launch_bounds__(256) sqrelu_vnm_compress_m_kernel(const uint16_t* __restrict__ y1, int64_t F,
                                                                   uint16_t* __restrict__ vals, uint8_t* __restrict__ meta,
                                                                   uint8_t* __restrict__ colidx) {
    constexpr int NB = 64 / M;                           // blocks per wavefront tile
    __shared__ __attribute__((aligned(16))) unsigned char tiles[4][64 * kPitch];
    __shared__ uint8_t nibs[64][256 / M];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tb = blockIdx.y;
    const int64_t c0 = (int64_t)blockIdx.x * 256 + wave * 64;
    const bool active = c0 < F;                          // F is a multiple of 64
    unsigned char* tl = tiles[wave];
    if (active) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 8 + (lane >> 3), seg = lane & 7;
            const uint4 w = *reinterpret_cast<const uint4*>(y1 + (tb * 64 + row) * F + c0 + seg * 8);
            *reinterpret_cast<uint4*>(tl + row * kPitch + seg * 16) =
                make_uint4(sqrelu_pair_g(w.x), sqrelu_pair_g(w.y), sqrelu_pair_g(w.z), sqrelu_pair_g(w.w));
        }
    }
    __syncthreads();
    if (active) {
        // column score: strict ascending-row fp32 sum of y2 (non-negative, so |y2| = y2)
        float sc = 0.0f;
#pragma unroll 8
        for (int r = 0; r < 64; ++r) sc = sc + bf2f(*reinterpret_cast<const uint16_t*>(tl + r * kPitch + lane * 2));
        const int c = lane % M, base = lane - c;
        int rank = 0;
        for (int k = 0; k < M; ++k) {
            const float o = __shfl(sc, base + k, 64);
            rank += (k < c) ? (o >= sc) : ((k > c) ? (o > sc) : 0);
        }
        const unsigned long long kept = __ballot(rank < 4);
        unsigned long long bits = (M == 64) ? kept : ((kept >> base) & ((1ull << (M & 63)) - 1ull));
        uint32_t cw = 0;                                 // the block's four kept offsets, ascending, one per byte
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            cw |= (uint32_t)__builtin_ctzll(bits) << (8 * n);
            bits &= bits - 1ull;
        }
        if (c == 0) *reinterpret_cast<uint32_t*>(colidx + (tb * (F / M) + (c0 + base) / M) * 4) = cw;
        // per-row 2:4 among the four kept columns
#pragma unroll
        for (int sweep = 0; sweep < NB; ++sweep) {
            const int pair = sweep * 64 + lane, row = pair / NB, b = pair % NB;
            const uint32_t cb = (uint32_t)__shfl((int)cw, b * M, 64);
            const unsigned char* rp = tl + row * kPitch + b * M * 2;
            const uint32_t y0 = *reinterpret_cast<const uint16_t*>(rp + (cb & 0xFFu) * 2);
            const uint32_t y1v = *reinterpret_cast<const uint16_t*>(rp + ((cb >> 8) & 0xFFu) * 2);
            const uint32_t y2v = *reinterpret_cast<const uint16_t*>(rp + ((cb >> 16) & 0xFFu) * 2);
            const uint32_t y3v = *reinterpret_cast<const uint16_t*>(rp + (cb >> 24) * 2);
            uint32_t nib;
            const uint32_t v = select24<false>(y0, y1v, y2v, y3v, nib);
            *reinterpret_cast<uint32_t*>(vals + (tb * 64 + row) * (2 * F / M) + (c0 / M + b) * 2) = v;
            nibs[row][wave * NB + b] = (uint8_t)nib;
        }
    }
    __syncthreads();
    constexpr int BYTES = 128 / M;                       // metadata bytes per row of the workgroup's 256 columns
    for (int e = threadIdx.x; e < 64 * BYTES; e += 256) {
        const int row = e / BYTES, j = e % BYTES;
        if ((int64_t)blockIdx.x * 256 + 2 * j * M < F)
            meta[(tb * 64 + row) * (F / (2 * M)) + (int64_t)blockIdx.x * BYTES + j] = (uint8_t)(nibs[row][2 * j] | (nibs[row][2 * j + 1] << 4));
    }
}

// eq. (6) on y2's kept slots; one thread per (token, block).
__global__ void __launch_bounds__(256) dsqrelu_vnm_m_kernel(const uint16_t* __restrict__ dy2, const uint16_t* __restrict__ y1,
                                                           const uint8_t* __restrict__ meta, const uint8_t* __restrict__ colidx,
                                                           int64_t F, int M, int nblk, uint16_t* __restrict__ dvals) {
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (blk >= nblk) return;
    const int64_t t = blockIdx.y;
    const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + ((t >> 6) * nblk + blk) * 4);
    const uint32_t nib = (meta[t * (nblk / 2) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;
    const int64_t base = t * F + (int64_t)blk * M;
    const float ya = bf2f(y1[base + o0]), yb = bf2f(y1[base + o1]);
    const float ga = 2.0f * bf2f(dy2[base + o0]) * (ya > 0.0f ? ya : 0.0f);
    const float gb = 2.0f * bf2f(dy2[base + o1]) * (yb > 0.0f ? yb : 0.0f);
    *reinterpret_cast<uint32_t*>(dvals + t * (2 * (int64_t)nblk) + (int64_t)blk * 2) = f2bf2(ga, gb);
}

// The V:2:M matrix as a plain 2:4 matrix over all F columns: vals24 [T, F/2], meta24 [T, F/8] (row-major).  One thread
// per (token, block) writes the block's M / 4 groups; a group holds both survivors, one (next to an empty slot) or none.
__global__ void __launch_bounds__(256) vnm_to_24_m_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                         const uint8_t* __restrict__ colidx, int64_t F, int M, int nblk,
                                                         uint16_t* __restrict__ vals24, uint8_t* __restrict__ meta24) {
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (blk >= nblk) return;
    const int64_t t = blockIdx.y;
    const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + ((t >> 6) * nblk + blk) * 4);
    const uint32_t nib = (meta[t * (nblk / 2) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
    const uint32_t v = *reinterpret_cast<const uint32_t*>(vals + t * (2 * (int64_t)nblk) + (int64_t)blk * 2);
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;    // o0 < o1
    const uint32_t v0 = v & 0xFFFFu, v1 = v >> 16;
    uint32_t* vo = reinterpret_cast<uint32_t*>(vals24 + t * (F / 2) + (int64_t)blk * (M / 2));
    uint8_t* mo = meta24 + t * (F / 8) + (int64_t)blk * (M / 8);
    uint32_t prev = 0;
    for (int g = 0; g < M / 4; ++g) {
        const bool in0 = (o0 >> 2) == (uint32_t)g, in1 = (o1 >> 2) == (uint32_t)g;
        const uint32_t p = o0 & 3u, q = o1 & 3u;
        uint32_t a = 0, n = 0x4u;                                   // empty group: +0 at positions 0, 1
        if (in0 && in1) { a = v; n = p | (q << 2); }
        else if (in0)   { a = (p < 3) ? v0 : (v0 << 16); n = (p < 3) ? (p | (3u << 2)) : (3u << 2); }
        else if (in1)   { a = (q > 0) ? (v1 << 16) : v1; n = (q > 0) ? (q << 2) : 0x4u; }
        vo[g] = a;
        if (g & 1) mo[g >> 1] = (uint8_t)(prev | (n << 4)); else prev = n;
    }
}

// Dense transposed expansion AT[f, t] (row-major [F, T]); one workgroup = 64 tokens x 64 columns through LDS.
__global__ void __launch_bounds__(256) vnm_expand_t_m_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                            const uint8_t* __restrict__ colidx, int64_t T, int64_t F, int M,
                                                            int nblk, uint16_t* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64][64 + 8];
    const int tid = threadIdx.x;
    for (int i = tid; i < 64 * 72 / 2; i += 256) reinterpret_cast<uint32_t*>(&tile[0][0])[i] = 0;
    __syncthreads();
    const int64_t tb = blockIdx.y;
    const int nb = 64 / M, b0 = blockIdx.x * nb;                   // first block of this 64-column tile
    for (int e = tid; e < 64 * nb; e += 256) {
        const int r = e / nb, bl = e % nb, blk = b0 + bl;
        const int64_t t = tb * 64 + r;
        const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + (tb * nblk + blk) * 4);
        const uint32_t nib = (meta[t * (nblk / 2) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
        const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(vals + t * (2 * (int64_t)nblk) + (int64_t)blk * 2);
        tile[bl * M + o0][r] = (uint16_t)(v & 0xFFFFu);
        tile[bl * M + o1][r] = (uint16_t)(v >> 16);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i, fr = e >> 3, seg = e & 7;     // 64 rows x 8 segments of 8 tokens
        *reinterpret_cast<uint4*>(out + ((int64_t)blockIdx.x * 64 + fr) * T + tb * 64 + seg * 8) = *reinterpret_cast<const uint4*>(&tile[fr][seg * 8]);
    }
}

hipError_t launch_sqrelu_vnm_compress_m(const uint16_t* y1, int64_t T, int64_t F, int M, uint16_t* vals, uint8_t* meta, uint8_t* colidx,
                                        hipStream_t s) {
    dim3 grid((unsigned)((F + 255) / 256), (unsigned)(T / 64));
    if (M == 8)       hipLaunchKernelGGL((sqrelu_vnm_compress_m_kernel<8>), grid, dim3(256), 0, s, y1, F, vals, meta, colidx);
    else if (M == 16) hipLaunchKernelGGL((sqrelu_vnm_compress_m_kernel<16>), grid, dim3(256), 0, s, y1, F, vals, meta, colidx);
    else if (M == 32) hipLaunchKernelGGL((sqrelu_vnm_compress_m_kernel<32>), grid, dim3(256), 0, s, y1, F, vals, meta, colidx);
    else if (M == 64) hipLaunchKernelGGL((sqrelu_vnm_compress_m_kernel<64>), grid, dim3(256), 0, s, y1, F, vals, meta, colidx);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_dsqrelu_vnm_m(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                                int M, uint16_t* dvals, hipStream_t s) {
    const int nblk = (int)(F / M);
    dim3 grid((unsigned)((nblk + 255) / 256), (unsigned)T);
    hipLaunchKernelGGL(dsqrelu_vnm_m_kernel, grid, dim3(256), 0, s, dy2, y1, meta, colidx, F, M, nblk, dvals);
    return hipGetLastError();
}

hipError_t launch_vnm_to_24_m(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M,
                              uint16_t* vals24, uint8_t* meta24, hipStream_t s) {
    const int nblk = (int)(F / M);
    dim3 grid((unsigned)((nblk + 255) / 256), (unsigned)T);
    hipLaunchKernelGGL(vnm_to_24_m_kernel, grid, dim3(256), 0, s, vals, meta, colidx, F, M, nblk, vals24, meta24);
    return hipGetLastError();
}

hipError_t launch_vnm_expand_t_m(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M,
                                 uint16_t* out, hipStream_t s) {
    const int nblk = (int)(F / M);
    dim3 grid((unsigned)(F / 64), (unsigned)(T / 64));
    hipLaunchKernelGGL(vnm_expand_t_m_kernel, grid, dim3(256), 0, s, vals, meta, colidx, T, F, M, nblk, out);
    return hipGetLastError();
}

}  // namespace sffn
