// V:N:M (V=64, N=2, M=8) kernels: eq. (6) on the kept slots (Alg. 2 line 4) and the layout helpers the GEMMs
// consume (re-expression as plain 2:4 over all columns, dense transposed expansion, bf16 transpose).  All of them
// are HBM-bound scans.  The stand-alone compressor of eq. (2) + Section 2.3 lives in vnm_general.hip, for every M.
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

__device__ __forceinline__ uint32_t pick16(const uint32_t (&w)[4], uint32_t c) {
    const uint32_t d = c >> 1;
    const uint32_t lo = (d == 0) ? w[0] : (d == 1) ? w[1] : (d == 2) ? w[2] : w[3];
    return (c & 1u) ? (lo >> 16) : (lo & 0xFFFFu);
}

// eq. (6) evaluated only where y2 was kept.  One thread per (row, column block).
__global__ void __launch_bounds__(256) dsqrelu_vnm_kernel(const uint16_t* __restrict__ dy2, const uint16_t* __restrict__ y1,
                                                         const uint8_t* __restrict__ meta, const uint8_t* __restrict__ colidx,
                                                         int64_t F, int nblk, uint16_t* __restrict__ dvals) {
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (blk >= nblk) return;          // nblk is a multiple of 8, so groups of 4 lanes are in or out together
    const int64_t t = blockIdx.y;
    const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + ((t >> 6) * nblk + blk) * 4);
    const uint32_t nib = (meta[t * (F / 16) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
    const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;
    const uint4 d4 = *reinterpret_cast<const uint4*>(dy2 + t * F + (int64_t)blk * 8);
    const uint4 y4 = *reinterpret_cast<const uint4*>(y1 + t * F + (int64_t)blk * 8);
    const uint32_t dw[4] = {d4.x, d4.y, d4.z, d4.w}, yw[4] = {y4.x, y4.y, y4.z, y4.w};
    const float ya = bf2f(pick16(yw, o0)), yb = bf2f(pick16(yw, o1));
    const float ga = 2.0f * bf2f(pick16(dw, o0)) * (ya > 0.0f ? ya : 0.0f);
    const float gb = 2.0f * bf2f(pick16(dw, o1)) * (yb > 0.0f ? yb : 0.0f);
    const uint32_t v = f2bf2(ga, gb);
    *reinterpret_cast<uint32_t*>(dvals + t * (F / 4) + (int64_t)blk * 2) = v;
}

// Two survivors per 8 columns leave at most two per aligned group of four, so a V:2:8 matrix is
// also a plain 2:4 matrix over all F columns.  This writes that view: vals24 [T, F/2], meta24
// [T, F/8] in the 2:4 packed format (empty slots are +0 at unused positions).
__global__ void __launch_bounds__(256) vnm_to_24_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                       const uint8_t* __restrict__ colidx, int64_t F, int nblk,
                                                       uint16_t* __restrict__ vals24, uint8_t* __restrict__ meta24) {
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (blk >= nblk) return;
    const int64_t t = blockIdx.y;
    const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + ((t >> 6) * nblk + blk) * 4);
    const uint32_t nib = (meta[t * (F / 16) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
    const uint32_t v = *reinterpret_cast<const uint32_t*>(vals + t * (F / 4) + (int64_t)blk * 2);
    uint32_t a, b, mb;
    vnm_block_to_24(v, nib, cw, a, b, mb);
    *reinterpret_cast<uint2*>(vals24 + t * (F / 2) + (int64_t)blk * 4) = make_uint2(a, b);
    meta24[t * (F / 8) + blk] = (uint8_t)mb;
}

// Dense, transposed expansion AT[f, t] of a V:N:M matrix (K-contiguous operand for the
// weight-gradient GEMMs).  One workgroup = 64 rows x 8 column blocks.
__global__ void __launch_bounds__(256) vnm_expand_t_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                          const uint8_t* __restrict__ colidx, int64_t T, int64_t F, int nblk,
                                                          uint16_t* __restrict__ out, int blocked) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64][64 + 8];
    const int tid = threadIdx.x;
    for (int i = tid; i < 64 * 72 / 2; i += 256) reinterpret_cast<uint32_t*>(&tile[0][0])[i] = 0;
    __syncthreads();
    const int64_t tb = blockIdx.y;
    const int b0 = blockIdx.x * 8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i;           // 64 rows x 8 blocks
        const int r = e >> 3, bl = e & 7, blk = b0 + bl;
        const int64_t t = tb * 64 + r;
        const uint32_t cw = *reinterpret_cast<const uint32_t*>(colidx + (tb * nblk + blk) * 4);
        const uint32_t nib = (meta[t * (F / 16) + (blk >> 1)] >> (4 * (blk & 1))) & 0xFu;
        const uint32_t o0 = (cw >> (8 * (nib & 3u))) & 0xFFu, o1 = (cw >> (8 * (nib >> 2))) & 0xFFu;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(vals + t * (F / 4) + (int64_t)blk * 2);
        tile[bl * 8 + o0][r] = (uint16_t)(v & 0xFFFFu);
        tile[bl * 8 + o1][r] = (uint16_t)(v >> 16);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i;           // 64 f rows x 8 segments of 8 tokens
        if (blocked) {                      // 8 blocks of 16 f-rows x 32 tokens, one per 64 consecutive e
            const int bk = e >> 6, l = e & 63, fr = (bk >> 1) * 16 + (l >> 2), tc = (bk & 1) * 32 + (l & 3) * 8;
            *reinterpret_cast<uint4*>(out + blk_off((int64_t)b0 * 8 + fr, tb * 64 + tc, T / 32)) =
                *reinterpret_cast<const uint4*>(&tile[fr][tc]);
        } else {
            const int fr = e >> 3, seg = e & 7;
            *reinterpret_cast<uint4*>(out + ((int64_t)b0 * 8 + fr) * T + tb * 64 + seg * 8) =
                *reinterpret_cast<const uint4*>(&tile[fr][seg * 8]);
        }
    }
}

// out[c, r] = in[r, c]; R, C multiples of 64.
// blocked = 1: out (the transpose) and, when given, out_same (a copy of `in`) are written in the blocked
// operand layout instead of row-major.
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const uint16_t* __restrict__ in, int64_t R, int64_t C, int64_t ld,
                                                            uint16_t* __restrict__ out, int blocked, uint16_t* __restrict__ out_same, int map_logM,
                                                            const int32_t* __restrict__ in_perm) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[64][64 + 2];
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    {   // batched form: matrix blockIdx.z of a stack of [R, C] matrices (map_logM: all read the one source, see the launcher)
        const int64_t m = (int64_t)blockIdx.z * R * C;
        if (!map_logM) in += m;
        if (out) out += m;
        if (out_same) out_same += m;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i, rr = e >> 3, seg = e & 7;
        int64_t rs = r0 + rr;
        if (map_logM) rs = ((rs >> 2) << map_logM) + 4 * blockIdx.z + (rs & 3);
        if (in_perm) rs = in_perm[rs];                       // row r of the matrix is row in_perm[r] of `in`; negative: a zero row
        uint4 w = make_uint4(0, 0, 0, 0);
        if (rs >= 0) w = *reinterpret_cast<const uint4*>(in + rs * ld + c0 + seg * 8);
        uint32_t* p = reinterpret_cast<uint32_t*>(&tile[rr][seg * 8]);
        p[0] = w.x; p[1] = w.y; p[2] = w.z; p[3] = w.w;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i;
        int cc, rs;                          // output row (a column of `in`) and first of 8 source rows
        if (blocked) { const int bk = e >> 6, l = e & 63; cc = (bk >> 1) * 16 + (l >> 2); rs = (bk & 1) * 32 + (l & 3) * 8; }
        else { cc = e >> 3; rs = (e & 7) * 8; }
        if (out) {                           // (out = nullptr: only the blocked copy of `in` is wanted)
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = tile[rs + 2 * j][cc] | ((uint32_t)tile[rs + 2 * j + 1][cc] << 16);
            uint16_t* dst = blocked ? out + blk_off(c0 + cc, r0 + rs, R / 32) : out + (c0 + cc) * R + r0 + rs;
            *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
        }
        if (out_same) {
            const int bk = e >> 6, l = e & 63, rr = (bk >> 1) * 16 + (l >> 2), cs = (bk & 1) * 32 + (l & 3) * 8;
            const uint32_t* p = reinterpret_cast<const uint32_t*>(&tile[rr][cs]);
            *reinterpret_cast<uint4*>(out_same + blk_off(r0 + rr, c0 + cs, C / 32)) = make_uint4(p[0], p[1], p[2], p[3]);
        }
    }
}

hipError_t launch_dsqrelu_vnm(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx, int64_t T,
                              int64_t F, uint16_t* dvals, hipStream_t s) {
    const int nblk = (int)(F / 8);
    dim3 grid((unsigned)((nblk + 255) / 256), (unsigned)T);
    hipLaunchKernelGGL(dsqrelu_vnm_kernel, grid, dim3(256), 0, s, dy2, y1, meta, colidx, F, nblk, dvals);
    return hipGetLastError();
}

// The canonical V:2:8 arrays regrouped into the units of the V:2:8 activation GEMM (gemm_vnm8.hip; the fused epilogues write them directly):
// one thread per (token, 64 hidden units) moves 16 survivors and 4 metadata bytes; the first 8 threads of a token block also build the 8
// offset words of their (token block, 64 hidden units).
__global__ void __launch_bounds__(256) vnm8_repack_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                         const uint8_t* __restrict__ colidx, int64_t T, int F, uint16_t* __restrict__ vcb,
                                                         uint8_t* __restrict__ mcb, uint8_t* __restrict__ cixt) {
    const int KS = F >> 6;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= T * KS) return;
    const int64_t t = i / KS;
    const int kt = (int)(i - t * KS);
    const uint4* src = reinterpret_cast<const uint4*>(vals + t * (F >> 2) + kt * 16);
    uint4* dst = reinterpret_cast<uint4*>(vcb + vcb_off(t, (int64_t)kt * 8, F));
    dst[0] = src[0];
    dst[1] = src[1];
    *reinterpret_cast<uint32_t*>(mcb + mcb_off(t, kt, F)) = *reinterpret_cast<const uint32_t*>(meta + t * (F >> 4) + kt * 4);
    const int q = (int)(t & 63);
    if (q < 8) {        // word (h, r), byte j = kept column r of column block 4 (j / 2) + j % 2 + 2 h
        const int h = q >> 2, r = q & 3;
        const uint8_t* c = colidx + ((t >> 6) * (F >> 3) + kt * 8) * 4;
        uint32_t dw = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) dw |= (uint32_t)c[(4 * (j >> 1) + (j & 1) + 2 * h) * 4 + r] << (8 * j);
        *reinterpret_cast<uint32_t*>(cixt + cixt_off(t >> 6, kt, T >> 6) + q * 4) = dw;
    }
}

hipError_t launch_vnm8_repack(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, uint16_t* vcb, uint8_t* mcb,
                              uint8_t* cixt, hipStream_t s) {
    const int64_t n = T * (F / 64);
    hipLaunchKernelGGL(vnm8_repack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, vals, meta, colidx, T, (int)F, vcb, mcb, cixt);
    return hipGetLastError();
}

hipError_t launch_vnm_to_24(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                            uint16_t* vals24, uint8_t* meta24, hipStream_t s) {
    const int nblk = (int)(F / 8);
    dim3 grid((unsigned)((nblk + 255) / 256), (unsigned)T);
    hipLaunchKernelGGL(vnm_to_24_kernel, grid, dim3(256), 0, s, vals, meta, colidx, F, nblk, vals24, meta24);
    return hipGetLastError();
}

hipError_t launch_vnm_expand_t(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                               uint16_t* out, int blocked, hipStream_t s) {
    const int nblk = (int)(F / 8);
    dim3 grid((unsigned)(nblk / 8), (unsigned)(T / 64));
    hipLaunchKernelGGL(vnm_expand_t_kernel, grid, dim3(256), 0, s, vals, meta, colidx, T, F, nblk, out, blocked);
    return hipGetLastError();
}

hipError_t launch_transpose(const uint16_t* in, int64_t R, int64_t C, int64_t ld, uint16_t* out, int blocked, uint16_t* out_same,
                            hipStream_t s, int batch, int cluster_M, const int32_t* in_perm) {
    if (batch > 1 && ld != C) return hipErrorInvalidValue;
    if (in_perm && (batch > 1 || cluster_M)) return hipErrorInvalidValue;
    if (cluster_M && batch * 4 != cluster_M) return hipErrorInvalidValue;
    const int logM = cluster_M == 8 ? 3 : cluster_M == 16 ? 4 : cluster_M == 32 ? 5 : cluster_M == 64 ? 6 : 0;
    if (cluster_M && !logM) return hipErrorInvalidValue;
    dim3 grid((unsigned)(C / 64), (unsigned)(R / 64), (unsigned)batch);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, s, in, R, C, ld, out, blocked, out_same, logM, in_perm);
    return hipGetLastError();
}

}  // namespace sffn
