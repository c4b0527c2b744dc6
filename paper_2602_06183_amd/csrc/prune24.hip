// prune24_compress: per-iteration 2:4 prune-and-pack of a weight matrix (paper Section 2.2 and the
// "sparsify24" calls of Alg. 1 line 4 / Alg. 2 line 2).  HBM-bound element-wise scan: every input
// element is read once (16-byte loads), 0.5 element of values and 1/16 byte of metadata are written.
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

// ---- rows are K-contiguous: one thread per 8 consecutive elements (two groups) -----------------
template <bool SOFT, bool FLAT>
__global__ void __launch_bounds__(256) prune24_rows_kernel(const uint16_t* __restrict__ src, int64_t nchunks, int cpr,
                                                          int64_t ld, uint16_t* __restrict__ vals,
                                                          uint8_t* __restrict__ meta) {
    constexpr int UNROLL = 4;
    const int64_t base = (int64_t)blockIdx.x * (256 * UNROLL) + threadIdx.x;
    uint4 w[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = base + u * 256;
        if (c < nchunks) {
            int64_t off;
            if (FLAT) off = c * 8;
            else { const int64_t r = c / cpr; off = r * ld + (c - r * cpr) * 8; }
            w[u] = *reinterpret_cast<const uint4*>(src + off);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t c = base + u * 256;
        if (c < nchunks) {
            uint32_t n0, n1;
            const uint32_t o0 = select24<SOFT>(w[u].x & 0xFFFFu, w[u].x >> 16, w[u].y & 0xFFFFu, w[u].y >> 16, n0);
            const uint32_t o1 = select24<SOFT>(w[u].z & 0xFFFFu, w[u].z >> 16, w[u].w & 0xFFFFu, w[u].w >> 16, n1);
            *reinterpret_cast<uint2*>(vals + c * 4) = make_uint2(o0, o1);
            meta[c] = (uint8_t)(n0 | (n1 << 4));
        }
    }
}

// ---- groups run along the strided axis: S[r,k] = src[k*ld + r] ---------------------------------
// A workgroup takes 64 logical rows x 128 k: the 128 x 64 source tile goes through LDS so that
// both the HBM reads (128 B row segments) and the packed writes (32 B per thread, 128 B per row)
// stay contiguous.
template <bool SOFT>
__global__ void __launch_bounds__(256) prune24_cols_kernel(const uint16_t* __restrict__ src, int64_t R, int K, int64_t ld,
                                                          uint16_t* __restrict__ vals, uint8_t* __restrict__ meta,
                                                          uint16_t* __restrict__ vblk, uint8_t* __restrict__ mblk,
                                                          uint16_t* __restrict__ src_blk, uint16_t* __restrict__ src_t = nullptr) {
    constexpr int TK = 128, TR = 64, PITCH = TR + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[TK * PITCH];
    const int64_t r0 = (int64_t)blockIdx.x * TR;
    const int k0 = blockIdx.y * TK;
    const int tid = threadIdx.x;
    if (blockIdx.z) {   // batched form: matrix blockIdx.z of a stack of [K, R] sources (ld = R)
        const int64_t m = (int64_t)blockIdx.z * R * K;
        src += m;
        if (vals) { vals += m / 2; meta += m / 8; }
        if (vblk) { vblk += m / 2; mblk += m / 8; }
        if (src_blk) src_blk += m;
        if (src_t) src_t += m;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int kk = tid / 8 + 32 * i, seg = tid % 8;
        uint4 w = make_uint4(0, 0, 0, 0);
        if (k0 + kk < K) w = *reinterpret_cast<const uint4*>(src + (int64_t)(k0 + kk) * ld + r0 + seg * 8);
        *reinterpret_cast<uint4*>(&tile[kk * PITCH + seg * 8]) = w;
    }
    __syncthreads();
    if (src_blk) {      // blocked copy of the source tile itself: rows = k (128), columns = r (64) -> 16 blocks of 1 KB
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i, bk = e >> 6, l = e & 63;
            const int kr = (bk >> 1) * 16 + (l >> 2), rc = (bk & 1) * 32 + (l & 3) * 8;
            if (k0 + kr < K)
                *reinterpret_cast<uint4*>(src_blk + blk_off(k0 + kr, r0 + rc, R / 32)) = *reinterpret_cast<const uint4*>(&tile[kr * PITCH + rc]);
        }
    }
    if (src_t) {        // the unpruned transposed tile: logical rows r (64) x k (128) -> [R, K] row-major, 16 bytes per thread and pass
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // row r0 + tr, k segment of 8 starting at 8 ks; neighbouring lanes take the two halves of a 32-byte piece of one output row
            // (whole sectors in HBM; the LDS reads of a wavefront then fall into two bank groups x 16 words: no conflicts)
            const int e = tid + 256 * i, tr = (e >> 1) & 63, ks = ((e >> 7) << 1) | (e & 1);
            if (k0 + 8 * ks < K) {
                uint32_t w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    w[j] = tile[(8 * ks + 2 * j) * PITCH + tr] | ((uint32_t)tile[(8 * ks + 2 * j + 1) * PITCH + tr] << 16);
                *reinterpret_cast<uint4*>(src_t + (r0 + tr) * K + k0 + 8 * ks) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
    const int rr = tid % 64, q = tid / 64;
    if (k0 + 32 * q >= K) return;
    uint32_t ov[8], mbytes = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const uint16_t* p = &tile[(32 * q + 4 * g) * PITCH + rr];
        uint32_t nib;
        ov[g] = select24<SOFT>(p[0], p[PITCH], p[2 * PITCH], p[3 * PITCH], nib);
        mbytes |= nib << (4 * g);
    }
    const int64_t r = r0 + rr;
    if (vals) {         // (the fused step's lean form passes no canonical outputs: only the blocked copies are consumed)
        uint16_t* vo = vals + r * (K / 2) + (k0 + 32 * q) / 2;
        *reinterpret_cast<uint4*>(vo) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
        *reinterpret_cast<uint4*>(vo + 8) = make_uint4(ov[4], ov[5], ov[6], ov[7]);
        *reinterpret_cast<uint32_t*>(meta + r * (K / 8) + (k0 + 32 * q) / 8) = mbytes;
    }
    if (vblk) {
        uint16_t* vb = vblk + blk_off(r, (k0 + 32 * q) / 2, K / 64);
        *reinterpret_cast<uint4*>(vb) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
        *reinterpret_cast<uint4*>(vb + 8) = make_uint4(ov[4], ov[5], ov[6], ov[7]);
        // 32 k = one step of the matrix instruction: its two 16-k halves belong to different lanes of the unit
        *reinterpret_cast<uint16_t*>(mblk + mblk_off(r, k0 + 32 * q, K / 64)) = (uint16_t)mbytes;
        *reinterpret_cast<uint16_t*>(mblk + mblk_off(r, k0 + 32 * q + 16, K / 64)) = (uint16_t)(mbytes >> 16);
    }
}

// Rows K-contiguous, fused-step variant: a wavefront owns 16 rows x 64 k, i.e. exactly one 1 KB block of the
// blocked packed output; lane = (row, 16 k), two 16-byte loads, one 16-byte store per output.
// logM > 0 (neuron-level experts, Section 3.3): output row e * Kc + j takes source row (j / 4) * M + 4 e + j % 4, i.e.
// the rows of every expert's hidden units come out consecutively (expert-major), ready for one grouped contraction.
template <bool SOFT>
__global__ void __launch_bounds__(256) prune24_rows_step_kernel(const uint16_t* __restrict__ src, int K, int64_t ld,
                                                               uint16_t* __restrict__ vals, uint8_t* __restrict__ meta,
                                                               uint16_t* __restrict__ vblk, uint8_t* __restrict__ mblk, int logM, int Kc) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x * 4 + wave;            // 64-k column
    if (chunk * 64 >= K) return;
    const int64_t r = (int64_t)blockIdx.y * 16 + (lane >> 2);
    int64_t rs = r;                                     // source row
    if (logM) { const int e = (int)(r / Kc), j = (int)(r - (int64_t)e * Kc); rs = ((int64_t)(j >> 2) << logM) + 4 * e + (j & 3); }
    const int q = lane & 3, k = chunk * 64 + 16 * q;
    const uint4 w0 = *reinterpret_cast<const uint4*>(src + rs * ld + k);
    const uint4 w1 = *reinterpret_cast<const uint4*>(src + rs * ld + k + 8);
    uint32_t n0, n1, n2, n3;
    const uint32_t o0 = select24<SOFT>(w0.x & 0xFFFFu, w0.x >> 16, w0.y & 0xFFFFu, w0.y >> 16, n0);
    const uint32_t o1 = select24<SOFT>(w0.z & 0xFFFFu, w0.z >> 16, w0.w & 0xFFFFu, w0.w >> 16, n1);
    const uint32_t o2 = select24<SOFT>(w1.x & 0xFFFFu, w1.x >> 16, w1.y & 0xFFFFu, w1.y >> 16, n2);
    const uint32_t o3 = select24<SOFT>(w1.z & 0xFFFFu, w1.z >> 16, w1.w & 0xFFFFu, w1.w >> 16, n3);
    const uint4 ov = make_uint4(o0, o1, o2, o3);
    const uint16_t mb = (uint16_t)(n0 | (n1 << 4) | (n2 << 8) | (n3 << 12));
    if (vals) {
        *reinterpret_cast<uint4*>(vals + r * (K / 2) + k / 2) = ov;
        *reinterpret_cast<uint16_t*>(meta + r * (K / 8) + k / 8) = mb;
    }
    *reinterpret_cast<uint4*>(vblk + blk_off(r, k / 2, K / 64)) = ov;
    *reinterpret_cast<uint16_t*>(mblk + mblk_off(r, k, K / 64)) = mb;
}

hipError_t launch_prune24(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, uint16_t* vals,
                          uint8_t* meta, hipStream_t stream) {
    if (!trans) {
        const int64_t nchunks = R * (K / 8);
        const unsigned grid = (unsigned)((nchunks + 1023) / 1024);
        const int cpr = (int)(K / 8);
        const bool flat = (ld == K);
        if (mode == 0) {
            if (flat) hipLaunchKernelGGL((prune24_rows_kernel<false, true>), dim3(grid), dim3(256), 0, stream, src, nchunks, cpr, ld, vals, meta);
            else      hipLaunchKernelGGL((prune24_rows_kernel<false, false>), dim3(grid), dim3(256), 0, stream, src, nchunks, cpr, ld, vals, meta);
        } else {
            if (flat) hipLaunchKernelGGL((prune24_rows_kernel<true, true>), dim3(grid), dim3(256), 0, stream, src, nchunks, cpr, ld, vals, meta);
            else      hipLaunchKernelGGL((prune24_rows_kernel<true, false>), dim3(grid), dim3(256), 0, stream, src, nchunks, cpr, ld, vals, meta);
        }
    } else {
        dim3 grid((unsigned)(R / 64), (unsigned)((K + 127) / 128));
        if (mode == 0) hipLaunchKernelGGL((prune24_cols_kernel<false>), grid, dim3(256), 0, stream, src, R, (int)K, ld, vals, meta, (uint16_t*)nullptr, (uint8_t*)nullptr, (uint16_t*)nullptr);
        else           hipLaunchKernelGGL((prune24_cols_kernel<true>), grid, dim3(256), 0, stream, src, R, (int)K, ld, vals, meta, (uint16_t*)nullptr, (uint8_t*)nullptr, (uint16_t*)nullptr);
    }
    return hipGetLastError();
}

hipError_t launch_prune24_step(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, uint16_t* vals,
                               uint8_t* meta, uint16_t* vblk, uint8_t* mblk, uint16_t* src_blk, hipStream_t stream, int batch, int cluster_M,
                               uint16_t* src_t) {
    if (batch > 1 && (!trans || ld != R)) return hipErrorInvalidValue;
    if (cluster_M && (trans || (cluster_M != 8 && cluster_M != 16 && cluster_M != 32 && cluster_M != 64) || R % cluster_M)) return hipErrorInvalidValue;
    if (!trans) {
        dim3 grid((unsigned)((K / 64 + 3) / 4), (unsigned)(R / 16));
        const int logM = cluster_M == 8 ? 3 : cluster_M == 16 ? 4 : cluster_M == 32 ? 5 : cluster_M == 64 ? 6 : 0;
        const int Kc = cluster_M ? (int)(4 * R / cluster_M) : 0;
        if (mode == 0) hipLaunchKernelGGL((prune24_rows_step_kernel<false>), grid, dim3(256), 0, stream, src, (int)K, ld, vals, meta, vblk, mblk, logM, Kc);
        else           hipLaunchKernelGGL((prune24_rows_step_kernel<true>), grid, dim3(256), 0, stream, src, (int)K, ld, vals, meta, vblk, mblk, logM, Kc);
    } else {
        dim3 grid((unsigned)(R / 64), (unsigned)((K + 127) / 128), (unsigned)batch);
        if (mode == 0) hipLaunchKernelGGL((prune24_cols_kernel<false>), grid, dim3(256), 0, stream, src, R, (int)K, ld, vals, meta, vblk, mblk, src_blk, src_t);
        else           hipLaunchKernelGGL((prune24_cols_kernel<true>), grid, dim3(256), 0, stream, src, R, (int)K, ld, vals, meta, vblk, mblk, src_blk, src_t);
    }
    return hipGetLastError();
}

}  // namespace sffn
