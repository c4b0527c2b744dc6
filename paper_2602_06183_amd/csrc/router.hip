// Neuron-level router of Section 3.3 / Alg. 3, steps 1 and 2 of the conversion listed in Section 3.4, and the small
// data-movement kernels of step 3:
//   route:   s[t, e] = x[t] . mean[e] (float32, fixed summation order), expert[t] = argmax_e (ties to the lower e)
//   permute: stable grouping of the tokens by expert, every run padded to 64 rows (perm, row_of_token, seg)
//   gather:  X rows in permuted order, written in the blocked operand layout; colidx of the V:N:M result
// HBM-bound: the route kernel reads X once (16 bytes per lane), the others move indices and one copy of X.
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

// One wavefront scores TOK tokens against all E experts.  Summation order (part of the parity contract, the argmax
// depends on it): the products are cut into chunks of 8 consecutive d; lane l accumulates chunks l, l + 64, ... in
// ascending d, then the 64 partial sums are folded by 32, 16, 8, 4, 2, 1.  A bf16 x bf16 product is exact in
// float32, so fmaf rounds exactly like the separate add.
template <int E, int TOK>
__global__ void __launch_bounds__(256) venom_route_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ means, int T, int D,
                                                         int32_t* __restrict__ expert, float* __restrict__ scores) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = (blockIdx.x * 4 + wave) * TOK;
    if (t0 >= T) return;
    float acc[TOK][E];
#pragma unroll
    for (int q = 0; q < TOK; ++q)
#pragma unroll
        for (int e = 0; e < E; ++e) acc[q][e] = 0.0f;
    for (int d = lane * 8; d < D; d += 512) {
        uint4 mv[E];
#pragma unroll
        for (int e = 0; e < E; ++e) mv[e] = *reinterpret_cast<const uint4*>(means + (int64_t)e * D + d);
#pragma unroll
        for (int q = 0; q < TOK; ++q) {
            const int t = t0 + q < T ? t0 + q : T - 1;
            const uint4 xv = *reinterpret_cast<const uint4*>(X + (int64_t)t * D + d);
            const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const uint32_t mw[4] = {mv[e].x, mv[e].y, mv[e].z, mv[e].w};
                float a = acc[q][e];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    a = __builtin_fmaf(bf2f(xw[k] & 0xFFFFu), bf2f(mw[k] & 0xFFFFu), a);
                    a = __builtin_fmaf(bf2f(xw[k] >> 16), bf2f(mw[k] >> 16), a);
                }
                acc[q][e] = a;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < TOK; ++q) {
        float best = 0.0f;
        int arg = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float s = acc[q][e];
#pragma unroll
            for (int w = 32; w >= 1; w >>= 1) s = s + __shfl_xor(s, w, 64);     // both partners add the same two numbers
            if (e == 0 || s > best) { best = s; arg = e; }
            if (scores && lane == 0 && t0 + q < T) scores[(int64_t)(t0 + q) * E + e] = s;
        }
        if (lane == 0 && t0 + q < T) expert[t0 + q] = arg;
    }
}

// ---- stable grouping by expert ------------------------------------------------------------------------------------
// Pass 1: per block of 1024 tokens, how many go to each expert; also clears perm to -1 (padding).
__global__ void __launch_bounds__(256) venom_count_kernel(const int32_t* __restrict__ expert, int T, int E, int cap,
                                                         int32_t* __restrict__ blockcnt, int32_t* __restrict__ perm) {
    __shared__ int cnt[16];
    if (threadIdx.x < 16) cnt[threadIdx.x] = 0;
    __syncthreads();
    const int base = blockIdx.x * 1024;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int t = base + k * 256 + threadIdx.x;
        if (t < cap) perm[t] = -1;
        if (t < T) atomicAdd(&cnt[expert[t]], 1);            // integer counts: the result does not depend on the order
    }
    __syncthreads();
    if ((int)threadIdx.x < E) blockcnt[blockIdx.x * E + threadIdx.x] = cnt[threadIdx.x];
}

// Pass 2 (one workgroup): first row of every (block, expert) and the 64-row padded run offsets.
__global__ void __launch_bounds__(64) venom_scan_kernel(int32_t* __restrict__ blockcnt, int nblk, int E, int32_t* __restrict__ seg) {
    __shared__ int total[16];
    const int e = threadIdx.x;
    if (e < E) {
        int run = 0;
        for (int b = 0; b < nblk; ++b) {
            const int c = blockcnt[b * E + e];
            blockcnt[b * E + e] = run;                        // becomes: tokens of expert e in earlier blocks
            run += c;
        }
        total[e] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int off = 0;
        seg[0] = 0;
        for (int q = 0; q < E; ++q) { off += (total[q] + 63) & ~63; seg[q + 1] = off; }
    }
}

// Pass 3: every token's row = seg[e] + tokens of e in earlier blocks + rank among the block's earlier tokens of e.
__global__ void __launch_bounds__(256) venom_scatter_kernel(const int32_t* __restrict__ expert, int T, int E,
                                                           const int32_t* __restrict__ blockbase, const int32_t* __restrict__ seg,
                                                           int32_t* __restrict__ perm, int32_t* __restrict__ row_of_token) {
    __shared__ int run[16];
    __shared__ int wcnt[4][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)threadIdx.x < E) run[threadIdx.x] = seg[threadIdx.x] + blockbase[blockIdx.x * E + threadIdx.x];
    __syncthreads();
    const int base = blockIdx.x * 1024;
    for (int k = 0; k < 4; ++k) {
        const int t = base + k * 256 + threadIdx.x;
        const int e = t < T ? expert[t] : -1;
        int rank = 0;
        for (int q = 0; q < E; ++q) {                         // E <= 16 ballots: rank among the wave's earlier lanes of the same expert
            const unsigned long long m = __ballot(e == q);
            if (e == q) rank = __popcll(m & ((1ull << lane) - 1ull));
            if (lane == 0) wcnt[wave][q] = __popcll(m);
        }
        __syncthreads();
        if (e >= 0) {
            int r = run[e] + rank;
            for (int w = 0; w < wave; ++w) r += wcnt[w][e];
            perm[r] = t;
            row_of_token[t] = r;
        }
        __syncthreads();
        if ((int)threadIdx.x < E) run[threadIdx.x] += wcnt[0][threadIdx.x] + wcnt[1][threadIdx.x] + wcnt[2][threadIdx.x] + wcnt[3][threadIdx.x];
        __syncthreads();
    }
}

// X rows in permuted order (zero rows for padding), blocked operand layout: one thread per 16 bytes.
__global__ void __launch_bounds__(256) venom_gather_x_kernel(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm, int cap, int D,
                                                            uint16_t* __restrict__ xb) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int cpr = D >> 3;
    const int64_t r = idx / cpr;
    const int c = (int)(idx - r * cpr);
    if (r >= cap) return;
    const int t = perm[r];
    uint4 v = make_uint4(0, 0, 0, 0);
    if (t >= 0) v = *reinterpret_cast<const uint4*>(X + (int64_t)t * D + c * 8);
    *reinterpret_cast<uint4*>(xb + blk_off(r, c * 8, D >> 5)) = v;
}

// (vals [rows, Kc / 2], meta [rows, Kc / 8]) -> the dense transposed matrix at[j, r] ([Kc, rows], row-major), zeros at the
// dropped positions: the A operand of the weight-gradient contractions over each expert's run.  64 x 64 tiles through LDS.
__global__ void __launch_bounds__(256) venom_expand_t_compact_kernel(const uint16_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                                                                    int64_t rows, int Kc, uint16_t* __restrict__ at) {
    __shared__ uint16_t tile[64][64 + 2];           // [compact column][row]
    const int tid = threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * 64;
    const int j0 = blockIdx.x * 64;
    // 64 rows x 16 groups: thread -> (row = tid / 4 [+ 0], groups 4 (tid % 4) .. + 3)
    {
        const int rr = tid >> 2, g4 = (tid & 3) * 4;
        const uint4 v = *reinterpret_cast<const uint4*>(vals + (r0 + rr) * (Kc / 2) + (j0 / 2) + g4 * 2);      // 4 groups x 2 survivors
        const uint32_t mb = *reinterpret_cast<const uint16_t*>(meta + (r0 + rr) * (Kc / 8) + (j0 / 8) + g4 / 2);  // 4 nibbles
        const uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t nib = (mb >> (4 * g)) & 0xFu, p0 = nib & 3u, p1 = nib >> 2;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                tile[(g4 + g) * 4 + c][rr] = (uint16_t)((c == (int)p0) ? (vw[g] & 0xFFFFu) : (c == (int)p1) ? (vw[g] >> 16) : 0u);
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 256 * i, jj = e >> 3, seg8 = (e & 7) * 8;
        const uint32_t* p = reinterpret_cast<const uint32_t*>(&tile[jj][seg8]);
        *reinterpret_cast<uint4*>(at + (int64_t)(j0 + jj) * rows + r0 + seg8) = make_uint4(p[0], p[1], p[2], p[3]);
    }
}

// colidx[tb, g, :] = (4e, 4e + 1, 4e + 2, 4e + 3) for the 64-row blocks of expert e's run; blocks past the last run: e = 0.
__global__ void __launch_bounds__(256) venom_colidx_kernel(GemmGroup g, int nblocks, int groups, uint32_t* __restrict__ colidx) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)nblocks * groups) return;
    const int tb = (int)(idx / groups);
    int e = 0;
    for (int q = 0; q < g.n; ++q)
        if (tb * 64 >= (g.seg_dev ? g.seg_dev[q] : g.seg[q]) && tb * 64 < (g.seg_dev ? g.seg_dev[q + 1] : g.seg[q + 1])) e = q;
    colidx[idx] = 0x03020100u + 0x04040404u * (uint32_t)e;
}

// Padding rows past the last run: rows first .. rows - 1 of up to five [rows, row_words] arrays <- their fill words, in one
// launch.  `first` comes from the device (first_dev[0], the end of the last run) or as an immediate.
__global__ void __launch_bounds__(256) fill_tail_rows_kernel(TailFill f, const int32_t* __restrict__ first_dev, int first_imm, int64_t rows) {
    const int a = blockIdx.y;
    const int64_t first = first_dev ? first_dev[0] : first_imm;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x + first * f.row_words[a];
    if (i < rows * f.row_words[a]) f.p[a][i] = f.v[a];
}

hipError_t launch_fill_tail_rows(const TailFill& f, const int32_t* first_dev, int64_t first_imm, int64_t rows, int64_t max_tail_rows,
                                 hipStream_t s) {
    int64_t widest = 0;
    for (int a = 0; a < f.n; ++a) widest = f.row_words[a] > widest ? f.row_words[a] : widest;
    const int64_t n = max_tail_rows * widest;
    if (n == 0 || f.n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_tail_rows_kernel, dim3((unsigned)((n + 255) / 256), (unsigned)f.n), dim3(256), 0, s, f, first_dev, (int)first_imm, rows);
    return hipGetLastError();
}

hipError_t launch_venom_route(const uint16_t* X, const uint16_t* means, int64_t T, int64_t D, int E, int32_t* expert, float* scores,
                              hipStream_t s) {
    if (T == 0) return hipSuccess;
    // two tokens per wavefront: enough wavefronts in flight to hide the load latency (8 tokens per wavefront: 1.2-2.2 TB/s of X)
    constexpr int TOK = 2;
    dim3 grid((unsigned)((T + 4 * TOK - 1) / (4 * TOK)));
    switch (E) {
        case 2:  hipLaunchKernelGGL((venom_route_kernel<2, TOK>), grid, dim3(256), 0, s, X, means, (int)T, (int)D, expert, scores); break;
        case 4:  hipLaunchKernelGGL((venom_route_kernel<4, TOK>), grid, dim3(256), 0, s, X, means, (int)T, (int)D, expert, scores); break;
        case 8:  hipLaunchKernelGGL((venom_route_kernel<8, TOK>), grid, dim3(256), 0, s, X, means, (int)T, (int)D, expert, scores); break;
        case 16: hipLaunchKernelGGL((venom_route_kernel<16, 4>), dim3((unsigned)((T + 15) / 16)), dim3(256), 0, s, X, means, (int)T, (int)D, expert, scores); break;   // 16 experts: the means' L2 traffic weighs more
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_venom_permute(const int32_t* expert, int64_t T, int E, int64_t cap, int32_t* blockcnt, int32_t* seg, int32_t* perm,
                                int32_t* row_of_token, hipStream_t s) {
    const int nblk = (int)((cap + 1023) / 1024);
    hipLaunchKernelGGL(venom_count_kernel, dim3(nblk), dim3(256), 0, s, expert, (int)T, E, (int)cap, blockcnt, perm);
    hipLaunchKernelGGL(venom_scan_kernel, dim3(1), dim3(64), 0, s, blockcnt, nblk, E, seg);
    hipLaunchKernelGGL(venom_scatter_kernel, dim3(nblk), dim3(256), 0, s, expert, (int)T, E, blockcnt, seg, perm, row_of_token);
    return hipGetLastError();
}

hipError_t launch_venom_gather_x(const uint16_t* X, const int32_t* perm, int64_t cap, int64_t D, uint16_t* xb, hipStream_t s) {
    const int64_t n = cap * (D / 8);
    hipLaunchKernelGGL(venom_gather_x_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, X, perm, (int)cap, (int)D, xb);
    return hipGetLastError();
}

hipError_t launch_venom_expand_t_compact(const uint16_t* vals, const uint8_t* meta, int64_t rows, int64_t Kc, uint16_t* at, hipStream_t s) {
    dim3 grid((unsigned)(Kc / 64), (unsigned)(rows / 64));
    hipLaunchKernelGGL(venom_expand_t_compact_kernel, grid, dim3(256), 0, s, vals, meta, rows, (int)Kc, at);
    return hipGetLastError();
}

hipError_t launch_venom_colidx(const GemmGroup& g, int64_t cap, int64_t groups, uint8_t* colidx, hipStream_t s) {
    const int64_t n = (cap / 64) * groups;
    hipLaunchKernelGGL(venom_colidx_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, g, (int)(cap / 64), (int)groups,
                       reinterpret_cast<uint32_t*>(colidx));
    return hipGetLastError();
}

}  // namespace sffn
