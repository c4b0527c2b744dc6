// The six contractions of the sparsified FFN step (paper eqs. (1), (3), (4), (5), (7), (8)) as one
// tiled kernel family: C[i, j] = sum_k A[i, k] * B[j, k], both operands K-contiguous in HBM.
//   SPARSE: A is a 2:4 packed matrix and the products run on the gfx950 structured-sparse matrix
//           cores (v_smfmac_f32_32x32x32_bf16: A holds the 16 survivors of 32 k per row plus a
//           2-bit position per survivor; B is dense).
//   dense : v_mfma_f32_32x32x16_bf16.
// Register layouts used below (measured on gfx950 with one-hot operands):
//   smfmac 32x32x32  A: lane l -> row l%32, survivors 8*(l/32)..+7 of the 16 (k in 16*(l/32)..+15),
//                       index VGPR bits [2e+1:2e] = position of survivor e inside its group of 4;
//                    B: lane l -> column l%32; elements 0-7 = k 8*(l/32)..+7, elements 8-15 = k 16+8*(l/32)..+7;
//                    D: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32.
//   mfma 32x32x16    A, B: lane l -> row/column l%32, k 8*(l/32)..+7;  D as above.
// The 2-bit positions are exactly the packed format's metadata nibbles, so metadata bytes go from
// HBM to the index VGPR without re-encoding.
#include "common.hpp"
#include "kernels.hpp"

namespace sffn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;

union Frag8 { uint4 u; bf16x8 v; };
union Frag16 { uint4 u[2]; bf16x16 v; };

constexpr int BK = 64;            // k per main-loop step
constexpr int DPITCH = 144;       // LDS row pitch of a dense 64-k row (128 B + 16 B: conflict-free b128 reads)
constexpr int SPITCH = 80;        // LDS row pitch of a packed 64-k row (64 B + 16 B)

template <bool SPARSE, int BM, int BN>
struct Smem {
    static constexpr int A_BYTES = BM * (SPARSE ? SPITCH : DPITCH);
    static constexpr int META_BYTES = SPARSE ? BM * 8 : 0;
    static constexpr int B_BYTES = BN * DPITCH;
    static constexpr int STAGE = A_BYTES + META_BYTES + B_BYTES;
};

template <bool SPARSE, int BM, int BN, bool OUT_I_CONTIG>
__global__ void __launch_bounds__(256) gemm_nt_kernel(const uint16_t* __restrict__ a_vals, const uint8_t* __restrict__ a_meta,
                                                     const uint16_t* __restrict__ B, const float* __restrict__ bias,
                                                     int Ra, int Rb, int K, uint16_t* __restrict__ out, int64_t ldo,
                                                     int tiles_m, int tiles_n) {
    using S = Smem<SPARSE, BM, BN>;
    constexpr int WM = BM / 2, WN = BN / 2, FM = WM / 32, FN = WN / 32;
    constexpr int A_PASSES = SPARSE ? BM / 64 : BM / 32;
    constexpr int B_PASSES = BN / 32;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * S::STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    // workgroup -> tile: consecutive ids of one XCD (ids are dealt round-robin over the 8 XCDs) walk
    // down a band of 8 tile rows, so an XCD's L2 sees few distinct operand panels at a time.
    int tm, tn;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        const int L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
        constexpr int GROUP = 8;
        const int width = GROUP * tiles_n, group = L / width, first = group * GROUP;
        const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
        tm = first + (L % width) % gsz;
        tn = (L % width) / gsz;
    }
    const int i0 = tm * BM, j0 = tn * BN;
    const int lda = SPARSE ? K / 2 : K;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    uint4 ga[A_PASSES], gb[B_PASSES];
    uint2 gm = make_uint2(0, 0);

    auto load_global = [&](int kt) {
        if (SPARSE) {
#pragma unroll
            for (int p = 0; p < A_PASSES; ++p) {
                const int row = (tid >> 2) + 64 * p, seg = tid & 3;
                ga[p] = make_uint4(0, 0, 0, 0);
                if (i0 + row < Ra) ga[p] = *reinterpret_cast<const uint4*>(a_vals + (int64_t)(i0 + row) * lda + kt * 32 + seg * 8);
            }
            gm = make_uint2(0x44444444u, 0x44444444u);
            if (tid < BM && i0 + tid < Ra) gm = *reinterpret_cast<const uint2*>(a_meta + (int64_t)(i0 + tid) * (K / 8) + kt * 8);
        } else {
#pragma unroll
            for (int p = 0; p < A_PASSES; ++p) {
                const int row = (tid >> 3) + 32 * p, seg = tid & 7;
                ga[p] = make_uint4(0, 0, 0, 0);
                if (i0 + row < Ra) ga[p] = *reinterpret_cast<const uint4*>(a_vals + (int64_t)(i0 + row) * lda + kt * 64 + seg * 8);
            }
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int row = (tid >> 3) + 32 * p, seg = tid & 7;
            gb[p] = make_uint4(0, 0, 0, 0);
            if (j0 + row < Rb) gb[p] = *reinterpret_cast<const uint4*>(B + (int64_t)(j0 + row) * K + kt * 64 + seg * 8);
        }
    };
    auto store_lds = [&](int buf) {
        unsigned char* sa = smem + buf * S::STAGE;
        unsigned char* sm = sa + S::A_BYTES;
        unsigned char* sb = sm + S::META_BYTES;
        if (SPARSE) {
#pragma unroll
            for (int p = 0; p < A_PASSES; ++p) {
                const int row = (tid >> 2) + 64 * p, seg = tid & 3;
                *reinterpret_cast<uint4*>(sa + row * SPITCH + seg * 16) = ga[p];
            }
            if (tid < BM) *reinterpret_cast<uint2*>(sm + tid * 8) = gm;
        } else {
#pragma unroll
            for (int p = 0; p < A_PASSES; ++p) {
                const int row = (tid >> 3) + 32 * p, seg = tid & 7;
                *reinterpret_cast<uint4*>(sa + row * DPITCH + seg * 16) = ga[p];
            }
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int row = (tid >> 3) + 32 * p, seg = tid & 7;
            *reinterpret_cast<uint4*>(sb + row * DPITCH + seg * 16) = gb[p];
        }
    };
    auto compute = [&](int buf) {
        const unsigned char* sa = smem + buf * S::STAGE;
        const unsigned char* sm = sa + S::A_BYTES;
        const unsigned char* sb = sm + S::META_BYTES;
        if (SPARSE) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                Frag8 fa[FM];
                int idx[FM];
                Frag16 fb[FN];
#pragma unroll
                for (int a = 0; a < FM; ++a) {
                    const int row = wm * WM + a * 32 + l32;
                    fa[a].u = *reinterpret_cast<const uint4*>(sa + row * SPITCH + 32 * ks + 16 * lh);
                    idx[a] = *reinterpret_cast<const uint16_t*>(sm + row * 8 + 4 * ks + 2 * lh);
                }
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                    const int row = wn * WN + b * 32 + l32;
                    fb[b].u[0] = *reinterpret_cast<const uint4*>(sb + row * DPITCH + 64 * ks + 16 * lh);
                    fb[b].u[1] = *reinterpret_cast<const uint4*>(sb + row * DPITCH + 64 * ks + 16 * lh + 32);
                }
#pragma unroll
                for (int a = 0; a < FM; ++a)
#pragma unroll
                    for (int b = 0; b < FN; ++b)
                        acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(fa[a].v, fb[b].v, acc[a][b], idx[a], 0, 0);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                Frag8 fa[FM], fb[FN];
#pragma unroll
                for (int a = 0; a < FM; ++a) {
                    const int row = wm * WM + a * 32 + l32;
                    fa[a].u = *reinterpret_cast<const uint4*>(sa + row * DPITCH + 32 * ks + 16 * lh);
                }
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                    const int row = wn * WN + b * 32 + l32;
                    fb[b].u = *reinterpret_cast<const uint4*>(sb + row * DPITCH + 32 * ks + 16 * lh);
                }
#pragma unroll
                for (int a = 0; a < FM; ++a)
#pragma unroll
                    for (int b = 0; b < FN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a].v, fb[b].v, acc[a][b], 0, 0, 0);
            }
        }
    };

    const int nk = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_global(kt + 1);
        compute(kt & 1);
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    if (OUT_I_CONTIG) {
        // a lane owns 4 consecutive i for one j: 8-byte stores, bias indexed by i
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int b = 0; b < FN; ++b) {
                const int j = j0 + wn * WN + b * 32 + l32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int i = i0 + wm * WM + a * 32 + 8 * g + 4 * lh;
                    if (j < Rb && i < Ra) {
                        float v0 = acc[a][b][4 * g], v1 = acc[a][b][4 * g + 1], v2 = acc[a][b][4 * g + 2], v3 = acc[a][b][4 * g + 3];
                        if (bias) { const float4 bb = *reinterpret_cast<const float4*>(bias + i); v0 += bb.x; v1 += bb.y; v2 += bb.z; v3 += bb.w; }
                        *reinterpret_cast<uint2*>(out + (int64_t)j * ldo + i) = make_uint2(f2bf(v0) | (f2bf(v1) << 16), f2bf(v2) | (f2bf(v3) << 16));
                    }
                }
            }
    } else {
        // j is the contiguous output axis: transpose each 32-row slab of the wave tile through LDS
        constexpr int EP = WN * 2 + 16;
        unsigned char* scratch = smem + wave * (32 * EP);
        static_assert(4 * 32 * EP <= 2 * S::STAGE, "epilogue scratch must fit in the main-loop LDS");
#pragma unroll
        for (int a = 0; a < FM; ++a) {
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
                    *reinterpret_cast<uint16_t*>(scratch + row * EP + (b * 32 + l32) * 2) = (uint16_t)f2bf(acc[a][b][r]);
                }
            __syncthreads();
            constexpr int CH = WN / 8;                  // 16-byte chunks per row
#pragma unroll
            for (int p = 0; p < 32 * CH / 64; ++p) {
                const int e = lane + 64 * p, row = e / CH, ch = e % CH;
                const int i = i0 + wm * WM + a * 32 + row, j = j0 + wn * WN + ch * 8;
                if (i < Ra && j < Rb)
                    *reinterpret_cast<uint4*>(out + (int64_t)i * ldo + j) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
            }
            __syncthreads();
        }
    }
}

template <bool SPARSE, int BM, int BN>
static hipError_t launch_one(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t Ra,
                             int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s) {
    const int tiles_m = (int)((Ra + BM - 1) / BM), tiles_n = (int)((Rb + BN - 1) / BN);
    dim3 grid((unsigned)(tiles_m * tiles_n));
    if (out_i_contig)
        hipLaunchKernelGGL((gemm_nt_kernel<SPARSE, BM, BN, true>), grid, dim3(256), 0, s, a_vals, a_meta, B, bias, (int)Ra, (int)Rb,
                           (int)K, out, ldo, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((gemm_nt_kernel<SPARSE, BM, BN, false>), grid, dim3(256), 0, s, a_vals, a_meta, B, bias, (int)Ra, (int)Rb,
                           (int)K, out, ldo, tiles_m, tiles_n);
    return hipGetLastError();
}

int g_tile_sparse = 4, g_tile_dense = 4;   // 0: 128x128, 1: 256x128, 2: 128x256, 3: 256x256 (BM x BN), 4: pipelined 256x256

hipError_t launch_gemm_nt_v2(int sparse_a, const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias,
                             int64_t Ra, int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s);

hipError_t launch_gemm_nt(int sparse_a, const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias,
                          int64_t Ra, int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s) {
    if ((sparse_a ? g_tile_sparse : g_tile_dense) == 4)
        return launch_gemm_nt_v2(sparse_a, a_vals, a_meta, B, bias, Ra, Rb, K, out_i_contig, out, ldo, s);
#define GO(SP, BM, BN) return launch_one<SP, BM, BN>(a_vals, a_meta, B, bias, Ra, Rb, K, out_i_contig, out, ldo, s)
    if (sparse_a) {
        switch (g_tile_sparse) { case 1: GO(true, 256, 128); case 2: GO(true, 128, 256); case 3: GO(true, 256, 256); default: GO(true, 128, 128); }
    }
    switch (g_tile_dense) { case 1: GO(false, 256, 128); case 2: GO(false, 128, 256); case 3: GO(false, 256, 256); default: GO(false, 128, 128); }
#undef GO
}

}  // namespace sffn
