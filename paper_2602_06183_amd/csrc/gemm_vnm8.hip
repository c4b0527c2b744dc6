// Eqs. (3), (7) of the paper for V:2:8 activations (V = 64, M = 8: the fused step's own format) without re-expressing the activation as a
// plain 2:4 matrix over all F columns:
//     out[t, n] = sum_k' Ac[t, k'] * Wk[row(t / 64, k'), n],      row(tb, k') = (k' / 4) * 8 + colidx[tb, k' / 4, k' % 4]
// Ac = the packed activation read as a 2:4 matrix of logical width K' = F / 2 (two survivors per four kept columns), Wk = [F, ldw]
// with the contraction index as row (W2.T for eq. (3), W1 as it is for eq. (7)).  The plain-2:4 route of gemm_v2.hip issues one
// structured-sparse matrix instruction per 32 columns of F; this kernel issues one per 64, and fetches half the activation bytes.
//
// Tile: 256 tokens x 256 output columns, 8 wavefronts as 4 (token blocks) x 2 (column halves).  A 64-row tile (the
// gathered-row kernel of gemm_gather.hip, which fetches only the kept rows) halves the reuse of Wk and is bound by L2 -> LDS delivery at
// M = 8; here the whole [64 f x 256 n] slab of Wk of a stage goes to LDS once for the tile's four token blocks, and each token block picks
// its kept rows when it READS its B fragments: ds_read_b64_tr_b16 takes one address per lane (inside a group of 16 lanes, lane s supplies 4
// consecutive elements of row s / 4, lane l receives element l of those 4 rows), so the 4 rows of a read are the 4 kept hidden units of
// one column block.  The 64-byte pieces of a slab row are XOR-swizzled by f % 8: the four rows of a read lie in one group of 8 rows and
// therefore in four different pieces.
//
// Operands as the fused epilogues of eqs. (1), (4) write them (common.hpp: vcb_off, mcb_off, cixt_off):
//   values    [T / 32][F / 64][32 tokens][16 values]   1 KB per (32 tokens, 64 hidden units): one wave-wide LDS-DMA load
//   metadata  [T / 64][F / 64][64 tokens][4 bytes]     the canonical nibbles of the 8 column blocks of a stage
//   offsets   [F / 64][T / 64][8 words]                word (h, r), byte j = kept column r of column block 4 (j / 2) + j % 2 + 2 h of the
//                                                      stage: the four rows that lane (h = lane / 32, r = (lane % 16) / 4) addresses in read j
// A stage = 64 hidden units = 32 k' = one matrix instruction step per fragment pair; 3 stages of 41.25 KB.
//
// FP8 (the fp8 step): the same kernel on E4M3 codes with v_smfmac_f32_32x32x64_fp8_fp8, out = bf16(alpha * sum).  A stage is 128 hidden
// units = 64 k' (the instruction's K): the slab is 128 rows x 256 bytes, the survivors' codes fill the same 32 bytes per token and stage,
// the metadata 8 bytes.  The B fragments are read with ds_read_b64_tr_b8 (inside a group of 16 lanes, lane s supplies 8 consecutive bytes of
// row s / 2, lane l receives byte l of those 8 rows), so a read covers the kept rows of TWO column blocks; the offsets unit of a (128 hidden
// units, token block) is 16 words: word (h, p), byte j = kept column p % 4 of column block 8 (j / 2) + 4 h + 2 (j % 2) + p / 4.  The 32-byte
// pieces of a slab row are swizzled by f % 8.
#include "common.hpp"
#include "kernels.hpp"
#include "lds_dma.hpp"

// Tile rows per band of the workgroup -> tile map (see SFFN_TILE_GROUP in common.hpp).  A tile fetches four times as many bytes of Wk as of
// the packed activation, so the 32 tiles that an XCD runs at a time should share few column slabs of Wk: tall bands (measured at
// T = D = 8192, F = 28672: 1.49 / 1.42 / 1.38 / 1.36 ms per launch with 2 / 4 / 8 / 16 tile rows per band).
#ifndef SFFN_VNM8_GROUP
#define SFFN_VNM8_GROUP 16
#endif

namespace sffn {

namespace {

constexpr int kStages = 3;
template <bool FP8>
struct G {
    static constexpr int SLAB = FP8 ? 128 : 64;         // hidden units per stage
    static constexpr int kB = 64 * 512;                 // slab bytes (64 x 512 or 128 x 256)
    static constexpr int kA = 256 * 32;
    static constexpr int kMt = FP8 ? 256 * 8 : 256 * 4;
    static constexpr int kC = 256;
    static constexpr int kStage = kB + kA + kMt + kC;   // 42240 / 43264 bytes
};
constexpr int kLoads = 4 + 1 + 1 + 1;                // per wave per stage
// Measurement switches (wrong results by design): SFFN_VNM8_NO_MFMA leaves the matrix instructions out, SFFN_VNM8_NO_DMA the loads after the
// prologue, SFFN_VNM8_NO_BREAD the transposing reads of the B fragments.

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef int v2i __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) v2i lds_v2i;

}  // namespace

// Wk / ldw: bf16 elements, or (FP8) code bytes
template <bool FP8>
__global__ void __launch_bounds__(512) vnm8_gemm_kernel(const uint16_t* __restrict__ vcb, const uint8_t* __restrict__ mcb,
                                                       const uint8_t* __restrict__ cixt, const uint8_t* __restrict__ Wk, int ldw,
                                                       int Ra, int N, int F, int Ttot, uint16_t* __restrict__ out, int64_t ldo,
                                                       int tiles_m, int tiles_n, GemmGroup grp, float alpha) {
    constexpr int kB = G<FP8>::kB, kA = G<FP8>::kA, kMt = G<FP8>::kMt, kStage = G<FP8>::kStage;
    constexpr int ES = FP8 ? 1 : 2;                      // bytes per element of Wk
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kStages * kStage];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    // Grouped form (role 0): the token tiles of segment e meet expert e's matrix
    int i_base = 0;
    if (grp.n) {
        int e = 0, cnt = 0;
        for (; e < grp.n; ++e) {
            cnt = ((grp.seg[e + 1] - grp.seg[e] + 255) >> 8) * tiles_n;
            if (L < cnt) break;
            L -= cnt;
        }
        if (e == grp.n) return;
        tiles_m = cnt / tiles_n; i_base = grp.seg[e]; Ra = grp.seg[e + 1];
        Wk += (int64_t)e * grp.b_stride * ES;
    }
    int tm, tn;
    {
        constexpr int GROUP = SFFN_VNM8_GROUP;
        const int width = GROUP * tiles_n, group = L / width, first = group * GROUP;
        const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
        tm = first + (L % width) % gsz;
        tn = (L % width) / gsz;
    }
    const int i0 = i_base + tm * 256, n0 = tn * 256;
    const int KS = F / G<FP8>::SLAB;                     // stages = slabs of 64 (128) hidden units
    const int NTB = Ttot >> 6;

    // ---- DMA sources (wave-uniform 64-bit base + 32-bit per-lane offset).  Token groups past the end of the operand are clamped into it:
    //      they only feed outputs that are never stored. ----------------------------------------------------------------------------------
    // B: load i of wave w (i = 0..3) brings slab rows 2 (4 w + i) + lane / 32; lane % 32 is the 16-byte slot inside the 512-byte row and
    // fetches the chunk whose 64-byte piece the swizzle puts there (FP8: rows 4 (4 w + i) + lane / 16 of 256 bytes, 32-byte pieces).
    // Chunks past the right edge of Wk are redirected into the first 64 columns.
    const uint64_t w_base = uniform64(Wk);
    uint32_t b_lane[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (FP8) {
            const int row = 4 * (4 * wave + i) + (lane >> 4), slot = lane & 15;
            int c = (((slot >> 1) ^ (row & 7)) << 1) | (slot & 1);
            if (n0 + c * 16 >= N) c &= 3;
            b_lane[i] = (uint32_t)row * (uint32_t)ldw + (uint32_t)(n0 + c * 16);
        } else {
            const int row = 2 * (4 * wave + i) + lh, slot = l32;
            int c = (((slot >> 2) ^ (row & 7)) << 2) | (slot & 3);
            if (n0 + c * 8 >= N) c &= 7;
            b_lane[i] = (uint32_t)row * (uint32_t)ldw * 2u + (uint32_t)(n0 + c * 8) * 2u;
        }
    }
    const uint32_t b_kstep = (uint32_t)G<FP8>::SLAB * (uint32_t)ldw * ES;
    uint64_t a_base, m_base, c_base;
    uint32_t a_lane, m_lane, c_lane;
    {
        int g32 = (i0 >> 5) + wave;                      // the wave's 32 tokens of the tile
        g32 = g32 < (Ttot >> 5) ? g32 : (Ttot >> 5) - 1;
        a_base = uniform64(vcb + (int64_t)g32 * KS * 512);
        const int row = lane >> 1, slot = lane & 1;
        a_lane = (uint32_t)(row * 32 + ((slot ^ ((row >> 3) & 1)) << 4));
        if (FP8) {          // 8 bytes per token and stage: the wave's own 32 tokens, 256 bytes of the 512-byte unit of their token block
            int g64 = (i0 >> 6) + (wave >> 1);
            g64 = g64 < NTB ? g64 : NTB - 1;
            m_base = uniform64(mcb + (int64_t)g64 * KS * 512 + (wave & 1) * 256);
        } else {            // 4 bytes: waves w and w + 4 fetch the same 64 tokens' metadata
            int g64 = (i0 >> 6) + (wave & 3);
            g64 = g64 < NTB ? g64 : NTB - 1;
            m_base = uniform64(mcb + (int64_t)g64 * KS * 256);
        }
        m_lane = lane * 4;
        // offsets of the tile's four token blocks: 4 x 32 (FP8: 4 x 64) bytes, every wave fetches all of them
        const int words = FP8 ? 16 : 8;
        int tb = (i0 >> 6) + (FP8 ? (lane >> 4) : (l32 >> 3));
        tb = tb < NTB ? tb : NTB - 1;
        c_base = uniform64(cixt);
        c_lane = (uint32_t)(tb * words * 4 + (lane & (words - 1)) * 4);
    }
    const uint32_t c_kstep = (uint32_t)NTB * (FP8 ? 64u : 32u);
    constexpr uint32_t m_kstep = FP8 ? 512u : 256u;
    auto issue_half = [&](int kt, int stage, int h) {
#ifdef SFFN_VNM8_NO_DMA
        if (kt >= kStages) return;
#endif
        unsigned char* sb = smem + stage * kStage;
        unsigned char* sa = sb + kB;
        unsigned char* sm = sa + kA;
        unsigned char* sc = sm + kMt;
        if (h == 0) {
            dma16(w_base, b_lane[0] + (uint32_t)kt * b_kstep, sb + (4 * wave + 0) * 1024);
            dma16(w_base, b_lane[1] + (uint32_t)kt * b_kstep, sb + (4 * wave + 1) * 1024);
            dma16(a_base, a_lane + (uint32_t)kt * 1024u, sa + wave * 1024);
            dma4(c_base, c_lane + (uint32_t)kt * c_kstep, sc);
        } else {
            dma16(w_base, b_lane[2] + (uint32_t)kt * b_kstep, sb + (4 * wave + 2) * 1024);
            dma16(w_base, b_lane[3] + (uint32_t)kt * b_kstep, sb + (4 * wave + 3) * 1024);
            dma4(m_base, m_lane + (uint32_t)kt * m_kstep, sm + (FP8 ? wave : (wave & 3)) * 256);
        }
    };
    auto issue = [&](int kt, int stage) { issue_half(kt, stage, 0); issue_half(kt, stage, 1); };

    // ---- per-lane LDS offsets of the fragment reads (inside a stage).  A wave owns one token block (64 tokens) x 128 output columns: its two
    //      A fragments are read by one other wave only, and the four B fragments it gathers belong to one column selection. ----------------------
    const int tbw = wave >> 1, nh = wave & 1;
    int a_off[2], m_off[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int row = tbw * 64 + a * 32 + l32;
        a_off[a] = kB + row * 32 + ((lh ^ ((row >> 3) & 1)) << 4);
        m_off[a] = kB + kA + (FP8 ? row * 8 + 4 * lh : row * 4 + 2 * lh);
    }
    // bf16: transpose read j of fragment fn: slab row = 8 cb(j) + c with cb(j) = 4 (j / 2) + j % 2 + 2 h and c = byte j of the lane's offsets
    // word; byte address = row * 512 + ((4 nh + fn) ^ c) * 64 + 32 (column half) + 8 (lane % 4)
    // FP8: the lane addresses row p = (lane % 16) / 2 of the read's 8: cb(j) = 8 (j / 2) + 4 h + 2 (j % 2) + p / 4, c = byte j of word (h, p);
    // byte address = row * 256 + ((4 nh + fn) ^ c) * 32 + 16 (column half) + 8 (lane % 2)
    const int r4 = (lane & 15) >> 2, p8 = (lane & 15) >> 1, g = lane >> 4;
    const int c_off = kB + kA + kMt + (FP8 ? 64 * tbw + (lh * 8 + p8) * 4 : 32 * tbw + (lh * 4 + r4) * 4);
    const int b_fix = FP8 ? ((g & 1) << 4) + ((lane & 1) << 3) : ((g & 1) << 5) + ((lane & 3) << 3);
    int b_cb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        b_cb[j] = FP8 ? (8 * (j >> 1) + 4 * lh + 2 * (j & 1) + (p8 >> 2)) * 8 * 256 + b_fix : (4 * (j >> 1) + (j & 1) + 2 * lh) * 8 * 512 + b_fix;

    f32x16 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    // The stage's fragments in two halves: P = both A fragments, the offsets word and B fragments 0, 1; Q = B fragments 2, 3 (the A
    // fragments of P stay live until Q's matrix instructions, so A is double-buffered by stage parity)
    struct BPair { union { s16x4 q[4]; v2i q8[4]; bf16x16 v; i32x8 v8; } b[2]; };
    struct AFrags { Frag8 a[2]; int idx[2]; uint32_t cw; };
    auto read_a = [&](AFrags& f, const unsigned char* st) {
        f.cw = *reinterpret_cast<const uint32_t*>(st + c_off);
#pragma unroll
        for (int a2 = 0; a2 < 2; ++a2) {
            f.a[a2].u = *reinterpret_cast<const uint4*>(st + a_off[a2]);
            f.idx[a2] = FP8 ? (int)*reinterpret_cast<const uint32_t*>(st + m_off[a2]) : (int)*reinterpret_cast<const uint16_t*>(st + m_off[a2]);
        }
    };
    auto read_b = [&](BPair& f, const unsigned char* st, uint32_t cw, int half) {
#ifdef SFFN_VNM8_NO_BREAD
        f.b[0].q[0][0] = (short)cw; f.b[1].q[0][0] = (short)(cw >> 16);
        return;
#endif
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t c = (cw >> (8 * j)) & 7u;
            if (FP8) {
                const uint32_t addr = (uint32_t)b_cb[j] + c * 256u + (((4u * nh + 2u * half) ^ c) << 5);
                f.b[0].q8[j] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(st + addr));
                f.b[1].q8[j] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(st + (addr ^ 32u)));
            } else {
                const uint32_t addr = (uint32_t)b_cb[j] + c * 512u + (((4u * nh + 2u * half) ^ c) << 6);
                f.b[0].q[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(st + addr));
                f.b[1].q[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(st + (addr ^ 64u)));
            }
        }
    };
    auto mma_half = [&](const AFrags& fa, const BPair& fb, int half) {
#ifdef SFFN_VNM8_NO_MFMA
        acc[0][2 * half][0] += __builtin_bit_cast(float, fa.a[0].u.x) + __builtin_bit_cast(float, fa.a[1].u.x) + (float)fb.b[0].q[0][0] + (float)fb.b[1].q[3][3] + (float)fa.idx[0] + (float)fa.idx[1];
        return;
#endif
#pragma unroll
        for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
                if (FP8) acc[a2][2 * half + fn] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(fa.a[a2].q, fb.b[fn].v8, acc[a2][2 * half + fn], fa.idx[a2], 0, 0);
                else     acc[a2][2 * half + fn] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(fa.a[a2].v, fb.b[fn].v, acc[a2][2 * half + fn], fa.idx[a2], 0, 0);
    };
#define SB() __builtin_amdgcn_sched_barrier(0)

    const int nk = KS;
#pragma unroll
    for (int p = 0; p < kStages; ++p) issue(p < nk ? p : nk - 1, p);
    wait_vmcnt<(kStages - 1) * kLoads>();
    __syncthreads();
    AFrags A0, A1;
    BPair P, Q;
    read_a(A0, smem);
    read_b(P, smem, A0.cw, 0);
    int stage = 0;
    // two stages per trip so that the A fragment buffers alternate without copies
    auto step = [&](int kt, AFrags& cur, AFrags& nxt_a) {
        const int nxt = (kt + kStages < nk) ? kt + kStages : nk - 1;
        const int next_stage = (stage + 1 == kStages) ? 0 : stage + 1;
        const unsigned char* st = smem + stage * kStage;
        const unsigned char* sn = smem + next_stage * kStage;
        mma_half(cur, P, 0); SB();
        read_b(Q, st, cur.cw, 1); SB();
        // Q has arrived and this wave's part of tile kt + 1 has landed; after the barrier every wave is done reading this stage, which is
        // refilled at once
        wait_vmcnt_lgkm0<(kStages - 2) * kLoads>();
        __builtin_amdgcn_s_barrier();
        SB();
        issue_half(nxt, stage, 0); SB();
        read_a(nxt_a, sn); SB();
        mma_half(cur, Q, 1); SB();
        issue_half(nxt, stage, 1); SB();
        read_b(P, sn, nxt_a.cw, 0); SB();
        stage = next_stage;
    };
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        step(kt, A0, A1);
        step(kt + 1, A1, A0);
    }
    if (kt < nk) step(kt, A0, A1);
#undef SB
    wait_vmcnt<0>();
    __syncthreads();

    // ---- output: the wave's 32 x 64 sub-tiles go through LDS as [t][n] so that HBM sees 128-byte row segments -----------------------------
    constexpr int EP = 64 * 2 + 16;
    unsigned char* scratch = smem + wave * (32 * EP);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
                    *reinterpret_cast<uint16_t*>(scratch + row * EP + (b * 32 + l32) * 2) = (uint16_t)f2bf(FP8 ? acc[a][2 * half + b][r] * alpha : acc[a][2 * half + b][r]);
                }
            wave_lds_sync();
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int e = lane + 64 * p, row = e >> 3, ch = e & 7;
                const int i = i0 + tbw * 64 + a * 32 + row, j = n0 + nh * 128 + half * 64 + ch * 8;
                if (i < Ra && j < N) *reinterpret_cast<uint4*>(out + (int64_t)i * ldo + j) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
            }
            wave_lds_sync();
        }
}

bool vnm8_gemm_ok(int64_t T, int64_t N, int64_t F, int64_t ldw) {
    // (32-bit offsets inside the kernel: the dense operand and the offsets array stay below 2 GiB, so every offset is also a non-negative int)
    return T > 0 && T % 64 == 0 && N > 0 && N % 64 == 0 && F > 0 && F % 64 == 0 && ldw >= N && ldw % 8 == 0 && F * ldw * 2 < ((int64_t)1 << 31) &&
           T * F < ((int64_t)1 << 38);
}
bool vnm8_gemm_fp8_ok(int64_t T, int64_t N, int64_t F, int64_t ldw) {
    return T > 0 && T % 64 == 0 && N > 0 && N % 64 == 0 && F > 0 && F % 128 == 0 && ldw >= N && ldw % 16 == 0 && F * ldw < ((int64_t)1 << 31) &&
           T * F < ((int64_t)1 << 38);
}

template <bool FP8>
static hipError_t launch_impl(const uint16_t* vcb, const uint8_t* mcb, const uint8_t* cixt, const uint8_t* Wk, int64_t ldw, float alpha, int64_t T,
                              int64_t N, int64_t F, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n && (g.role != 0 || g.seg_dev || g.n > GemmGroup::kMaxExperts)) return hipErrorInvalidValue;
    const int tiles_m = (int)((T + 255) / 256), tiles_n = (int)((N + 255) / 256);
    int tiles = tiles_m * tiles_n;
    if (g.n) {
        tiles = 0;
        for (int e = 0; e < g.n; ++e) tiles += (g.seg[e + 1] - g.seg[e] + 255) / 256 * tiles_n;
    }
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL((vnm8_gemm_kernel<FP8>), dim3((unsigned)tiles), dim3(512), 0, s, vcb, mcb, cixt, Wk, (int)ldw, (int)T, (int)N, (int)F, (int)T, out,
                       ldo, tiles_m, tiles_n, g, alpha);
    return hipGetLastError();
}

hipError_t launch_vnm8_gemm(const uint16_t* vcb, const uint8_t* mcb, const uint8_t* cixt, const uint16_t* Wk, int64_t ldw, int64_t T, int64_t N,
                            int64_t F, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    if (!vnm8_gemm_ok(T, N, F, ldw)) return hipErrorInvalidValue;
    return launch_impl<false>(vcb, mcb, cixt, reinterpret_cast<const uint8_t*>(Wk), ldw, 1.0f, T, N, F, out, ldo, s, grp);
}

hipError_t launch_vnm8_gemm_fp8(const uint8_t* vcb, const uint8_t* mcb, const uint8_t* cixt, const uint8_t* Wq, int64_t ldw, float alpha, int64_t T,
                                int64_t N, int64_t F, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    if (!vnm8_gemm_fp8_ok(T, N, F, ldw)) return hipErrorInvalidValue;
    return launch_impl<true>(reinterpret_cast<const uint16_t*>(vcb), mcb, cixt, Wq, ldw, alpha, T, N, F, out, ldo, s, grp);
}

}  // namespace sffn
