// V:N:M activation x dense matrix with the dense operand's rows gathered per token block (eqs. (3), (7) of the paper
// for blocks of M >= 16 columns, the regime of Table 5; also the stand-alone vnm_spmm at M = 8 when Wk is given as is):
//     out[t, n] = sum_k' Ac[t, k'] * Wk[row(t / 64, k'), n],      row(tb, k') = (k' / 4) * M + colidx[tb, k' / 4, k' % 4]
// Ac = the packed activation read as a plain 2:4 matrix of logical width K' = 4 F / M (vals [T, K' / 2], meta
// [T, K' / 8], both row-major: exactly the canonical V:N:M arrays), Wk = [F, ldw] with the contraction index as row.
// Only the K' selected rows of Wk take part, so the matrix work and the operand traffic shrink with 4 / M; the
// plain-2:4 route of gemm_v2.hip contracts over all F instead.
//
// A workgroup owns one V = 64 token block (the unit that shares a column selection) x 256 output columns; 4 wavefronts,
// 64 x 64 each.  Per 64-k' stage it streams 64 gathered 512-byte row segments of Wk (LDS-DMA, two rows per wave-wide
// load; the per-lane source offset carries the row), the 64 x 32 packed values and their metadata.  The rows arrive
// k-major while v_smfmac_f32_32x32x32_bf16 wants 16 consecutive k per lane, so the B fragments are read with the
// LDS transpose read ds_read_b64_tr_b16: inside each group of 16 lanes, lane s supplies the address of 4 consecutive
// elements of row s / 4 (element chunk s % 4) and lane l receives element l of rows 0..3 (measured with an index
// pattern).  64-byte pieces of a row are XOR-swizzled by k' % 4 so that the four rows of one read hit disjoint banks.
// With 64-row tiles the kernel is bound by L2 -> LDS delivery, not by the matrix cores, and for large M a tile has
// only a few stages, so start-up and drain matter: the ring has 2 stages and the footprint is exactly 80 KB, which
// lets two workgroups share a CU and cover each other's prologue and epilogue (measured faster than one workgroup
// with a 4-stage ring at every M).  Workgroups of one XCD share a column slab of Wk and walk k' together.
#include "common.hpp"
#include "kernels.hpp"
#include "lds_dma.hpp"

namespace sffn {

namespace {

constexpr int kGStages = 2;
constexpr int kGB = 64 * 512, kGA = 64 * 64, kGM = 64 * 8;
constexpr int kGStage = kGB + kGA + kGM;               // 37376 bytes
constexpr int kGLoads = 8 + 1 + 1;                     // per wave per stage
constexpr int kGMaxKc = 7168;                          // column offsets of one token block kept in LDS (2 stages + this = 80 KB)

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

}  // namespace

__global__ void __launch_bounds__(256) vnm_spmm_gather_kernel(const uint16_t* __restrict__ a_vals, const uint8_t* __restrict__ a_meta,
                                                             const uint8_t* __restrict__ colidx, const uint16_t* __restrict__ Wk,
                                                             int ldw, int N, int Kc, int logM, int nblk_tok, int tiles_n,
                                                             uint16_t* __restrict__ out, int64_t ldo, GemmGroup grp) {
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kGStages * kGStage];
    __shared__ __attribute__((aligned(16))) unsigned char cix[kGMaxKc];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    // Consecutive workgroup ids go to different XCDs; give each XCD a run of consecutive logical ids, and let logical
    // ids walk the token blocks of one column slab, so an XCD's L2 holds one slab of Wk at a time.
    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    const int tn = L / nblk_tok, tb = L - tn * nblk_tok;
    const int t0 = tb * 64, n0 = tn * 256;
    if (grp.n) {                                         // grouped form: the token block's segment names the expert whose matrix it meets
        int e = 0;
        while (e + 1 < grp.n && t0 >= grp.seg[e + 1]) ++e;
        Wk += e * grp.b_stride;
    }

    // ---- column offsets of this token block -> LDS ------------------------------------------------------------
    {
        const uint4* src = reinterpret_cast<const uint4*>(colidx + (int64_t)tb * Kc);
        for (int i = tid; i < (Kc >> 4); i += 256) reinterpret_cast<uint4*>(cix)[i] = src[i];
    }
    __syncthreads();

    // ---- DMA sources ---------------------------------------------------------------------------------------------
    // B: load i of wave w (i = 0..7) brings rows k' = 2 (8 w + i) + lane / 32 of the stage; lane % 32 is the 16-byte
    // slot inside the row and fetches the chunk that the swizzle puts there (chunk ^ 4 (k' % 4)).  Chunks past the
    // right edge of Wk are redirected to the first 64 columns of the tile: they only feed outputs that are not stored.
    const uint64_t w_base = uniform64(Wk);
    uint32_t b_col[2];                                   // byte offset of the lane's chunk inside a row, for even / odd load index
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        int c = l32 ^ ((par * 2 + lh) << 2);
        if (n0 + c * 8 >= N) c &= 7;
        b_col[par] = (uint32_t)(n0 + c * 8) * 2;
    }
    const uint32_t row_bytes = (uint32_t)ldw * 2;
    // A (16 rows x 64 bytes per load, as in gemm_v2.hip) and metadata ([row][8 bytes]; waves 2, 3 repeat the loads of
    // waves 0, 1 so that every wave has the same number of loads in flight)
    const int lda = Kc >> 1;
    const uint64_t a_base = uniform64(a_vals + (int64_t)(t0 + 16 * wave) * lda);
    const uint64_t m_base = uniform64(a_meta + (int64_t)(t0 + 32 * (wave & 1)) * (Kc >> 3));
    uint32_t a_lane, m_lane;
    {
        const int rb = lane >> 2, c = (lane & 3) ^ ((rb >> 2) & 3);
        a_lane = (uint32_t)(rb * lda + c * 8) * 2;
        m_lane = (uint32_t)((lane >> 1) * (Kc >> 3) + (lane & 1) * 4);
    }
    // byte offsets of the gathered rows for the next refill, looked up ahead of the loads that use them
    uint32_t b_row[8];
    auto lookup = [&](int kt) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = kt * 64 + 2 * (8 * wave + i) + lh;
            b_row[i] = (uint32_t)(((k >> 2) << logM) + cix[k]) * row_bytes;
        }
    };
    auto issue = [&](int kt, int stage) {
        unsigned char* sb = smem + stage * kGStage;
        unsigned char* sa = sb + kGB;
        unsigned char* sm = sa + kGA;
#pragma unroll
        for (int i = 0; i < 8; ++i) dma16(w_base, b_row[i] + b_col[i & 1], sb + (8 * wave + i) * 1024);
        dma16(a_base, a_lane + (uint32_t)kt * 64, sa + wave * 1024);
        dma4(m_base, m_lane + (uint32_t)kt * 8, sm + (wave & 1) * 256);
    };

    // ---- fragment read offsets inside a stage ----------------------------------------------------------------------
    int a_off[2], m_off[2], b_off[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int row = a * 32 + l32;
        a_off[a] = kGB + row * 64 + ((lh ^ ((row >> 2) & 3)) << 4);
        m_off[a] = kGB + kGA + row * 8 + 2 * lh;
    }
    {
        // transpose read: lane supplies row r = (lane % 16) / 4 and 8-byte piece c = lane % 4 of its 16-lane group's
        // 16 columns; groups 0, 1 are the two column halves of the 32-wide fragment, groups 2, 3 the same for k + 8
        const int r = (lane & 15) >> 2, c = lane & 3, g = lane >> 4;
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
            b_off[fn] = (8 * (g >> 1) + r) * 512 + (((2 * wave + fn) ^ r) << 6) + ((g & 1) << 5) + (c << 3);
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    struct FragSet {
        Frag8 a[2];
        int idx[2];
        union { s16x4 q[4]; bf16x16 v; } b[2];
    };
    auto read_frags = [&](FragSet& f, const unsigned char* st, int ks) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            f.a[a].u = *reinterpret_cast<const uint4*>(st + (a_off[a] ^ (32 * ks)));
            f.idx[a] = *reinterpret_cast<const uint16_t*>(st + m_off[a] + 4 * ks);
        }
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int j = 0; j < 4; ++j)      // k rows 32 ks + 16 (j / 2) + 4 (j % 2) + (8 h + r): elements 4 j .. 4 j + 3 of the operand
                f.b[fn].q[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_s16x4*)(st + b_off[fn] + (32 * ks + 16 * (j >> 1) + 4 * (j & 1)) * 512));
    };
    auto mma = [&](const FragSet& f) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
                acc[a][fn] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[a].v, f.b[fn].v, acc[a][fn], f.idx[a], 0, 0);
    };
#define SB() __builtin_amdgcn_sched_barrier(0)

    const int nk = Kc >> 6;
#pragma unroll
    for (int p = 0; p < kGStages; ++p) {
        const int kt = p < nk ? p : nk - 1;
        lookup(kt);
        issue(kt, p);
    }
    wait_vmcnt<(kGStages - 1) * kGLoads>();
    __syncthreads();
    FragSet P, Q;
    read_frags(P, smem, 0);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int nxt = (kt + kGStages < nk) ? kt + kGStages : nk - 1;
        const int next_stage = (stage + 1 == kGStages) ? 0 : stage + 1;
        const unsigned char* st = smem + stage * kGStage;
        const unsigned char* sn = smem + next_stage * kGStage;
        lookup(nxt); SB();
        mma(P); SB();
        read_frags(Q, st, 1); SB();
        // Q has arrived and this wave's part of tile kt + 1 has landed; after the barrier every wave is done reading
        // this stage, which is refilled at once
        wait_vmcnt_lgkm0<(kGStages - 2) * kGLoads>();
        __builtin_amdgcn_s_barrier();
        SB();
        issue(nxt, stage); SB();
        mma(Q); SB();
        read_frags(P, sn, 0); SB();
        stage = next_stage;
    }
#undef SB
    wait_vmcnt<0>();
    __syncthreads();

    // ---- output: the wave's 64 x 64 tile goes through LDS as [t][n] so that HBM sees 128-byte row segments --------
    constexpr int EP = 64 * 2 + 16;
    unsigned char* scratch = smem + wave * (64 * EP);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                // registers r, r + 1 are rows t, t + 1 of the same column: one 16-bit LDS store each
                const int t = a * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const uint32_t pr = f2bf2(acc[a][fn][r], acc[a][fn][r + 1]);
                *reinterpret_cast<uint16_t*>(scratch + t * EP + (fn * 32 + l32) * 2) = (uint16_t)pr;
                *reinterpret_cast<uint16_t*>(scratch + (t + 1) * EP + (fn * 32 + l32) * 2) = (uint16_t)(pr >> 16);
            }
    wave_lds_sync();
    const int nw = n0 + 64 * wave;
    if (nw < N) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = p * 8 + (lane >> 3), ch = lane & 7;
            *reinterpret_cast<uint4*>(out + (int64_t)(t0 + row) * ldo + nw + ch * 8) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
        }
    }
}

// The same contraction on E4M3 codes (the fp8 step with blocks of M >= 16 columns): Ac = the survivors' codes [T, K' / 2] + the same
// metadata, Wq = codes [F, ldw bytes] with the contraction index as row, out = bf16(alpha * sum), alpha = the product of the two tensor scales.
// v_smfmac_f32_32x32x64_fp8_fp8 contracts 64 k' per instruction, so a stage holds 128 k' and occupies the same LDS as above: 128 gathered
// 256-byte row segments (four rows per wave-wide load), 64 x 64 bytes of codes, 64 x 16 bytes of metadata.  The B operand wants 16
// consecutive k' per lane and half (lds_dma.hpp); it is read with ds_read_b64_tr_b8: inside a group of 16 lanes, lane s supplies the address
// of 8 consecutive bytes of row s / 2 (piece s % 2) and lane l receives byte l of rows 0..7 (measured with an index pattern).  The 32-byte
// pieces of a row are XOR-swizzled by k' % 8, so the eight rows that the lower or upper 32 lanes read together cover all 64 banks once.
__global__ void __launch_bounds__(256) vnm_spmm_gather_fp8_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_meta,
                                                                 const uint8_t* __restrict__ colidx, const uint8_t* __restrict__ Wq,
                                                                 int ldw, int N, int Kc, int logM, int nblk_tok, int tiles_n, float alpha,
                                                                 uint16_t* __restrict__ out, int64_t ldo, GemmGroup grp) {
    constexpr int kB = 128 * 256, kA = 64 * 64, kMt = 64 * 16, kStage = kB + kA + kMt;      // 37888 bytes; two stages = 74 KB: two workgroups per CU
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kGStages * kStage];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;

    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    const int tn = L / nblk_tok, tb = L - tn * nblk_tok;
    const int t0 = tb * 64, n0 = tn * 256;
    if (grp.n) {
        int e = 0;
        while (e + 1 < grp.n && t0 >= grp.seg[e + 1]) ++e;
        Wq += e * grp.b_stride;
    }
    // column offsets of this token block: a wave's 32 rows of a stage are 8 consecutive blocks = 32 consecutive bytes, read as is (same address
    // in every lane) one stage ahead of the loads that use them
    const uint4* cix = reinterpret_cast<const uint4*>(colidx + (int64_t)tb * Kc + 32 * wave);

    // B: load i of wave w (i = 0..7) brings rows k' = 4 (8 w + i) + lane / 16 of the stage; lane % 16 is the 16-byte slot inside the row and
    // fetches the chunk whose 32-byte piece the swizzle puts there.  Chunks past the right edge of Wq are redirected into the first 64 columns.
    const uint64_t w_base = uniform64(Wq);
    uint32_t b_col[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int slot = lane & 15, k7 = 4 * par + (lane >> 4);
        int c = (((slot >> 1) ^ k7) << 1) | (slot & 1);
        if (n0 + c * 16 >= N) c &= 3;
        b_col[par] = (uint32_t)(n0 + c * 16);
    }
    const uint32_t row_bytes = (uint32_t)ldw;
    const int lda = Kc >> 1;                              // bytes per row of codes
    const uint64_t a_base = uniform64(a_codes + (int64_t)(t0 + 16 * wave) * lda);
    const uint64_t m_base = uniform64(a_meta + (int64_t)(t0 + 16 * wave) * (Kc >> 3));
    uint32_t a_lane, m_lane;
    {
        const int rb = lane >> 2, c = (lane & 3) ^ ((rb >> 2) & 3);
        a_lane = (uint32_t)(rb * lda + c * 16);
        m_lane = (uint32_t)(rb * (Kc >> 3) + (lane & 3) * 4);
    }
    uint4 cw[2];                                         // the 8 blocks' offsets of the stage to be issued next
    auto lookup = [&](int kt) {
        cw[0] = cix[kt * 8];
        cw[1] = cix[kt * 8 + 1];
    };
    const int bsh = (lane >> 4) * 8;                     // the lane's row inside a block of four
    auto issue = [&](int kt, int stage) {
        unsigned char* sb = smem + stage * kStage;
        unsigned char* sa = sb + kB;
        unsigned char* sm = sa + kA;
        const uint32_t w8[8] = {cw[0].x, cw[0].y, cw[0].z, cw[0].w, cw[1].x, cw[1].y, cw[1].z, cw[1].w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // row k' = 4 (32 kt + 8 w + i) + lane / 16 of the compact operand = row block * M + offset of the dense one
            const uint32_t row = (uint32_t)((kt * 32 + 8 * wave + i) << logM) + ((w8[i] >> bsh) & 0xFFu);
            dma16(w_base, row * row_bytes + b_col[i & 1], sb + (8 * wave + i) * 1024);
        }
        dma16(a_base, a_lane + (uint32_t)kt * 64, sa + wave * 1024);
        dma4(m_base, m_lane + (uint32_t)kt * 16, sm + wave * 256);
    };

    int a_off[2], m_off[2], b_off[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int row = a * 32 + l32;
        a_off[a] = kB + row * 64 + ((lh ^ ((row >> 2) & 3)) << 4);
        m_off[a] = kB + kA + row * 16 + 4 * lh;
    }
    {
        // transpose read: lane supplies row r = (lane % 16) / 2 and 8-byte piece c = lane % 2 of its 16-lane group's 16 columns; groups 0, 1
        // are the two column halves of the 32-wide fragment, groups 2, 3 the same for k' + 16
        const int r = (lane & 15) >> 1, c = lane & 1, g = lane >> 4;
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
            b_off[fn] = (16 * (g >> 1) + r) * 256 + (((2 * wave + fn) ^ r) << 5) + ((g & 1) << 4) + (c << 3);
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    typedef int v2i __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) v2i lds_v2i;
    struct FragSet {
        Frag8 a[2];
        int idx[2];
        union { v2i q[4]; i32x8 v; } b[2];
    };
    auto read_frags = [&](FragSet& f, const unsigned char* st, int ks) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            f.a[a].u = *reinterpret_cast<const uint4*>(st + (a_off[a] ^ (32 * ks)));
            f.idx[a] = *reinterpret_cast<const uint32_t*>(st + m_off[a] + 8 * ks);
        }
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int j = 0; j < 4; ++j)      // k' rows 64 ks + 32 (j / 2) + 8 (j % 2) + (16 h + r): bytes 8 j .. 8 j + 7 of the operand
                f.b[fn].q[j] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(st + b_off[fn] + (64 * ks + 32 * (j >> 1) + 8 * (j & 1)) * 256));
    };
    auto mma = [&](const FragSet& f) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
                acc[a][fn] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(f.a[a].q, f.b[fn].v, acc[a][fn], f.idx[a], 0, 0);
    };
#define SB() __builtin_amdgcn_sched_barrier(0)

    const int nk = Kc >> 7;
#pragma unroll
    for (int p = 0; p < kGStages; ++p) {
        const int kt = p < nk ? p : nk - 1;
        lookup(kt);
        issue(kt, p);
    }
    wait_vmcnt<(kGStages - 1) * kGLoads>();
    __syncthreads();
    FragSet P, Q;
    read_frags(P, smem, 0);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int nxt = (kt + kGStages < nk) ? kt + kGStages : nk - 1;
        const int next_stage = (stage + 1 == kGStages) ? 0 : stage + 1;
        const unsigned char* st = smem + stage * kStage;
        const unsigned char* sn = smem + next_stage * kStage;
        lookup(nxt); SB();
        mma(P); SB();
        read_frags(Q, st, 1); SB();
        wait_vmcnt_lgkm0<(kGStages - 2) * kGLoads>();
        __builtin_amdgcn_s_barrier();
        SB();
        issue(nxt, stage); SB();
        mma(Q); SB();
        read_frags(P, sn, 0); SB();
        stage = next_stage;
    }
#undef SB
    wait_vmcnt<0>();
    __syncthreads();

    constexpr int EP = 64 * 2 + 16;
    unsigned char* scratch = smem + wave * (64 * EP);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int fn = 0; fn < 2; ++fn)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const int t = a * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const uint32_t pr = f2bf2(acc[a][fn][r] * alpha, acc[a][fn][r + 1] * alpha);
                *reinterpret_cast<uint16_t*>(scratch + t * EP + (fn * 32 + l32) * 2) = (uint16_t)pr;
                *reinterpret_cast<uint16_t*>(scratch + (t + 1) * EP + (fn * 32 + l32) * 2) = (uint16_t)(pr >> 16);
            }
    wave_lds_sync();
    const int nw = n0 + 64 * wave;
    if (nw < N) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = p * 8 + (lane >> 3), ch = lane & 7;
            *reinterpret_cast<uint4*>(out + (int64_t)(t0 + row) * ldo + nw + ch * 8) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
        }
    }
}

bool vnm_spmm_gather_ok(int64_t T, int64_t N, int64_t F, int M) {
    const int64_t Kc = 4 * F / M;
    return M >= 8 && T % 64 == 0 && N % 64 == 0 && Kc % 64 == 0 && Kc <= kGMaxKc;
}

hipError_t launch_vnm_spmm_gather(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* colidx, const uint16_t* Wk, int64_t ldw,
                                  int64_t T, int64_t N, int64_t F, int M, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    if (!vnm_spmm_gather_ok(T, N, F, M) || ldw < N || F * ldw * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n && (g.role != 0 || g.seg_dev || g.n > GemmGroup::kMaxExperts)) return hipErrorInvalidValue;
    const int Kc = (int)(4 * F / M), logM = M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
    const int nblk_tok = (int)(T / 64), tiles_n = (int)((N + 255) / 256);
    hipLaunchKernelGGL(vnm_spmm_gather_kernel, dim3((unsigned)(nblk_tok * tiles_n)), dim3(256), 0, s, a_vals, a_meta, colidx, Wk, (int)ldw, (int)N,
                       Kc, logM, nblk_tok, tiles_n, out, ldo, g);
    return hipGetLastError();
}

bool vnm_spmm_gather_fp8_ok(int64_t T, int64_t N, int64_t F, int M) {
    const int64_t Kc = 4 * F / M;
    return M >= 8 && T % 64 == 0 && N % 64 == 0 && Kc % 128 == 0;
}

hipError_t launch_vnm_spmm_gather_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* colidx, const uint8_t* Wq, int64_t ldw, float alpha,
                                      int64_t T, int64_t N, int64_t F, int M, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    if (!vnm_spmm_gather_fp8_ok(T, N, F, M) || ldw < N || ldw % 16 != 0 || F * ldw >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n && (g.role != 0 || g.seg_dev || g.n > GemmGroup::kMaxExperts)) return hipErrorInvalidValue;
    const int Kc = (int)(4 * F / M), logM = M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
    const int nblk_tok = (int)(T / 64), tiles_n = (int)((N + 255) / 256);
    hipLaunchKernelGGL(vnm_spmm_gather_fp8_kernel, dim3((unsigned)(nblk_tok * tiles_n)), dim3(256), 0, s, a_codes, a_meta, colidx, Wq, (int)ldw, (int)N,
                       Kc, logM, nblk_tok, tiles_n, alpha, out, ldo, g);
    return hipGetLastError();
}

}  // namespace sffn
