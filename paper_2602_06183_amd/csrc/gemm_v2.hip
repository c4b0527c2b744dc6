// Pipelined tile kernel: C[i, j] = sum_k A[i, k] * B[j, k] with a 256 x 256 workgroup tile, 8 wavefronts
// (2 along i x 4 along j, 128 x 64 each, two wavefronts per SIMD so one hides the other's LDS latency), operand
// tiles streamed HBM -> LDS with global_load_lds_dwordx4 into a ring of LDS stages (no register staging),
// XOR-swizzled 16-byte chunks so that the b128 fragment reads are bank-conflict free without padding.
//   SPARSE: A packed 2:4 -> v_smfmac_f32_32x32x32_bf16; ring of 3 stages of 64 k (50 KB each).  Eqs. (1), (3), (4), (7):
//           in the fused step on blocked operands (eqs. (1), (4) with the V:N:M epilogue), stand-alone on row-major ones.
//   dense : v_mfma_f32_32x32x16_bf16; ring of 4 stages of 32 k (32 KB each); row-major operands only (stand-alone
//           vnm_wgrad; the fused step's weight gradients have their own kernel, gemm_wgrad.hip).
// Register layouts of the two instructions are documented in lds_dma.hpp.
#include "common.hpp"
#include "kernels.hpp"
#include "lds_dma.hpp"

namespace sffn {

namespace {

// FP8 (structured-sparse kernel): both operands are 1-byte E4M3 codes, row-major (stand-alone entry points) or blocked with a pair
// of codes per 2-byte element (fused fp8 step); the metadata is row-major [R, K/8] for row-major operands and in 512-byte units
// (m8blk_off, common.hpp) for blocked ones: 16-byte row pieces fetched one by one cost 17 % of eq. (3) at the 70B-scale layer.  In BYTES the tiles are those of
// the bf16 kernel (a stage is 128 k instead of 64: 64 survivor bytes per A row, 128 bytes per B row, and the fragment a lane of
// v_smfmac_f32_32x32x64_fp8_fp8 wants is the same 16 / 2 x 16 bytes), so the kernel runs with K counted in byte pairs and only
// the metadata differs: 16 survivors per lane and step need a whole 32-bit index word, 16 bytes per row and stage.
// Measurement switches (never set in the shipped build; results are wrong with the last two): -DSFFN_SPARSE_NSTAGE=2 shortens the
// structured-sparse kernel's ring, -DSFFN_LOOP_NO_MFMA drops the matrix instructions of its blocked main loop (operand delivery alone),
// -DSFFN_LOOP_NO_DMA drops the loads after the prologue (matrix pipe, fragment reads and barriers alone).
#ifndef SFFN_SPARSE_NSTAGE
#define SFFN_SPARSE_NSTAGE 3
#endif
template <bool SPARSE, bool FP8 = false>
struct Cfg {
    static constexpr int BM = 256, BN = 256;
    static constexpr int BK = SPARSE ? 64 : 32;
    static constexpr int NSTAGE = SPARSE ? SFFN_SPARSE_NSTAGE : 4;
    static constexpr int A_ROW = 64;                        // bytes per A row per stage (32 survivors or 32 dense k)
    static constexpr int B_ROW = SPARSE ? 128 : 64;
    static constexpr int META_ROW = FP8 ? 16 : 8;
    static constexpr int A_BYTES = BM * A_ROW, B_BYTES = BN * B_ROW, META_BYTES = SPARSE ? BM * META_ROW : 0;
    static constexpr int STAGE = A_BYTES + B_BYTES + META_BYTES;
    static constexpr int LOADS = (A_BYTES + B_BYTES) / 1024 / 8 + (SPARSE ? (FP8 ? 2 : 1) : 0);   // per wave per stage
};

}  // namespace

// bf16 bits -> max(y, 0)^2 rounded to bf16 (RNE), returned as the fp32 bit pattern (low half zero).
// r * r is never NaN here (a NaN input fails the comparison and becomes 0), so no NaN path is needed.
__device__ __forceinline__ uint32_t sqrelu16(uint32_t y) {
    const float f = bf2f(y), r = f > 0.0f ? f : 0.0f;
    return f2bf(r * r);
}
__device__ __forceinline__ uint32_t sqrelu_hi(uint32_t y) { return sqrelu16(y) << 16; }
template <bool SPARSE, bool OUT_I_CONTIG, int EPI, bool BLOCKED, bool FP8 = false>
__global__ void __launch_bounds__(512) gemm_nt_v2_kernel(const uint16_t* __restrict__ a_vals, const uint8_t* __restrict__ a_meta,
                                                        const uint16_t* __restrict__ B, const float* __restrict__ bias,
                                                        int Ra, int Rb, int K, uint16_t* __restrict__ out, int64_t ldo,
                                                        int tiles_m, int tiles_n, VnmEpilogue ep, GemmGroup grp, float alpha = 1.0f) {
    static_assert(EPI == 0 || (SPARSE && OUT_I_CONTIG && BLOCKED), "the V:N:M epilogues belong to the 2:4-weight GEMMs of the fused step");
    // EPI 16 + log2(M) / 32 + log2(M): the forward (eq. (2) + compression) / backward (eq. (6)) epilogue for blocks of M = 16, 32, 64 columns
    constexpr bool GEN_F = EPI >= 16 && EPI < 32, GEN_B = EPI >= 32;
    constexpr int LOGM = (GEN_F || GEN_B) ? (EPI & 15) : 3;
    static_assert(!(GEN_F || GEN_B) || (LOGM >= 4 && LOGM <= 6), "wide V:N:M blocks: M = 16, 32 or 64");
    static_assert(!FP8 || (SPARSE && (EPI == 0 || (BLOCKED && (EPI == 1 || EPI == 2 || GEN_F || GEN_B)))), "fp8 operands: structured-sparse kernel; the step's fused epilogues");
    constexpr bool blocked = BLOCKED;       // operands in the blocked layout of common.hpp (fused step) or row-major (stand-alone entry points)
    using C = Cfg<SPARSE, FP8>;
    constexpr int BM = C::BM, BN = C::BN, WM = 128, WN = 64, FM = 4, FN = 2;
    constexpr int EPI_LDS = (EPI != 0) ? 8 * (64 + 32) * (64 * 2 + 16) : 0;        // the epilogues' scratch (see below) when the ring is shorter
    __shared__ __attribute__((aligned(1024))) unsigned char smem[C::NSTAGE * C::STAGE > EPI_LDS ? C::NSTAGE * C::STAGE : EPI_LDS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: everything derived from it stays in SGPRs
    const int wm = wave >> 2, wn = wave & 3;
    const int l32 = lane & 31, lh = lane >> 5;

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs; the remap gives each XCD a run of
    // consecutive logical ids, and logical ids walk bands of 4 tile rows, so an XCD's L2 sees few operand panels.
    int L;
    {
        const int n = gridDim.x, pid = blockIdx.x, per = n >> 3;
        L = (pid < per * 8) ? (pid & 7) * per + (pid >> 3) : pid;
    }
    // Grouped form: find the expert of this tile and narrow the problem to its token segment.
    const int Kld = K;                   // K extent of the stored operands (block-row stride)
#define SEG(i) (grp.seg_dev ? grp.seg_dev[i] : grp.seg[i])
    const int tok_ld = grp.n ? SEG(grp.n) : Rb;       // tokens in the token-indexed outputs of the V:N:M epilogue
    int i_base = 0, j_base = 0;
    int expert_id = 0;
    if (!SPARSE && !BLOCKED && grp.n && grp.role == 2) {
        // every expert has its own tiles_m x tiles_n output and contracts over its own k range of the shared operands
        const int per = tiles_m * tiles_n;
        expert_id = L / per;
        L -= expert_id * per;
        if (expert_id >= grp.n) return;
        const int k0 = SEG(expert_id);
        K = SEG(expert_id + 1) - k0;
        a_vals += k0; B += k0;
        out += expert_id * grp.out_stride;
    } else if (grp.n) {
        int e = 0;
        {
            const int other = grp.role == 0 ? tiles_n : tiles_m;
            int cnt = 0;
            for (; e < grp.n; ++e) {
                cnt = ((SEG(e + 1) - SEG(e) + 255) >> 8) * other;
                if (L < cnt) break;
                L -= cnt;
            }
            if (e == grp.n) return;      // (the launcher sizes the grid exactly; kept as a guard)
            if (grp.role == 0) { tiles_m = cnt / other; i_base = SEG(e); Ra = SEG(e + 1); }
            else               { tiles_n = cnt / other; j_base = SEG(e); Rb = SEG(e + 1); }
#undef SEG
        }
        if (grp.role != 0) { a_vals += e * grp.a_stride; if (SPARSE) a_meta += e * grp.m_stride; }
        if (grp.role != 1) B += e * grp.b_stride;
        if (bias) bias += e * grp.bias_stride;
        out += e * grp.out_stride;
    }
    int tm, tn;
    {
        constexpr int GROUP = SFFN_TILE_GROUP;
        const int width = GROUP * tiles_n, group = L / width, first = group * GROUP;
        const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
        tm = first + (L % width) % gsz;
        tn = (L % width) / gsz;
    }
    const int i0 = i_base + tm * BM, j0 = j_base + tn * BN;
    const int lda = SPARSE ? Kld / 2 : Kld;

    // ---- per-lane source addresses of the DMA loads.  A wave-wide load fills 1 KB of LDS = 16 tile rows x
    //      64 bytes; lane l lands at (row l / 4, 16-byte chunk l % 4) and therefore fetches the chunk that the
    //      XOR swizzle assigns to that slot.  Row-major sources: 16 row segments per load; blocked sources
    //      (common.hpp): the 16 rows x 64 bytes are one contiguous block.  Tile rows past the matrix edge
    //      are clamped into it: they only feed outputs that are never stored. --------------------------
    constexpr int A_LD = C::A_BYTES / 1024 / 8;          // dma16 issues per wave for A
    constexpr int B_LD = C::B_BYTES / 1024 / 8;
    // Row-major operands of the sparse kernel: a B row's 64 k of a stage are one 128-byte line, fetched whole (8 rows per
    // load, tile [256][128 bytes], 16-byte chunks swizzled by (row / 2) % 8) rather than as two 64-byte halves.
    constexpr bool lineB = SPARSE && !BLOCKED;
    uint64_t a_base[A_LD], b_base[B_LD], m_base = 0;     // wave-uniform byte addresses of kt = 0
    uint32_t a_lane, b_lane, b_lane1 = 0, m_lane;        // per-lane byte offsets (b_lane1: odd loads of the line layout)
    uint32_t a_kstep, b_kstep, m_kstep;                  // bytes per main-loop step
    {
        const int rb = lane >> 2;                                        // row inside the 16-row group
        const int c = (lane & 3) ^ ((rb >> 2) & 3);                      // source chunk for this lane's LDS slot
        const int KCa = SPARSE ? Kld / 64 : Kld / 32, KCb = Kld / 32;    // 32-element chunks per row
#pragma unroll
        for (int n = 0; n < A_LD; ++n) {
            int gr = i0 + (wave * A_LD + n) * 16; gr = gr < Ra ? gr : Ra - 16;
            a_base[n] = uniform64(blocked ? a_vals + ((int64_t)(gr >> 4) * KCa << 9) : a_vals + (int64_t)gr * lda);
        }
#pragma unroll
        for (int n = 0; n < B_LD; ++n) {
            // SPARSE: a stage holds 64 k of B as two half-tiles (k 0-31, k 32-63), each laid out like the A tile
            const int bk = wave * B_LD + n, h = SPARSE ? (bk >> 4) : 0;
            int gr = j0 + (bk & 15) * 16; gr = gr < Rb ? gr : Rb - 16;
            if (lineB) { gr = j0 + bk * 8; gr = gr < Rb ? gr : Rb - 8; }
            b_base[n] = uniform64(blocked ? B + (((int64_t)(gr >> 4) * KCb + h) << 9) : lineB ? B + (int64_t)gr * Kld : B + (int64_t)gr * Kld + h * 32);
        }
        a_lane = blocked ? (rb * 32 + c * 8) * 2 : (uint32_t)(rb * lda + c * 8) * 2;
        b_lane = blocked ? (rb * 32 + c * 8) * 2 : (uint32_t)(rb * Kld + c * 8) * 2;
        if (lineB) {        // lane -> (row lane / 8 of the load's 8 rows, slot lane % 8); tile row = 8 * load + row, load parity = n % 2
            const int r8 = lane >> 3, slot = lane & 7;
            b_lane = (uint32_t)(r8 * Kld + ((slot ^ (r8 >> 1)) * 8)) * 2;
            b_lane1 = (uint32_t)(r8 * Kld + ((slot ^ (4 + (r8 >> 1))) * 8)) * 2;
        }
        // metadata: one 4-byte-per-lane load brings 32 rows x 64 k; blocked: one unit of common.hpp, lane-linear;
        // row-major: lane -> (row lane / 2, 4-byte half lane % 2), landing as [row][8 bytes]
        m_lane = blocked ? lane * 4 : (uint32_t)((lane >> 1) * (Kld / 8) + (lane & 1) * 4);
        // fp8: a row has Kld / 4 metadata bytes, 16 per stage; one load brings 16 rows (lane -> row lane / 4, word lane % 4), two per wave
        if (FP8) m_lane = (uint32_t)((lane >> 2) * (Kld / 4) + (lane & 3) * 4);
        if (SPARSE) {
            int gr = i0 + wave * 32; gr = gr < Ra ? gr : Ra - 32;
            m_base = uniform64(FP8 ? a_meta + (int64_t)gr * (Kld / 4) : blocked ? a_meta + ((int64_t)(gr >> 5) * (Kld / 64) << 8) : a_meta + (int64_t)gr * (Kld / 8));
        }
        a_kstep = blocked ? 1024 : 64;
        b_kstep = blocked ? 1024 * (C::BK / 32) : C::BK * 2;
        m_kstep = (blocked && !FP8) ? 256 : C::META_ROW;
        if (FP8 && blocked) {       // fp8 metadata units of common.hpp (m8blk_off): 512 contiguous bytes per (32 rows, 128 k), row-major inside
            m_lane = lane * 4; m_kstep = 512;
            int gr = i0 + wave * 32; gr = gr < Ra ? gr : Ra - 32;
            m_base = uniform64(a_meta + (int64_t)(gr >> 5) * (Kld / 64) * 512);
        }
    }
    // the DMA loads of one stage, issued in two halves (h = 0, 1) so that they can sit between matrix instructions
    auto issue_half = [&](int kt, int stage, int h) {
#ifdef SFFN_LOOP_NO_DMA
        if (SPARSE && BLOCKED && kt >= C::NSTAGE) return;
#endif
        unsigned char* sa = smem + stage * C::STAGE;
        unsigned char* sb = sa + C::A_BYTES;
        unsigned char* sm = sb + C::B_BYTES;
        // the k position goes into the 32-bit per-lane offset (one vector add per operand); the bases stay put in SGPRs
        if (h == 0) {
            const uint32_t ao = a_lane + (uint32_t)kt * a_kstep, bo = b_lane + (uint32_t)kt * b_kstep, bo1 = b_lane1 + (uint32_t)kt * b_kstep;
#pragma unroll
            for (int n = 0; n < A_LD; ++n) dma16(a_base[n], ao, sa + (wave * A_LD + n) * 1024);
#pragma unroll
            for (int n = 0; n < B_LD / 2; ++n) dma16(b_base[n], (lineB && (n & 1)) ? bo1 : bo, sb + (wave * B_LD + n) * 1024);
        } else {
            const uint32_t bo = b_lane + (uint32_t)kt * b_kstep, bo1 = b_lane1 + (uint32_t)kt * b_kstep;
#pragma unroll
            for (int n = B_LD / 2; n < B_LD; ++n) dma16(b_base[n], (lineB && (n & 1)) ? bo1 : bo, sb + (wave * B_LD + n) * 1024);
            if (SPARSE && !FP8) dma4(m_base, m_lane + (uint32_t)kt * m_kstep, sm + wave * 256);
            if (FP8) {
                dma4(m_base, m_lane + (uint32_t)kt * m_kstep, sm + wave * 512);
                // second half of the wave's 32 rows: the next 256 bytes of a blocked unit, or 16 rows further down a row-major array
                dma4(m_base, m_lane + (blocked ? 256u : (uint32_t)(16 * (Kld / 4))) + (uint32_t)kt * m_kstep, sm + wave * 512 + 256);
            }
        }
    };
    auto issue = [&](int kt, int stage) { issue_half(kt, stage, 0); issue_half(kt, stage, 1); };

    // ---- per-lane LDS offsets of the fragment reads (inside a stage) --------------------------------
    int a_off[FM], b_off[FN], m_off[FM];
#pragma unroll
    for (int a = 0; a < FM; ++a) {
        const int row = wm * WM + a * 32 + l32;
        a_off[a] = row * 64 + ((lh ^ ((row >> 2) & 3)) << 4);
        // blocked: the lane's word of unit row / 32 holds both 32-k steps (picked by ABID); row-major: [row][8 bytes]
        m_off[a] = C::A_BYTES + C::B_BYTES + (FP8 ? row * 16 + 4 * lh : blocked ? (row >> 5) * 256 + lane * 4 : row * 8 + 2 * lh);
    }
#pragma unroll
    for (int b = 0; b < FN; ++b) {
        const int row = wn * WN + b * 32 + l32;
        b_off[b] = C::A_BYTES + row * 64 + ((lh ^ ((row >> 2) & 3)) << 4);      // SPARSE: + 16 KB for the second k half
        if (lineB) b_off[b] = C::A_BYTES + row * 128 + ((lh ^ ((row >> 1) & 7)) << 4);   // chunk = 4 ks + 2 u + lh
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

    // Fragment sets: P feeds the first half of a stage's k range, Q the second.  Reads of one set are
    // issued while the matrix cores work on the other, so LDS latency stays behind MFMA time.
    struct FragSet {
        Frag8 a[FM];
        int idx[FM];
        Frag16 b16[FN];     // SPARSE: 16 k-values per lane
        Frag8 b8[FN];       // dense: 8 k-values per lane
    };
    // `prev` = the set that holds the first 32-k step of the same tile (its index word serves both steps)
    auto read_a = [&](FragSet& f, const FragSet& prev, const unsigned char* st, int ks, int a) {
        f.a[a].u = *reinterpret_cast<const uint4*>(st + (a_off[a] ^ (32 * ks)));
        if (SPARSE) {
            if (FP8) f.idx[a] = *reinterpret_cast<const uint32_t*>(st + m_off[a] + 8 * ks);
            else if (!blocked) f.idx[a] = *reinterpret_cast<const uint16_t*>(st + m_off[a] + 4 * ks);
            else if (ks == 0) f.idx[a] = *reinterpret_cast<const uint32_t*>(st + m_off[a]);
            else f.idx[a] = prev.idx[a];
        }
    };
    auto read_b = [&](FragSet& f, const unsigned char* st, int ks, int b) {
        if (lineB) {
            f.b16[b].u[0] = *reinterpret_cast<const uint4*>(st + (b_off[b] ^ (64 * ks)));
            f.b16[b].u[1] = *reinterpret_cast<const uint4*>(st + (b_off[b] ^ (64 * ks + 32)));
        } else if (SPARSE) {
            f.b16[b].u[0] = *reinterpret_cast<const uint4*>(st + b_off[b] + 16384 * ks);
            f.b16[b].u[1] = *reinterpret_cast<const uint4*>(st + (b_off[b] ^ 32) + 16384 * ks);
        } else {
            f.b8[b].u = *reinterpret_cast<const uint4*>(st + (b_off[b] ^ (32 * ks)));
        }
    };
    auto read_frags = [&](FragSet& f, int stage, int ks) {
        const unsigned char* st = smem + stage * C::STAGE;
#pragma unroll
        for (int a = 0; a < FM; ++a) read_a(f, f, st, ks, a);
#pragma unroll
        for (int b = 0; b < FN; ++b) read_b(f, st, ks, b);
    };
    // second = the set holds the second 32-k step of its tile: blocked metadata then sits in the high half of the index word
    auto mma_row = [&](const FragSet& f, int a, bool second) {
#ifdef SFFN_LOOP_NO_MFMA
        if (SPARSE && BLOCKED) { acc[a][0][0] += __builtin_bit_cast(float, f.a[a].u.x) + __builtin_bit_cast(float, f.b16[a & 1].u[0].x); return; }
#endif
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            if (FP8)                    acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(f.a[a].q, f.b16[b].q, acc[a][b], f.idx[a], 0, 0);
            else if (!SPARSE)           acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[a].v, f.b8[b].v, acc[a][b], 0, 0, 0);
            else if (blocked && second) acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[a].v, f.b16[b].v, acc[a][b], f.idx[a], 0, 1);
            else                        acc[a][b] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[a].v, f.b16[b].v, acc[a][b], f.idx[a], 0, 0);
        }
    };
#define SB() __builtin_amdgcn_sched_barrier(0)

    const int nk = K / C::BK;            // 0 for an expert without tokens (weight gradients): the output is zeros
    if (nk > 0) {
    // The ring holds NSTAGE tiles: the one being multiplied, the next one (landed by the middle of the step,
    // when its first fragments are read) and NSTAGE - 2 in flight.  A stage is refilled right after the
    // barrier that ends its last fragment reads, so a tile has almost NSTAGE - 1 steps to arrive.
#pragma unroll
    for (int p = 0; p < C::NSTAGE; ++p) issue(p < nk ? p : nk - 1, p);
    wait_vmcnt<(C::NSTAGE - 1) * C::LOADS>();
    __syncthreads();
    FragSet P, Q;
    read_frags(P, 0, 0);
    int stage = 0;
    // One step = two halves of eight matrix instructions.  Each pair of matrix instructions (64+ cycles of
    // the matrix pipe) is followed in program order by a few LDS reads for the other fragment set or by
    // half of a stage's DMA issue, so the non-matrix work of a wave hides behind its own MFMAs.
    for (int kt = 0; kt < nk; ++kt) {
        const int nxt = (kt + C::NSTAGE < nk) ? kt + C::NSTAGE : nk - 1;
        const int next_stage = (stage + 1 == C::NSTAGE) ? 0 : stage + 1;
        const unsigned char* st = smem + stage * C::STAGE;
        const unsigned char* sn = smem + next_stage * C::STAGE;
        mma_row(P, 0, false); SB();
        read_a(Q, P, st, 1, 0); read_a(Q, P, st, 1, 1); read_b(Q, st, 1, 0); SB();
        mma_row(P, 1, false); SB();
        read_a(Q, P, st, 1, 2); read_a(Q, P, st, 1, 3); read_b(Q, st, 1, 1); SB();
        mma_row(P, 2, false); SB();
        mma_row(P, 3, false); SB();
        // Q has arrived and tile kt+1 has landed (this wave's part); after the barrier every wave is done
        // reading this stage, which is refilled at once, and every wave's part of tile kt+1 is in LDS
        wait_vmcnt_lgkm0<(C::NSTAGE - 2) * C::LOADS>();
        __builtin_amdgcn_s_barrier();
        SB();
        mma_row(Q, 0, true); SB();
        issue_half(nxt, stage, 0); SB();
        read_a(P, P, sn, 0, 0); read_a(P, P, sn, 0, 1); read_b(P, sn, 0, 0); SB();
        mma_row(Q, 1, true); SB();
        issue_half(nxt, stage, 1); SB();
        read_a(P, P, sn, 0, 2); read_a(P, P, sn, 0, 3); read_b(P, sn, 0, 1); SB();
        mma_row(Q, 2, true); SB();
        mma_row(Q, 3, true); SB();
        stage = next_stage;
    }
#undef SB
    wait_vmcnt<0>();
    }
    __syncthreads();

    if (OUT_I_CONTIG) {
        // i is the contiguous output axis and a lane owns 4 consecutive i of one j.  Stage the wave's tile
        // through LDS as [j][i] (two halves of 64 i) so that HBM sees 128-byte row segments instead of
        // 16-byte ones; the bias (indexed by i) is added before the single rounding to bf16.
        constexpr int EP = 64 * 2 + 16;
        // EPI: second tile (32 compact rows) for the transposed output
        constexpr int WAVE_LDS = (EPI != 0) ? (WN + 32) * EP : WN * EP;
        unsigned char* scratch = smem + wave * WAVE_LDS;
        static_assert(8 * WAVE_LDS <= sizeof(smem), "epilogue scratch must fit in the main-loop LDS");
        unsigned char* ttile = scratch + WN * EP;
        // EPI: i = hidden unit f, j = token t; the wave's 64 tokens are exactly one V = 64 block and each half of
        // 64 f holds 8 whole column blocks, so the V:N:M work is wave-local.
        const int t0 = j0 + wn * WN;
        const int nblk = Ra >> 3;
        const int64_t F = Ra;
        uint32_t nib_h0 = 0;                                  // M = 64: the metadata nibble of the first half waits for the second's
        // The lane's 32 bias values of each half, and (EPI 2) the saved column offsets, metadata and y1 of its 8 sweeps: all fetched here, for
        // both halves.  Loads and stores share one in-order counter, so a load issued after the first half's stores would wait for all of them
        // (and for its own latency) in the middle of the epilogue.
        float4 bb_all[2][2][4];
        uint32_t pre_cw[2] = {0x03020100u, 0x03020100u}, pre_m_all[2][8], pre_y_all[2][8];
        const uint32_t amax_seen = (FP8 && EPI != 0) ? amax_slot_peek(ep.amax) : 0u;
        float vmax_tile = 0.0f;                                 // fp8: largest survivor magnitude of the wave's tile
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int f0 = i0 + wm * WM + h * 64;
#pragma unroll
            for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bb_all[h][a2][g] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (bias) {
                        int i = f0 + a2 * 32 + 8 * g + 4 * lh; i = i < Ra ? i : Ra - 4;
                        // EPI 3: compact column i of the expert is hidden unit (i / 4) * M + 4 e + i % 4 (bias already points at 4 e)
                        bb_all[h][a2][g] = *reinterpret_cast<const float4*>(EPI == 3 ? bias + ((int64_t)(i >> 2) << ep.logM) : bias + i);
                    }
                }
            if (EPI == 2 && t0 < Rb && f0 < Ra) {
                const int64_t blk = (f0 >> 3) + (lane & 7);
                pre_cw[h] = *reinterpret_cast<const uint32_t*>(ep.colidx + ((int64_t)(t0 >> 6) * nblk + blk) * 4);
                const uint32_t* kp = reinterpret_cast<const uint32_t*>(ep.ykept) + ykept_off(t0 + (lane >> 3), blk, F);
                const uint8_t* mp = ep.meta + (int64_t)(t0 + (lane >> 3)) * (F / 16) + (blk >> 1);
#pragma unroll
                for (int it = 0; it < 8; ++it) {
                    pre_m_all[h][it] = mp[(int64_t)it * 8 * (F / 16)];
                    pre_y_all[h][it] = kp[it * 64];
                }
            }
        }
        // (the same for the backward epilogue of the wide blocks)
        constexpr int GNB = (GEN_F || GEN_B) ? (64 >> LOGM) : 1;
        uint32_t gpre_cb[2] = {0x03020100u, 0x03020100u}, gpre_m[2][GNB], gpre_y[2][GNB];
        if (GEN_B) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int f0 = i0 + wm * WM + h * 64;
                if (t0 < Rb && f0 < Ra) {
                    const int b = lane & (GNB - 1), r_lane = lane >> (6 - LOGM);
                    const int64_t blk = (f0 >> LOGM) + b;
                    gpre_cb[h] = *reinterpret_cast<const uint32_t*>(ep.colidx + ((int64_t)(t0 >> 6) * (F >> LOGM) + blk) * 4);
                    const uint32_t* kp = reinterpret_cast<const uint32_t*>(ep.ykept) + ((((int64_t)(t0 >> 6) * (F >> 6) + (f0 >> 6)) << 6) + r_lane) * GNB + b;
                    const uint8_t* mp = ep.meta + (int64_t)(t0 + r_lane) * (F >> (LOGM + 1)) + (blk >> 1);
#pragma unroll
                    for (int sw = 0; sw < GNB; ++sw) {
                        gpre_m[h][sw] = mp[(int64_t)sw * (1 << LOGM) * (F >> (LOGM + 1))];
                        gpre_y[h][sw] = kp[sw * (1 << LOGM) * GNB];
                    }
                }
            }
        }
        bool tok_ok[FN];                                       // EPI 3: padding rows of the permuted token order come out as zeros
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            tok_ok[b] = true;
            if (EPI == 3) { int j = t0 + b * 32 + l32; j = j < Rb ? j : Rb - 1; tok_ok[b] = ep.perm[j] >= 0; }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int f0 = i0 + wm * WM + h * 64;
            const bool valid = t0 < Rb && f0 < Ra;
            float4 (&bb)[2][4] = bb_all[h];
#pragma unroll
            for (int a2 = 0; a2 < 2; ++a2)
#pragma unroll
                for (int b = 0; b < FN; ++b)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int a = 2 * h + a2;
                        const int il = a2 * 32 + 8 * g + 4 * lh;              // i inside the 64-wide half
                        float v0, v1, v2, v3;
                        if (FP8) {      // codes were multiplied: the product of the two tensor scales comes first, one rounding, then the bias
                            v0 = acc[a][b][4 * g] * alpha + bb[a2][g].x;     v1 = acc[a][b][4 * g + 1] * alpha + bb[a2][g].y;
                            v2 = acc[a][b][4 * g + 2] * alpha + bb[a2][g].z; v3 = acc[a][b][4 * g + 3] * alpha + bb[a2][g].w;
                        } else {
                            v0 = acc[a][b][4 * g] + bb[a2][g].x;     v1 = acc[a][b][4 * g + 1] + bb[a2][g].y;
                            v2 = acc[a][b][4 * g + 2] + bb[a2][g].z; v3 = acc[a][b][4 * g + 3] + bb[a2][g].w;
                        }
                        *reinterpret_cast<uint2*>(scratch + (b * 32 + l32) * EP + il * 2) =
                            tok_ok[b] ? make_uint2(f2bf2(v0, v1), f2bf2(v2, v3)) : make_uint2(0u, 0u);
                    }
            if (EPI == 1 || EPI == 2 || GEN_F || GEN_B) {
#pragma unroll
                for (int q = 0; q < (32 * EP + 1023) / 1024; ++q)
                    if ((q * 64 + lane) * 16 < 32 * EP) *reinterpret_cast<uint4*>(ttile + (q * 64 + lane) * 16) = make_uint4(0, 0, 0, 0);
            }
            wave_lds_sync();
            if (EPI == 0 || ep.store_dense) {
#pragma unroll
                for (int p = 0; p < WN / 8; ++p) {
                    const int row = p * 8 + (lane >> 3), ch = lane & 7;
                    const int j = t0 + row, i = f0 + ch * 8;
                    if (j < Rb && i < Ra) {
                        const uint4 w = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
                        if (EPI == 0 && grp.map_logM) {     // 8 consecutive compact columns = two groups of four hidden units, M apart
                            uint16_t* o = out + (int64_t)j * ldo + ((int64_t)(i >> 2) << grp.map_logM) + 4 * expert_id;
                            *reinterpret_cast<uint2*>(o) = make_uint2(w.x, w.y);
                            *reinterpret_cast<uint2*>(o + ((int64_t)1 << grp.map_logM)) = make_uint2(w.z, w.w);
                        } else {
                            *reinterpret_cast<uint4*>(out + (int64_t)j * ldo + i) = w;
                        }
                    }
                }
            }
            if (EPI == 3) {
                // lane = (token t = lane / 16 + 4 it, group of four compact columns g = lane % 16): eq. (2), then the 2:4 rule
                const int g = lane & 15;
#pragma unroll
                for (int it = 0; it < 16; ++it) {
                    const int t = (lane >> 4) + 4 * it;
                    const uint2 w = *reinterpret_cast<const uint2*>(scratch + t * EP + g * 8);
                    uint32_t nib;
                    const uint32_t v = select24<false>(sqrelu16(w.x & 0xFFFFu), sqrelu16(w.x >> 16), sqrelu16(w.y & 0xFFFFu), sqrelu16(w.y >> 16), nib);
                    uint32_t mw = nib | (row_shl<1>(nib) << 4);            // metadata of 8 groups -> one 32-bit store from every eighth lane
                    mw |= row_shl<2>(mw) << 8;
                    mw |= row_shl<4>(mw) << 16;
                    if (valid && t0 + t < Rb) {
                        *reinterpret_cast<uint32_t*>(ep.vals + (int64_t)(t0 + t) * (F / 2) + (f0 >> 1) + 2 * g) = v;
                        if ((g & 7) == 0) *reinterpret_cast<uint32_t*>(ep.meta + (int64_t)(t0 + t) * (F / 8) + (f0 >> 3) + (g >> 1)) = mw;
                        if (ep.v24) {       // the same packed matrix in the blocked operand layout (A operand of eqs. (3), (7) over the expert's run)
                            *reinterpret_cast<uint32_t*>(ep.v24 + blk_off(t0 + t, (f0 >> 1) + 2 * g, F / 64)) = v;
                            if ((g & 3) == 0) *reinterpret_cast<uint16_t*>(ep.m24 + mblk_off(t0 + t, f0 + 4 * g, F / 64)) = (uint16_t)mw;
                        }
                    }
                }
            }
            if (EPI == 4) {
                // eq. (6) on the compact tile: lane = (token, group of four compact columns); the two kept positions come from the
                // forward pass's metadata, y1 from the stored compact y1c (ep.ykept); dy2 is the bf16-rounded tile in LDS
                const int g = lane & 15;
                uint2 yv[16];
                uint32_t mb[16];
#pragma unroll
                for (int it = 0; it < 16; ++it) {
                    const int t = (lane >> 4) + 4 * it;
                    const bool ok = valid && t0 + t < Rb;
                    yv[it] = ok ? *reinterpret_cast<const uint2*>(ep.ykept + (int64_t)(t0 + t) * F + f0 + 4 * g) : make_uint2(0u, 0u);
                    mb[it] = ok ? ep.meta[(int64_t)(t0 + t) * (F / 8) + (f0 >> 3) + (g >> 1)] : 0x44u;
                }
#pragma unroll
                for (int it = 0; it < 16; ++it) {
                    const int t = (lane >> 4) + 4 * it;
                    const uint2 w = *reinterpret_cast<const uint2*>(scratch + t * EP + g * 8);
                    const uint32_t nib = (mb[it] >> (4 * (g & 1))) & 0xFu, p0 = nib & 3u, p1 = nib >> 2;
                    const uint32_t d0 = ((p0 >> 1) ? w.y : w.x) >> (16 * (p0 & 1)), d1 = ((p1 >> 1) ? w.y : w.x) >> (16 * (p1 & 1));
                    const uint32_t y0 = ((p0 >> 1) ? yv[it].y : yv[it].x) >> (16 * (p0 & 1)), y1 = ((p1 >> 1) ? yv[it].y : yv[it].x) >> (16 * (p1 & 1));
                    const float ya = bf2f(y0 & 0xFFFFu), yb = bf2f(y1 & 0xFFFFu);
                    const uint32_t v = f2bf2(2.0f * bf2f(d0 & 0xFFFFu) * (ya > 0.0f ? ya : 0.0f), 2.0f * bf2f(d1 & 0xFFFFu) * (yb > 0.0f ? yb : 0.0f));
                    if (valid && t0 + t < Rb) {
                        *reinterpret_cast<uint32_t*>(ep.vals + (int64_t)(t0 + t) * (F / 2) + (f0 >> 1) + 2 * g) = v;
                        *reinterpret_cast<uint32_t*>(ep.v24 + blk_off(t0 + t, (f0 >> 1) + 2 * g, F / 64)) = v;
                    }
                }
            }
            if (GEN_F || GEN_B) {
                // Blocks of M = 16 / 32 / 64 columns (Table 5): the wave's 64 tokens x 64 hidden units hold NB = 64 / M whole blocks.
                // Lane = column for the ordered scores and the ranking inside a block; lane = (token, block) for the per-row 2:4 choice,
                // block = lane % NB in every sweep.  The survivors also go into the compacted transposed tile of the weight-gradient GEMM,
                // in the SAME format as for M = 8 (4 rows per group of 8 hidden units + one kept-column mask byte per group): a block of
                // M columns keeps 4, so none of its M / 8 groups keeps more than 4; row = 4 * group + number of kept units below it.
                constexpr int M = 1 << LOGM, NB = 64 >> LOGM;
                const int64_t nblkM = F >> LOGM, blk0 = f0 >> LOGM;
                const int b = lane & (NB - 1);
                uint32_t cb;                                              // the four kept column offsets of block b
                unsigned long long bmask;                                 // and the same as a bit mask over the block's M columns
                if (GEN_F) {
                    float sc = 0.0f;
#pragma unroll 8
                    for (int r = 0; r < WN; ++r)
                        sc = sc + __uint_as_float(sqrelu_hi(*reinterpret_cast<const uint16_t*>(scratch + r * EP + lane * 2)));
                    const int c = lane & (M - 1), base = lane - c;
                    int rank = 0;
#pragma unroll 8
                    for (int k = 0; k < M; ++k) {
                        const float o = __shfl(sc, base + k, 64);
                        rank += (k < c) ? (o >= sc) : ((k > c) ? (o > sc) : 0);
                    }
                    const unsigned long long kept = __ballot(rank < 4);
                    unsigned long long bits = (M == 64) ? kept : ((kept >> base) & ((1ull << (M & 63)) - 1ull));
                    const unsigned long long mine = bits;
                    uint32_t cw = 0;
#pragma unroll
                    for (int n = 0; n < 4; ++n) {
                        cw |= (uint32_t)__builtin_ctzll(bits) << (8 * n);
                        bits &= bits - 1ull;
                    }
                    if (valid && c < M / 8) {          // lane c of a block: its column offsets (c = 0) and the mask byte of its group c of 8 hidden units
                        if (c == 0) *reinterpret_cast<uint32_t*>(ep.colidx + ((int64_t)(t0 >> 6) * nblkM + blk0 + (lane >> LOGM)) * 4) = cw;
                        ep.kmask[(int64_t)(t0 >> 6) * (F >> 3) + (f0 >> 3) + (lane >> LOGM) * (M / 8) + c] = (uint8_t)(mine >> (8 * c));
                    }
                    cb = (uint32_t)__shfl((int)cw, b << LOGM, 64);
                    bmask = (unsigned long long)(uint32_t)__shfl((int)(uint32_t)mine, b << LOGM, 64);
                    if (M == 64) bmask |= (unsigned long long)(uint32_t)__shfl((int)(uint32_t)(mine >> 32), b << LOGM, 64) << 32;
                } else {
                    cb = gpre_cb[h];
                    bmask = (1ull << (cb & 0xFFu)) | (1ull << ((cb >> 8) & 0xFFu)) | (1ull << ((cb >> 16) & 0xFFu)) | (1ull << (cb >> 24));
                }
                const uint32_t q0 = (cb & 0xFFu) * 2, q1 = ((cb >> 8) & 0xFFu) * 2, q2 = ((cb >> 16) & 0xFFu) * 2, q3 = (cb >> 24) * 2;
                const int r_lane = lane >> (6 - LOGM);                    // token of sweep 0; sweep s adds s * M
                // survivors of (token, block): a pair of bf16, or (fp8 operands) a pair of codes
                uint32_t* vals_p = reinterpret_cast<uint32_t*>(ep.vals) + (int64_t)(t0 + r_lane) * (F >> LOGM) + blk0 + b;
                uint16_t* codes_p = ep.vals + (int64_t)(t0 + r_lane) * (F >> LOGM) + blk0 + b;
                float vmax = 0.0f;                                        // fp8: largest survivor magnitude of this half tile
                uint32_t* kept_p = reinterpret_cast<uint32_t*>(ep.ykept) + ((((int64_t)(t0 >> 6) * (F >> 6) + (f0 >> 6)) << 6) + r_lane) * NB + b;
                uint8_t* meta_p = ep.meta + (int64_t)(t0 + r_lane) * (F >> (LOGM + 1)) + ((blk0 + b) >> 1);
                const uint32_t (&pre_m)[GNB] = gpre_m[h];                 // backward: saved metadata and y1 of the sweeps (fetched above)
                const uint32_t (&pre_y)[GNB] = gpre_y[h];
                if (valid) {
#pragma unroll
                    for (int sw = 0; sw < NB; ++sw) {
                        const int t = r_lane + sw * M;
                        const unsigned char* row = scratch + t * EP + (b << LOGM) * 2;
                        uint32_t v, nib;
                        if (GEN_F) {
                            const uint32_t y0 = *reinterpret_cast<const uint16_t*>(row + q0);
                            const uint32_t y1 = *reinterpret_cast<const uint16_t*>(row + q1);
                            const uint32_t y2 = *reinterpret_cast<const uint16_t*>(row + q2);
                            const uint32_t y3 = *reinterpret_cast<const uint16_t*>(row + q3);
                            v = select24<false>(sqrelu16(y0), sqrelu16(y1), sqrelu16(y2), sqrelu16(y3), nib);
                            const uint32_t p0 = nib & 3u, p1 = nib >> 2;
                            const uint32_t k0 = (p0 == 0) ? y0 : (p0 == 1) ? y1 : y2;
                            const uint32_t k1 = (p1 == 3) ? y3 : (p1 == 2) ? y2 : y1;
                            if (FP8) codes_p[(int64_t)sw * M * (F >> LOGM)] = (uint16_t)fp8_enc2(bf2f(v & 0xFFFFu), bf2f(v >> 16), ep.inv_out);
                            else vals_p[(int64_t)sw * M * (F >> LOGM)] = v;
                            kept_p[sw * M * NB] = k0 | (k1 << 16);
                            // two blocks share a metadata byte: neighbours in the lane order (M = 16, 32) or the two halves of the wave tile (M = 64)
                            if (LOGM == 4) {
                                uint32_t mw = nib | (row_shl<1>(nib) << 4);
                                mw |= row_shl<2>(mw) << 8;
                                if (b == 0) *reinterpret_cast<uint16_t*>(meta_p + (int64_t)sw * M * (F >> (LOGM + 1))) = (uint16_t)mw;
                            } else if (LOGM == 5) {
                                const uint32_t mw = nib | (row_shl<1>(nib) << 4);
                                if (b == 0) meta_p[(int64_t)sw * M * (F >> (LOGM + 1))] = (uint8_t)mw;
                            } else {
                                if (h == 0) nib_h0 = nib;
                                else meta_p[0] = (uint8_t)(nib_h0 | (nib << 4));
                            }
                        } else {
                            const uint32_t yk = pre_y[sw];
                            nib = (pre_m[sw] >> (4 * ((blk0 + b) & 1))) & 0xFu;
                            const uint32_t o0 = (cb >> (8 * (nib & 3u))) & 0xFFu, o1 = (cb >> (8 * (nib >> 2))) & 0xFFu;
                            const float d0 = bf2f(*reinterpret_cast<const uint16_t*>(row + o0 * 2));
                            const float d1 = bf2f(*reinterpret_cast<const uint16_t*>(row + o1 * 2));
                            const float ya = bf2f(yk & 0xFFFFu), yb = bf2f(yk >> 16);
                            v = f2bf2(2.0f * d0 * (ya > 0.0f ? ya : 0.0f), 2.0f * d1 * (yb > 0.0f ? yb : 0.0f));
                            if (FP8) codes_p[(int64_t)sw * M * (F >> LOGM)] = (uint16_t)fp8_enc2(bf2f(v & 0xFFFFu), bf2f(v >> 16), ep.inv_out);
                            else vals_p[(int64_t)sw * M * (F >> LOGM)] = v;
                        }
                        if (FP8) vmax = __builtin_fmaxf(vmax, __builtin_fmaxf(__builtin_fabsf(bf2f(v & 0xFFFFu)), __builtin_fabsf(bf2f(v >> 16))));
                        // compact row of a survivor at column o of the block: group (b M + o) / 8 of the half tile, position = kept columns of
                        // that group below o
                        const uint32_t o0 = (cb >> (8 * (nib & 3u))) & 0xFFu, o1 = (cb >> (8 * (nib >> 2))) & 0xFFu;
                        const uint32_t g0 = (uint32_t)(bmask >> (o0 & ~7u)) & 0xFFu, g1 = (uint32_t)(bmask >> (o1 & ~7u)) & 0xFFu;
                        const uint32_t r0 = ((b * (M / 8) + (o0 >> 3)) << 2) + __builtin_popcount(g0 & ((1u << (o0 & 7u)) - 1u));
                        const uint32_t r1 = ((b * (M / 8) + (o1 >> 3)) << 2) + __builtin_popcount(g1 & ((1u << (o1 & 7u)) - 1u));
                        *reinterpret_cast<uint16_t*>(ttile + r0 * EP + t * 2) = (uint16_t)(v & 0xFFFFu);
                        *reinterpret_cast<uint16_t*>(ttile + r1 * EP + t * 2) = (uint16_t)(v >> 16);
                    }
                }
                if (FP8) vmax_tile = __builtin_fmaxf(vmax_tile, vmax);
                wave_lds_sync();
#pragma unroll
                for (int q = 0; q < 4; ++q) {          // 2 groups of 16 compact rows x 2 chunks of 32 tokens, 1 KB each
                    const int fr = (q >> 1) * 16 + (lane >> 2), tc = (q & 1) * 32 + (lane & 3) * 8;
                    const uint4 w = *reinterpret_cast<const uint4*>(ttile + fr * EP + tc * 2);
                    if (FP8 && ep.at_fp8) {     // fp8 weight gradients: codes, as in the M = 8 epilogues below
                        if (valid)
                            *reinterpret_cast<uint2*>(ep.at + blk_off(f0 / 2 + fr, (t0 + tc) / 2, tok_ld / 64)) =
                                make_uint2(fp8_enc2(bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), ep.inv_out) | (fp8_enc2(bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16), ep.inv_out) << 16),
                                           fp8_enc2(bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), ep.inv_out) | (fp8_enc2(bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16), ep.inv_out) << 16));
                    } else if (valid) {
                        *reinterpret_cast<uint4*>(ep.at + blk_off(f0 / 2 + fr, t0 + tc, tok_ld / 32)) = w;
                    }
                }
            }
            if (EPI == 1 || EPI == 2) {
                const int bl = lane & 7;                                  // column block handled in the per-row pass
                const int64_t blk_g = (f0 >> 3) + bl;
                uint32_t cw;                                              // the four kept column offsets of block bl
                if (EPI == 1) {
                    // column scores: lane = column, strict ascending-row fp32 sum of y2 = bf16(max(y1, 0)^2)
                    float sc = 0.0f;
#pragma unroll 8
                    for (int r = 0; r < WN; ++r)
                        sc = sc + __uint_as_float(sqrelu_hi(*reinterpret_cast<const uint16_t*>(scratch + r * EP + lane * 2)));
                    int rank = 0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const float o = __shfl(sc, (lane & ~7) + k, 64);
                        rank += (k < bl) ? (o >= sc) : ((k > bl) ? (o > sc) : 0);
                    }
                    const unsigned long long kept = __ballot(rank < 4);
                    const uint32_t bits = (uint32_t)(kept >> (lane & ~7)) & 0xFFu;
                    uint32_t mine = 0, n = 0;
#pragma unroll
                    for (int c = 0; c < 8; ++c)
                        if ((bits >> c) & 1u) { mine |= (uint32_t)c << (8 * n); ++n; }
                    if (valid && bl == 0)
                    {
                        *reinterpret_cast<uint32_t*>(ep.colidx + ((int64_t)(t0 >> 6) * nblk + (f0 >> 3) + (lane >> 3)) * 4) = mine;
                        ep.kmask[(int64_t)(t0 >> 6) * nblk + (f0 >> 3) + (lane >> 3)] = (uint8_t)bits;
                    }
                    cw = (uint32_t)__shfl((int)mine, bl * 8, 64);
                    if (FP8 && ep.cixt) {       // fp8 form: 16 words per 128 hidden units, word q = (h, p); this half of them (64 hidden units) fills two bytes
                        const int q = lane & 15, hq = q >> 3, pq = q & 7, hf = (f0 >> 6) & 1;
                        const uint32_t b0 = ((uint32_t)__shfl((int)mine, (4 * hq + (pq >> 2)) * 8, 64) >> (8 * (pq & 3))) & 0xFFu;
                        const uint32_t b1 = ((uint32_t)__shfl((int)mine, (4 * hq + 2 + (pq >> 2)) * 8, 64) >> (8 * (pq & 3))) & 0xFFu;
                        if (valid && lane < 16)
                            *reinterpret_cast<uint16_t*>(ep.cixt + cixt8_off(t0 >> 6, f0 >> 7, tok_ld >> 6) + q * 4 + 2 * hf) = (uint16_t)(b0 | (b1 << 8));
                    }
                    if (!FP8 && ep.cixt) {      // the same offsets regrouped for the transposing reads of gemm_vnm8.hip: word q = (h, r), byte j
                        const int q = lane & 7, hq = q >> 2, rq = q & 3;
                        uint32_t dw = 0;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            dw |= (((uint32_t)__shfl((int)mine, (4 * (j >> 1) + (j & 1) + 2 * hq) * 8, 64) >> (8 * rq)) & 0xFFu) << (8 * j);
                        if (valid && lane < 8) *reinterpret_cast<uint32_t*>(ep.cixt + cixt_off(t0 >> 6, f0 >> 6, tok_ld >> 6) + q * 4) = dw;
                    }
                } else {
                    cw = pre_cw[h];
                }
                // per-row pass: lane = (column block bl, token t); 8 tokens per sweep, 8 sweeps
                uint32_t* vals_p = reinterpret_cast<uint32_t*>(ep.vals) + ((int64_t)(t0 + (lane >> 3)) * (F / 4) + blk_g * 2) / 2;
                uint32_t* kept_p = reinterpret_cast<uint32_t*>(ep.ykept) + ykept_off(t0 + (lane >> 3), blk_g, F);
                uint8_t* meta_p = ep.meta + (int64_t)(t0 + (lane >> 3)) * (F / 16) + (blk_g >> 1);
                // operands of eq. (3) / eq. (7) on the V:2:8 kernel (gemm_vnm8.hip); sweep it: + (it / 4) 32-token groups + 8 (it % 4) tokens
                uint32_t* vcb_p = FP8 ? nullptr : reinterpret_cast<uint32_t*>(ep.vcb + vcb_off(t0 + (lane >> 3), blk_g, F));
                uint8_t* vcb8_p = FP8 ? reinterpret_cast<uint8_t*>(ep.vcb) + vcb8_off(t0 + (lane >> 3), blk_g, F) : nullptr;   // (the lane of block 0 stores its row's 8 pairs of codes)
                uint8_t* mcb_p = FP8 ? ep.mcb + mcb8_off(t0 + (lane >> 3), f0 >> 6, F) : ep.mcb + mcb_off(t0 + (lane >> 3), f0 >> 6, F);
                const uint32_t c0 = (cw & 0xFFu) * 2, c1 = ((cw >> 8) & 0xFFu) * 2, c2 = ((cw >> 16) & 0xFFu) * 2, c3 = (cw >> 24) * 2;
                const uint32_t (&pre_m)[8] = pre_m_all[h];                  // EPI 2: saved metadata and y1 of the 8 sweeps
                const uint32_t (&pre_y)[8] = pre_y_all[h];
                float vmax = 0.0f;                                         // fp8: largest survivor magnitude of this half tile
                if (valid) {
#pragma unroll
                    for (int it = 0; it < 8; ++it) {
                        const int t = (lane >> 3) + 8 * it;
                        const unsigned char* row = scratch + t * EP + bl * 16;
                        uint32_t v, nib;
                        if (EPI == 1) {
                            const uint32_t y0 = *reinterpret_cast<const uint16_t*>(row + c0);
                            const uint32_t y1 = *reinterpret_cast<const uint16_t*>(row + c1);
                            const uint32_t y2 = *reinterpret_cast<const uint16_t*>(row + c2);
                            const uint32_t y3 = *reinterpret_cast<const uint16_t*>(row + c3);
                            v = select24<false>(sqrelu16(y0), sqrelu16(y1), sqrelu16(y2), sqrelu16(y3), nib);
                            const uint32_t p0 = nib & 3u, p1 = nib >> 2;
                            const uint32_t k0 = (p0 == 0) ? y0 : (p0 == 1) ? y1 : y2;
                            const uint32_t k1 = (p1 == 3) ? y3 : (p1 == 2) ? y2 : y1;
                            if (FP8) {  // canonical values are the survivors' codes [T, F / 4]
                                if (ep.vals)
                                    reinterpret_cast<uint16_t*>(ep.vals)[(int64_t)(t0 + t) * (F / 8) + blk_g] = (uint16_t)fp8_enc2(bf2f(v & 0xFFFFu), bf2f(v >> 16), ep.inv_out);
                            } else if (ep.vals)       // (lean form: no canonical copy; the 2:4 view and the compact transpose carry the values)
                                vals_p[(int64_t)it * 8 * (F / 8)] = v;
                            kept_p[it * 64] = k0 | (k1 << 16);
                            // metadata bytes of the row's 8 blocks -> one 32-bit store from the lane of block 0
                            uint32_t mw = nib | (row_shl<1>(nib) << 4);
                            mw |= row_shl<2>(mw) << 8;
                            mw |= row_shl<4>(mw) << 16;
                            if (bl == 0) *reinterpret_cast<uint32_t*>(meta_p + (int64_t)it * 8 * (F / 16)) = mw;
                            if (ep.mcb && bl == 0) *reinterpret_cast<uint32_t*>(mcb_p + it * (FP8 ? 64 : 32)) = mw;
                        } else {
                            const uint32_t mb = pre_m[it];
                            const uint32_t yk = pre_y[it];
                            nib = (mb >> (4 * (bl & 1))) & 0xFu;
                            const uint32_t q0 = (cw >> (8 * (nib & 3u))) & 0xFFu, q1 = (cw >> (8 * (nib >> 2))) & 0xFFu;
                            const float d0 = bf2f(*reinterpret_cast<const uint16_t*>(row + q0 * 2));
                            const float d1 = bf2f(*reinterpret_cast<const uint16_t*>(row + q1 * 2));
                            const float ya = bf2f(yk & 0xFFFFu), yb = bf2f(yk >> 16);
                            const float ga = 2.0f * d0 * (ya > 0.0f ? ya : 0.0f), gb = 2.0f * d1 * (yb > 0.0f ? yb : 0.0f);
                            v = f2bf2(ga, gb);
                            if (ep.vals) vals_p[(int64_t)it * 8 * (F / 8)] = v;
                        }
                        if (FP8) vmax = __builtin_fmaxf(vmax, __builtin_fmaxf(__builtin_fabsf(bf2f(v & 0xFFFFu)), __builtin_fabsf(bf2f(v >> 16))));
                        if (!FP8 && ep.vcb) vcb_p[(int64_t)(it >> 2) * (F >> 6) * 256 + (it & 3) * 64] = v;
                        if (FP8 && ep.vcb) {    // the survivors' codes: the row's 8 pairs gathered into the lane of block 0, one 16-byte store
                            const uint32_t q2 = fp8_enc2(bf2f(v & 0xFFFFu), bf2f(v >> 16), ep.inv_out);
                            const uint32_t w2 = q2 | (row_shl<1>(q2) << 16);
                            const uint4 w8 = make_uint4(w2, row_shl<2>(w2), row_shl<4>(w2), row_shl<6>(w2));
                            if (bl == 0) *reinterpret_cast<uint4*>(vcb8_p + (int64_t)(it >> 2) * (F >> 7) * 1024 + (it & 3) * 256) = w8;
                        }
                        // transposed tile for the weight-gradient GEMM, compacted to the block's four kept hidden units:
                        // row = 4 * block + position among the kept units, column = token
                        *reinterpret_cast<uint16_t*>(ttile + (bl * 4 + (nib & 3u)) * EP + t * 2) = (uint16_t)(v & 0xFFFFu);
                        *reinterpret_cast<uint16_t*>(ttile + (bl * 4 + (nib >> 2)) * EP + t * 2) = (uint16_t)(v >> 16);
                    }
                }
                if (FP8) vmax_tile = __builtin_fmaxf(vmax_tile, vmax);
                wave_lds_sync();
#pragma unroll
                for (int q = 0; q < 4; ++q) {          // 2 groups of 16 compact rows x 2 chunks of 32 tokens, 1 KB each
                    const int fr = (q >> 1) * 16 + (lane >> 2), tc = (q & 1) * 32 + (lane & 3) * 8;
                    const uint4 w = *reinterpret_cast<const uint4*>(ttile + fr * EP + tc * 2);
                    if (FP8 && ep.at_fp8) {     // fp8 weight gradients: the compact transposed survivors leave as codes (a 64-token block = one 64-byte chunk)
                        if (valid)
                            *reinterpret_cast<uint2*>(ep.at + blk_off(f0 / 2 + fr, (t0 + tc) / 2, tok_ld / 64)) =
                                make_uint2(fp8_enc2(bf2f(w.x & 0xFFFFu), bf2f(w.x >> 16), ep.inv_out) | (fp8_enc2(bf2f(w.y & 0xFFFFu), bf2f(w.y >> 16), ep.inv_out) << 16),
                                           fp8_enc2(bf2f(w.z & 0xFFFFu), bf2f(w.z >> 16), ep.inv_out) | (fp8_enc2(bf2f(w.w & 0xFFFFu), bf2f(w.w >> 16), ep.inv_out) << 16));
                    } else if (valid) {
                        *reinterpret_cast<uint4*>(ep.at + blk_off(f0 / 2 + fr, t0 + tc, tok_ld / 32)) = w;
                    }
                }
            }
            wave_lds_sync();
        }
        if (FP8 && EPI != 0 && ep.amax) note_amax_slots_seen(ep.amax, vmax_tile, amax_seen);
    } else {
        constexpr int EP = WN * 2 + 16;
        constexpr int CH = WN / 8;
        unsigned char* scratch = smem + wave * (32 * EP);
        // destination rows of the lane's 16 stores, looked up before the first store (loads and stores share one in-order counter: a look-up
        // between two stores would wait for the earlier one)
        int32_t io_map[FM][32 * CH / 64];
        if (grp.out_row_map) {
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int p = 0; p < 32 * CH / 64; ++p) {
                    const int i = i0 + wm * WM + a * 32 + (lane + 64 * p) / CH;
                    io_map[a][p] = i < Ra ? grp.out_row_map[i] : -1;
                }
        }
#pragma unroll
        for (int a = 0; a < FM; ++a) {
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r >> 2) + 4 * lh + (r & 3);
                    *reinterpret_cast<uint16_t*>(scratch + row * EP + (b * 32 + l32) * 2) = (uint16_t)f2bf(FP8 ? acc[a][b][r] * alpha : acc[a][b][r]);
                }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < 32 * CH / 64; ++p) {
                const int e = lane + 64 * p, row = e / CH, ch = e % CH;
                const int i = i0 + wm * WM + a * 32 + row, j = j0 + wn * WN + ch * 8;
                if (i < Ra && j < Rb) {
                    int64_t io = grp.map_logM ? ((int64_t)(i >> 2) << grp.map_logM) + 4 * expert_id + (i & 3) : i;
                    if (grp.out_row_map) io = io_map[a][p];
                    if (io >= 0) *reinterpret_cast<uint4*>(out + io * ldo + j) = *reinterpret_cast<const uint4*>(scratch + row * EP + ch * 16);
                }
            }
            __syncthreads();
        }
    }
}

// Grid of a launch: one workgroup per 256 x 256 output tile; grouped: per expert, over its token segment.
static unsigned grid_tiles(int tiles_m, int tiles_n, const GemmGroup& g) {
    if (g.n == 0) return (unsigned)(tiles_m * tiles_n);
    if (g.role == 2) return (unsigned)(g.n * tiles_m * tiles_n);
    if (g.seg_dev) return (unsigned)(((g.cap_rows + 255) / 256 + g.n) * (g.role == 0 ? tiles_n : tiles_m));   // worst case over all run lengths
    int tok_tiles = 0;
    for (int e = 0; e < g.n; ++e) tok_tiles += (g.seg[e + 1] - g.seg[e] + 255) / 256;
    return (unsigned)(tok_tiles * (g.role == 0 ? tiles_n : tiles_m));
}

template <bool SPARSE>
static hipError_t launch_v2(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t Ra,
                            int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, int blocked, hipStream_t s,
                            const GemmGroup* grp) {
    const int tiles_m = (int)((Ra + 255) / 256), tiles_n = (int)((Rb + 255) / 256);
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n > GemmGroup::kMaxExperts) return hipErrorInvalidValue;
    if (g.n && g.role == 2 ? (SPARSE || blocked) : (g.n && !blocked)) return hipErrorInvalidValue;   // role 2: dense row-major only; roles 0, 1: blocked only
    const unsigned tiles = grid_tiles(tiles_m, tiles_n, g);
    if (tiles == 0) return hipSuccess;
    dim3 grid(tiles);
    const VnmEpilogue none;
#define SFFN_LAUNCH(ICONTIG, BLK) hipLaunchKernelGGL((gemm_nt_v2_kernel<SPARSE, ICONTIG, 0, BLK>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, \
                                                   (int)Ra, (int)Rb, (int)K, out, ldo, tiles_m, tiles_n, none, g)
    if (blocked) {      // fused step: only eqs. (3), (7) come here (structured-sparse A, tokens along i, j-contiguous output)
        if constexpr (SPARSE) { if (out_i_contig) return hipErrorInvalidValue; SFFN_LAUNCH(false, true); }
        else return hipErrorInvalidValue;
    } else if (out_i_contig) SFFN_LAUNCH(true, false);
    else SFFN_LAUNCH(false, false);
#undef SFFN_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemm_nt(int sparse_a, const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias,
                             int64_t Ra, int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s,
                             const GemmGroup* grp) {
    if (sparse_a) return grp ? hipErrorInvalidValue : launch_v2<true>(a_vals, a_meta, B, bias, Ra, Rb, K, out_i_contig, out, ldo, 0, s, nullptr);
    return launch_v2<false>(a_vals, a_meta, B, bias, Ra, Rb, K, out_i_contig, out, ldo, 0, s, grp);
}

hipError_t launch_spmm24_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* Bq, const float* bias, float alpha, int64_t Ra, int64_t Rb,
                             int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s) {
    if (K % 128 != 0) return hipErrorInvalidValue;
    const int tiles_m = (int)((Ra + 255) / 256), tiles_n = (int)((Rb + 255) / 256);
    const VnmEpilogue none;
    const GemmGroup g;
    dim3 grid((unsigned)(tiles_m * tiles_n));
    // the kernel addresses its operands in 2-byte units: K / 2 of them per B row, K / 4 per A row
    const uint16_t* a = reinterpret_cast<const uint16_t*>(a_codes);
    const uint16_t* b = reinterpret_cast<const uint16_t*>(Bq);
    if (out_i_contig)
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 0, false, true>), grid, dim3(512), 0, s, a, a_meta, b, bias, (int)Ra, (int)Rb, (int)(K / 2), out, ldo,
                           tiles_m, tiles_n, none, g, alpha);
    else
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, false, 0, false, true>), grid, dim3(512), 0, s, a, a_meta, b, bias, (int)Ra, (int)Rb, (int)(K / 2), out, ldo,
                           tiles_m, tiles_n, none, g, alpha);
    return hipGetLastError();
}

hipError_t launch_gemm_fp8_blocked(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* Bq, const float* bias, float alpha, int64_t Ra,
                                   int64_t Rb, int64_t K, uint16_t* out, int64_t ldo, const VnmEpilogue* ep, hipStream_t s, const GemmGroup* grp) {
    if (K % 128 != 0 || !ep || (ep->mode != 1 && ep->mode != 2 && ep->mode != 5 && ep->mode != 6)) return hipErrorInvalidValue;
    if (ep->mode >= 5 && (ep->logM < 4 || ep->logM > 6)) return hipErrorInvalidValue;
    const int tiles_m = (int)((Ra + 255) / 256), tiles_n = (int)((Rb + 255) / 256);
    const VnmEpilogue e = *ep;
    const GemmGroup g = grp ? *grp : GemmGroup();
    // grouped: the tokens are the j rows (role 1: A = the expert's packed weights)
    if (g.n && (g.n > GemmGroup::kMaxExperts || g.role != 1 || g.seg_dev)) return hipErrorInvalidValue;
    const unsigned tiles = grid_tiles(tiles_m, tiles_n, g);
    if (tiles == 0) return hipSuccess;
    dim3 grid(tiles);
    const uint16_t* a = reinterpret_cast<const uint16_t*>(a_codes);
    const uint16_t* b = reinterpret_cast<const uint16_t*>(Bq);
#define SFFN_F8(ICONTIG, E) hipLaunchKernelGGL((gemm_nt_v2_kernel<true, ICONTIG, E, true, true>), grid, dim3(512), 0, s, a, a_meta, b, bias, (int)Ra, (int)Rb, \
                                              (int)(K / 2), out, ldo, tiles_m, tiles_n, e, g, alpha)
    if (ep->mode == 1) SFFN_F8(true, 1);
    else if (ep->mode == 2) SFFN_F8(true, 2);
    else if (ep->mode == 5) { if (ep->logM == 4) SFFN_F8(true, 20); else if (ep->logM == 5) SFFN_F8(true, 21); else SFFN_F8(true, 22); }
    else                    { if (ep->logM == 4) SFFN_F8(true, 36); else if (ep->logM == 5) SFFN_F8(true, 37); else SFFN_F8(true, 38); }
#undef SFFN_F8
    return hipGetLastError();
}

hipError_t launch_spmm_blocked(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t Ra, int64_t Rb,
                               int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp) {
    return launch_v2<true>(a_vals, a_meta, B, bias, Ra, Rb, K, out_i_contig, out, ldo, 1, s, grp);
}

hipError_t launch_gemm_vnm_epilogue(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t F,
                                    int64_t T, int64_t K, uint16_t* out, const VnmEpilogue& ep, hipStream_t s, const GemmGroup* grp) {
    const int tiles_m = (int)((F + 255) / 256), tiles_n = (int)((T + 255) / 256);
    const GemmGroup g = grp ? *grp : GemmGroup();
    if (g.n && (g.n > GemmGroup::kMaxExperts || g.role != 1)) return hipErrorInvalidValue;
    const unsigned tiles = grid_tiles(tiles_m, tiles_n, g);
    if (tiles == 0) return hipSuccess;
    dim3 grid(tiles);
#define SFFN_EPI(E) hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, E, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F, \
                                      tiles_m, tiles_n, ep, g)
    if (ep.mode == 5 || ep.mode == 6) {     // wide blocks: forward / backward epilogue for M = 16, 32, 64
        if (ep.logM < 4 || ep.logM > 6) return hipErrorInvalidValue;
        if (ep.mode == 5) { if (ep.logM == 4) SFFN_EPI(20); else if (ep.logM == 5) SFFN_EPI(21); else SFFN_EPI(22); }
        else              { if (ep.logM == 4) SFFN_EPI(36); else if (ep.logM == 5) SFFN_EPI(37); else SFFN_EPI(38); }
        return hipGetLastError();
    }
#undef SFFN_EPI
    if (ep.mode == 0)       // no V:N:M work: the dense output only
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 0, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F,
                           tiles_m, tiles_n, ep, g);
    else if (ep.mode == 4)
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 4, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F,
                           tiles_m, tiles_n, ep, g);
    else if (ep.mode == 3)
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 3, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F,
                           tiles_m, tiles_n, ep, g);
    else if (ep.mode == 1)
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 1, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F,
                           tiles_m, tiles_n, ep, g);
    else
        hipLaunchKernelGGL((gemm_nt_v2_kernel<true, true, 2, true>), grid, dim3(512), 0, s, a_vals, a_meta, B, bias, (int)F, (int)T, (int)K, out, F,
                           tiles_m, tiles_n, ep, g);
    return hipGetLastError();
}

}  // namespace sffn
